"""GPU parity of the W8A8 reference kernel (the baseline without dequantisation of Sec. 3.2 /
7.3) against the oracle, element by element, and against the W4A8 path on the dequantised
LiquidQuant weights, where both must give the same integers."""
import sys

import numpy as np
import pytest

from oracle import lqq_oracle as O
from paper_2509_01229_amd import api
from paper_2509_01229_amd import workloads as WL

import gpu_helpers as H
import inputs as I

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


CASES = [
    # M, N, K
    (8, 64, 256),          # smallest legal problem
    (77, 448, 768),        # ragged M over one tile, N tail (inactive waves), 6 stages
    (200, 256, 256),       # 2 stages only; last row tile with 72 rows
    (300, 320, 1792),      # last row tile with 44 rows (two-fragment form), 14 stages
    (513, 512, 1024),      # 5 row tiles, the last with one row
]


@pytest.mark.parametrize("M,N,K", CASES)
def test_w8a8_matches_oracle(M, N, K):
    import torch

    _say(f"w8a8 M={M} N={N} K={K}")
    rng = np.random.default_rng(M + N + K)
    W = WL.make_weights(N, K, 0.02, rng=rng)
    Q_i8, s_w = O.level1_quantize(W)
    X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=M)
    ACC_ref, _ = O.w8a8_gemm(X, s_x, Q_i8, s_w)
    ref64 = O.scale_epilogue_f64(ACC_ref, s_x, s_w)
    dW = torch.from_numpy(api.w8a8_pack_weights(Q_i8)).cuda()
    dX, dsx, dsw = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda(), torch.from_numpy(s_w).cuda()
    Y, ACC = api.w8a8_gemm(dX, dsx, dW, dsw, N, K, want_y=True, want_acc=True)
    torch.cuda.synchronize()
    assert np.array_equal(ACC.cpu().numpy(), ACC_ref), "INT32 accumulators differ"
    H.assert_fp16_close(Y.cpu().numpy(), ref64, "w8a8")
    # extreme weights and activations: the full INT8 range on both sides
    Wx = rng.integers(-128, 128, size=(N, K), dtype=np.int64).astype(np.int8)
    Xx = rng.integers(-128, 128, size=(M, K), dtype=np.int64).astype(np.int8)
    ACCx = api.w8a8_gemm(torch.from_numpy(Xx).cuda(), None, torch.from_numpy(api.w8a8_pack_weights(Wx)).cuda(),
                         None, N, K, want_y=False, want_acc=True)
    torch.cuda.synchronize()
    assert np.array_equal(ACCx.cpu().numpy(), O.matmul_i64(Xx, Wx))


def test_w8a8_on_dequantised_weights_equals_w4a8():
    """W8A8 on Wd = dequant(LQQ codes) and W4A8 on the codes compute the same integers."""
    import torch

    M, N, K, g = 260, 512, 2048, 64
    _say("w8a8 vs w4a8 on the same dequantised weights")
    P = H.Problem(N, K, g, seed=9)
    X, s_x = I.make_activations(M, K, outlier_frac=0.002, seed=10)
    Wd = api.w4a8_dequant_dump(P.d_packed, P.d_gparams, N, K, g)
    torch.cuda.synchronize()
    Wd_ref, _ = P.oracle_wd()
    assert np.array_equal(Wd.cpu().numpy(), Wd_ref)
    dW8 = torch.from_numpy(api.w8a8_pack_weights(Wd.cpu().numpy())).cuda()
    dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
    Y8, ACC8 = api.w8a8_gemm(dX, dsx, dW8, P.d_w_scales, N, K, want_y=True, want_acc=True)
    Y4 = api.w4a8_gemm(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
    ACC4 = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g)
    torch.cuda.synchronize()
    ACC_ref, _ = P.oracle_gemm(X, s_x)
    assert np.array_equal(ACC8.cpu().numpy(), ACC_ref)
    assert np.array_equal(ACC4.cpu().numpy(), ACC_ref)
    assert np.array_equal(Y8.cpu().numpy().view(np.uint16), Y4.cpu().numpy().view(np.uint16))


def test_w8a8_rejects_bad_arguments():
    import torch

    with pytest.raises(api.LiquidGemmError):
        api.w8a8_pack_weights(np.zeros((100, 256), dtype=np.int8))      # N % 64 != 0
    X = torch.zeros((4, 256), dtype=torch.int8, device="cuda")
    Wp = torch.zeros(64 * 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(api.LiquidGemmError):
        api.w8a8_gemm(X, None, Wp, None, 64, 256, want_y=False, want_acc=False)   # no output
    with pytest.raises(ValueError):
        api.w8a8_gemm(X, None, Wp[:100], None, 64, 256, want_y=False, want_acc=True)
    E = torch.zeros((0, 256), dtype=torch.int8, device="cuda")
    assert tuple(api.w8a8_gemm(E, None, Wp, None, 64, 256, want_y=False, want_acc=True).shape) == (0, 64)
