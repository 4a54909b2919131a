"""GPU parity of the per-token activation quantisation kernel (Sec. 6 of the paper) against
the CPU oracle: INT8 codes and FP32 scales must match bit for bit (every step is one
correctly rounded FP32 operation on both sides), and the chain quantise -> W4A8 GEMM must
reproduce the oracle chain."""
import sys

import numpy as np
import pytest

from oracle import lqq_oracle as O
from paper_2509_01229_amd import api
from paper_2509_01229_amd import workloads as WL

import gpu_helpers as H

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _run(X16, smooth):
    import torch

    dX = torch.from_numpy(X16).cuda()
    ds = torch.from_numpy(smooth).cuda() if smooth is not None else None
    q, s = api.w4a8_quantize_activations(dX, ds)
    torch.cuda.synchronize()
    return q.cpu().numpy(), s.cpu().numpy()


SHAPES = [
    (1, 8), (1, 256), (7, 4096), (33, 11008), (16, 8192), (3, 16384),  # register-resident tokens
    (2, 16392), (5, 28672), (3, 32768),                               # register-resident on 1024 threads, ragged tail
    (2, 32776), (2, 131072),                                          # two-pass tokens
    (300, 512),                                                       # many short tokens
]


@pytest.mark.parametrize("M,K", SHAPES)
@pytest.mark.parametrize("with_smooth", [False, True])
def test_quantize_activations_bit_exact(M, K, with_smooth):
    _say(f"actquant M={M} K={K} smooth={with_smooth}")
    X16 = WL.make_activations_f16(M, K, outlier_frac=0.001, seed=M + K)
    smooth = WL.make_smooth(K, seed=K) if with_smooth else None
    q_ref, s_ref = O.quantize_activations(X16, smooth)
    q, s = _run(X16, smooth)
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32)), "per-token scales differ"
    assert np.array_equal(q, q_ref), f"{np.count_nonzero(q != q_ref)} codes differ"


@pytest.mark.parametrize("M,K", [(1027, 2048), (2051, 4096), (4096, 512), (1027, 12288), (600, 16384)])
def test_several_tokens_per_block(M, K):
    """From 1024 tokens on a block quantises 2 or 4 consecutive tokens (ragged last block) and
    shares the reciprocals of the smooth scales between them."""
    _say(f"actquant rows per block M={M} K={K}")
    X16 = WL.make_activations_f16(M, K, outlier_frac=0.001, seed=M)
    smooth = WL.make_smooth(K, seed=K + 1)
    q_ref, s_ref = O.quantize_activations(X16, smooth)
    q, s = _run(X16, smooth)
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32)), "per-token scales differ"
    assert np.array_equal(q, q_ref), f"{np.count_nonzero(q != q_ref)} codes differ"


def test_smooth_scales_outside_the_short_division_range():
    """Smooth scales below 2^-40 or above 2^40 (and FP32 subnormals) take the full IEEE
    division; scales at the edges of the range and powers of two take the short one."""
    _say("actquant extreme smooth scales")
    K = 2048
    rng = np.random.default_rng(5)
    X16 = (rng.standard_normal((5, K)) * 3).astype(np.float16)
    X16[1] = (rng.standard_normal(K) * 1e-4).astype(np.float16)       # FP16 subnormals among them
    smooth = np.exp2(rng.integers(-45, 46, size=K)).astype(np.float32)
    smooth[::7] *= np.float32(1.2345)
    smooth[3] = np.float32(2.0 ** -40)
    smooth[4] = np.float32(2.0 ** 40)
    smooth[5] = np.float32(1e-38)      # the quotients overflow or are huge: codes saturate
    smooth[6] = np.float32(1e-44)      # FP32 subnormal
    X16[:3, 5:7] = 0                   # tokens 0..2 stay finite; 3 and 4 overflow (unspecified codes)
    with np.errstate(over="ignore", invalid="ignore"):
        q_ref, s_ref = O.quantize_activations(X16, smooth)
    finite = np.isfinite(s_ref)
    assert finite[:3].all() and not finite[3:].any()
    q, s = _run(X16, smooth)
    assert np.array_equal(s.view(np.uint32)[finite], s_ref.view(np.uint32)[finite])
    assert np.array_equal(q[finite], q_ref[finite])
    # and a moderate range, where every token stays finite and every thread takes the short division
    smooth = np.exp2(rng.uniform(-12, 12, size=K)).astype(np.float32)
    q_ref, s_ref = O.quantize_activations(X16, smooth)
    q, s = _run(X16, smooth)
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(q, q_ref)


def test_quantize_activations_edge_values():
    _say("actquant edge values")
    K = 512
    X = np.zeros((6, K), dtype=np.float16)
    X[1, 5] = 65504.0                       # largest FP16
    X[1, 6] = -65504.0
    X[1, 7] = 257.9                         # rounds to a small code
    X[2, :] = 6e-8                          # FP16 subnormals only
    X[3, :] = np.float16(-1.0)              # constant token
    X[4, ::2] = 0.5
    X[4, 1::2] = 1.0                        # exact ties: 0.5 / (1/127) = 63.5 -> 64
    X[5, 3] = 1.0                           # one-hot
    q_ref, s_ref = O.quantize_activations(X)
    q, s = _run(X, None)
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(q, q_ref)
    assert s[0] == 1.0 and not q[0].any()
    assert q[1, 5] == 127 and q[1, 6] == -127 and q[3].tolist() == [-127] * K
    assert q[4, 0] == 64 and q[4, 1] == 127


def test_quantize_activations_near_ties():
    """Tokens whose quotients sit on or next to rounding ties: x = k/2 * s for all k, and the
    FP16 neighbours of those values."""
    _say("actquant near ties")
    K = 512
    rows = []
    for amax in (1.0, 127.0, 0.3333, 100.0):
        base = (np.arange(K) % 255 - 127).astype(np.float64) * 0.5 * (amax / 127.0)
        for bump in (0, 1, -1):
            x = base.astype(np.float16)
            x = (x.view(np.int16) + np.int16(bump)).view(np.float16) if bump else x
            x[0] = amax
            rows.append(np.nan_to_num(x, nan=0.0, posinf=0.0, neginf=0.0))
    X = np.stack(rows).astype(np.float16)
    for smooth in (None, WL.make_smooth(K, seed=3)):
        q_ref, s_ref = O.quantize_activations(X, smooth)
        q, s = _run(X, smooth)
        assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32))
        assert np.array_equal(q, q_ref), f"{np.count_nonzero(q != q_ref)} codes differ"


def test_empty_and_bad_arguments():
    import torch

    X0 = torch.empty((0, 256), dtype=torch.float16, device="cuda")
    q, s = api.w4a8_quantize_activations(X0)
    assert tuple(q.shape) == (0, 256) and tuple(s.shape) == (0,)
    with pytest.raises(api.LiquidGemmError):
        api.w4a8_quantize_activations(torch.zeros((2, 12), dtype=torch.float16, device="cuda"))
    with pytest.raises(TypeError):
        api.w4a8_quantize_activations(torch.zeros((2, 16), dtype=torch.float32, device="cuda"))
    with pytest.raises(ValueError):
        api.w4a8_quantize_activations(torch.zeros((2, 16), dtype=torch.float16, device="cuda"),
                                      torch.ones(8, dtype=torch.float32, device="cuda"))


def test_quantize_then_gemm_matches_oracle_chain():
    import torch

    M, N, K, g = 24, 256, 1024, 64
    _say("actquant -> gemm chain")
    P = H.Problem(N, K, g, seed=21)
    X16 = WL.make_activations_f16(M, K, outlier_frac=0.002, seed=22)
    smooth = WL.make_smooth(K, seed=23)
    q_ref, s_ref = O.quantize_activations(X16, smooth)
    ACC_ref, _ = P.oracle_gemm(q_ref, s_ref)
    ref64 = O.scale_epilogue_f64(ACC_ref, s_ref, P.oracle_full()["s_w"])
    dq, ds = api.w4a8_quantize_activations(torch.from_numpy(X16).cuda(), torch.from_numpy(smooth).cuda())
    Y = api.w4a8_gemm(dq, ds, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
    ACC = api.w4a8_gemm_i32(dq, P.d_packed, P.d_gparams, N, K, g)
    torch.cuda.synchronize()
    assert np.array_equal(ACC.cpu().numpy(), ACC_ref)
    H.assert_fp16_close(Y.cpu().numpy(), ref64, "chain")
