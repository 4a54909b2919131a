"""GPU parity of the grouped (mixture-of-experts) W4A8 GEMM against the CPU oracle: INT32
accumulators bit for bit, FP16 outputs within one ulp, for mixes of expert sizes that reach
all three kernel families, empty experts, ragged tails, and the limits of the interface."""
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


class Experts:
    def __init__(self, E, N, K, g, seed):
        import torch

        self.E, self.N, self.K, self.g = E, N, K, g
        Ws = [WL.make_weights(N, K, 0.02, seed=seed + e) for e in range(E)]
        packs = [api.liquidquant_pack_weights(W, g) for W in Ws]
        self.oracle = [O.quantize_weights(W, g) for W in Ws]
        self.d_packed = torch.from_numpy(np.concatenate([p[0] for p in packs])).cuda()
        self.d_gparams = torch.from_numpy(np.concatenate([p[1] for p in packs])).cuda()
        self.w_scales = np.stack([p[2] for p in packs])
        self.d_w_scales = torch.from_numpy(self.w_scales).cuda()

    def check(self, rows, seed, what):
        import torch

        offs = np.concatenate([[0], np.cumsum(rows)]).astype(int)
        M = int(offs[-1])
        X, s_x = I.make_activations(M, self.K, outlier_frac=0.01, seed=seed)
        ACC_ref, _ = O.grouped_w4a8_gemm(X, s_x, offs, self.oracle)
        s_w_rows = np.concatenate([np.repeat(self.oracle[e]["s_w"][None, :], rows[e], axis=0)
                                   for e in range(self.E)]) if M else np.zeros((0, self.N), np.float32)
        ref64 = ACC_ref.astype(np.float64) * s_x.astype(np.float64)[:, None] * s_w_rows.astype(np.float64)
        dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
        Y, ACC = api.w4a8_grouped_gemm(offs, dX, dsx, self.d_packed, self.d_gparams, self.d_w_scales,
                                       self.N, self.K, self.g, want_y=True, want_acc=True)
        torch.cuda.synchronize()
        assert np.array_equal(ACC.cpu().numpy(), ACC_ref), f"{what}: INT32 accumulators differ"
        H.assert_fp16_close(Y.cpu().numpy(), ref64, what)
        return dX, dsx, offs, ACC


CASES = [
    # E, N, K, g, rows per expert
    (5, 256, 512, 64, [3, 0, 20, 40, 200]),        # all three families and an empty expert
    (8, 448, 768, 128, [1, 16, 7, 0, 2, 16, 9, 4]),  # decode-like: every expert small
    (3, 320, 1024, 64, [130, 77, 300]),            # only tiled experts, ragged rows, N tail
    (4, 128, 256, 64, [32, 17, 33, 31]),           # around the family boundaries, one k unit
    (2, 64, 2048, 128, [0, 5]),                    # smallest N, leading empty expert
    # wide layers with many experts: large grids in every family
    (4, 16384, 256, 64, [20, 64, 33, 50]),
    (8, 16384, 256, 128, [17, 32, 25, 30, 64, 40, 50, 60]),
    (16, 16384, 256, 64, [18, 33] * 8),
    (6, 16384, 512, 128, [70, 96, 65, 80, 128, 90]),   # one k group per block, tiles of three row fragments
    # more blocks than CUs and larger experts: the direct-to-LDS tiles (2, 3 and 4 row fragments; 6 and 10 stages)
    (4, 16384, 768, 64, [200, 130, 75, 300]),
    (3, 16384, 1280, 128, [129, 260, 100]),
]


@pytest.mark.parametrize("E,N,K,g,rows", CASES)
def test_grouped_gemm_matches_oracle(E, N, K, g, rows):
    _say(f"grouped E={E} N={N} K={K} g={g} rows={rows}")
    ex = Experts(E, N, K, g, seed=N + K)
    ex.check(rows, seed=E, what=f"rows={rows}")


def test_grouped_equals_separate_calls_and_many_experts():
    import torch

    E, N, K, g = 64, 64, 256, 64
    _say("grouped E=64")
    ex = Experts(E, N, K, g, seed=500)
    rng = np.random.default_rng(3)
    rows = rng.integers(0, 40, size=E).tolist()
    dX, dsx, offs, ACC = ex.check(rows, seed=9, what="64 experts")
    cb, gb = api.liquidquant_packed_size(N, K, g)
    for e in (0, 17, 63):
        r0, r1 = offs[e], offs[e + 1]
        if r1 == r0:
            continue
        one = api.w4a8_gemm_i32(dX[r0:r1].contiguous(), ex.d_packed[e * cb:(e + 1) * cb],
                                ex.d_gparams[e * gb:(e + 1) * gb], N, K, g)
        torch.cuda.synchronize()
        assert torch.equal(one, ACC[r0:r1])


def test_grouped_interface_limits():
    import torch

    N, K, g = 64, 256, 64
    ex = Experts(1, N, K, g, seed=1)
    X = torch.zeros((4, K), dtype=torch.int8, device="cuda")
    sx = torch.ones(4, dtype=torch.float32, device="cuda")
    # no tokens at all: a successful no-op
    Y, _ = api.w4a8_grouped_gemm([0, 0], X[:0], sx[:0], ex.d_packed, ex.d_gparams, ex.d_w_scales, N, K, g)
    assert tuple(Y.shape) == (0, N)
    L = api.lib()
    import ctypes

    def raw(E, offs):
        arr = (ctypes.c_int * len(offs))(*offs)
        return L.w4a8_grouped_gemm(E, arr, N, K, g, ctypes.c_void_p(X.data_ptr()), ctypes.c_void_p(sx.data_ptr()),
                                   ctypes.c_void_p(ex.d_packed.data_ptr()), ctypes.c_void_p(ex.d_gparams.data_ptr()),
                                   ctypes.c_void_p(ex.d_w_scales.data_ptr()), None, None, None)

    assert raw(65, [0] * 66) == -1          # too many experts
    assert raw(0, [0]) == -1
    assert raw(1, [1, 4]) == -1             # must start at 0
    assert raw(2, [0, 3, 2]) == -1          # must not decrease
    assert raw(1, [0, 4]) == -1             # no output pointer


def test_grouped_full_size_layer_all_families():
    """A layer of realistic width (N = K = 4096, 8 experts) with expert sizes in every kernel
    family, checked in full: per expert the float64 BLAS product of the oracle's dequantised
    weights is exact (|ACC| < 2^53)."""
    import torch

    E, N, K, g = 8, 4096, 4096, 64
    rows = [5, 0, 16, 33, 64, 65, 130, 700]
    _say(f"grouped full size E={E} N={N} K={K} rows={rows}")
    Ws = [WL.make_weights(N, K, 0.02, seed=900 + e) for e in range(E)]
    packs = [api.liquidquant_pack_weights(W, g) for W in Ws]
    d_packed = torch.from_numpy(np.concatenate([p[0] for p in packs])).cuda()
    d_gparams = torch.from_numpy(np.concatenate([p[1] for p in packs])).cuda()
    d_sw = torch.from_numpy(np.stack([p[2] for p in packs])).cuda()
    offs = np.concatenate([[0], np.cumsum(rows)]).astype(int)
    X, s_x = I.make_activations(int(offs[-1]), K, outlier_frac=0.001, seed=77)
    Y, ACC = api.w4a8_grouped_gemm(offs, torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda(), d_packed,
                                   d_gparams, d_sw, N, K, g, want_y=True, want_acc=True)
    torch.cuda.synchronize()
    ACC, Y = ACC.cpu().numpy(), Y.cpu().numpy()
    for e in range(E):
        r0, r1 = offs[e], offs[e + 1]
        if r1 == r0:
            continue
        q = O.quantize_weights(Ws[e], g)
        assert np.array_equal(q["s_w"].view(np.uint32), packs[e][2].view(np.uint32))
        Wd = O.dequant_plain(q["Q_u4"], q["s_u8"], q["mn"], g)
        ref = X[r0:r1].astype(np.float64) @ Wd.astype(np.float64).T
        assert np.array_equal(ACC[r0:r1].astype(np.float64), ref), f"expert {e}: accumulators differ"
        H.assert_fp16_close(Y[r0:r1], ref * s_x[r0:r1, None].astype(np.float64) * q["s_w"][None, :].astype(np.float64),
                            f"expert {e}")


@pytest.mark.parametrize("K", [1024, 768])
def test_grouped_large_experts_take_256_row_tiles(K):
    """Experts of several hundred rows on a layer wide enough that whole rounds of 256 x 256 tiles
    pay: the big experts run as one persistent launch of the one-wave-per-SIMD kernel over all of
    them (ragged last row tiles of 8, 132 and 188 rows, an expert of exactly 256 rows, tile
    boundaries between experts inside a block's stream), the small ones in their own families.
    Also with K % 512 == 256 (two added stages of zero weights per tile).
    Checked in full against the exact float64 product of the oracle's dequantised weights."""
    import torch

    E, N, g = 7, 4096, 128
    rows = [700, 5, 520, 900, 40, 256, 1000]
    _say(f"grouped 256-row tiles E={E} N={N} K={K} rows={rows}")
    Ws = [WL.make_weights(N, K, 0.02, seed=300 + e) for e in range(E)]
    packs = [api.liquidquant_pack_weights(W, g) for W in Ws]
    d_packed = torch.from_numpy(np.concatenate([p[0] for p in packs])).cuda()
    d_gparams = torch.from_numpy(np.concatenate([p[1] for p in packs])).cuda()
    d_sw = torch.from_numpy(np.stack([p[2] for p in packs])).cuda()
    offs = np.concatenate([[0], np.cumsum(rows)]).astype(int)
    X, s_x = I.make_activations(int(offs[-1]), K, outlier_frac=0.001, seed=78)
    dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
    Y, ACC = api.w4a8_grouped_gemm(offs, dX, dsx, d_packed, d_gparams, d_sw, N, K, g, want_y=True, want_acc=True)
    # the accumulators alone: no scales are passed, none may be read
    _, ACC2 = api.w4a8_grouped_gemm(offs, dX, None, d_packed, d_gparams, None, N, K, g, want_y=False, want_acc=True)
    torch.cuda.synchronize()
    ACC, Y, ACC2 = ACC.cpu().numpy(), Y.cpu().numpy(), ACC2.cpu().numpy()
    assert np.array_equal(ACC, ACC2), "accumulator-only call differs"
    for e in range(E):
        r0, r1 = offs[e], offs[e + 1]
        q = O.quantize_weights(Ws[e], g)
        Wd = O.dequant_plain(q["Q_u4"], q["s_u8"], q["mn"], g)
        ref = X[r0:r1].astype(np.float64) @ Wd.astype(np.float64).T
        assert np.array_equal(ACC[r0:r1].astype(np.float64), ref), f"expert {e}: accumulators differ"
        H.assert_fp16_close(Y[r0:r1], ref * s_x[r0:r1, None].astype(np.float64) * q["s_w"][None, :].astype(np.float64),
                            f"expert {e}")
