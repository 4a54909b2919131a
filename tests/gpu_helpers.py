"""Shared helpers of the GPU parity tests: build a problem once per weight shape, keep
its device tensors, and compute oracle results (full or sampled)."""
from __future__ import annotations

import functools

import numpy as np

from oracle import c_oracle
from oracle import lqq_oracle as O
from paper_2509_01229_amd import api
from paper_2509_01229_amd import workloads as WL


class Problem:
    """Weights of one (N, K, group) packed by the library and resident on the GPU."""

    def __init__(self, N, K, group, sigma=0.02, seed=0, W=None, Q_i8=None):
        import torch

        self.N, self.K, self.group = N, K, group
        if Q_i8 is not None:
            self.W = None
            self.Q_i8 = np.ascontiguousarray(Q_i8, dtype=np.int8)
            self.packed, self.gparams = api.liquidquant_pack_from_i8(self.Q_i8, group)
            self.w_scales = np.linspace(0.5, 1.5, N).astype(np.float32) * np.float32(1e-3)
        else:
            self.W = WL.make_weights(N, K, sigma, seed=seed) if W is None else W
            self.Q_i8 = None
            self.packed, self.gparams, self.w_scales = api.liquidquant_pack_weights(self.W, group)
        dev = "cuda:0"
        self.d_packed = torch.from_numpy(self.packed).to(dev)
        self.d_gparams = torch.from_numpy(self.gparams).to(dev)
        self.d_w_scales = torch.from_numpy(self.w_scales).to(dev)
        self._oracle_q = None

    # -- oracle side ---------------------------------------------------------------
    def oracle_rows(self, rows):
        """Oracle quantisation of the selected output channels only (per-channel
        independent): returns dict with Q_u4, s_u8, mn, a, s_w for those rows."""
        rows = np.asarray(rows)
        if self.W is not None:
            Q_i8, s_w = O.level1_quantize(self.W[rows])
        else:
            Q_i8, s_w = self.Q_i8[rows], self.w_scales[rows]
        Q_u4, s_u8, mn = O.level2_quantize(Q_i8, self.group)
        return {"Q_u4": Q_u4, "s_u8": s_u8, "mn": mn, "a": O.offset_a(mn), "s_w": s_w}

    def oracle_full(self):
        if self._oracle_q is None:
            self._oracle_q = self.oracle_rows(np.arange(self.N))
            q = self._oracle_q
            q["packed"] = O.pack_canonical(q["Q_u4"])
        return self._oracle_q

    def oracle_wd(self, rows=None):
        q = self.oracle_full() if rows is None else self.oracle_rows(rows)
        return O.dequant_plain(q["Q_u4"], q["s_u8"], q["mn"], self.group), q["s_w"]

    def oracle_gemm(self, X_i8, s_x):
        """Full oracle result through the C oracle (same steps as the numpy one)."""
        q = self.oracle_full()
        return c_oracle.w4a8_gemm(X_i8, s_x, q["packed"], q["s_u8"], q["a"], q["s_w"], self.group)

    def oracle_sampled(self, X_i8, s_x, m_idx, n_idx):
        """Oracle ACC and Y (float64, unrounded) on the sub-matrix m_idx x n_idx."""
        Wd, s_w = self.oracle_wd(n_idx)
        ACC = O.matmul_i64(X_i8[m_idx], Wd)
        return ACC, O.scale_epilogue_f64(ACC, s_x[m_idx], s_w)

    # -- device side ---------------------------------------------------------------
    def run(self, X_i8, s_x, variant=-1, want_y=True, want_acc=True):
        import torch

        dX = torch.from_numpy(np.ascontiguousarray(X_i8)).to("cuda:0")
        dsx = torch.from_numpy(np.ascontiguousarray(s_x)).to("cuda:0")
        Y, ACC = api.w4a8_gemm_variant(variant, dX, dsx, self.d_packed, self.d_gparams, self.d_w_scales,
                                       self.N, self.K, self.group, want_y=want_y, want_acc=want_acc)
        torch.cuda.synchronize()
        return (Y.cpu().numpy() if want_y else None), (ACC.cpu().numpy() if want_acc else None)


@functools.lru_cache(maxsize=4)
def problem(N, K, group, sigma=0.02, seed=0):
    return Problem(N, K, group, sigma, seed)


def assert_fp16_close(Y, ref_f64, what=""):
    """|Y - ref| <= 1e-3 |ref| + 2^-24: one FP16 ulp is at most 2^-10 = 9.8e-4 relative,
    and 2^-24 is the subnormal spacing.  Values that overflow FP16 must be infinite."""
    Y = np.asarray(Y, dtype=np.float64)
    ref = np.asarray(ref_f64, dtype=np.float64)
    over = np.abs(ref) > 65520.0
    assert np.isinf(Y[over]).all(), f"{what}: overflow not mapped to inf"
    ok = ~over
    err = np.abs(Y[ok] - ref[ok])
    tol = 1e-3 * np.abs(ref[ok]) + 2.0 ** -24
    bad = err > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outputs off, worst rel {np.max(err / (np.abs(ref[ok]) + 1e-30)):.3e}"


def variants_for(M, N, K, group):
    """Indices of every kernel variant able to run this shape."""
    return [i for i in range(api.w4a8_variant_count()) if api.w4a8_variant_supports(i, M, N, K, group)]
