"""The allocation-free entry point (w4a8_gemm_static: split-K state in the library's built-in
static workspace) against w4a8_gemm with a caller's workspace: same kernels, so the FP16
outputs must be equal bit for bit -- on consecutive calls that share the built-in workspace,
each smaller than the one before, on shapes whose kernels split K across blocks."""
import sys

import numpy as np
import pytest

from paper_2509_01229_amd import api

import gpu_helpers as H
import inputs as I

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_static_workspace_entry_point_matches_w4a8_gemm():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    # 256-row tiles with K slices (a matrix of partial sums per slice: nearly all of the built-in
    # workspace), the 128-row tiled kernel with K slices, then the 64-row and 16-row stream kernels
    # with K slices (smaller each time), then a shape that uses no workspace at all
    cases = [(256, 6144, 16384, 128), (200, 1024, 4096, 128), (48, 4096, 2048, 64), (8, 1024, 8192, 64),
             (4096 + 40, 512, 512, 64)]
    for M, N, K, g in cases:
        picked = api.w4a8_variant_name(api.w4a8_select_variant(M, N, K, g))
        need = api.w4a8_gemm_workspace_size(M, N, K, g)
        _say(f"static workspace: M={M} N={N} K={K} g={g} -> {picked} (caller workspace {need} bytes)")
        P = H.Problem(N, K, g, seed=M)
        X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=M + 7)
        dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
        ref = api.w4a8_gemm(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
        torch.cuda.synchronize()
        out = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        for rep in range(2):   # two calls in a row on the same state
            api.w4a8_gemm_static(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g, out)
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), f"M={M} call {rep}: outputs differ"
            out.fill_(float("nan"))
        # and against the oracle on a sample (the comparison above is between two library paths)
        m_idx = np.arange(min(M, 24))
        n_idx = np.arange(0, N, max(1, N // 96))
        _, Y_ref = P.oracle_sampled(X, s_x, m_idx, n_idx)
        H.assert_fp16_close(ref.cpu().numpy()[np.ix_(m_idx, n_idx)], Y_ref, f"M={M}")
    # empty batch: a successful no-op
    api.w4a8_gemm_static(dX[:0], dsx[:0], P.d_packed, P.d_gparams, P.d_w_scales, N, K, g,
                         torch.empty((0, N), dtype=torch.float16, device="cuda"))
    with pytest.raises(api.LiquidGemmError):
        api.lib().w4a8_gemm_static.argtypes  # (binding present)
        api._check(api.lib().w4a8_gemm_static(4, 100, 256, 64, None, None, None, None, None, None, None))
