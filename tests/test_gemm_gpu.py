"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  INT32 accumulators and the dequantised INT8 matrix must match bit
for bit; FP16 outputs within 1e-3 relative (one FP16 ulp) of the double-precision oracle.
"""
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


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    import torch

    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' elsewhere)")
    api.lib()  # must load: there is no fallback


# ---------------------------------------------------------------------------------------
# Layout + dequantisation alone (no MFMA): kernels' unpack/Eq. 12 path vs oracle Eq. 8
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,K,g", [(64, 256, 64), (256, 512, 64), (192, 1280, 128), (64, 256, 128)])
def test_dequant_dump_matches_oracle(N, K, g):
    import torch

    _say(f"dequant_dump N={N} K={K} g={g}")
    P = H.Problem(N, K, g, seed=N + K)
    Wd_ref, _ = P.oracle_wd()
    Wd = api.w4a8_dequant_dump(P.d_packed, P.d_gparams, N, K, g)
    torch.cuda.synchronize()
    assert np.array_equal(Wd.cpu().numpy(), Wd_ref)


@pytest.mark.parametrize("style", ["extreme", "constant", "narrow", "uniform"])
def test_dequant_dump_edge_distributions(style):
    import torch

    N, K, g = 128, 512, 64
    _say(f"dequant_dump style={style}")
    Q = WL.make_q_i8(N, K, seed=5, style=style)
    P = H.Problem(N, K, g, Q_i8=Q)
    Wd_ref, _ = P.oracle_wd()
    Wd = api.w4a8_dequant_dump(P.d_packed, P.d_gparams, N, K, g)
    torch.cuda.synchronize()
    assert np.array_equal(Wd.cpu().numpy(), Wd_ref)


# ---------------------------------------------------------------------------------------
# Every kernel variant on small shapes spanning several tiles and ragged tails
# ---------------------------------------------------------------------------------------
SMALL = [
    # M, N, K, g
    (8, 256, 512, 64),       # the tiny config
    (1, 64, 256, 64),        # smallest legal problem
    (16, 320, 768, 128),     # N not a multiple of 256
    (13, 192, 1024, 64),     # ragged M inside one fragment
    (31, 128, 512, 128),
    (50, 192, 768, 64),      # two row fragments of the 64-row stream kernel, ragged
    (64, 128, 512, 128),     # exactly 64 rows
    (77, 448, 768, 64),      # ragged M over several row tiles, N tail
    (128, 64, 512, 64),      # exactly 128 rows: four row fragments of the stream kernel
    (200, 256, 256, 64),     # one k unit only
    (130, 576, 1280, 128),
    (300, 320, 1792, 64),    # 14 stages of 128 k; last row tile with 44 rows, N tail
]


@pytest.mark.parametrize("M,N,K,g", SMALL)
def test_every_variant_bit_exact(M, N, K, g):
    P = H.Problem(N, K, g, seed=M * 7 + N)
    X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=M + K)
    ACC_ref, Y_ref = P.oracle_gemm(X, s_x)
    q = P.oracle_full()
    ref64 = O.scale_epilogue_f64(ACC_ref, s_x, q["s_w"])
    ran = 0
    for v in H.variants_for(M, N, K, g):
        name = api.w4a8_variant_name(v)
        _say(f"variant {name} M={M} N={N} K={K} g={g}")
        Y, ACC = P.run(X, s_x, variant=v)
        assert np.array_equal(ACC, ACC_ref), f"{name}: INT32 accumulators differ"
        H.assert_fp16_close(Y, ref64, name)
        ran += 1
    assert ran >= 2
    # the dispatcher's own choice, through the two public entry points
    import torch

    dX = torch.from_numpy(X).cuda()
    dsx = torch.from_numpy(s_x).cuda()
    Y = api.w4a8_gemm(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
    ACC = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g)
    torch.cuda.synchronize()
    assert np.array_equal(ACC.cpu().numpy(), ACC_ref)
    H.assert_fp16_close(Y.cpu().numpy(), ref64, "dispatcher")


# ---------------------------------------------------------------------------------------
# Degenerate inputs
# ---------------------------------------------------------------------------------------
def test_degenerate_inputs():
    N, K, g = 128, 512, 64
    P = H.Problem(N, K, g, seed=3)
    Wd, s_w = P.oracle_wd()
    for M in (5, 40):
        _say(f"degenerate M={M}")
        X = np.zeros((M, K), dtype=np.int8)
        X[1, 77] = 1            # one-hot row: picks column 77 of Wd^T
        X[2, :] = 1             # all ones: row sums
        X[3, :] = -127          # extreme negative
        X[4, :] = 127           # extreme positive
        s_x = np.ones(M, dtype=np.float32)
        for v in H.variants_for(M, N, K, g):
            _, ACC = P.run(X, s_x, variant=v, want_y=False)
            assert (ACC[0] == 0).all()
            assert np.array_equal(ACC[1], Wd[:, 77].astype(np.int32))
            assert np.array_equal(ACC[2], Wd.astype(np.int64).sum(axis=1))
            assert np.array_equal(ACC[3], -127 * Wd.astype(np.int64).sum(axis=1))
            assert np.array_equal(ACC[4], 127 * Wd.astype(np.int64).sum(axis=1))


@pytest.mark.parametrize("style", ["extreme", "constant"])
def test_extreme_weight_ranges(style):
    M, N, K, g = 24, 128, 1024, 128
    _say(f"extreme weights style={style}")
    Q = WL.make_q_i8(N, K, seed=9, style=style)
    P = H.Problem(N, K, g, Q_i8=Q)
    X, s_x = I.make_activations(M, K, seed=1)
    X[0, :] = 127
    ACC_ref, _ = P.oracle_gemm(X, s_x)
    for v in H.variants_for(M, N, K, g):
        _, ACC = P.run(X, s_x, variant=v, want_y=False)
        assert np.array_equal(ACC, ACC_ref), api.w4a8_variant_name(v)


def test_fp16_overflow_and_tiny_scales():
    M, N, K, g = 4, 64, 256, 64
    _say("fp16 overflow / underflow")
    P = H.Problem(N, K, g, seed=2)
    X, _ = I.make_activations(M, K, seed=2)
    s_x = np.array([1e4, 1e-3, 1e-9, 1.0], dtype=np.float32)
    ACC_ref, _ = P.oracle_gemm(X, s_x)
    ref64 = O.scale_epilogue_f64(ACC_ref, s_x, P.oracle_full()["s_w"])
    Y, ACC = P.run(X, s_x)
    assert np.array_equal(ACC, ACC_ref)
    H.assert_fp16_close(Y, ref64, "overflow")


def test_empty_batch_and_determinism():
    import torch

    N, K, g = 256, 1024, 64
    P = H.Problem(N, K, g, seed=4)
    _say("M=0")
    X0 = torch.empty((0, K), dtype=torch.int8, device="cuda")
    s0 = torch.empty((0,), dtype=torch.float32, device="cuda")
    Y0 = api.w4a8_gemm(X0, s0, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
    assert tuple(Y0.shape) == (0, N)
    _say("determinism")
    X, s_x = I.make_activations(16, K, seed=8)
    a1 = P.run(X, s_x)
    a2 = P.run(X, s_x)
    assert np.array_equal(a1[1], a2[1]) and np.array_equal(a1[0].view(np.uint16), a2[0].view(np.uint16))


def test_binding_rejects_bad_tensors():
    import torch

    N, K, g = 64, 256, 64
    P = H.Problem(N, K, g, seed=1)
    X = torch.zeros((4, K), dtype=torch.int8, device="cuda")
    sx = torch.ones(4, dtype=torch.float32, device="cuda")
    with pytest.raises(TypeError):
        api.w4a8_gemm(X.cpu(), sx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
    with pytest.raises(TypeError):
        api.w4a8_gemm(X.to(torch.int32), sx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
    with pytest.raises(ValueError):
        api.w4a8_gemm(X, sx[:3], P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
    with pytest.raises(api.LiquidGemmError):
        api.w4a8_gemm_variant(0, torch.zeros((64, K), dtype=torch.int8, device="cuda"),
                              torch.ones(64, device="cuda"), P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)


def test_workspace_is_optional_for_the_dispatcher():
    """Without room for split-K partials the dispatcher runs unsplit and stays exact; a
    variant that names its split reports the missing workspace."""
    import torch

    for M, N, K, g in [(8, 256, 2048, 64), (160, 512, 2048, 128)]:
        _say(f"small workspace M={M} N={N} K={K}")
        assert api.w4a8_gemm_workspace_size(M, N, K, g) > 16
        P = H.Problem(N, K, g, seed=11)
        X, s_x = I.make_activations(M, K, seed=12)
        ACC_ref, _ = P.oracle_gemm(X, s_x)
        dX = torch.from_numpy(X).cuda()
        tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
        ACC = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g, workspace=tiny)
        torch.cuda.synchronize()
        assert np.array_equal(ACC.cpu().numpy(), ACC_ref)
        split = [v for v in H.variants_for(M, N, K, g) if api.w4a8_variant_name(v).endswith("_s2")]
        assert split
        for v in split:
            with pytest.raises(api.LiquidGemmError) as e:
                api.w4a8_gemm_variant(v, dX, torch.from_numpy(s_x).cuda(), P.d_packed, P.d_gparams,
                                      P.d_w_scales, N, K, g, workspace=tiny)
            assert e.value.code == -3


def test_calibration_kernels_run():
    import torch

    _say("calibration kernels")
    buf = torch.zeros((1 << 20) + 8, dtype=torch.uint8, device="cuda")
    assert api.w4a8_calib_stream_read(buf[: 1 << 20]) == 1 << 20
    ops = api.w4a8_calib_mfma_i8(2, True)
    assert ops == 512 * 4 * 2 * 64 * 2.0 * 32 ** 3
    assert api.w4a8_calib_mfma_i8(1, False) == ops / 2
    torch.cuda.synchronize()
    with pytest.raises(api.LiquidGemmError):
        api.w4a8_calib_mfma_i8(0, True)
    with pytest.raises(api.LiquidGemmError):
        api.w4a8_calib_stream_read(buf[8:])  # not 16-byte aligned


def test_random_shapes_through_the_dispatcher():
    """A seeded sweep of legal shapes (every row-count family, ragged tails in M and N, one
    to many k units, both group sizes) through w4a8_gemm / w4a8_gemm_i32 as a caller would
    use them, with and without the optional workspace."""
    import torch

    rng = np.random.default_rng(2024)
    Ms = [1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 191, 257, 300]
    for case in range(34):
        M = Ms[case % len(Ms)]
        N = 64 * int(rng.integers(1, 13))
        K = 256 * int(rng.integers(1, 9))
        g = (64, 128)[case % 2]
        picked = api.w4a8_variant_name(api.w4a8_select_variant(M, N, K, g))
        _say(f"random shape {case}: M={M} N={N} K={K} g={g} -> {picked}")
        P = H.Problem(N, K, g, seed=1000 + case)
        X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=2000 + case)
        ACC_ref, _ = P.oracle_gemm(X, s_x)
        ref64 = O.scale_epilogue_f64(ACC_ref, s_x, P.oracle_full()["s_w"])
        dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
        ws = None if case % 3 else torch.empty(16, dtype=torch.uint8, device="cuda")  # every third: no room to split
        Y = api.w4a8_gemm(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g, workspace=ws)
        ACC = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(ACC.cpu().numpy(), ACC_ref), f"case {case}: accumulators differ"
        H.assert_fp16_close(Y.cpu().numpy(), ref64, f"case {case}")


def test_random_large_grids_through_the_dispatcher():
    """Seeded shapes with more than 256 tiles of 128 x 256 (the direct-to-LDS tiled kernels and the
    256-row tiles with one wave per SIMD: ragged
    last row tiles, N tails, 2 to 24 stages so that every remainder of the three-stage loop of the
    former occurs, and the added stages of the latter for K % 512 == 256, K = 256 included) and a few
    just below; the accumulators are compared with the exact float64
    product on the oracle's dequantised weights, the FP16 output with the epilogue definition."""
    import torch

    rng = np.random.default_rng(11)
    seen = set()
    for case in range(14):
        N = 64 * int(rng.integers(40, 65))
        K = 256 * int(rng.integers(1, 13))
        g = (64, 128)[case % 2]
        M = int(rng.integers(2600, 4600)) if case % 5 != 4 else int(rng.integers(1400, 2000))
        picked = api.w4a8_variant_name(api.w4a8_select_variant(M, N, K, g))
        seen.add(picked)
        _say(f"large grid {case}: M={M} N={N} K={K} g={g} -> {picked}")
        P = H.Problem(N, K, g, seed=500 + case)
        X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=900 + case)
        Wd, s_w = P.oracle_wd()
        ref = X.astype(np.float64) @ Wd.astype(np.float64).T      # exact: |acc| < 2^31 << 2^53
        dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
        ACC = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g)
        Y = api.w4a8_gemm(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
        torch.cuda.synchronize()
        assert np.array_equal(ACC.cpu().numpy().astype(np.float64), ref), f"case {case}: accumulators differ"
        H.assert_fp16_close(Y.cpu().numpy(), O.scale_epilogue_f64(ref, s_x, s_w), f"case {case}")
        del P, dX, ACC, Y
    assert {"duo_dl_m128", "duo_pt_m128", "solo16_pt_m256", "solo16_g2_m256"} <= seen


def test_random_small_batches_through_the_dispatcher():
    """Seeded shapes with 1..64 rows over weight matrices of every aspect (the stream kernels as
    the dispatcher launches them: 16-, 32- and 64-row forms, one or two tiles per block, 4 to 16
    waves, K slices across blocks, X fragments direct or through LDS), with and without a
    workspace; accumulators against the exact float64 product on the oracle's dequantised
    weights, FP16 output against the epilogue definition."""
    import torch

    rng = np.random.default_rng(23)
    seen = set()
    for case in range(16):
        aspect = case // 4                      # generic / wide and short / narrow and long / wide
        if aspect == 0:
            N, K = 64 * int(rng.integers(1, 129)), 256 * int(rng.integers(1, 33))
        elif aspect == 1:
            N, K = 64 * int(rng.integers(100, 201)), 256 * int(rng.integers(1, 5))
        elif aspect == 2:
            N, K = 64 * int(rng.integers(4, 41)), 256 * int(rng.integers(48, 81))
        else:
            N, K = 64 * int(rng.integers(128, 257)), 256 * int(rng.integers(8, 17))
        g = (64, 128)[case % 2]
        lo, hi = ((1, 9), (9, 17), (17, 33), (33, 65))[case % 4]
        M = int(rng.integers(lo, hi))
        picked = api.w4a8_variant_name(api.w4a8_select_variant(M, N, K, g))
        seen.add(picked)
        _say(f"small batch {case}: M={M} N={N} K={K} g={g} -> {picked}")
        P = H.Problem(N, K, g, seed=700 + case)
        X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=1100 + case)
        Wd, s_w = P.oracle_wd()
        ref = X.astype(np.float64) @ Wd.astype(np.float64).T      # exact: |acc| < 2^31 << 2^53
        dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
        ws = None if case % 4 else torch.empty(16, dtype=torch.uint8, device="cuda")  # every fourth: no room to split
        ACC = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g, workspace=ws)
        Y = api.w4a8_gemm(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(ACC.cpu().numpy().astype(np.float64), ref), f"case {case}: accumulators differ"
        H.assert_fp16_close(Y.cpu().numpy(), O.scale_epilogue_f64(ref, s_x, s_w), f"case {case}")
        del P, dX, ACC, Y
    assert len(seen) >= 5, seen


def test_maximum_k_and_accumulator_range():
    """K at the interface limit (131072) with inputs that drive the accumulators to the edge
    of INT32: |ACC| up to K * 127 * 121 = 2 014 183 424 < 2^31 must come out exactly."""
    import torch

    N, K, g = 64, 131072, 128
    _say("maximum K, extreme accumulators")
    Q = np.full((N, K), 119, dtype=np.int8)
    Q[1::2] = -119
    Q[:, ::128] = -119          # every group spans the whole protective range: s = 16, top code 15 -> 121
    Q[1::2, ::128] = 119
    P = H.Problem(N, K, g, Q_i8=Q)
    Wd, _ = P.oracle_wd()
    assert Wd.max() == 121 and Wd.min() == -119
    for M in (3, 40, 70):
        X = np.full((M, K), 127, dtype=np.int8)
        X[1] = -127
        X[2, ::2] = -127
        s_x = np.ones(M, dtype=np.float32)
        ACC_ref = X.astype(np.float64) @ Wd.astype(np.float64).T   # exact: below 2^53
        assert np.abs(ACC_ref).max() < 2.0 ** 31
        dX = torch.from_numpy(X).cuda()
        ACC = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g)
        torch.cuda.synchronize()
        assert np.array_equal(ACC.cpu().numpy().astype(np.float64), ACC_ref), f"M={M}"
    with pytest.raises(api.LiquidGemmError):
        api.liquidquant_packed_size(64, 131072 + 256, 64)


def test_wide_layer_large_grid():
    """N = 65536: grids of thousands of blocks in the stream kernels and many column tiles in
    the tiled kernel (one k unit keeps the oracle cheap)."""
    import torch

    N, K, g = 65536, 256, 64
    _say("wide layer")
    P = H.Problem(N, K, g, seed=31)
    Wd, _ = P.oracle_wd()
    for M in (2, 20, 50, 130):
        X, s_x = I.make_activations(M, K, seed=M)
        ACC = api.w4a8_gemm_i32(torch.from_numpy(X).cuda(), P.d_packed, P.d_gparams, N, K, g)
        torch.cuda.synchronize()
        ref = X.astype(np.float64) @ Wd.astype(np.float64).T
        assert np.array_equal(ACC.cpu().numpy().astype(np.float64), ref), f"M={M}"


def test_hip_graph_replays_of_split_k_kernels():
    """Split-K launches (arrival tickets that reset themselves, partial tiles in the workspace)
    captured in a HIP graph: every replay, with eager work of the same kind in between, must
    reproduce the eager result."""
    import torch

    # stream16 / stream_m64 / duo_m64 / 256-row tiles with K slices and their finish kernel
    cases = [(8, 2048, 4096, 64), (48, 4096, 2048, 64), (200, 1024, 4096, 128), (256, 6144, 16384, 128)]
    stream = torch.cuda.Stream()
    for M, N, K, g in cases:
        picked = api.w4a8_variant_name(api.w4a8_select_variant(M, N, K, g))
        _say(f"graph replay M={M} N={N} K={K} -> {picked}")
        P = H.Problem(N, K, g, seed=M)
        X, s_x = I.make_activations(M, K, seed=M + 1)
        X2, s_x2 = I.make_activations(M, K, seed=M + 2)
        dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
        dX2, dsx2 = torch.from_numpy(X2).cuda(), torch.from_numpy(s_x2).cuda()
        ws = torch.zeros(api.w4a8_gemm_workspace_size(M, N, K, g) + 16, dtype=torch.uint8, device="cuda")
        out = torch.empty((M, N), dtype=torch.int32, device="cuda")
        eager = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g, workspace=ws).clone()
        eager2 = api.w4a8_gemm_i32(dX2, P.d_packed, P.d_gparams, N, K, g, workspace=ws).clone()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(stream):
            with torch.cuda.graph(graph, stream=stream):
                api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g, out=out, workspace=ws,
                                  stream=stream.cuda_stream)
        for rep in range(3):
            out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
            other = api.w4a8_gemm_i32(dX2, P.d_packed, P.d_gparams, N, K, g, workspace=ws)   # eager work in between
            torch.cuda.synchronize()
            assert torch.equal(other, eager2)


def test_workspace_init_and_concurrent_streams():
    """The split-K state lives in the caller's workspace: a dirty buffer works after
    w4a8_workspace_init, and calls that overlap on two streams, each with its own workspace,
    do not disturb each other."""
    import torch

    M, N, K, g = 8, 1024, 8192, 64          # stream16 with grid split-K
    assert api.w4a8_variant_name(api.w4a8_select_variant(M, N, K, g)).startswith("stream16")
    P = H.Problem(N, K, g, seed=77)
    X, s_x = I.make_activations(M, K, seed=78)
    ACC_ref, _ = P.oracle_gemm(X, s_x)
    ref = torch.from_numpy(ACC_ref).cuda()
    dX = torch.from_numpy(X).cuda()
    need = api.w4a8_gemm_workspace_size(M, N, K, g)
    assert need > 32768
    _say("dirty workspace + init")
    dirty = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")
    api.w4a8_workspace_init(dirty)
    for _ in range(3):
        out = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g, workspace=dirty)
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
    _say("two streams")
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    spaces = [torch.zeros(need, dtype=torch.uint8, device="cuda") for _ in streams]
    outs = [[torch.empty((M, N), dtype=torch.int32, device="cuda") for _ in range(40)] for _ in streams]
    torch.cuda.synchronize()
    for i in range(40):
        for s, ws, o in zip(streams, spaces, outs):
            api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g, out=o[i], workspace=ws, stream=s.cuda_stream)
    torch.cuda.synchronize()
    for o in outs:
        for t in o:
            assert torch.equal(t, ref)


def test_batch_beyond_32_bit_offsets_of_x():
    """M * K just above 2^32 (the kernels address X with 32-bit byte offsets; the entry point
    runs such a batch as consecutive row chunks): every accumulator and every FP16 output
    against the exact float64 product of the oracle's weights, for the dispatcher's kernel
    (w4a8_gemm, w4a8_gemm_i32) and, on the rows around the chunk boundary, for a named tiled
    variant."""
    import torch

    N, K, g = 64, 131072, 128
    M = (1 << 32) // K + 64                       # 32832 rows: M * K = 2^32 + 2^23
    assert M * K > (1 << 32)
    _say(f"M*K beyond 2^32: M={M} N={N} K={K}")
    P = H.Problem(N, K, g, sigma=0.02, seed=5)
    Wd, s_w = P.oracle_wd()
    WfT = np.ascontiguousarray(Wd.astype(np.float64).T)
    rng = np.random.Generator(np.random.PCG64(6))
    X = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
    X[-1] = 127                                   # the last row of the last chunk is distinctive
    s_x = (0.5 + rng.random(M, dtype=np.float32)) * np.float32(1e-4)
    ref = np.empty((M, N), dtype=np.int32)
    for r0 in range(0, M, 2048):
        prod = X[r0:r0 + 2048].astype(np.float64) @ WfT
        assert np.abs(prod).max() < 2.0 ** 31
        ref[r0:r0 + 2048] = prod.astype(np.int32)
    _say("GPU run")
    dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
    ACC = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g)
    Y = api.w4a8_gemm(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
    torch.cuda.synchronize()
    assert np.array_equal(ACC.cpu().numpy(), ref), "accumulators differ"
    H.assert_fp16_close(Y.cpu().numpy(), O.scale_epilogue_f64(ref, s_x, s_w), "M*K beyond 2^32")
    names = api.w4a8_variant_names()
    _, ACC2 = api.w4a8_gemm_variant(names.index("duo_m128_s1"), dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales,
                                    N, K, g, want_y=False)
    torch.cuda.synchronize()
    assert np.array_equal(ACC2.cpu().numpy(), ref), "accumulators of the named variant differ"


@pytest.mark.parametrize("kernel", ["duo_pt_m128", "solo_pt_m256", "solo_g2_m256", "solo16_pt_m256", "solo16_g2_m256"])
@pytest.mark.parametrize("M,N,K,g", [(1541, 12352, 512, 64), (2048, 10240, 1024, 128), (700, 2048, 1536, 64),
                                     (1100, 4160, 768, 64), (600, 5120, 1280, 128), (520, 2048, 256, 64)])
def test_persistent_tile_kernel(M, N, K, g, kernel):
    """The persistent forms of the tiled kernel (blocks walk several tiles as one stream of
    stages; 128-row tiles with two waves per SIMD, 256-row tiles with one, also in its form of
    two k groups per block that finishes every tile with an exchange through LDS): more tiles than
    resident blocks, so that blocks cross tile boundaries; a ragged last row tile, an N tail,
    tile counts that are and are not multiples of the XCD count, and a grid smaller than the
    number of resident slots; K % 512 == 256 (the 16x16x64 forms: two added stages of zero weights
    per tile).  Every accumulator and every FP16 output against the exact float64 product of the
    oracle's weights."""
    names = api.w4a8_variant_names()
    v = names.index(kernel)
    if K % 512 != 0 and not kernel.startswith("solo16"):
        assert not api.w4a8_variant_supports(v, M, N, K, g)
        pytest.skip(f"{kernel} needs K % 512 == 0")
    assert api.w4a8_variant_supports(v, M, N, K, g)
    _say(f"persistent tiles {kernel} M={M} N={N} K={K} g={g}")
    P = H.Problem(N, K, g, seed=M)
    Wd, s_w = P.oracle_wd()
    X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=M + N)
    ref = (X.astype(np.float64) @ Wd.astype(np.float64).T).astype(np.int64)
    Y, ACC = P.run(X, s_x, variant=v)
    assert np.array_equal(ACC.astype(np.int64), ref), f"{np.count_nonzero(ACC != ref)} accumulators differ"
    H.assert_fp16_close(Y, O.scale_epilogue_f64(ref, s_x, s_w), "persistent tiles")
    # the accumulators alone: such a call passes no scales (null pointers), which no kernel may read
    import torch

    _, ACC2 = api.w4a8_gemm_variant(v, torch.from_numpy(X).cuda(), None, P.d_packed, P.d_gparams, None, N, K, g,
                                    want_y=False)
    torch.cuda.synchronize()
    assert np.array_equal(ACC2.cpu().numpy().astype(np.int64), ref), "accumulator-only call differs"


@pytest.mark.parametrize("kernel", ["solo16_g2_sk_m256", "solo16_pt_m256_s2", "solo16_g2_m256_s4"])
@pytest.mark.parametrize("M,N,K,g", [(300, 640, 2048, 64), (256, 1024, 4608, 128), (520, 320, 1024, 64),
                                     (200, 448, 4096, 128)])
def test_solo_k_slices(M, N, K, g, kernel):
    """The 256-row tile kernels with K slices across blocks (every slice writes an INT32 matrix of
    partial sums, a second kernel adds them up and scales): slice counts of 2, 3 and 4, ragged row
    tiles, an N tail, blocks that walk several (tile, slice) items.  Every accumulator and every
    FP16 output against the exact float64 product of the oracle's weights; then the accumulators
    alone (no scales passed)."""
    import torch

    names = api.w4a8_variant_names()
    v = names.index(kernel)
    if not api.w4a8_variant_supports(v, M, N, K, g):
        pytest.skip(f"{kernel} does not take M={M} K={K}")
    _say(f"K slices {kernel} M={M} N={N} K={K} g={g}")
    P = H.Problem(N, K, g, seed=M + 11)
    Wd, s_w = P.oracle_wd()
    X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=M + N)
    ref = (X.astype(np.float64) @ Wd.astype(np.float64).T).astype(np.int64)
    for rep in range(2):    # the second call finds the first one's partial sums in the workspace
        Y, ACC = P.run(X, s_x, variant=v)
        assert np.array_equal(ACC.astype(np.int64), ref), f"call {rep}: {np.count_nonzero(ACC != ref)} accumulators differ"
        H.assert_fp16_close(Y, O.scale_epilogue_f64(ref, s_x, s_w), "K slices")
    _, ACC2 = api.w4a8_gemm_variant(v, torch.from_numpy(X).cuda(), None, P.d_packed, P.d_gparams, None, N, K, g,
                                    want_y=False)
    torch.cuda.synchronize()
    assert np.array_equal(ACC2.cpu().numpy().astype(np.int64), ref), "accumulator-only call differs"


def test_k_slices_through_the_dispatcher():
    """A shape the dispatcher runs with K slices across blocks (very long K, one row tile):
    the public entry points with the workspace the library asks for, then with one that holds
    fewer slices and with none at all -- the launcher takes what fits."""
    import torch

    M, N, K, g = 250, 6144, 16384, 128
    assert api.w4a8_variant_name(api.w4a8_select_variant(M, N, K, g)) == "solo16_g2_sk_m256"
    need = api.w4a8_gemm_workspace_size(M, N, K, g)
    assert need >= 4 * M * N * 4
    _say(f"K slices through the dispatcher M={M} N={N} K={K} g={g}, workspace {need} bytes")
    P = H.Problem(N, K, g, seed=21)
    Wd, s_w = P.oracle_wd()
    X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=22)
    ref = X.astype(np.float64) @ Wd.astype(np.float64).T
    ref_y = O.scale_epilogue_f64(ref, s_x, s_w)
    dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
    for ws_bytes in (need, 32768 + 2 * M * N * 4 + 4096, 32768, 0):
        _say(f"  workspace of {ws_bytes} bytes")
        ws = torch.zeros(ws_bytes, dtype=torch.uint8, device="cuda")
        Y = api.w4a8_gemm(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g, workspace=ws)
        ACC = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(ACC.cpu().numpy().astype(np.float64), ref), "accumulators differ"
        H.assert_fp16_close(Y.cpu().numpy(), ref_y, "K slices through the dispatcher")


@pytest.mark.parametrize("M,N,K,g", [(2048 + 100, 8192, 4096, 64), (4096 + 40, 8192, 2048, 128), (1024 + 30, 16384, 4096, 128),
                                     (2048 + 700, 8192, 4096, 64), (2048 + 512, 8192, 4096, 128)])
def test_two_launch_plans(M, N, K, g):
    """Batches that the dispatcher runs as two launches over consecutive rows (whole rounds of
    256 x 256 tiles, then the rest with its own kernel; the last cases rests of several row tiles, on
    256 x 128 tiles with a ragged one and on 64-row tiles with K slices): every accumulator and every FP16 output
    against the exact float64 product, through both public entry points."""
    import torch

    plan = api.w4a8_select_plan(M, N, K, g)
    assert len(plan) == 2, plan
    _say(f"two launches M={M} N={N} K={K} g={g}: {[(r, api.w4a8_variant_name(v)) for r, v in plan]}")
    P = H.Problem(N, K, g, seed=M + 3)
    Wd, s_w = P.oracle_wd()
    X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=M + N)
    ref = X.astype(np.float64) @ Wd.astype(np.float64).T
    dX, dsx = torch.from_numpy(X).cuda(), torch.from_numpy(s_x).cuda()
    Y = api.w4a8_gemm(dX, dsx, P.d_packed, P.d_gparams, P.d_w_scales, N, K, g)
    ACC = api.w4a8_gemm_i32(dX, P.d_packed, P.d_gparams, N, K, g)
    torch.cuda.synchronize()
    assert np.array_equal(ACC.cpu().numpy().astype(np.float64), ref), "accumulators differ"
    H.assert_fp16_close(Y.cpu().numpy(), O.scale_epilogue_f64(ref, s_x, s_w), "two launches")
