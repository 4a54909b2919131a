"""Host logic of the library that needs no GPU: the shape -> kernel dispatcher, the variant
table and the workspace sizing."""
import pytest

from paper_2509_01229_amd import api
from paper_2509_01229_amd import workloads as WL


def _pick(M, N, K, g=64):
    return api.w4a8_variant_name(api.w4a8_select_variant(M, N, K, g))


def _pt_fits(M, N, K):
    return K % 512 == 0 and (M % 128 == 0 or M % 128 > 64)


def _solo_form(M, N, K):
    """The dispatcher's cost rule for the 256-row tiles, restated: costs fitted to measurements, in
    units of a round of 256 tiles of 128 x 256; 1 = 256 x 256 tiles, 2 = 256 x 128 tiles with two k
    groups, 0 = neither."""
    if K % 512:
        return 0
    bm = -(-M // 256)
    t256, t2, t128 = bm * -(-N // 256), bm * -(-N // 128), -(-M // 128) * -(-N // 256)
    def part(t):
        fill = t / 256
        return 0.0 if t == 0 else 0.24 + 0.90 * fill if t <= 128 else 0.47 + 0.52 * fill if t <= 256 else 0.80 + 0.51 * fill
    duo = 2.0 * (t128 // 512) + part(t128 % 512)
    short_k = 1.0 if K >= 4096 else 1.06
    solo = (0.734 + 0.94 * t256 / 256 if t256 <= 256 else 2.0 * -(-t256 // 256) * 0.86) * short_k * 0.92
    g2 = (0.406 + 0.56 * t2 / 256) * short_k if 136 < t2 <= 256 else 1e30
    if solo < duo and solo <= g2:
        return 1
    return 2 if g2 < duo else 0


def test_dispatcher_families_on_the_workloads():
    for s in WL.ALL_SHAPES:
        name = _pick(s.M, s.N, s.K, s.group)
        if s.M <= 16:
            assert name.startswith("stream16_"), (s.name, name)
        elif s.M <= 32:
            assert name == "stream_m32", (s.name, name)
        elif s.M <= 64 and s.N <= 16384:
            assert name == "stream_m64", (s.name, name)
        else:
            assert name in ("duo_m64", "duo_m128", "duo_dl_m128", "duo_pt_m128", "solo16_pt_m256", "solo16_g2_m256",
                            "solo16_g2_sk_m256"), (s.name, name)
            tiles128 = -(-s.M // 128) * -(-s.N // 256)
            form = _solo_form(s.M, s.N, s.K)
            if name == "solo16_g2_sk_m256":   # K slices across blocks: very long K, one round of 256 x 128 tiles x slices
                assert not form and s.K >= 16384 and -(-s.M // 256) * -(-s.N // 128) <= 128, (s.name, name)
            elif form:                  # 256-row tiles, one wave per SIMD, where their whole rounds come out ahead
                assert name == ("solo16_pt_m256" if form == 1 else "solo16_g2_m256"), (s.name, name)
            elif tiles128 > 256:      # more tiles than CUs: the direct-to-LDS pipeline, persistent where it fits
                assert name == ("duo_pt_m128" if _pt_fits(s.M, s.N, s.K) else "duo_dl_m128"), (s.name, name)
            elif tiles128 > 128 and s.K % 512 == 0:   # more than half a round: persistent, one block per CU
                assert name == "duo_pt_m128", (s.name, name)
            elif -(-s.M // 64) * -(-s.N // 256) > 256:
                assert name == "duo_m128", (s.name, name)
        v = api.w4a8_select_variant(s.M, s.N, s.K, s.group)
        assert api.w4a8_variant_supports(v, s.M, s.N, s.K, s.group)


def test_dispatcher_boundaries():
    assert _pick(8, 4096, 4096) == "stream16_f1_w16_s1"        # short K: sixteen waves per block, one tile
    assert _pick(16, 4096, 4096) == "stream16_f1_w16_s1" and _pick(16, 4096, 2048) == "stream16_f1_w16_s1"
    assert _pick(8, 8192, 8192) == "stream16_f1_w8_u4"         # K to 8192: deep prefetch, whole K in the block
    assert _pick(16, 8192, 8192) == "stream16_f1_w16_s1" and _pick(16, 4096, 8192) == "stream16_f1_w8"
    assert _pick(16, 4096, 11008) == "stream16_f1_w8"          # longer K: K slices across blocks
    assert _pick(16, 8192, 28672, 128) == "stream16_f2_w8"     # 129..256 tiles, long K: two tiles per block
    assert _pick(4, 8192, 28672, 128) == "stream16_f1_w16_s1"  # ... up to 8 rows: sixteen waves split K
    assert _pick(4, 4096, 16384) == "stream16_f1_w8" and _pick(16, 8192, 14336) == "stream16_f1_w8"
    assert _pick(16, 11008, 4096) == "stream16_f2_w16_s1"      # more than 256 tiles: two per block
    assert _pick(4, 16384, 4096) == "stream16_f1_w16_s1" and _pick(16, 16384, 8192) == "stream16_f2_w8"
    assert _pick(16, 28672, 2048) == "stream16_f2_w8"
    assert _pick(16, 28672, 8192, 128) == "stream16_f2_w4"     # N alone fills the chip
    assert _pick(17, 4096, 4096) == "stream_m32" and _pick(32, 28672, 8192) == "stream_m32"
    assert _pick(33, 4096, 4096) == "stream_m64" and _pick(64, 16384, 4096) == "stream_m64"
    # 33..64 rows: streamed (X through LDS) up to 512 tiles of 32 channels, whatever K
    assert _pick(64, 8192, 8192) == "stream_m64" and _pick(48, 8192, 8192) == "stream_m64"
    assert _pick(40, 8192, 28672, 128) == "stream_m64" and _pick(64, 4096, 11008) == "stream_m64"
    # ... except 129..256 tiles with very long K from 48 rows on: the tiles' split-K grid
    assert _pick(64, 8192, 28672, 128) in ("duo_m64", "duo_m128") and _pick(48, 6144, 28672, 128) in ("duo_m64", "duo_m128")
    assert _pick(64, 4096, 28672, 128) == "stream_m64" and _pick(64, 8192, 16384, 128) == "stream_m64"
    assert _pick(64, 28672, 8192) == "duo_m64" and _pick(65, 4096, 4096) == "duo_m64"
    assert _pick(256, 28672, 8192) == "solo16_g2_m256"           # 224 tiles of 256 x 128: one round, 62 against 66 us
    assert _pick(192, 28672, 8192) == "solo16_g2_m256" and _pick(128, 28672, 8192) == "duo_m128"
    assert _pick(512, 4096, 4096) == "duo_m64" and _pick(1025, 4096, 4096) == "solo16_g2_m256"
    # very long K, nearly full 256-row tiles: the 256 x 128 tiles with K slices across blocks
    assert _pick(256, 8192, 28672, 128) == "solo16_g2_sk_m256" and _pick(512, 8192, 28672, 128) == "solo16_g2_sk_m256"
    assert _pick(256, 6144, 16384, 128) == "solo16_g2_sk_m256" and _pick(250, 8192, 16384) == "solo16_g2_sk_m256"
    assert _pick(256, 4096, 16384, 128) == "duo_m64"           # (four slices of 32 tiles: half a round)
    assert _pick(128, 8192, 28672, 128) in ("duo_m64", "duo_m128") and _pick(384, 8192, 28672, 128) == "duo_m128"
    assert _pick(256, 8192, 14336, 128) in ("duo_m64", "duo_m128")
    assert _pick(256, 8192, 8192) == "duo_m64" and _pick(256, 10240, 8192, 128) == "duo_m128"
    assert _pick(128, 4096, 256) == "duo_m128"                 # one k unit: no room for two k groups
    # 256-row tiles, one wave per SIMD: 256 x 128 as one round on more than half of the CUs ...
    assert _pick(1024, 8192, 8192) == "solo16_g2_m256" and _pick(960, 8192, 8192) == "solo16_g2_m256"
    assert _pick(2048, 4096, 11264) == "solo16_g2_m256"
    assert _pick(768, 8192, 8192) == "solo16_g2_m256"            # 192 tiles: 54 against 58 us
    assert _pick(512, 9216, 8192) == "solo16_g2_m256" and _pick(512, 11008, 4096) == "solo16_g2_m256"   # 144 / 172 tiles
    assert _pick(512, 10240, 2048) in ("solo16_g2_m256", "duo_pt_m128") and _pick(1024, 5120, 8192) == "solo16_g2_m256"
    assert _pick(512, 8192, 8192) == "duo_m128" and _pick(1024, 4096, 8192) in ("duo_m64", "duo_m128")   # 128 tiles: equal or behind
    assert _pick(384, 8192, 8192) == "duo_m128"                # (a third of the second row tile's work is lost)
    # ... 256 x 256 where their whole rounds cost less than the rounds of 128-row tiles, two blocks to a CU
    assert _pick(1152, 8192, 8192) == "solo16_pt_m256" and _pick(1280, 8192, 8192) == "solo16_pt_m256"   # 160 tiles, one round
    assert _pick(4096, 8192, 8192) == "solo16_pt_m256" and _pick(2048, 8192, 28672, 128) == "solo16_pt_m256"
    assert _pick(8192, 8192, 8192) == "solo16_pt_m256" and _pick(4096, 8192, 2048) == "solo16_pt_m256"
    assert _pick(1024, 28672, 8192, 128) == "solo16_pt_m256" and _pick(2048, 28672, 8192, 128) == "solo16_pt_m256"
    assert _pick(1024, 10240, 8192, 128) == "solo16_pt_m256" and _pick(1024, 11008, 4096) == "solo16_pt_m256"
    # ... and the 128-row tiles where a last round of 256-row tiles would be mostly empty
    assert _pick(2560, 8192, 8192) == "duo_pt_m128" and _pick(3072, 8192, 8192) == "duo_pt_m128"
    assert _pick(2048, 10240, 8192, 128) == "duo_pt_m128" and _pick(2048, 11008, 4096) == "duo_pt_m128"
    # K % 512 == 256: the 16x16x64 forms of the 256-row tiles take it (two added stages of zero weights),
    # the persistent 128-row tiles do not
    assert _pick(4096, 8192, 11008) == "solo16_pt_m256" and _pick(4096, 4096, 11008) == "solo16_pt_m256"
    assert _pick(2048, 4096, 11008) == "solo16_g2_m256" and _pick(2560, 8192, 11008) == "duo_dl_m128"
    assert _pick(4096 + 40, 8192, 8192) == "duo_dl_m128"       # (rounds of 256-row tiles: 3 against 2.06) ragged last row tile of at most 64 rows: its two-fragment path
    assert _pick(4096 + 100, 8192, 8192) == "duo_pt_m128"
    with pytest.raises(api.LiquidGemmError):
        api.w4a8_select_variant(8, 100, 512, 64)                # bad shape


def _plan(M, N, K, g=64):
    return [(rows, api.w4a8_variant_name(v)) for rows, v in api.w4a8_select_plan(M, N, K, g)]


def test_two_launch_plans():
    """Batches whose 256 x 256 tiles make whole rounds of the chip plus a rest of at most 256 rows,
    or a larger rest that does not take 256 x 256 tiles itself, run as two launches over consecutive
    rows where the cost rule says so; everything else as one, which is then the dispatcher's choice."""
    assert _plan(4096 + 40, 8192, 8192) == [(4096, "solo16_pt_m256"), (40, "stream_m64")]      # a ragged tail of the batch
    assert _plan(2048 + 100, 8192, 4096) == [(2048, "solo16_pt_m256"), (100, "duo_m64")]
    assert _plan(1024 + 30, 16384, 4096, 128) == [(1024, "solo16_pt_m256"), (30, "stream_m32")]
    # larger rests that fill most of a round of 256 x 128 tiles (143 against 150 us, 157 against 162, 240 against 255)
    assert _plan(2048, 10240, 8192, 128) == [(1536, "solo16_pt_m256"), (512, "solo16_g2_m256")]
    assert _plan(3072, 8192, 8192) == [(2048, "solo16_pt_m256"), (1024, "solo16_g2_m256")]
    assert _plan(1280, 28672, 8192, 128) == [(1024, "solo16_pt_m256"), (256, "solo16_g2_m256")]
    assert _plan(2748, 8192, 4096) == [(2048, "solo16_pt_m256"), (700, "solo16_g2_m256")]
    # ... also a rest on 128-row tiles (143 against 156 us, 423 against 513)
    assert _plan(2560, 8192, 8192) == [(2048, "solo16_pt_m256"), (512, "duo_m128")]
    assert _plan(2560, 8192, 28672, 128) == [(2048, "solo16_pt_m256"), (512, "solo16_g2_sk_m256")]
    # ... but not a rest that would be 256 x 256 tiles again, nor with short K
    assert _plan(3584, 8192, 8192) == [(3584, "solo16_pt_m256")] and _plan(2304, 11008, 4096) == [(2304, "solo16_pt_m256")]
    assert _plan(2748, 8192, 512) == [(2748, _pick(2748, 8192, 512))]
    # K % 512 == 256 splits like any other K (the 16x16x64 forms take it)
    assert _plan(3072, 8192, 8448) == [(2048, "solo16_pt_m256"), (1024, "solo16_g2_m256")]
    for M, N, K, g in [(4096, 8192, 8192, 64), (2048, 28672, 8192, 128), (1536, 8192, 8192, 64), (16, 8192, 8192, 64),
                       (256, 8192, 8192, 64), (2048, 11008, 4096, 64), (0, 4096, 4096, 64)]:
        assert _plan(M, N, K, g) == [(M, _pick(M, N, K, g))], (M, N, K)
    for s in WL.ALL_SHAPES:
        plan = api.w4a8_select_plan(s.M, s.N, s.K, s.group)
        assert sum(rows for rows, _ in plan) == s.M and all(rows > 0 for rows, _ in plan)
        assert all(api.w4a8_variant_supports(v, rows, s.N, s.K, s.group) for rows, v in plan)
        assert len(plan) == 1 or plan[0][0] % 256 == 0


def test_variant_table_is_consistent():
    names = api.w4a8_variant_names()
    assert len(names) == len(set(names)) == api.w4a8_variant_count()
    for v, name in enumerate(names):
        # row limits are part of the names' families
        limit = (16 if name.startswith("stream16") else 64 if name.startswith("stream_m64")
                 else 32 if name.startswith(("stream_f", "stream_x_", "stream_m32"))
                 else 256 if name in ("solo16_pt_m256_s2", "solo16_g2_m256_s4") else None)
        if limit:
            assert api.w4a8_variant_supports(v, limit, 256, 2048, 64)
            assert not api.w4a8_variant_supports(v, limit + 1, 256, 2048, 64)
        else:
            assert api.w4a8_variant_supports(v, 4096, 256, 1024, 64)
        assert not api.w4a8_variant_supports(v, 8, 96, 1024, 64)   # N % 64 != 0
        assert not api.w4a8_variant_supports(v, 8, (1 << 26) + 64, 1024, 64)   # rows addressed in 32 bits
        assert not api.w4a8_variant_supports(v, 8, 256, 131072 + 256, 64)      # the accumulator's range
    assert not api.w4a8_variant_supports(-1, 8, 256, 1024, 64)
    assert not api.w4a8_variant_supports(len(names), 8, 256, 1024, 64)


def test_workspace_sizes():
    ws = api.w4a8_gemm_workspace_size
    assert ws(0, 4096, 4096, 64) == 0 and ws(16, 100, 4096, 64) == 0     # nothing to do / bad shape
    assert ws(4096, 8192, 8192, 64) == 0                                  # enough tiles: no split-K
    small = ws(16, 4096, 4096, 64)
    assert small > 0 and small % 16 == 0
    # room for 16 slices of the 16-row kernels' partial tiles at least
    assert small >= 16 * (4096 // 32) * 8 * 64 * 4
    # the tiled kernel's partial tiles (128 x 256 INT32 per tile and slice, up to 8 slices)
    assert ws(128, 4096, 4096, 64) >= 16 * 8 * 128 * 256 * 4
    assert ws(128, 4096, 4096, 64) <= 1 << 30


def test_workload_names():
    # the listed shapes by name, and any other shape spelled <label>_M.._N.._K..[_g..]
    s = WL.by_name("l70b_up_M16_N28672_K8192")
    assert (s.M, s.N, s.K, s.group) == (16, 28672, 8192, 128)
    s = WL.by_name("curve_M64_N8192_K8192_g128")
    assert (s.M, s.N, s.K, s.group) == (64, 8192, 8192, 128)
    assert WL.by_name("x_M3_N64_K256").group == 64
    for bad in ("bogus", "x_M3_N64", "x_M3_N64_K256_g32", "_M3_N64_K256"):
        with pytest.raises(KeyError):
            WL.by_name(bad)
