"""CPU tests of the C-ABI library: symbols, the offline LiquidQuant packer against the
oracle (through liquidquant_unpack_weights), and host-side argument checking.
No test here launches GPU work."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import lqq_oracle as O
from paper_2509_01229_amd import api
from paper_2509_01229_amd import workloads as WL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "liquidgemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(w4a8_\w+|liquidquant_\w+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = api.lib()
    names = _declared_symbols()
    assert len(names) >= 14
    for name in names:
        assert hasattr(L, name), f"{name} declared in liquidgemm.h but not exported"
    assert api.w4a8_version() >= 1
    assert api.w4a8_variant_count() >= 2
    assert all(api.w4a8_variant_names())
    assert api.w4a8_variant_name(10**6) is None


def test_packed_size_and_shape_rules():
    assert api.liquidquant_packed_size(256, 512, 64) == (256 * 512 // 2, 256 * 8 * 2)
    assert api.liquidquant_packed_size(64, 256, 128) == (64 * 128, 64 * 2 * 2)
    for bad in [(100, 512, 64), (256, 500, 64), (256, 512, 32), (0, 512, 64), (256, 262144, 64)]:
        with pytest.raises(api.LiquidGemmError) as e:
            api.liquidquant_packed_size(*bad)
        assert e.value.code == api.LQ_ERR_INVALID
    assert api.w4a8_gemm_workspace_size(16, 4096, 4096, 64) >= 0


@pytest.mark.parametrize("N,K,g,seed", [(256, 512, 64, 0), (64, 256, 128, 1), (192, 1024, 128, 2),
                                        (128, 768, 64, 3)])
def test_packer_matches_oracle_quantizer(N, K, g, seed):
    W = WL.make_weights(N, K, sigma=0.02, seed=seed)
    ref = O.quantize_weights(W, g)
    packed, gparams, w_scales = api.liquidquant_pack_weights(W, g)
    codes, s_u8, a = api.liquidquant_unpack_weights(packed, gparams, N, K, g)
    assert np.array_equal(w_scales.view(np.uint32), ref["s_w"].view(np.uint32))
    assert np.array_equal(codes, ref["Q_u4"])
    assert np.array_equal(s_u8, ref["s_u8"])
    assert np.array_equal(a, ref["a"])
    # FP16 entry point gives the same blob
    p16, g16, s16 = api.liquidquant_pack_weights(W.astype(np.float16), g)
    assert np.array_equal(p16, packed) and np.array_equal(g16, gparams) and np.array_equal(s16, w_scales)
    # level-2-only entry point from the oracle's level-1 integers
    p8, g8 = api.liquidquant_pack_from_i8(ref["Q_i8"], g)
    assert np.array_equal(p8, packed) and np.array_equal(g8, gparams)


@pytest.mark.parametrize("style", ["uniform", "extreme", "constant", "narrow"])
@pytest.mark.parametrize("g", [64, 128])
def test_pack_from_i8_edge_distributions(style, g):
    N, K = 64, 512
    Q = WL.make_q_i8(N, K, seed=7, style=style)
    Q_u4, s_u8, mn = O.level2_quantize(Q, g)
    packed, gparams = api.liquidquant_pack_from_i8(Q, g)
    codes, s_lib, a_lib = api.liquidquant_unpack_weights(packed, gparams, N, K, g)
    assert np.array_equal(codes, Q_u4)
    assert np.array_equal(s_lib, s_u8)
    assert np.array_equal(a_lib, O.offset_a(mn))
    # Eq. 11 holds for every triple the packer emits
    t = codes.astype(np.int32) * np.repeat(s_lib, g, axis=1) + np.repeat(a_lib, g, axis=1)
    assert t.max() <= 255


def test_packed_blob_is_a_permutation_of_the_codes():
    # every (n, k) owns exactly one nibble: mark one element at a time in a tiny matrix
    N, K, g = 64, 256, 64
    rng = np.random.default_rng(0)
    for _ in range(12):
        n, k = int(rng.integers(N)), int(rng.integers(K))
        Q = np.zeros((N, K), dtype=np.int8)
        Q[n, k] = 15                      # group range 15 -> s = 1, code 15 at (n, k) only
        packed, gparams = api.liquidquant_pack_from_i8(Q, g)
        nz = np.flatnonzero(packed)
        assert len(nz) == 1 and packed[nz[0]] in (0x0F, 0xF0)
        codes, s_u8, a = api.liquidquant_unpack_weights(packed, gparams, N, K, g)
        assert codes[n, k] == 15 and codes.sum() == 15
        assert s_u8[n, k // g] == 1 and (a == 128).all()


def test_fp16_subnormals_and_zero_rows():
    N, K, g = 64, 256, 64
    W = np.zeros((N, K), dtype=np.float16)
    W[1, :] = np.float16(6e-8)            # smallest subnormal
    W[2, 0::2] = np.float16(1e-6)
    W[2, 1::2] = np.float16(-3e-6)
    packed, gparams, s_w = api.liquidquant_pack_weights(W, g)
    ref = O.quantize_weights(W.astype(np.float32), g)
    codes, s_u8, a = api.liquidquant_unpack_weights(packed, gparams, N, K, g)
    assert np.array_equal(s_w.view(np.uint32), ref["s_w"].view(np.uint32))
    assert np.array_equal(codes, ref["Q_u4"]) and np.array_equal(a, ref["a"])
    assert s_w[0] == 1.0


def test_host_argument_checks():
    W = np.zeros((64, 256), dtype=np.float32)
    W[0, 0] = np.inf
    with pytest.raises(api.LiquidGemmError):
        api.liquidquant_pack_weights(W, 64)
    Q = np.zeros((64, 256), dtype=np.int8)
    Q[3, 3] = 120
    with pytest.raises(api.LiquidGemmError) as e:
        api.liquidquant_pack_from_i8(Q, 64)
    assert "protective range" in str(e.value)
    with pytest.raises(api.LiquidGemmError):
        api.liquidquant_pack_weights(np.zeros((65, 256), np.float32), 64)
    # device entry points validate shapes and pointers on the host before any launch
    L = api.lib()
    null = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(0x1000)
    assert L.w4a8_gemm(4, 100, 256, 64, fake, fake, fake, fake, fake, fake, null, 0, null) == api.LQ_ERR_INVALID
    assert L.w4a8_gemm(4, 64, 256, 64, null, fake, fake, fake, fake, fake, null, 0, null) == api.LQ_ERR_INVALID
    assert L.w4a8_gemm(-1, 64, 256, 64, fake, fake, fake, fake, fake, fake, null, 0, null) == api.LQ_ERR_INVALID
    mis = ctypes.c_void_p(0x1008)
    assert L.w4a8_gemm(4, 64, 256, 64, mis, fake, fake, fake, fake, fake, null, 0, null) == api.LQ_ERR_ALIGN
    assert b"aligned" in L.w4a8_last_error()
    assert L.w4a8_gemm_variant(999, 4, 64, 256, 64, fake, fake, fake, fake, fake, fake, null, null, 0,
                               null) == api.LQ_ERR_INVALID
    assert L.w4a8_dequant_dump(fake, fake, 64, 100, 64, fake, null) == api.LQ_ERR_INVALID
    # M = 0 is a successful no-op
    assert L.w4a8_gemm(0, 64, 256, 64, fake, fake, fake, fake, fake, fake, null, 0, null) == api.LQ_OK
    assert api.w4a8_select_variant(1, 4096, 4096, 64) >= 0
    with pytest.raises(api.LiquidGemmError):
        api.w4a8_select_variant(1, 4000, 4096, 64)


def test_w8a8_packer_layout():
    """INT8 weights of the W8A8 reference: per tile of 32 channels and k-step of 32, lane
    32*kb + j holds W[n][32*step + 16*kb + 0..15] in 16 consecutive bytes, n = 64*(tile//2) +
    2*j + tile%2 (the two tiles of a 64-channel group interleave)."""
    rng = np.random.default_rng(3)
    N, K = 128, 512
    W = rng.integers(-128, 128, size=(N, K), dtype=np.int64).astype(np.int8)
    blob = api.w8a8_pack_weights(W).view(np.int8).reshape(N // 32, K // 32, 2, 32, 16)   # tile, step, kb, j, byte
    for tile in range(N // 32):
        for step in (0, 5, K // 32 - 1):
            for kb in range(2):
                rows = 64 * (tile // 2) + 2 * np.arange(32) + tile % 2
                want = W[rows, 32 * step + 16 * kb:32 * step + 16 * kb + 16]
                assert np.array_equal(blob[tile, step, kb], want)
    # every weight appears exactly once
    assert np.array_equal(np.sort(blob.ravel()), np.sort(W.ravel()))
    with pytest.raises(api.LiquidGemmError):
        api.w8a8_pack_weights(np.zeros((64, 100), dtype=np.int8))
