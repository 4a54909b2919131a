"""Plain, slow, obviously-correct CPU oracle of the LiquidQuant (LQQ) W4A8 GEMM.

TEST INFRASTRUCTURE ONLY: used by tests/, the smoke check and the cpu_baseline
leg of the benchmark.  It shares no code with the HIP library and never imports
it.  Every function is the definition in the paper written out with numpy,
without blocking, fusion or reordering.

Notation follows the paper: W is [N, K] (N output channels, K reduction), X is
[M, K], Y = X W^T is [M, N]; g is the group size along K and G = K / g.

Pinning status (tests/test_oracle_pins.py):
  level1_quantize    pinned: closed forms (scale = amax/119, range, sign symmetry,
                     exact grid recovery), brute-force scalar re-derivation.
  level2_quantize    pinned: the paper's worked example (Sec. 4), the bounds of
                     Sec. 4 (s <= 16, code*s <= 240, code*s + a <= 255) by
                     exhaustive enumeration, reconstruction-error bound.
  dequant_plain /    pinned: exhaustive identity Eq. 8 == Eq. 12 over every
  dequant_bits       admissible (min, max, q); the worked example (121, bit patterns).
  pack/unpack        pinned: round trip, hand-written byte example.
  matmul_i64         pinned: pure-Python brute force on tiny shapes, exact float64
                     BLAS product on larger ones, one-hot / all-ones special cases.
  scale_epilogue     double-precision product then one RNE rounding to FP16;
                     pinned on exactly representable cases only.  The exact FP16
                     rounding of the product is not fixed by the paper:
                     "parity unpinned" beyond the 1-ulp tolerance.
  quantize_activations  pinned: hand example with a tie (round half to even), the
                     extreme element maps to +-127, zero row, exact power-of-two scale
                     invariance, reconstruction error <= s_x / 2, smooth divide
                     against exact rational arithmetic.

  w8a8_gemm          matmul_i64 + scale_epilogue on INT8 weights: pinned through them.

  grouped_w4a8_gemm  pinned: brute force in Python integers on a tiny case, independence of
                     every expert's rows from the other experts' weights, empty experts,
                     the single-expert case.

Readings of the paper taken here (the paper is silent or ambiguous on them):
  * s_u8 is an integer: round(R / 15) with R = max - min of the group, computed
    as (2R + 15) // 30 (no ties are possible since 15 is odd); matches the
    worked example 223/15 -> 15 and the bound 238/15 -> 16 of Sec. 4.
  * a constant group (R = 0) takes s_u8 = 1.
  * codes are rounded half-up in integers, (2 q_u + s) // (2 s), and clamped to
    15 (s rounded down can otherwise give 16 or more).
  * activations (Sec. 6 "Serving System": dynamic per-token INT8 after dividing by the
    smooth scale) are quantized symmetrically per token over the full INT8 range:
    x' = X / smooth in FP32, s_x = max_k |x'| / 127 in FP32 (1 for an all-zero token),
    Q = clamp(rint(x' / s_x), -127, 127).
  * level 1 is symmetric per output channel with the protective range:
    s_w = amax / 119 in FP32, Q = clamp(rint(W / s_w), -119, 119); an all-zero
    channel takes s_w = 1.
"""
from __future__ import annotations

import numpy as np

Q_PROTECT = 119  # protective INT8 range of Sec. 4 ("Quantization")
U4_MAX = 15


# --------------------------------------------------------------------------
# Activations: FP16 -> INT8, per token  (Sec. 6 "Serving System")
# --------------------------------------------------------------------------
def quantize_activations(X, smooth=None):
    """Dynamic per-token symmetric INT8 quantization after the smooth divide.

    X: [M, K] FP16 values (any float dtype holding them); smooth: [K] positive FP32
    smooth scales or None.  The arithmetic is FP32 because its roundings decide
    integers and the library takes the same decisions in FP32: every operation below is
    one correctly rounded IEEE binary32 operation.  Returns (Q_i8 [M, K] int8,
    s_x [M] float32).
    """
    Xs = np.asarray(X, dtype=np.float32)
    if smooth is not None:
        Xs = Xs / np.asarray(smooth, dtype=np.float32)[None, :]
    amax = np.max(np.abs(Xs), axis=1).astype(np.float32) if Xs.shape[1] else np.zeros(Xs.shape[0], np.float32)
    s_x = np.where(amax > 0, amax / np.float32(127), np.float32(1.0)).astype(np.float32)
    q = np.rint(Xs / s_x[:, None])  # FP32 quotient, round half to even
    return np.clip(q, -127, 127).astype(np.int8), s_x


# --------------------------------------------------------------------------
# Level 1: FP -> INT8, per output channel  (Sec. 4 "Quantization"; Eq. 1 with z = 0)
# --------------------------------------------------------------------------
def level1_quantize(W):
    """Per-channel symmetric quantization into the protective range [-119, 119].

    W: [N, K] float (FP16 values are passed widened to FP32; the arithmetic is
    FP32 because the rounding decides an integer and the library takes the same
    decision in FP32).  Returns (Q_i8 [N, K] int8, s_w [N] float32).
    """
    W = np.asarray(W, dtype=np.float32)
    amax = np.max(np.abs(W), axis=1).astype(np.float32)
    s_w = np.where(amax > 0, amax / np.float32(Q_PROTECT), np.float32(1.0)).astype(np.float32)
    q = np.rint(W / s_w[:, None])  # FP32 quotient, round half to even
    q = np.clip(q, -Q_PROTECT, Q_PROTECT)
    return q.astype(np.int8), s_w


# --------------------------------------------------------------------------
# Level 2: INT8 -> UINT4, per group of g along K  (Sec. 4, Eq. 7)
# --------------------------------------------------------------------------
def level2_quantize(Q_i8, g):
    """Shift each group to the unsigned domain and quantize to 4 bits (Eq. 7).

    Returns (Q_u4 [N, K] uint8 in 0..15, s_u8 [N, G] uint8 in 1..16,
             mn [N, G] int16 = min(Q_i8) of the group).
    """
    Q = np.asarray(Q_i8).astype(np.int32)
    N, K = Q.shape
    assert K % g == 0
    G = K // g
    Qg = Q.reshape(N, G, g)
    mn = Qg.min(axis=2)                       # min(Q_i8)
    mx = Qg.max(axis=2)
    R = mx - mn                               # max(Q_u8), in 0..238
    s = np.maximum(1, (2 * R + U4_MAX) // (2 * U4_MAX))   # round(R / 15), at least 1
    Qu8 = Qg - mn[:, :, None]                 # Q_u8 = Q_i8 - min(Q_i8)
    s3 = s[:, :, None]
    Qu4 = (2 * Qu8 + s3) // (2 * s3)          # round(Q_u8 / s_u8), half up
    Qu4 = np.minimum(Qu4, U4_MAX)
    return (Qu4.reshape(N, K).astype(np.uint8), s.astype(np.uint8), mn.astype(np.int16))


def offset_a(mn):
    """a = 2^7 + min(Q_i8), the per-group offset stored offline (Eq. 10 / Eq. 12)."""
    a = 128 + np.asarray(mn).astype(np.int32)
    assert a.min() >= 0 and a.max() <= 255
    return a.astype(np.uint8)


# --------------------------------------------------------------------------
# Canonical nibble packing (oracle-private storage: two codes per byte, row-major)
# --------------------------------------------------------------------------
def pack_canonical(Q_u4):
    """byte[n, k/2] = code[n, k] | code[n, k+1] << 4 for even k."""
    Q = np.asarray(Q_u4, dtype=np.uint8)
    assert Q.shape[1] % 2 == 0 and Q.max(initial=0) <= U4_MAX
    return (Q[:, 0::2] | (Q[:, 1::2] << 4)).astype(np.uint8)


def unpack_canonical(packed):
    P = np.asarray(packed, dtype=np.uint8)
    N, Kh = P.shape
    Q = np.empty((N, 2 * Kh), dtype=np.uint8)
    Q[:, 0::2] = P & 0x0F
    Q[:, 1::2] = P >> 4
    return Q


# --------------------------------------------------------------------------
# Dequantization UINT4 -> INT8
# --------------------------------------------------------------------------
def _expand(per_group, g):
    return np.repeat(np.asarray(per_group), g, axis=1)


def dequant_plain(Q_u4, s_u8, mn, g):
    """Eq. 8: Q^_i8 = Q_u4 * s_u8 + min(Q_i8), in ordinary signed integers."""
    v = np.asarray(Q_u4).astype(np.int32) * _expand(s_u8, g).astype(np.int32) \
        + _expand(mn, g).astype(np.int32)
    assert v.min(initial=0) >= -128 and v.max(initial=0) <= 127, "Eq. 8 left the INT8 range"
    return v.astype(np.int8)


def dequant_bits(Q_u4, s_u8, a, g):
    """Eq. 12: (Q_u4 * s_u8 + a) XOR 0x80, every intermediate held in UINT8."""
    t = np.asarray(Q_u4).astype(np.int32) * _expand(s_u8, g).astype(np.int32) \
        + _expand(a, g).astype(np.int32)
    assert t.max(initial=0) <= 255, "Eq. 11 violated: q^_u + a exceeds UINT8"
    u = t.astype(np.uint8) ^ np.uint8(0x80)
    return u.view(np.int8)


# --------------------------------------------------------------------------
# Main loop: integer matmul  (Sec. 2 "GEMM on GPUs": Y = X W^T, INT8 x INT8 -> INT32)
# --------------------------------------------------------------------------
def matmul_i64(X_i8, Wd_i8):
    """ACC[m, n] = sum_k X[m, k] * Wd[n, k] accumulated in int64, checked to fit int32."""
    acc = np.asarray(X_i8).astype(np.int64) @ np.asarray(Wd_i8).astype(np.int64).T
    assert np.abs(acc).max(initial=0) < 2**31, "accumulator leaves INT32"
    return acc.astype(np.int32)


# --------------------------------------------------------------------------
# Epilogue: first-level dequantization to FP16  (Sec. 4 last sentence; Sec. 5.3; Sec. 6)
# --------------------------------------------------------------------------
def scale_epilogue(ACC, s_x, s_w):
    """Y[m, n] = fp16( ACC[m, n] * s_x[m] * s_w[n] ), product in double, one rounding."""
    y = np.asarray(ACC).astype(np.float64) \
        * np.asarray(s_x, dtype=np.float64)[:, None] \
        * np.asarray(s_w, dtype=np.float64)[None, :]
    with np.errstate(over="ignore"):
        return y.astype(np.float16)


def scale_epilogue_f64(ACC, s_x, s_w):
    """The same product before the FP16 rounding (for tolerance checks)."""
    return np.asarray(ACC).astype(np.float64) \
        * np.asarray(s_x, dtype=np.float64)[:, None] \
        * np.asarray(s_w, dtype=np.float64)[None, :]


# --------------------------------------------------------------------------
# Whole path
# --------------------------------------------------------------------------
def quantize_weights(W, g):
    """Offline path: W (float) -> dict of LQQ arrays in canonical (unpermuted) form."""
    Q_i8, s_w = level1_quantize(W)
    Q_u4, s_u8, mn = level2_quantize(Q_i8, g)
    return {
        "Q_i8": Q_i8, "s_w": s_w, "Q_u4": Q_u4, "s_u8": s_u8, "mn": mn,
        "a": offset_a(mn), "packed": pack_canonical(Q_u4), "g": g,
    }


def w4a8_gemm(X_i8, s_x, packed, s_u8, a, s_w, g):
    """unpack -> Eq. 8 dequant (checked against Eq. 12) -> int64 matmul -> scale -> FP16.

    Returns (ACC int32 [M, N], Y float16 [M, N]).
    """
    Q_u4 = unpack_canonical(packed)
    mn = np.asarray(a).astype(np.int16) - 128
    Wd = dequant_plain(Q_u4, s_u8, mn, g)
    assert np.array_equal(Wd, dequant_bits(Q_u4, s_u8, a, g)), "Eq. 8 and Eq. 12 disagree"
    ACC = matmul_i64(X_i8, Wd)
    return ACC, scale_epilogue(ACC, s_x, s_w)


def w8a8_gemm(X_i8, s_x, W_i8, s_w):
    """The W8A8 baseline of Sec. 3.2 / 7.3 (INT8 weights, no second-level dequantization):
    the same main loop and epilogue on the level-1 weights.  Returns (ACC int32, Y float16)."""
    ACC = matmul_i64(X_i8, W_i8)
    return ACC, scale_epilogue(ACC, s_x, s_w)


# --------------------------------------------------------------------------
# Grouped GEMM (mixture-of-experts layers, Sec. 7.3: a batch of independent GEMMs, one
# per expert, over disjoint runs of tokens)
# --------------------------------------------------------------------------
def grouped_w4a8_gemm(X_i8, s_x, row_offsets, experts):
    """Expert e owns tokens row_offsets[e] .. row_offsets[e+1]-1 of X and multiplies them
    with its own quantized weights experts[e] (a dict as returned by quantize_weights);
    nothing is shared between experts.  Returns (ACC int32 [M, N], Y float16 [M, N])."""
    X_i8 = np.asarray(X_i8)
    row_offsets = [int(r) for r in row_offsets]
    assert len(row_offsets) == len(experts) + 1 and row_offsets[0] == 0 and row_offsets[-1] == X_i8.shape[0]
    N = experts[0]["Q_u4"].shape[0]
    ACC = np.zeros((X_i8.shape[0], N), dtype=np.int32)
    Y = np.zeros((X_i8.shape[0], N), dtype=np.float16)
    for e, q in enumerate(experts):
        r0, r1 = row_offsets[e], row_offsets[e + 1]
        assert r1 >= r0
        if r1 == r0:
            continue
        ACC[r0:r1], Y[r0:r1] = w4a8_gemm(X_i8[r0:r1], np.asarray(s_x)[r0:r1], q["packed"], q["s_u8"], q["a"],
                                         q["s_w"], q["g"])
    return ACC, Y
