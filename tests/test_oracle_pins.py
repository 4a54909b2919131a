"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP library.  Each pin compares the oracle with
something other than itself: values the paper prints (tests/golden/), closed forms,
exhaustive enumeration of the Sec. 4 bounds, pure-Python brute force, or a library
routine that is exact for the case (float64 BLAS on small integers).
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import c_oracle
from oracle import lqq_oracle as O
from paper_2509_01229_amd import workloads as WL

import inputs as I


# --------------------------------------------------------------------------
# Worked example of Sec. 4 (values from tests/golden/worked_example_sec4.txt)
# --------------------------------------------------------------------------
def test_worked_example_values(golden_sec4):
    gd = golden_sec4
    mn, mx = int(gd["min_q_i8"]), int(gd["max_q_i8"])
    g = 64
    row = np.full(g, mn, dtype=np.int8)
    row[5] = mx
    row[9] = 0
    Q_u4, s_u8, mn_out = O.level2_quantize(row[None, :], g)
    assert int(s_u8[0, 0]) == int(gd["s_u8"])
    assert int(mn_out[0, 0]) == mn
    assert int(Q_u4[0, 5]) == int(gd["q_u4"])
    assert mx - mn == int(gd["range_u8"])
    a = O.offset_a(mn_out)
    assert int(a[0, 0]) == 128 + mn
    Wd = O.dequant_plain(Q_u4, s_u8, mn_out, g)
    assert int(Wd[0, 5]) == int(gd["q_i8_hat"])
    assert int(O.dequant_bits(Q_u4, s_u8, a, g)[0, 5]) == int(gd["q_i8_hat"])
    assert int(Q_u4[0, 5]) * int(s_u8[0, 0]) == int(gd["q_u8_hat"])


def test_worked_example_bit_patterns(golden_sec4):
    gd = golden_sec4
    q_u8_hat = int(gd["q_u8_hat"])
    mn = int(gd["min_q_i8"])
    assert format(q_u8_hat, "08b") == gd["q_u8_hat_bits"]
    assert format(mn & 0xFF, "08b") == gd["min_q_i8_bits"]
    assert format(q_u8_hat + (mn & 0xFF), "b") == gd["naive_sum_bits"]      # 9 bits: overflow
    assert int(np.array([q_u8_hat], dtype=np.uint8).view(np.int8)[0]) == int(gd["q_u8_hat_as_int8"])
    # two's complement congruence example
    i, j = int(gd["congruent_i8"]), int(gd["congruent_u8"])
    assert (i - j) % 256 == 0 and format(j, "08b") == gd["congruent_bits"]
    assert int(np.array([i], dtype=np.int8).view(np.uint8)[0]) == j


# --------------------------------------------------------------------------
# Exhaustive enumeration over every admissible (min, max) pair of a group
# --------------------------------------------------------------------------
@pytest.fixture(scope="module")
def all_groups():
    """One row per (min, max) with min <= max in [-119, 119]; the row holds every
    integer of [min, max] once (padded with min), so every reachable q appears."""
    P = O.Q_PROTECT
    pairs = [(mn, mx) for mn in range(-P, P + 1) for mx in range(mn, P + 1)]
    g = 2 * P + 2  # 240 >= 239 distinct values
    rows = np.empty((len(pairs), g), dtype=np.int8)
    for i, (mn, mx) in enumerate(pairs):
        vals = np.arange(mn, mx + 1)
        rows[i, :len(vals)] = vals
        rows[i, len(vals):] = mn
    return pairs, rows, g


def test_exhaustive_bounds_and_identity(all_groups, golden_sec4):
    pairs, rows, g = all_groups
    assert len(pairs) == 239 * 240 // 2
    Q_u4, s_u8, mn = O.level2_quantize(rows, g)
    a = O.offset_a(mn)
    s = s_u8.astype(np.int32)[:, 0]
    assert np.array_equal(mn[:, 0], np.array([p[0] for p in pairs]))
    # Sec. 4 bounds
    assert s.min() >= 1 and s.max() == int(golden_sec4["s_u8_max"])
    assert Q_u4.max() == 15 and Q_u4.min() == 0
    prod = Q_u4.astype(np.int32) * s[:, None]
    assert prod.max() <= int(golden_sec4["q_u8_hat_max"])
    pre_xor = prod + a.astype(np.int32)
    assert pre_xor.max() <= int(golden_sec4["eq11_bound"])        # Eq. 11
    assert pre_xor.min() >= 0
    # Eq. 8 == Eq. 12 for every reachable element
    plain = O.dequant_plain(Q_u4, s_u8, mn, g)
    bits = O.dequant_bits(Q_u4, s_u8, a, g)
    assert np.array_equal(plain, bits)
    # MSB flip == adding b = +-128 (proof of Sec. 4): x = 0 iff q^_u + a >= 128
    b = np.where(pre_xor >= 128, -128, 128)
    assert np.array_equal((pre_xor + b).astype(np.int32) % 256, bits.view(np.uint8).astype(np.int32))
    # dequantised values stay a valid INT8 and never fall below the group minimum
    assert plain.min() >= -119 and plain.max() <= 127
    assert (plain.astype(np.int32) >= mn.astype(np.int32)).all()


def test_exhaustive_scale_is_round_to_nearest(all_groups):
    pairs, rows, g = all_groups
    _, s_u8, _ = O.level2_quantize(rows, g)
    for (mn, mx), s in zip(pairs[::37], s_u8[::37, 0]):
        R = mx - mn
        exact = Fraction(R, 15)
        nearest = int(exact + Fraction(1, 2))        # floor(x + 1/2)
        assert (exact - int(exact)) != Fraction(1, 2)  # no tie can occur: 15 is odd
        assert int(s) == max(1, nearest)


def test_exhaustive_reconstruction_error(all_groups):
    pairs, rows, g = all_groups
    Q_u4, s_u8, mn = O.level2_quantize(rows, g)
    Wd = O.dequant_plain(Q_u4, s_u8, mn, g).astype(np.int32)
    err = np.abs(Wd - rows.astype(np.int32))
    s = s_u8.astype(np.int32)
    unclamped = (2 * (rows.astype(np.int32) - mn) + s) // (2 * s) <= 15
    # rounding to the nearest multiple of s: error at most s/2 where no clamp happened
    assert (2 * err[unclamped] <= np.broadcast_to(s, err.shape)[unclamped]).all()
    # with the clamp to code 15 the error stays below one INT8 step of 8
    assert err.max() <= 8
    # the group minimum is reproduced exactly (code 0)
    assert (Wd[np.arange(len(pairs)), 0] == mn[:, 0]).all()


def test_constant_group_takes_scale_one():
    Q = np.full((3, 128), -7, dtype=np.int8)
    Q_u4, s_u8, mn = O.level2_quantize(Q, 64)
    assert (s_u8 == 1).all() and (Q_u4 == 0).all() and (mn == -7).all()
    assert (O.dequant_plain(Q_u4, s_u8, mn, 64) == -7).all()


def test_level2_codes_round_half_up_hand_example():
    """The tie rule of Eq. 7's rounding to nearest, worked by hand.  A group whose values
    span 0..30 has s_u8 = round(30 / 15) = 2, so every odd Q_u8 is a tie: 1/2 = 0.5,
    3/2 = 1.5, 5/2 = 2.5.  Half-up (the reading taken) gives codes 1, 2, 3; half-to-even
    would give 0, 2, 2 and half-down 0, 1, 2, so this one group tells the three apart.
    The shifted group (min = -50) must give the same codes."""
    for shift in (0, -50):
        Q = np.zeros((1, 64), dtype=np.int8)
        Q[0, :6] = np.array([0, 1, 3, 5, 29, 30]) + shift
        Q[0, 6:] = shift
        Q_u4, s_u8, mn = O.level2_quantize(Q, 64)
        assert s_u8[0, 0] == 2 and mn[0, 0] == shift
        assert Q_u4[0, :6].tolist() == [0, 1, 2, 3, 15, 15]
        # what the codes decode to (Eq. 8): multiples of s above the minimum
        assert O.dequant_plain(Q_u4, s_u8, mn, 64)[0, :6].tolist() == [shift + v for v in (0, 2, 4, 6, 30, 30)]
    # a tie at s = 4 (R = 60): Q_u8 = 2, 6, 10 -> 0.5, 1.5, 2.5 -> codes 1, 2, 3
    Q = np.zeros((1, 64), dtype=np.int8)
    Q[0, :4] = [2, 6, 10, 60]
    Q_u4, s_u8, _ = O.level2_quantize(Q, 64)
    assert s_u8[0, 0] == 4 and Q_u4[0, :4].tolist() == [1, 2, 3, 15]


def test_groups_run_along_k():
    # group j of every row is the constant j - 3: a grouping along N would mix them
    N, g, G = 5, 64, 6
    Q = np.repeat(np.arange(G, dtype=np.int8)[None, :] - 3, g, axis=1).repeat(N, axis=0)
    Q_u4, s_u8, mn = O.level2_quantize(Q, g)
    assert mn.shape == (N, G)
    assert np.array_equal(mn, np.broadcast_to(np.arange(G) - 3, (N, G)))
    assert (Q_u4 == 0).all() and (s_u8 == 1).all()


# --------------------------------------------------------------------------
# Level 1
# --------------------------------------------------------------------------
def test_level1_closed_forms():
    step = np.float32(2.0 ** -10)
    q = np.arange(-119, 120, dtype=np.float32)
    W = np.stack([q * step, -q * step, np.zeros_like(q), 0.5 * q * step])
    Q, s_w = O.level1_quantize(W)
    assert s_w[0] == step and s_w[1] == step            # amax / 119 exactly
    assert np.array_equal(Q[0], q.astype(np.int8))      # the grid is recovered exactly
    assert np.array_equal(Q[1], -Q[0])                  # symmetric: Q(-W) = -Q(W)
    assert s_w[2] == 1.0 and (Q[2] == 0).all()          # all-zero channel
    assert s_w[3] == np.float32(0.5) * step and np.array_equal(Q[3], Q[0])  # scale invariance
    assert Q.min() == -119 and Q.max() == 119


def test_level1_rounds_half_to_even_and_matches_scalar_definition():
    W = np.array([[119.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49, -3.51]], dtype=np.float32)
    Q, s_w = O.level1_quantize(W)
    assert s_w[0] == 1.0
    assert Q[0].tolist() == [119, 0, 2, 2, 0, -2, -2, 3, -4]
    # scalar re-derivation with exact rationals on random FP16 data
    Wr = WL.make_weights(4, 96, sigma=0.02, seed=11)
    Qr, sr = O.level1_quantize(Wr)
    for n in range(4):
        amax = max(abs(float(v)) for v in Wr[n])
        assert sr[n] == np.float32(np.float32(amax) / np.float32(119))
        for k in range(96):
            quot = np.float32(Wr[n, k]) / sr[n]                 # the FP32 quotient decides
            fr = Fraction(float(quot))
            lo = fr.numerator // fr.denominator
            rem = fr - lo
            r = lo + (1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2) else 0)
            assert int(Qr[n, k]) == max(-119, min(119, r))


# --------------------------------------------------------------------------
# Canonical packing
# --------------------------------------------------------------------------
def test_pack_hand_example_and_round_trip():
    codes = np.array([[1, 2, 15, 0, 7, 8]], dtype=np.uint8)
    assert O.pack_canonical(codes).tolist() == [[0x21, 0x0F, 0x87]]
    rng = np.random.default_rng(3)
    Q = rng.integers(0, 16, size=(7, 64), dtype=np.uint8)
    assert np.array_equal(O.unpack_canonical(O.pack_canonical(Q)), Q)


# --------------------------------------------------------------------------
# Integer matmul and epilogue
# --------------------------------------------------------------------------
def _brute_matmul(X, Wd):
    M, K = X.shape
    N = Wd.shape[0]
    return [[sum(int(X[m, k]) * int(Wd[n, k]) for k in range(K)) for n in range(N)] for m in range(M)]


def test_matmul_brute_force_tiny():
    rng = np.random.default_rng(5)
    X = rng.integers(-127, 128, size=(3, 40), dtype=np.int8)
    Wd = rng.integers(-119, 127, size=(5, 40), dtype=np.int8)
    assert O.matmul_i64(X, Wd).tolist() == _brute_matmul(X, Wd)
    ACC_c, _ = c_oracle.matmul_scale(X, np.ones(3, np.float32), Wd, np.ones(5, np.float32))
    assert ACC_c.tolist() == _brute_matmul(X, Wd)


def test_matmul_special_cases_and_exact_blas():
    rng = np.random.default_rng(6)
    M, N, K = 9, 33, 256
    X = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
    Wd = rng.integers(-119, 127, size=(N, K), dtype=np.int8)
    X[2] = 0
    X[2, 17] = 1                       # one-hot row picks column 17 of Wd^T
    X[3] = 1                           # all-ones row gives row sums of Wd
    ACC = O.matmul_i64(X, Wd)
    assert np.array_equal(ACC[2], Wd[:, 17].astype(np.int32))
    assert np.array_equal(ACC[3], Wd.astype(np.int64).sum(axis=1))
    exact = X.astype(np.float64) @ Wd.astype(np.float64).T     # exact: |ACC| << 2^53
    assert np.array_equal(ACC.astype(np.float64), exact)
    ACC_c, _ = c_oracle.matmul_scale(X, np.ones(M, np.float32), Wd, np.ones(N, np.float32))
    assert np.array_equal(ACC_c, ACC)
    # worst case of the largest supported K stays inside INT32
    assert 131072 * 127 * 127 < 2**31


def test_epilogue_exact_cases():
    ACC = np.array([[3, -5], [1 << 20, 0]], dtype=np.int32)
    s_x = np.array([0.5, 1.0], dtype=np.float32)
    s_w = np.array([0.25, 2.0], dtype=np.float32)
    Y = O.scale_epilogue(ACC, s_x, s_w)
    assert Y.dtype == np.float16
    assert Y.tolist() == [[0.375, -5.0], [float("inf"), 0.0]]   # 2^18 overflows FP16
    # rows take s_x, columns take s_w (a swapped epilogue fails here)
    Y2 = O.scale_epilogue(np.ones((2, 3), np.int32), np.array([1, 2], np.float32),
                          np.array([1, 4, 16], np.float32))
    assert Y2.tolist() == [[1, 4, 16], [2, 8, 32]]
    # one rounding, to nearest even: 2049 -> 2048, 2051 -> 2052
    Y3 = O.scale_epilogue(np.array([[2049, 2051]], np.int32), np.ones(1, np.float32), np.ones(2, np.float32))
    assert Y3.tolist() == [[2048.0, 2052.0]]


# --------------------------------------------------------------------------
# Whole path: numpy oracle == C oracle == brute force
# --------------------------------------------------------------------------
def test_whole_path_tiny_config_three_ways():
    shp = WL.TINY[0]
    W, X, s_x = I.make_problem(shp)
    q = O.quantize_weights(W, shp.group)
    ACC, Y = O.w4a8_gemm(X, s_x, q["packed"], q["s_u8"], q["a"], q["s_w"], shp.group)
    ACC_c, Y_c = c_oracle.w4a8_gemm(X, s_x, q["packed"], q["s_u8"], q["a"], q["s_w"], shp.group)
    assert np.array_equal(ACC, ACC_c) and np.array_equal(Y.view(np.uint16), Y_c.view(np.uint16))
    # pure-Python brute force of the definition on a corner of the problem
    g, Kc, Nc, Mc = shp.group, 128, 6, 3
    for m in range(Mc):
        for n in range(Nc):
            acc = 0
            for k in range(shp.K):
                code = int(q["Q_u4"][n, k])
                acc += int(X[m, k]) * (code * int(q["s_u8"][n, k // g]) + int(q["mn"][n, k // g]))
            assert acc == int(ACC[m, n])
    # the quantised weights reproduce W to within the step sizes of both levels
    Wd = O.dequant_plain(q["Q_u4"], q["s_u8"], q["mn"], g).astype(np.float32) * q["s_w"][:, None]
    bound = q["s_w"][:, None] * (np.repeat(q["s_u8"], g, axis=1).astype(np.float32) / 2 + 8.5)
    assert (np.abs(Wd - W) <= bound).all()
    rel = np.linalg.norm(Wd - W) / np.linalg.norm(W)
    assert rel < 0.15
    # and the GEMM approximates the FP product of the unquantised operands
    ref = (X.astype(np.float64) * s_x[:, None]) @ W.astype(np.float64).T
    got = Y.astype(np.float64)
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 0.15


@pytest.mark.parametrize("M,N,K,g,seed", [(1, 64, 256, 64, 1), (5, 128, 512, 128, 2), (17, 64, 768, 64, 3)])
def test_c_oracle_matches_numpy_oracle(M, N, K, g, seed):
    W = WL.make_weights(N, K, seed=seed)
    X, s_x = I.make_activations(M, K, outlier_frac=0.01, seed=seed + 100)
    q = O.quantize_weights(W, g)
    ACC, Y = O.w4a8_gemm(X, s_x, q["packed"], q["s_u8"], q["a"], q["s_w"], g)
    ACC_c, Y_c = c_oracle.w4a8_gemm(X, s_x, q["packed"], q["s_u8"], q["a"], q["s_w"], g)
    assert np.array_equal(ACC, ACC_c)
    assert np.array_equal(Y.view(np.uint16), Y_c.view(np.uint16))
    assert np.array_equal(c_oracle.dequant(q["packed"], q["s_u8"], q["a"], g),
                          O.dequant_plain(q["Q_u4"], q["s_u8"], q["mn"], g))


def test_c_oracle_rejects_inadmissible_triples():
    # code 15 with s = 16 and a = 247 breaks Eq. 11 (240 + 247 > 255); Eq. 8 gives 359 > 127
    packed = np.full((1, 32), 0xFF, dtype=np.uint8)
    with pytest.raises(ArithmeticError):
        c_oracle.dequant(packed, np.array([[16]], np.uint8), np.array([[247]], np.uint8), 64)
    with pytest.raises(AssertionError):
        O.dequant_plain(np.full((1, 64), 15, np.uint8), np.array([[16]], np.uint8),
                        np.array([[119]], np.int16), 64)


# --------------------------------------------------------------------------
# Planted mistakes: each plausible slip in the oracle is caught by a pin above
# --------------------------------------------------------------------------
def test_planted_mistakes_are_caught(all_groups):
    pairs, rows, g = all_groups
    Q_u4, s_u8, mn = O.level2_quantize(rows, g)
    a = O.offset_a(mn)
    good = O.dequant_plain(Q_u4, s_u8, mn, g)
    t = Q_u4.astype(np.int32) * s_u8.astype(np.int32) + a.astype(np.int32)
    no_xor = t.astype(np.uint8).view(np.int8)                       # XOR dropped
    wrong_a = ((t - 1).astype(np.uint8) ^ np.uint8(0x80)).view(np.int8)   # a = 127 + min
    xor_7f = (t.astype(np.uint8) ^ np.uint8(0x7F)).view(np.int8)    # wrong mask
    for bad in (no_xor, wrong_a, xor_7f):
        assert not np.array_equal(bad, good)
    # floor instead of round for s would break the worked example (223/15 -> 14)
    assert 223 // 15 != 15


# ---------------------------------------------------------------------------------------
# Activation quantization (Sec. 6: dynamic per-token INT8 after the smooth divide)
# ---------------------------------------------------------------------------------------
def test_activation_quant_hand_example_with_tie():
    # amax = 1 -> s = 1/127; -0.5 -> -63.5 -> -64 (half to even), 0.25 -> 31.75 -> 32
    X = np.array([[1.0, -0.5, 0.25, 0.0], [0.0, 0.0, 0.0, 0.0], [-3.0, 3.0, 1.5, -1.5]], dtype=np.float16)
    q, s = O.quantize_activations(X)
    assert s.dtype == np.float32 and q.dtype == np.int8
    assert s[0] == np.float32(1.0) / np.float32(127) and s[1] == np.float32(1.0)
    assert q[0].tolist() == [127, -64, 32, 0]
    assert q[1].tolist() == [0, 0, 0, 0]
    # 1.5 / (3/127) = 63.5 -> 64 (half to even)
    assert q[2].tolist() == [-127, 127, 64, -64]


def test_activation_quant_properties():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((37, 512)).astype(np.float16)
    X[:, 7] *= 20
    q, s = O.quantize_activations(X)
    Xf = X.astype(np.float64)
    amax = np.abs(Xf).max(axis=1)
    # the extreme element of every token maps to +-127 and nothing exceeds it
    assert (np.abs(q).max(axis=1) == 127).all()
    pos = np.argmax(np.abs(Xf), axis=1)
    assert (np.abs(q[np.arange(37), pos]) == 127).all()
    assert np.array_equal(np.sign(q[np.abs(q) > 0]), np.sign(Xf[np.abs(q) > 0]))
    # scale = amax / 127 to FP32 accuracy; reconstruction within half a step (plus FP32 slack)
    assert np.allclose(s, amax / 127, rtol=2e-7, atol=0)
    assert (np.abs(q.astype(np.float64) * s[:, None].astype(np.float64) - Xf) <= 0.5 * s[:, None] * (1 + 1e-5)).all()
    # exact invariance under a power-of-two rescale of a token
    q2, s2 = O.quantize_activations(X * np.float16(4.0))
    assert np.array_equal(q2, q) and np.array_equal(s2, s * np.float32(4.0))
    # sign symmetry
    q3, s3 = O.quantize_activations(-X)
    assert np.array_equal(q3, -q) and np.array_equal(s3, s)


def test_activation_quant_smooth_divide_against_rationals():
    from fractions import Fraction

    rng = np.random.default_rng(6)
    M, K = 5, 24
    X = rng.standard_normal((M, K)).astype(np.float16)
    smooth = np.exp(rng.standard_normal(K) * 0.5).astype(np.float32)
    q, s = O.quantize_activations(X, smooth)

    for m in range(M):
        xs = []
        for k in range(K):
            # exact quotient, rounded once to FP32: float(Fraction) is correctly rounded to
            # FP64, and rounding a quotient of two 24-bit numbers to 53 bits and then to 24
            # bits gives the same result as rounding it once (53 >= 2 * 24 + 2)
            xs.append(np.float32(float(Fraction(float(X[m, k])) / Fraction(float(smooth[k])))))
        amax = max(abs(v) for v in xs)
        sm = np.float32(float(Fraction(float(amax)) / 127))
        assert s[m] == sm
        for k in range(K):
            exact = Fraction(float(xs[k])) / Fraction(float(sm))
            quo = np.float32(float(exact))          # the FP32 quotient the definition rounds
            want = int(np.clip(np.rint(quo), -127, 127))
            assert q[m, k] == want, (m, k)
    # planted mistake: multiplying by the smooth scale instead of dividing gives other codes
    q_mul, _ = O.quantize_activations(X, np.float32(1.0) / smooth)
    assert not np.array_equal(q_mul, q)


# ---------------------------------------------------------------------------------------
# Grouped (mixture-of-experts) GEMM: independent GEMMs over disjoint runs of tokens
# ---------------------------------------------------------------------------------------
def _tiny_experts(E, N, K, g, seed):
    rng = np.random.default_rng(seed)
    return [O.quantize_weights(rng.standard_normal((N, K)).astype(np.float16).astype(np.float32) * 0.05, g)
            for _ in range(E)]


def test_grouped_gemm_brute_force_and_independence():
    E, N, K, g = 3, 4, 64, 64
    experts = _tiny_experts(E, N, K, g, seed=11)
    offs = [0, 2, 2, 5]                     # expert 1 has no tokens
    rng = np.random.default_rng(12)
    X = rng.integers(-127, 128, size=(5, K)).astype(np.int8)
    s_x = np.ones(5, dtype=np.float32)
    ACC, Y = O.grouped_w4a8_gemm(X, s_x, offs, experts)
    owner = [0, 0, 2, 2, 2]
    for m in range(5):
        q = experts[owner[m]]
        for n in range(N):
            tot = 0
            for k in range(K):
                w = int(q["Q_u4"][n, k]) * int(q["s_u8"][n, k // g]) + int(q["mn"][n, k // g])
                tot += int(X[m, k]) * w
            assert ACC[m, n] == tot
            assert Y[m, n] == np.float16(float(tot) * float(q["s_w"][n]))
    # rows of one expert do not move when another expert's weights change
    other = list(experts)
    other[0] = _tiny_experts(1, N, K, g, seed=99)[0]
    ACC2, _ = O.grouped_w4a8_gemm(X, s_x, offs, other)
    assert np.array_equal(ACC2[2:], ACC[2:]) and not np.array_equal(ACC2[:2], ACC[:2])
    # one expert owning every token is the plain GEMM
    q = experts[2]
    A1, Y1 = O.grouped_w4a8_gemm(X, s_x, [0, 5], [q])
    A0, Y0 = O.w4a8_gemm(X, s_x, q["packed"], q["s_u8"], q["a"], q["s_w"], g)
    assert np.array_equal(A1, A0) and np.array_equal(Y1.view(np.uint16), Y0.view(np.uint16))
