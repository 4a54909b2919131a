"""The register-level form of Eq. 12 that the kernels use, replayed in numpy: four codes per
32-bit register, one multiply-add per 16-bit lane (s in both lanes, a in all four bytes), one
XOR with 0x80808080.  For every admissible (code, s, a) -- drawn through the oracle's
quantiser, as the interface requires -- no byte may carry into its neighbour and the result
must equal the per-element Eq. 8 of the oracle."""
import numpy as np

from oracle import lqq_oracle as O


def _packed_dequant(reg_codes, s, a):
    """reg_codes: uint32 registers holding 4 codes (one per byte); s, a: per-register scalars."""
    r = reg_codes.astype(np.uint32)
    lanes = np.stack([r & 0xFFFF, r >> 16], axis=-1).astype(np.uint32)            # two 16-bit lanes
    mad = (lanes * s[..., None].astype(np.uint32) + a[..., None].astype(np.uint32) * 0x0101) & 0xFFFF
    out = (mad[..., 0] | (mad[..., 1] << 16)) ^ np.uint32(0x80808080)
    return out.astype(np.uint32)


def test_packed_multiply_add_has_no_byte_carries_and_matches_eq8():
    rng = np.random.default_rng(7)
    g = 64
    # groups spanning every range width, including the extremes of the protective range
    Q = rng.integers(-119, 120, size=(4096, g)).astype(np.int8)
    width = rng.integers(0, 239, size=4096)
    lo = rng.integers(-119, 120 - np.minimum(width, 238))
    Q = (lo[:, None] + (rng.random((4096, g)) * (width[:, None] + 1)).astype(np.int64)).clip(-119, 119).astype(np.int8)
    Q[0, :] = 119
    Q[1, ::2], Q[1, 1::2] = -119, 119
    Q_u4, s_u8, mn = O.level2_quantize(Q, g)
    a = O.offset_a(mn)
    ref = O.dequant_plain(Q_u4, s_u8, mn, g)                                       # Eq. 8, element by element
    codes = Q_u4.reshape(4096, g // 4, 4).astype(np.uint32)
    regs = codes[..., 0] | (codes[..., 1] << 8) | (codes[..., 2] << 16) | (codes[..., 3] << 24)
    s = np.repeat(s_u8.astype(np.uint32), g // 4, axis=1)
    av = np.repeat(a.astype(np.uint32), g // 4, axis=1)
    # the premise of the trick: every byte of code*s + a stays below 256 (Eq. 11)
    assert int((codes * s[..., None] + av[..., None]).max()) <= 255
    out = _packed_dequant(regs, s, av)
    got = np.stack([(out >> (8 * b)) & 0xFF for b in range(4)], axis=-1).astype(np.uint8).view(np.int8)
    assert np.array_equal(got.reshape(4096, g), ref)


def test_a_violated_premise_does_carry():
    """With an inadmissible triple (code * s + a > 255) the packed form corrupts the neighbouring
    byte -- the reason the interface demands quantiser-made blobs."""
    regs = np.array([0x0000000F], dtype=np.uint32)                                 # code 15 in byte 0
    out = _packed_dequant(regs, np.array([16]), np.array([100]))                    # 15*16 + 100 = 340
    byte1 = (int(out[0]) >> 8) & 0xFF
    assert byte1 != ((0 * 16 + 100) ^ 0x80)
