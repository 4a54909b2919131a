// Device-side building blocks shared by the gfx950 kernels: vector types, the LiquidQuant
// register-level dequantisation (paper Sec. 5.3, Eq. 12) and the INT8 MFMA wrapper.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lqq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// (r * s + a) on two 16-bit lanes: one v_pk_mad_u16.  With every byte of r <= 15,
// s <= 16 and byte*s + a <= 255 (Eq. 11) no byte carries into its neighbour, so this is
// four independent UINT8 multiply-adds -- the gfx950 stand-in for the 32-bit IMAD of
// Sec. 5.3 (a 32-bit integer multiply is quarter rate on CDNA; the packed 16-bit one is
// full rate).
__device__ __forceinline__ uint32_t pk_mad_u16(uint32_t r, uint32_t s2, uint32_t a4)
{
    const u16x2 rv = __builtin_bit_cast(u16x2, r);
    const u16x2 sv = __builtin_bit_cast(u16x2, s2);
    const u16x2 av = __builtin_bit_cast(u16x2, a4);
    return __builtin_bit_cast(uint32_t, (u16x2)(rv * sv + av));
}

// Broadcast forms of one (s_u8, a) byte pair held in `word`: which = 0 takes bytes 0/1,
// which = 1 takes bytes 2/3.  s2 = s in both 16-bit lanes, a4 = a in all four bytes.
__device__ __forceinline__ void expand_params(uint32_t word, int which, uint32_t &s2, uint32_t &a4)
{
    s2 = __builtin_amdgcn_perm(word, word, which ? 0x0c020c02u : 0x0c000c00u);
    a4 = __builtin_amdgcn_perm(word, word, which ? 0x03030303u : 0x01010101u);
}

// Unpack + dequantise one 16-byte lane load (32 codes of one channel, one group): the low
// nibbles become the four operand registers of the first k-step, the high nibbles those
// of the second.  7 VALU instructions per 8 codes: and, shift, and, 2 x pk_mad, 2 x xor
// (Sec. 5.3).
__device__ __forceinline__ void dequant_chunk(const u32x4 p, uint32_t s2, uint32_t a4, v4i &lo, v4i &hi)
{
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t l = p[d] & 0x0F0F0F0Fu;
        const uint32_t h = (p[d] >> 4) & 0x0F0F0F0Fu;
        lo[d] = (int)(pk_mad_u16(l, s2, a4) ^ 0x80808080u);
        hi[d] = (int)(pk_mad_u16(h, s2, a4) ^ 0x80808080u);
    }
}

// Half of dequant_chunk: the low (h = 0) or high (h = 1) nibbles only, i.e. the operand
// registers of one k-step of 32.
__device__ __forceinline__ void dequant_half(const u32x4 p, uint32_t s2, uint32_t a4, int h, v4i &out)
{
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t v = (h ? (p[d] >> 4) : p[d]) & 0x0F0F0F0Fu;
        out[d] = (int)(pk_mad_u16(v, s2, a4) ^ 0x80808080u);
    }
}

// Group parameters of one lane's channel for one unit of 128 k (two chunks).
// group 64: two (s, a) pairs in 4 bytes; group 128: one pair in 2 bytes.
template <bool G128>
struct UnitParams;
template <>
struct UnitParams<false> {
    uint32_t raw;
    __device__ __forceinline__ void load(const uint8_t *gp, size_t tile_unit, int slot)
    {
        raw = *reinterpret_cast<const uint32_t *>(gp + (tile_unit * 32 + slot) * 4);
    }
    // broadcast parameters of chunk c (0 or 1) of the unit
    __device__ __forceinline__ void get(int c, uint32_t &s2, uint32_t &a4) const { expand_params(raw, c, s2, a4); }
};
template <>
struct UnitParams<true> {
    uint32_t raw;
    __device__ __forceinline__ void load(const uint8_t *gp, size_t tile_unit, int slot)
    {
        raw = *reinterpret_cast<const uint16_t *>(gp + (tile_unit * 32 + slot) * 2);
    }
    __device__ __forceinline__ void get(int, uint32_t &s2, uint32_t &a4) const { expand_params(raw, 0, s2, a4); }
};

// D(32x32) += A(32x32) * B(32x32), INT8 inputs, INT32 accumulate.  Lane l supplies row
// l%32 of A and column l%32 of B for k-block l/32 (16 bytes each); it receives
// D[8*(r/4) + 4*(l/32) + r%4][l%32] in element r (r = 0..15).
__device__ __forceinline__ v16i mfma_i8(const v4i a, const v4i b, const v16i c)
{
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}

// D(16x16) += A(16x64) * B(64x16), INT8 inputs, INT32 accumulate (decode-sized batches).
// Lane l supplies row l%16 of A and column l%16 of B for k-block l/16 (16 bytes each); it
// receives D[4*(l/16) + r][l%16] in element r (r = 0..3).
__device__ __forceinline__ v4i mfma16_i8(const v4i a, const v4i b, const v4i c)
{
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}

// Regroup one dequantised chunk (lo/hi = the two k-steps of a 32-channel x 64-k chunk in
// the 32x32x32 operand order) into the B operands of two 16x16x64 MFMAs: b1 covers slots
// 0..15, b2 slots 16..31 of the tile, each over the chunk's 64 k.  One
// v_permlane16_swap per register: it exchanges the odd 16-lane rows of `lo` with the even
// rows of `hi`.  The k-blocks end up in the order {0..15, 32..47, 16..31, 48..63}; the X
// operand is read in the same order (kStep16Offset).
__device__ __forceinline__ void regroup_16x16(const v4i lo, const v4i hi, v4i &b1, v4i &b2)
{
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const auto r = __builtin_amdgcn_permlane16_swap((unsigned)lo[d], (unsigned)hi[d], false, false);
        b1[d] = (int)r[0];
        b2[d] = (int)r[1];
    }
}
// byte offset inside a chunk's 64 k of the k-block that lane group q = l/16 must supply
__device__ __forceinline__ int kstep16_offset(int q) { return ((q & 1) << 5) | ((q & 2) << 3); }

// Row of the 32x32 MFMA result held in accumulator element r of lane l.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// Channel held by slot j of tile t (see lqq_layout.h).
__device__ __forceinline__ int channel_of(int t, int j) { return 64 * (t >> 1) + 2 * j + (t & 1); }

}  // namespace lqq
