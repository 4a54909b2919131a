// Packed weight layout for gfx950 (host-side index functions).
//
// The layout plays the role of the paper's dual-MMA packed layout (Sec. 5.2): what one
// lane needs for two consecutive matrix instructions is one contiguous 16-byte load, the
// global-memory order equals the register order, and the permutation is done offline.
// It is re-derived for v_mfma_i32_32x32x32_i8, whose weight operand holds, in lane l,
// 16 k values (4 registers x 4 bytes) of matrix column (l % 32) for k-block (l / 32).
//
// Codes.  The matrix is cut into chunks of 32 output channels x 64 k = 1 KiB:
//   tile  t = 2*(n/64) + (n%2)      slot j = (n%64)/2       (tile t, slot j holds channel
//                                   n = 64*(t/2) + 2*j + (t%2): the two tiles of a
//                                   64-channel group interleave, so a lane that owns slot
//                                   j of both writes 2 adjacent outputs and a half-wave
//                                   writes a full 128-byte line of FP16)
//   chunk c = k/64,  half h = (k%64)/32,  k-block kb = (k%32)/16,
//   dword d = (k%16)/4,  byte b = k%4
//   byte offset = (t*(K/64) + c)*1024 + (32*kb + j)*16 + 4*d + b
//   nibble      = low for h = 0, high for h = 1
// A wave reads a chunk with one 16-byte load per lane (lane = 32*kb + j); the low
// nibbles of its four dwords are the operand registers of k-step 2c (32 k), the high
// nibbles those of k-step 2c+1.  With group 64 a chunk is exactly one group, so one
// (s_u8, a) pair serves the whole 16-byte load.
//
// Group parameters (s_u8, a), two bytes per (channel, group), in units of 128 k:
//   offset = ((t*(K/128) + k/128)*32 + j) * (2*128/group) + 2*((k%128)/group)
// so the lanes of a wave fetch the parameters of their channel for two chunks with one
// 4-byte (group 64) or 2-byte (group 128) load from a contiguous 128/64-byte segment.
#pragma once
#include <cstddef>
#include <cstdint>

namespace lqq {

struct CodeLoc {
    size_t byte;
    int shift;  // 0 or 4
};

inline CodeLoc code_loc(int n, int k, int K)
{
    const int t = 2 * (n / 64) + (n % 2);
    const int j = (n % 64) / 2;
    const int c = k / 64, h = (k % 64) / 32, kb = (k % 32) / 16, d = (k % 16) / 4, b = k % 4;
    CodeLoc r;
    r.byte = ((size_t)t * (K / 64) + c) * 1024 + (size_t)(32 * kb + j) * 16 + 4 * d + b;
    r.shift = 4 * h;
    return r;
}

// Offset of the s_u8 byte of (channel n, group gi); the a byte follows it.
inline size_t gparam_loc(int n, int gi, int K, int group)
{
    const int t = 2 * (n / 64) + (n % 2);
    const int j = (n % 64) / 2;
    const int per_unit = 128 / group;  // groups per 128 k: 2 or 1
    const int unit = gi / per_unit, within = gi % per_unit;
    return (((size_t)t * (K / 128) + unit) * 32 + j) * (size_t)(2 * per_unit) + 2 * within;
}

}  // namespace lqq
