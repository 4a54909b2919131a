// Packed weight layout for gfx950 (host-side index functions).
//
// The layout plays the role of the paper's dual-MMA packed layout (Sec. 5.2): what one
// lane needs for two consecutive matrix instructions is one contiguous 16-byte load, the
// global-memory order equals the register order, and the permutation is done offline.
// It is re-derived for v_mfma_i32_16x16x64_i8, whose weight operand holds, in lane l,
// 16 consecutive-in-register k values of matrix column (l % 16) for k-block (l / 16).
//
// Codes.  The matrix is cut into chunks of 16 output channels x 128 k = 1 KiB:
//   tile  t = 4*(n/64) + (n%4)      slot j = (n%64)/4       (so tile t, slot j holds
//                                   channel n = 64*(t/4) + 4*j + (t%4): the four tiles of
//                                   a 64-channel group interleave, which lets a lane
//                                   that owns slot j of all four write 4 adjacent outputs)
//   chunk c = k/128,  half h = (k%128)/64,  k-block kb = (k%64)/16,
//   dword d = (k%16)/4,  byte b = k%4
//   byte offset = (t*(K/128) + c)*1024 + (16*kb + j)*16 + 4*d + b
//   nibble      = low for h = 0, high for h = 1
// A wave reads a chunk with one 16-byte load per lane (lane = 16*kb + j); the low
// nibbles of its four dwords are the operand registers of k-step 2c, the high nibbles
// those of k-step 2c+1.
//
// Group parameters (s_u8, a), two bytes per (channel, group), in units of 256 k:
//   offset = ((t*(K/256) + k/256)*16 + j) * (2*256/group) + 2*((k%256)/group)
// so the lanes of a wave fetch the parameters of their channel for four k-steps with one
// 8-byte (group 64) or 4-byte (group 128) load from a contiguous 128/64-byte segment.
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
    const int t = 4 * (n / 64) + (n % 4);
    const int j = (n % 64) / 4;
    const int c = k / 128, h = (k % 128) / 64, kb = (k % 64) / 16, d = (k % 16) / 4, b = k % 4;
    CodeLoc r;
    r.byte = ((size_t)t * (K / 128) + c) * 1024 + (size_t)(16 * kb + j) * 16 + 4 * d + b;
    r.shift = 4 * h;
    return r;
}

// Offset of the s_u8 byte of (channel n, group gi); the a byte follows it.
inline size_t gparam_loc(int n, int gi, int K, int group)
{
    const int t = 4 * (n / 64) + (n % 4);
    const int j = (n % 64) / 4;
    const int per_unit = 256 / group;  // groups per 256 k
    const int unit = gi / per_unit, within = gi % per_unit;
    return (((size_t)t * (K / 256) + unit) * 16 + j) * (size_t)(2 * per_unit) + 2 * within;
}

}  // namespace lqq
