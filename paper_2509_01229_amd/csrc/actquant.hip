// Dynamic per-token activation quantisation, the step directly upstream of the W4A8 GEMM
// (paper Sec. 6, "Serving System": FP16 activations are divided by the smooth scale and
// mapped to INT8 per token on the fly):
//
//     x'[m,k] = (float)X[m,k] / smooth[k]                (smooth optional)
//     s_x[m]  = max_k |x'[m,k]| / 127                    (1 for an all-zero token)
//     Q[m,k]  = clamp(rint(x'[m,k] / s_x[m]), -127, 127)
//
// Every operation is one correctly rounded FP32 operation, so the INT8 result is determined
// bit for bit; the kernel reproduces it exactly (see round8 for how the second division is
// avoided where it cannot matter).
//
// One block of 256 threads per token (or per R consecutive tokens, one after the other, so
// that the reciprocals of the smooth scales are computed once for R tokens).  A token of up
// to 32768 elements is read from HBM once and kept in registers between the max pass and the
// rounding pass (from 16392 elements on, on blocks of 512 or 1024 threads); longer tokens are
// read twice (the second read hits L2).  Traffic: 2 bytes in, 1 byte out per element.
#include <algorithm>

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "lqq_common.h"
#include "lqq_device.h"

namespace lqq {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr int kQuantThreads = 256;

// 8 FP16 values (one 16-byte load) -> FP32, optionally divided by their smooth scales
struct Raw8 {
    u32x4 x;
    float4 s0, s1;
};
template <bool SMOOTH>
__device__ __forceinline__ Raw8 load8(const u32x4 *xrow, const float *smooth, int i)
{
    Raw8 r;
    r.x = xrow[i];
    if (SMOOTH) {
        r.s0 = *reinterpret_cast<const float4 *>(smooth + 8 * (size_t)i);
        r.s1 = *reinterpret_cast<const float4 *>(smooth + 8 * (size_t)i + 4);
    }
    return r;
}
template <bool SMOOTH>
__device__ __forceinline__ void convert8(const Raw8 &r, float (&f)[8])
{
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t w = r.x[d];
        const f16x2 h = __builtin_bit_cast(f16x2, w);
        f[2 * d] = (float)h[0];
        f[2 * d + 1] = (float)h[1];
    }
    if (SMOOTH) {
        f[0] /= r.s0.x, f[1] /= r.s0.y, f[2] /= r.s0.z, f[3] /= r.s0.w;
        f[4] /= r.s1.x, f[5] /= r.s1.y, f[6] /= r.s1.z, f[7] /= r.s1.w;
    }
}

// x / s, correctly rounded, from a reciprocal refined once per smooth scale.  This is the
// instruction sequence of the IEEE division without its scaling and special-case steps
// (y1 = rcp refined by one Newton step; quotient x * y1 corrected twice with exact
// residuals), which change nothing while s is within [2^-40, 2^40] and x is zero or an FP16
// magnitude (2^-24 .. 65504): no intermediate leaves the normal range.  Callers check s.
struct Recip {
    float s, y1;
};
__device__ __forceinline__ Recip refine_recip(float s)
{
    const float y0 = __builtin_amdgcn_rcpf(s);
    const float e = __builtin_fmaf(-s, y0, 1.0f);
    return Recip{s, __builtin_fmaf(e, y0, y0)};
}
__device__ __forceinline__ float div_by(float x, const Recip r)
{
    const float q0 = x * r.y1;
    const float r0 = __builtin_fmaf(-r.s, q0, x);
    const float q1 = __builtin_fmaf(r0, r.y1, q0);
    const float r1 = __builtin_fmaf(-r.s, q1, x);
    return __builtin_fmaf(r1, r.y1, q1);
}
__device__ __forceinline__ bool recip_is_safe(float s) { return s >= 0x1p-40f && s <= 0x1p40f; }

// 8 FP16 values -> FP32 (no smooth divide)
__device__ __forceinline__ void widen8(const u32x4 x, float (&f)[8])
{
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t w = x[d];
        const f16x2 h = __builtin_bit_cast(f16x2, w);
        f[2 * d] = (float)h[0];
        f[2 * d + 1] = (float)h[1];
    }
}

__device__ __forceinline__ float max_abs8(const float (&f)[8], float m)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf(f[e]));
    return m;
}

// Q = clamp(rint(f / s)) for 8 values.  The FP32 quotient is only needed to decide an
// integer, so the common case multiplies by an approximate reciprocal: that product and
// the correctly rounded quotient both lie within 127 * (2^-23 + 2^-24 + 2^-24) < 3.1e-5 of
// the exact quotient (|f / s| <= 127), hence they round to the same integer unless the
// product is within 1e-4 of a tie.  Only then (about 1 lane-visit in 600) the 8 values
// are redone with the full IEEE division, so the result is always that of the division.
__device__ __forceinline__ uint2 round8(const float (&f)[8], float s, float rcp_s)
{
    float q[8];
    bool near_tie = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float t = f[e] * rcp_s;
        q[e] = __builtin_rintf(t);
        near_tie |= fabsf(t - q[e]) > 0.5f - 1e-4f;
    }
    if (near_tie) {
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = __builtin_rintf(f[e] / s);
    }
    uint32_t w[2] = {0, 0};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float c = fminf(fmaxf(q[e], -127.0f), 127.0f);
        w[e >> 2] |= ((uint32_t)(int)c & 0xffu) << (8 * (e & 3));
    }
    return uint2{w[0], w[1]};
}

// maximum over the block of NWAVES waves; every thread gets the result
template <int NWAVES = 4>
__device__ __forceinline__ float block_max(float m, float *s_part)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = m;
    __syncthreads();
    float r = s_part[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) r = fmaxf(r, s_part[w]);
    return r;
}

// Tokens of any length, one per block, read twice.  Loads of a pass are issued four pieces at
// a time, with indices past the end clamped to the last piece and their values ignored, so
// that no load waits behind a branch.
template <bool SMOOTH>
__global__ __launch_bounds__(kQuantThreads) void quantize_act_long_kernel(
    int K, const __half *__restrict__ X, const float *__restrict__ smooth, int8_t *__restrict__ Q,
    float *__restrict__ sx)
{
    __shared__ float s_part[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    const u32x4 *xrow = reinterpret_cast<const u32x4 *>(X + (size_t)m * K);
    uint2 *qrow = reinterpret_cast<uint2 *>(Q + (size_t)m * K);
    const int n8 = K >> 3;
    constexpr int U = 4;  // pieces in flight per thread

    float amax = 0.0f;
    float f[U][8];
    for (int i0 = tid; i0 < n8; i0 += U * kQuantThreads) {
        Raw8 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) raw[u] = load8<SMOOTH>(xrow, smooth, min(i0 + u * kQuantThreads, n8 - 1));
#pragma unroll
        for (int u = 0; u < U; ++u) {
            convert8<SMOOTH>(raw[u], f[u]);
            if (i0 + u * kQuantThreads < n8) amax = max_abs8(f[u], amax);
        }
    }
    amax = block_max(amax, s_part);
    const float s = amax > 0.0f ? amax / 127.0f : 1.0f;
    if (tid == 0) sx[m] = s;
    const float rcp_s = __builtin_amdgcn_rcpf(s);
    for (int i0 = tid; i0 < n8; i0 += U * kQuantThreads) {
        Raw8 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) raw[u] = load8<SMOOTH>(xrow, smooth, min(i0 + u * kQuantThreads, n8 - 1));
#pragma unroll
        for (int u = 0; u < U; ++u) {
            convert8<SMOOTH>(raw[u], f[u]);
            const int i = i0 + u * kQuantThreads;
            if (i < n8) qrow[i] = round8(f[u], s, rcp_s);
        }
    }
}

// Register-resident tokens (K <= ITERS x NT x 8), R consecutive tokens per block.  Thread t owns
// the 16-byte pieces t, t + NT, ... of every token of its block, i.e. fixed columns: their
// smooth scales and refined reciprocals are loaded and computed once.
// KEEP = false (tokens of 16392..32768 elements, on 512 or 1024 threads): what would not fit in
// registers is not kept -- with smooth scales the reciprocals (the scales are re-read for
// every token and divided by with the IEEE division), without them the widened values.
template <bool SMOOTH, int ITERS, int NT, bool KEEP = true>
__global__ __launch_bounds__(NT) void quantize_act_rows_kernel(
    int M, int K, int R, const __half *__restrict__ X, const float *__restrict__ smooth,
    int8_t *__restrict__ Q, float *__restrict__ sx)
{
    __shared__ float s_part[2][NT / 64];
    const int tid = threadIdx.x;
    const int n8 = K >> 3;
    int piece[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) piece[it] = min(it * NT + tid, n8 - 1);

    // the first token's loads go out before anything waits for the smooth scales
    const int m_begin = blockIdx.x * R, m_end = min(M, m_begin + R);
    u32x4 raw[ITERS];
    if (m_begin < m_end) {
        const u32x4 *xrow = reinterpret_cast<const u32x4 *>(X + (size_t)m_begin * K);
#pragma unroll
        for (int it = 0; it < ITERS; ++it) raw[it] = xrow[piece[it]];
    }

    Recip rc[SMOOTH && KEEP ? ITERS : 1][8];
    bool safe = true;  // every smooth scale of this thread allows the short division
    if (SMOOTH && KEEP) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const float4 a = *reinterpret_cast<const float4 *>(smooth + 8 * (size_t)piece[it]);
            const float4 b = *reinterpret_cast<const float4 *>(smooth + 8 * (size_t)piece[it] + 4);
            const float sm[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                rc[it][e] = refine_recip(sm[e]);
                safe &= recip_is_safe(sm[e]);
            }
        }
    }

    for (int m = m_begin; m < m_end; ++m) {
        uint2 *qrow = reinterpret_cast<uint2 *>(Q + (size_t)m * K);
        if (!SMOOTH && !KEEP) {
            // Long tokens without smooth scales: only the FP16 token itself stays in registers
            // between the two passes (4 registers per piece instead of 12) and widening is
            // repeated, so that several blocks still share a CU (34 instead of 41 us for
            // 2048 x 28672; shorter tokens are 5 % faster with the widened values kept).
            if (m > m_begin) {
                const u32x4 *xrow = reinterpret_cast<const u32x4 *>(X + (size_t)m * K);
#pragma unroll
                for (int it = 0; it < ITERS; ++it) raw[it] = xrow[piece[it]];
            }
            float amax = 0.0f;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                float f[8];
                widen8(raw[it], f);
                if (it * NT + tid < n8) amax = max_abs8(f, amax);
            }
            amax = block_max<NT / 64>(amax, s_part[(m - m_begin) & 1]);
            const float s = amax > 0.0f ? amax / 127.0f : 1.0f;
            if (tid == 0) sx[m] = s;
            const float rcp_s = __builtin_amdgcn_rcpf(s);
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                // (opaque to the compiler, so that it widens again instead of keeping the first pass's values)
                asm volatile("" : "+v"(raw[it]));
                float f[8];
                widen8(raw[it], f);
                const int i = it * NT + tid;
                if (i < n8) qrow[i] = round8(f, s, rcp_s);
            }
            continue;
        }
        float f[ITERS][8];
        float amax = 0.0f;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            widen8(raw[it], f[it]);
            if (!SMOOTH) {
            } else if (KEEP) {
                if (safe) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[it][e] = div_by(f[it][e], rc[KEEP ? it : 0][e]);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[it][e] = f[it][e] / rc[KEEP ? it : 0][e].s;
                }
            } else {
                const float4 a = *reinterpret_cast<const float4 *>(smooth + 8 * (size_t)piece[it]);
                const float4 b = *reinterpret_cast<const float4 *>(smooth + 8 * (size_t)piece[it] + 4);
                const float sm[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) f[it][e] = f[it][e] / sm[e];
            }
            if (it * NT + tid < n8) amax = max_abs8(f[it], amax);
        }
        if (m + 1 < m_end) {  // the next token's loads fly while this one is reduced, rounded and stored
            const u32x4 *xrow = reinterpret_cast<const u32x4 *>(X + (size_t)(m + 1) * K);
#pragma unroll
            for (int it = 0; it < ITERS; ++it) raw[it] = xrow[piece[it]];
        }
        amax = block_max<NT / 64>(amax, s_part[(m - m_begin) & 1]);
        const float s = amax > 0.0f ? amax / 127.0f : 1.0f;
        if (tid == 0) sx[m] = s;
        const float rcp_s = __builtin_amdgcn_rcpf(s);
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = it * NT + tid;
            if (i < n8) qrow[i] = round8(f[it], s, rcp_s);
        }
    }
}

template <bool SMOOTH>
static void launch_quantize(int M, int K, const __half *X, const float *smooth, int8_t *Q, float *sx,
                            hipStream_t st)
{
    const dim3 block(kQuantThreads);
    const int pieces = (K / 8 + kQuantThreads - 1) / kQuantThreads;  // 16-byte pieces per thread
    // tokens per block: as many as leave four blocks per CU (with smooth scales only: without
    // them there is nothing to share between tokens; three blocks of this kernel fit a CU, and
    // 1024 blocks measured 3 to 12 % faster than 512 on 4096 tokens of 8192 and 4096 elements)
    const int R = !SMOOTH ? 1 : std::max(1, (M + 1023) / 1024);
    const dim3 grid((unsigned)((M + R - 1) / R));
#define LQ_LAUNCH_Q(ITERS) \
    hipLaunchKernelGGL((quantize_act_rows_kernel<SMOOTH, ITERS, kQuantThreads>), grid, block, 0, st, M, K, R, X, \
                       smooth, Q, sx)
    if (pieces <= 1)
        LQ_LAUNCH_Q(1);
    else if (pieces <= 2)
        LQ_LAUNCH_Q(2);
    else if (pieces <= 4)
        LQ_LAUNCH_Q(4);
    else if (pieces <= 8) {
        // 8193..16384 columns.  With smooth scales the reciprocals triple the registers per
        // piece: blocks of 512 threads keep twice the waves on a CU (64 instead of 72 us for
        // 4096 x 16384, 32 instead of 38 for 2048 x 14336).
        if constexpr (SMOOTH) {
            if (pieces <= 6)
                hipLaunchKernelGGL((quantize_act_rows_kernel<SMOOTH, 3, 512>), grid, dim3(512), 0, st, M, K, R, X,
                                   smooth, Q, sx);
            else
                hipLaunchKernelGGL((quantize_act_rows_kernel<SMOOTH, 4, 512>), grid, dim3(512), 0, st, M, K, R, X,
                                   smooth, Q, sx);
        } else {
            if (pieces <= 6)
                LQ_LAUNCH_Q(6);
            else
                LQ_LAUNCH_Q(8);
        }
    } else if (pieces <= 16) {  // up to 32768 columns: still register-resident, on larger blocks
        if constexpr (SMOOTH)
            hipLaunchKernelGGL((quantize_act_rows_kernel<SMOOTH, 4, 1024, false>), dim3((unsigned)M), dim3(1024), 0, st,
                               M, K, 1, X, smooth, Q, sx);
        else
            hipLaunchKernelGGL((quantize_act_rows_kernel<false, 8, 512, false>), dim3((unsigned)M), dim3(512), 0, st, M,
                               K, 1, X, smooth, Q, sx);
    } else
        hipLaunchKernelGGL((quantize_act_long_kernel<SMOOTH>), dim3((unsigned)M), block, 0, st, K, X, smooth, Q, sx);
#undef LQ_LAUNCH_Q
}

}  // namespace lqq

using namespace lqq;

extern "C" int w4a8_quantize_activations(int M, int K, const uint16_t *X_f16, const float *smooth,
                                         int8_t *X_i8, float *act_scales, void *hip_stream)
{
    if (M < 0 || K <= 0 || K % 8 != 0 || K > (1 << 24))
        return fail(LQ_ERR_INVALID, "bad shape M=%d K=%d (need M>=0, K>0, K%%8==0)", M, K);
    if (M == 0) return LQ_OK;
    if (!X_f16 || !X_i8 || !act_scales) return fail(LQ_ERR_INVALID, "null pointer");
    const uintptr_t bits = (uintptr_t)X_f16 | (uintptr_t)smooth | (uintptr_t)X_i8 | (uintptr_t)act_scales;
    if (bits & 15) return fail(LQ_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const __half *X = reinterpret_cast<const __half *>(X_f16);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    if (smooth)
        launch_quantize<true>(M, K, X, smooth, X_i8, act_scales, st);
    else
        launch_quantize<false>(M, K, X, smooth, X_i8, act_scales, st);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LQ_ERR_HIP, "activation quantisation launch failed: %s", hipGetErrorString(e));
    return LQ_OK;
}
