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
// One block of 256 threads per token.  A token of up to 16384 elements is read from HBM
// once and kept in registers between the max pass and the rounding pass; longer tokens
// are read twice (the second read hits L2).  Traffic: 2 bytes in, 1 byte out per element.
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

// maximum over the block; every thread gets the result
__device__ __forceinline__ float block_max(float m, float *s_part)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = m;
    __syncthreads();
    return fmaxf(fmaxf(s_part[0], s_part[1]), fmaxf(s_part[2], s_part[3]));
}

// ITERS > 0: the token fits in ITERS x 256 x 8 elements and stays in registers between the
// two passes; ITERS = 0: any length, read twice.  Loads of a pass are issued together, with
// indices past the end clamped to the last piece and their values ignored, so that no load
// waits behind a branch.
template <bool SMOOTH, int ITERS>
__global__ __launch_bounds__(kQuantThreads) void quantize_act_kernel(
    int K, const __half *__restrict__ X, const float *__restrict__ smooth, int8_t *__restrict__ Q,
    float *__restrict__ sx)
{
    __shared__ float s_part[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    const u32x4 *xrow = reinterpret_cast<const u32x4 *>(X + (size_t)m * K);
    uint2 *qrow = reinterpret_cast<uint2 *>(Q + (size_t)m * K);
    const int n8 = K >> 3;
    constexpr int U = 4;  // pieces in flight per thread in the two-pass form

    float amax = 0.0f;
    float f[ITERS > 0 ? ITERS : U][8];
    if (ITERS > 0) {
        Raw8 raw[ITERS > 0 ? ITERS : 1];
#pragma unroll
        for (int it = 0; it < ITERS; ++it) raw[it] = load8<SMOOTH>(xrow, smooth, min(it * kQuantThreads + tid, n8 - 1));
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            convert8<SMOOTH>(raw[it], f[it]);
            if (it * kQuantThreads + tid < n8) amax = max_abs8(f[it], amax);
        }
    } else {
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
    }
    amax = block_max(amax, s_part);
    const float s = amax > 0.0f ? amax / 127.0f : 1.0f;
    if (tid == 0) sx[m] = s;
    const float rcp_s = __builtin_amdgcn_rcpf(s);
    if (ITERS > 0) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = it * kQuantThreads + tid;
            if (i < n8) qrow[i] = round8(f[it], s, rcp_s);
        }
    } else {
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
}

template <bool SMOOTH>
static void launch_quantize(int M, int K, const __half *X, const float *smooth, int8_t *Q, float *sx,
                            hipStream_t st)
{
    const dim3 grid((unsigned)M), block(kQuantThreads);
    const int pieces = (K / 8 + kQuantThreads - 1) / kQuantThreads;  // 16-byte pieces per thread
#define LQ_LAUNCH_Q(ITERS) \
    hipLaunchKernelGGL((quantize_act_kernel<SMOOTH, ITERS>), grid, block, 0, st, K, X, smooth, Q, sx)
    if (pieces <= 1)
        LQ_LAUNCH_Q(1);
    else if (pieces <= 2)
        LQ_LAUNCH_Q(2);
    else if (pieces <= 4)
        LQ_LAUNCH_Q(4);
    else if (pieces <= 6)
        LQ_LAUNCH_Q(6);
    else if (pieces <= 8)
        LQ_LAUNCH_Q(8);
    else
        LQ_LAUNCH_Q(0);
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
