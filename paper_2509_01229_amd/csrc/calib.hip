// Calibration kernels: what one MI355X actually delivers on the two resources that bound
// the W4A8 GEMM (the T_LD and T_MMA terms of the paper's cost model, Sec. 3.2), measured
// with nothing else in the way.  bench.py reports them beside the nominal peaks.
//
//   w4a8_calib_stream_read : every byte of a buffer read once with 16-byte non-temporal
//                            loads (one contiguous share per block), nothing computed,
//                            nothing of size written.
//   w4a8_calib_mfma_i8     : back-to-back v_mfma_i32_32x32x32_i8 on register operands,
//                            two waves per SIMD, with the register pressure of a real
//                            kernel (8 independent 32x32 accumulators per wave).
#include <hip/hip_runtime.h>

#include "lqq_common.h"
#include "lqq_device.h"

namespace lqq {

// Written only if a checksum takes one particular value, so that no load or MFMA can be
// dropped by the compiler while practically nothing is stored.
__device__ unsigned int g_calib_sink[64];

constexpr int kReadBlocksPerCU = 4, kCUs = 256;

// Every block streams its own contiguous share of the buffer, eight 16-byte loads per thread
// in flight: many concurrent sequential streams, the pattern of the GEMM kernels themselves
// (a block walks the contiguous code stream of its tiles) and, among the launch shapes tried
// (grid-stride or block-contiguous, 2 to 8 loads in flight, 256 to 4096 blocks), the fastest.
__global__ __launch_bounds__(256) void calib_read_kernel(const u32x4 *__restrict__ p, size_t n16)
{
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t begin = (size_t)blockIdx.x * per, end = begin + per < n16 ? begin + per : n16;
    size_t i = begin + threadIdx.x;
    u32x4 x = {0, 0, 0, 0};
    for (; i + 7 * 256 < end; i += 8 * 256) {
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(p + i + j * 256);
#pragma unroll
        for (int j = 0; j < 8; ++j) x ^= v[j];
    }
    for (; i < end; i += 256) x ^= __builtin_nontemporal_load(p + i);
    if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x5eed1234u) g_calib_sink[threadIdx.x & 63] = 1;
}

// RANDOM = false: the same operands every time (little switching in the multipliers);
// RANDOM = true: eight different pseudo-random A fragments and four B fragments taken in
// turn, so that consecutive MFMAs see unrelated bytes, as with real activations and weights.
template <bool RANDOM>
__global__ __launch_bounds__(256, 2) void calib_mfma_kernel(int iters)
{
    const unsigned lane_seed = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    v4i a[8], b[4];
    unsigned s = lane_seed;
    auto next = [&]() {
        s = s * 1664525u + 1013904223u;
        return (int)(s ^ (s >> 13));
    };
#pragma unroll
    for (int i = 0; i < 8; ++i)
        a[i] = RANDOM ? v4i{next(), next(), next(), next()} : v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
#pragma unroll
    for (int i = 0; i < 4; ++i)
        b[i] = RANDOM ? v4i{next(), next(), next(), next()} : v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
    v16i acc[4][2];
#pragma unroll
    for (int mf = 0; mf < 4; ++mf)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mf][t][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int mf = 0; mf < 4; ++mf)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    acc[mf][t] = mfma_i8(a[(u + mf) & 7], b[(u + t) & 3], acc[mf][t]);
    }
    int x = 0;
#pragma unroll
    for (int mf = 0; mf < 4; ++mf)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) x ^= acc[mf][t][r];
    if (x == 0x5eed1234 && iters < 0) g_calib_sink[threadIdx.x & 63] = (unsigned)x;
}

}  // namespace lqq

using namespace lqq;

extern "C" {

int w4a8_calib_stream_read(const void *buf, size_t bytes, void *hip_stream)
{
    if (!buf || bytes < 16) return fail(LQ_ERR_INVALID, "calibration read needs a buffer of at least 16 bytes");
    if ((uintptr_t)buf & 15) return fail(LQ_ERR_ALIGN, "device pointers must be 16-byte aligned");
    (void)hipGetLastError();
    hipLaunchKernelGGL(calib_read_kernel, dim3(kCUs * kReadBlocksPerCU), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const u32x4 *>(buf), bytes / 16);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LQ_ERR_HIP, "calibration read launch failed: %s", hipGetErrorString(e));
    return LQ_OK;
}

int w4a8_calib_mfma_i8(int iters, int random_operands, double *ops, void *hip_stream)
{
    if (iters < 1 || iters > (1 << 20)) return fail(LQ_ERR_INVALID, "calibration iterations out of range");
    constexpr int blocks = 2 * kCUs;
    if (ops) *ops = (double)blocks * 4 /*waves*/ * iters * 64 /*MFMAs per iteration*/ * (2.0 * 32 * 32 * 32);
    (void)hipGetLastError();
    if (random_operands)
        hipLaunchKernelGGL(calib_mfma_kernel<true>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), iters);
    else
        hipLaunchKernelGGL(calib_mfma_kernel<false>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), iters);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LQ_ERR_HIP, "calibration MFMA launch failed: %s", hipGetErrorString(e));
    return LQ_OK;
}

}  // extern "C"
