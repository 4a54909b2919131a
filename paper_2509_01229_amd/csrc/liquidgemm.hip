// gfx950 kernels and the C-ABI dispatcher of the LiquidQuant W4A8 GEMM.
//
// Two kernel families share the packed layout of lqq_layout.h and the dequantisation of
// lqq_device.h (paper Sec. 5.3):
//
//   stream  (M <= 16*MB): the memory-bound regime of the paper's cost model (Sec. 3.2,
//           T_LD dominates).  A block owns F tiles of 16 output channels; its NW waves
//           split K between them (in-block split-K), stream the packed weights straight
//           from HBM into registers with one 16-byte load per lane, dequantise, feed the
//           MFMA, and reduce their INT32 partials through LDS -- integer sums, so the
//           result does not depend on the order.  No workspace, one launch.
//
//   tile    (larger M): the compute-bound regime (T_DQ + T_MMA dominates).  A block of 4
//           waves owns WM rows of X and 256 output channels; the X tile is staged in LDS
//           (double buffered) and shared by the waves, each wave keeps its own 64
//           channels' weights in registers (global -> VGPR, never through LDS: the
//           dequantised operand is consumed by the MFMA of the same wave, which is the
//           point of the paper's implicit fine-grained pipeline, Sec. 5.1) and reuses
//           every dequantised fragment for WM/16 MFMAs.
//
// Both compute Y = X W^T with the weights on the B operand of v_mfma_i32_16x16x64_i8, so
// that a lane ends up with 4 adjacent output channels of one row (the tile interleave of
// the layout) and the epilogue writes 8-byte FP16 pieces that form full 128-byte lines.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>

#include "lqq_common.h"
#include "lqq_device.h"

namespace lqq {

// ------------------------------------------------------------------------------------
// Layout hook: packed -> INT8 [N,K] with the kernels' own unpack + Eq. 12 path.
// One wave per 1 KiB chunk (16 channels x 128 k).
// ------------------------------------------------------------------------------------
template <bool G128>
__global__ __launch_bounds__(256) void dequant_dump_kernel(const u32x4 *__restrict__ Wp,
                                                           const uint8_t *__restrict__ gp, int N, int K,
                                                           int8_t *__restrict__ Wd)
{
    const int lane = threadIdx.x & 63;
    const int j = lane & 15, kb = lane >> 4;
    const int chunks_per_tile = K >> 7;
    const int t = blockIdx.y;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= chunks_per_tile) return;
    const size_t chunk = (size_t)t * chunks_per_tile + c;
    const u32x4 p = Wp[chunk * 64 + lane];
    UnitParams<G128> up;
    up.load(gp, (size_t)t * (K >> 8) + (c >> 1), j);
    v4i lo, hi;
    dequant_unit_chunk<G128>(p, up, c & 1, lo, hi);
    int8_t *row = Wd + (size_t)channel_of(t, j) * K + (size_t)c * 128 + 16 * kb;
    *reinterpret_cast<v4i *>(row) = lo;
    *reinterpret_cast<v4i *>(row + 64) = hi;
}

// ------------------------------------------------------------------------------------
// Epilogue of one accumulator element (Sec. 4: first-level dequantisation; Sec. 5.3).
// ------------------------------------------------------------------------------------
__device__ __forceinline__ __half scale_to_half(int acc, float sx, float sw)
{
    return __float2half_rn((float)acc * sx * sw);
}

// ------------------------------------------------------------------------------------
// stream kernel
// ------------------------------------------------------------------------------------
template <int F, int MB, bool G128>
struct StreamRegs {
    u32x4 w[F][2];
    UnitParams<G128> p[F];
    u32x4 x[MB][4];
};

template <int F, int NW, int MB, bool G128>
__global__ __launch_bounds__(NW * 64) void w4a8_stream_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, kb = lane >> 4;
    const int t0 = blockIdx.x * F;
    const int units = K >> 8;
    const int chunks_per_tile = K >> 7;

    v4i acc[F][MB];
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[f][mb] = v4i{0, 0, 0, 0};

    auto load_unit = [&](int u, StreamRegs<F, MB, G128> &r) {
#pragma unroll
        for (int f = 0; f < F; ++f) {
            const u32x4 *base = Wp + ((size_t)(t0 + f) * chunks_per_tile + 2 * u) * 64 + lane;
            r.w[f][0] = __builtin_nontemporal_load(base);
            r.w[f][1] = __builtin_nontemporal_load(base + 64);
            r.p[f].load(gp, (size_t)(t0 + f) * units + u, j);
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            // rows past M read row M-1 (their outputs are never stored)
            const int m = min(16 * mb + j, M - 1);
            const int8_t *xr = X + (size_t)m * K + (size_t)u * 256 + 16 * kb;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) r.x[mb][ks] = *reinterpret_cast<const u32x4 *>(xr + 64 * ks);
        }
    };

    auto compute_unit = [&](const StreamRegs<F, MB, G128> &r) {
#pragma unroll
        for (int f = 0; f < F; ++f)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                v4i lo, hi;
                dequant_unit_chunk<G128>(r.w[f][c], r.p[f], c, lo, hi);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    acc[f][mb] = mfma_i8(__builtin_bit_cast(v4i, r.x[mb][2 * c]), lo, acc[f][mb]);
                    acc[f][mb] = mfma_i8(__builtin_bit_cast(v4i, r.x[mb][2 * c + 1]), hi, acc[f][mb]);
                }
            }
    };

    // Register double buffering: the loads of the next unit are in flight while the
    // current one is dequantised and multiplied.
    StreamRegs<F, MB, G128> cur, nxt;
    int u = wave;
    if (u < units) load_unit(u, cur);
    for (; u < units; u += NW) {
        const bool more = (u + NW) < units;
        if (more) load_unit(u + NW, nxt);
        compute_unit(cur);
        if (more) cur = nxt;
    }

    // In-block split-K reduction (integer, order independent) and epilogue.
    constexpr int VALS = F * MB * 4;  // accumulator registers per lane
    __shared__ int red[NW][VALS][64];
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave][(f * MB + mb) * 4 + r][lane] = acc[f][mb][r];
    __syncthreads();
    for (int idx = threadIdx.x; idx < VALS * 64; idx += NW * 64) {
        const int v = idx >> 6, l = idx & 63;
        int sum = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red[w][v][l];
        const int r = v & 3, fm = v >> 2;
        const int mb = fm % MB, f = fm / MB;
        const int m = 16 * mb + 4 * (l >> 4) + r;
        if (m < M) {
            const int n = channel_of(t0 + f, l & 15);
            if (ACC) ACC[(size_t)m * N + n] = sum;
            if (Y) Y[(size_t)m * N + n] = scale_to_half(sum, sx[m], sw[n]);
        }
    }
}

// ------------------------------------------------------------------------------------
// tile kernel
// ------------------------------------------------------------------------------------
constexpr int kTilePitch = 256 + 16;  // LDS row pitch in bytes: rows shift by 4 banks

template <int WM, bool G128>
__global__ __launch_bounds__(256) void w4a8_tile_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int blocks_n)
{
    constexpr int MI = WM / 16;        // m fragments per wave
    constexpr int XP = WM * 16 / 256;  // 16-byte X pieces per thread per unit
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, kb = lane >> 4;
    const int bn = blockIdx.x % blocks_n, bm = blockIdx.x / blocks_n;
    const int m0 = bm * WM;
    const int ng = bn * 4 + wave;  // 64-channel group of this wave
    const bool active = ng < (N >> 6);
    // A wave past the last group recomputes the last one and stores nothing, so that the
    // main loop has no divergent path around its barriers.
    const int t0 = 4 * (active ? ng : (N >> 6) - 1);
    const int units = K >> 8;
    const int chunks_per_tile = K >> 7;

    v4i acc[MI][4];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[mi][f] = v4i{0, 0, 0, 0};

    u32x4 xr[XP];
    u32x4 wc[4][2], wn[4][2];
    UnitParams<G128> pc[4], pn[4];

    // Rows past M read row M-1: an output row depends only on its own X row, and rows
    // past M are never stored.
    auto load_x = [&](int u) {
#pragma unroll
        for (int i = 0; i < XP; ++i) {
            const int q = tid + 256 * i;
            const int row = q >> 4, col = q & 15;
            const int m = min(m0 + row, M - 1);
            xr[i] = *reinterpret_cast<const u32x4 *>(X + (size_t)m * K + (size_t)u * 256 + 16 * col);
        }
    };
    auto store_x = [&](int stage) {
        int8_t *base = lds + stage * (WM * kTilePitch);
#pragma unroll
        for (int i = 0; i < XP; ++i) {
            const int q = tid + 256 * i;
            const int row = q >> 4, col = q & 15;
            *reinterpret_cast<u32x4 *>(base + row * kTilePitch + 16 * col) = xr[i];
        }
    };
    auto load_w = [&](int u, u32x4 (&w)[4][2], UnitParams<G128> (&p)[4]) {
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const u32x4 *base = Wp + ((size_t)(t0 + f) * chunks_per_tile + 2 * u) * 64 + lane;
            w[f][0] = base[0];
            w[f][1] = base[64];
            p[f].load(gp, (size_t)(t0 + f) * units + u, j);
        }
    };
    auto compute = [&](int stage) {
        const int8_t *xs = lds + stage * (WM * kTilePitch) + j * kTilePitch + 16 * kb;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            v4i blo[4], bhi[4];
#pragma unroll
            for (int f = 0; f < 4; ++f) dequant_unit_chunk<G128>(wc[f][c], pc[f], c, blo[f], bhi[f]);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const v4i a0 = *reinterpret_cast<const v4i *>(xs + mi * 16 * kTilePitch + 128 * c);
                const v4i a1 = *reinterpret_cast<const v4i *>(xs + mi * 16 * kTilePitch + 128 * c + 64);
#pragma unroll
                for (int f = 0; f < 4; ++f) acc[mi][f] = mfma_i8(a0, blo[f], acc[mi][f]);
#pragma unroll
                for (int f = 0; f < 4; ++f) acc[mi][f] = mfma_i8(a1, bhi[f], acc[mi][f]);
            }
        }
    };

    load_x(0);
    load_w(0, wc, pc);
    store_x(0);
    __syncthreads();

    // Steady state: the global loads of unit u+1 are issued before the MFMAs of unit u
    // and land in LDS / registers after them.
    for (int u = 0; u + 1 < units; ++u) {
        load_x(u + 1);
        load_w(u + 1, wn, pn);
        compute(u & 1);
        store_x((u + 1) & 1);
        __syncthreads();
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            wc[f][0] = wn[f][0];
            wc[f][1] = wn[f][1];
            pc[f] = pn[f];
        }
    }
    compute((units - 1) & 1);

    if (!active) return;
    // Epilogue: lane holds, for row m = m0 + 16*mi + 4*kb + r, the 4 adjacent channels
    // n0 + 4*j + f (f = 0..3).
    const int n = 64 * ng + 4 * j;
    float4 swv = float4{0, 0, 0, 0};
    if (Y) swv = *reinterpret_cast<const float4 *>(sw + n);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = m0 + 16 * mi + 4 * kb + r;
            if (m < M) {
                const int a0 = acc[mi][0][r], a1 = acc[mi][1][r], a2 = acc[mi][2][r], a3 = acc[mi][3][r];
                if (ACC) *reinterpret_cast<v4i *>(ACC + (size_t)m * N + n) = v4i{a0, a1, a2, a3};
                if (Y) {
                    const float s = sx[m];
                    union {
                        __half h[4];
                        uint2 u;
                    } o;
                    o.h[0] = scale_to_half(a0, s, swv.x);
                    o.h[1] = scale_to_half(a1, s, swv.y);
                    o.h[2] = scale_to_half(a2, s, swv.z);
                    o.h[3] = scale_to_half(a3, s, swv.w);
                    *reinterpret_cast<uint2 *>(Y + (size_t)m * N + n) = o.u;
                }
            }
        }
}

// ------------------------------------------------------------------------------------
// Variant table and dispatcher
// ------------------------------------------------------------------------------------
struct Args {
    int M, N, K, group;
    const int8_t *X;
    const float *sx;
    const u32x4 *Wp;
    const uint8_t *gp;
    const float *sw;
    __half *Y;
    int32_t *ACC;
    hipStream_t stream;
};

typedef int (*LaunchFn)(const Args &);

template <int F, int NW, int MB>
static int launch_stream(const Args &a)
{
    if (a.M > 16 * MB) return fail(LQ_ERR_INVALID, "stream variant handles M <= %d, got %d", 16 * MB, a.M);
    if ((a.N / 16) % F != 0) return fail(LQ_ERR_INVALID, "N/16 not a multiple of F=%d", F);
    const dim3 grid(a.N / (16 * F)), block(NW * 64);
    if (a.group == 128)
        hipLaunchKernelGGL((w4a8_stream_kernel<F, NW, MB, true>), grid, block, 0, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC);
    else
        hipLaunchKernelGGL((w4a8_stream_kernel<F, NW, MB, false>), grid, block, 0, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC);
    return LQ_OK;
}

template <int WM>
static int launch_tile(const Args &a)
{
    const int blocks_n = (a.N + 255) / 256, blocks_m = (a.M + WM - 1) / WM;
    const size_t lds_bytes = 2 * (size_t)WM * kTilePitch;
    const dim3 grid((unsigned)(blocks_n * blocks_m)), block(256);
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&w4a8_tile_kernel<WM, true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&w4a8_tile_kernel<WM, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess)
            return fail(LQ_ERR_HIP, "hipFuncSetAttribute(%zu bytes of LDS): %s", lds_bytes, hipGetErrorString(e));
        attr_done = true;
    }
    if (a.group == 128)
        hipLaunchKernelGGL((w4a8_tile_kernel<WM, true>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_n);
    else
        hipLaunchKernelGGL((w4a8_tile_kernel<WM, false>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_n);
    return LQ_OK;
}

struct Variant {
    const char *name;
    LaunchFn fn;
    int max_m;  // 0 = unlimited
};

static const Variant kVariants[] = {
    {"stream_f1_w16_m16", &launch_stream<1, 16, 1>, 16},
    {"stream_f1_w8_m16", &launch_stream<1, 8, 1>, 16},
    {"stream_f2_w8_m16", &launch_stream<2, 8, 1>, 16},
    {"stream_f4_w4_m16", &launch_stream<4, 4, 1>, 16},
    {"stream_f4_w8_m16", &launch_stream<4, 8, 1>, 16},
    {"stream_f2_w8_m32", &launch_stream<2, 8, 2>, 32},
    {"stream_f4_w4_m32", &launch_stream<4, 4, 2>, 32},
    {"tile_m32", &launch_tile<32>, 0},
    {"tile_m64", &launch_tile<64>, 0},
    {"tile_m128", &launch_tile<128>, 0},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

static int find_variant(const char *name)
{
    for (int i = 0; i < kNumVariants; ++i)
        if (!strcmp(kVariants[i].name, name)) return i;
    return -1;
}

// Shape -> kernel.  Decode-sized batches stream the weights with in-block split-K sized
// so that the grid fills the 256 CUs; larger batches use the LDS-tiled kernel with the
// largest row tile that M fills.
static int select_variant(int M, int N, int K)
{
    (void)K;
    if (M <= 16) {
        const int tiles = N / 16;
        if (tiles <= 512) return find_variant("stream_f1_w16_m16");
        if (tiles <= 1024) return find_variant("stream_f1_w8_m16");
        return find_variant("stream_f2_w8_m16");
    }
    if (M <= 32) return find_variant(N / 16 <= 1024 ? "stream_f2_w8_m32" : "stream_f4_w4_m32");
    if (M <= 64) return find_variant("tile_m64");
    return find_variant("tile_m128");
}

static int check_device_args(const Args &a, const void *ws, size_t ws_bytes)
{
    (void)ws;
    (void)ws_bytes;
    if (a.M < 0 || !shape_ok(a.N, a.K, a.group))
        return fail(LQ_ERR_INVALID,
                    "bad shape M=%d N=%d K=%d group=%d (need M>=0, N%%64==0, K%%256==0, group 64|128, K<=131072)",
                    a.M, a.N, a.K, a.group);
    if (a.M == 0) return LQ_OK;  // nothing to read or write; pointers may be null
    if (!a.Y && !a.ACC) return fail(LQ_ERR_INVALID, "no output pointer");
    if (!a.X || !a.Wp || !a.gp) return fail(LQ_ERR_INVALID, "null input pointer");
    if (a.Y && (!a.sx || !a.sw)) return fail(LQ_ERR_INVALID, "null scale pointer");
    const uintptr_t bits = (uintptr_t)a.X | (uintptr_t)a.Wp | (uintptr_t)a.gp | (uintptr_t)a.sx |
                           (uintptr_t)a.sw | (uintptr_t)a.Y | (uintptr_t)a.ACC;
    if (bits & 15) return fail(LQ_ERR_ALIGN, "device pointers must be 16-byte aligned");
    return LQ_OK;
}

static int run(int variant, const Args &a, const void *ws, size_t ws_bytes)
{
    if (int rc = check_device_args(a, ws, ws_bytes)) return rc;
    if (a.M == 0) return LQ_OK;
    if (variant < 0) variant = select_variant(a.M, a.N, a.K);
    if (variant < 0 || variant >= kNumVariants) return fail(LQ_ERR_INVALID, "unknown variant %d", variant);
    (void)hipGetLastError();
    if (int rc = kVariants[variant].fn(a)) return rc;
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(LQ_ERR_HIP, "launch of %s failed: %s", kVariants[variant].name, hipGetErrorString(e));
    return LQ_OK;
}

}  // namespace lqq

using namespace lqq;

extern "C" {

size_t w4a8_gemm_workspace_size(int M, int N, int K, int group)
{
    (void)M;
    (void)N;
    (void)K;
    (void)group;
    return 0;  // split-K is reduced inside the block, in LDS
}

int w4a8_gemm(int M, int N, int K, int group, const int8_t *X, const float *act_scales,
              const void *W_packed, const uint8_t *gparams, const float *w_scales, uint16_t *Y,
              void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!Y && M != 0) return fail(LQ_ERR_INVALID, "null Y");
    const Args a{M, N, K, group, X, act_scales, static_cast<const u32x4 *>(W_packed), gparams, w_scales,
                 reinterpret_cast<__half *>(Y), nullptr, static_cast<hipStream_t>(hip_stream)};
    return run(-1, a, workspace, workspace_bytes);
}

int w4a8_gemm_i32(int M, int N, int K, int group, const int8_t *X, const void *W_packed,
                  const uint8_t *gparams, int32_t *ACC, void *workspace, size_t workspace_bytes,
                  void *hip_stream)
{
    if (!ACC && M != 0) return fail(LQ_ERR_INVALID, "null ACC");
    const Args a{M, N, K, group, X, nullptr, static_cast<const u32x4 *>(W_packed), gparams, nullptr,
                 nullptr, ACC, static_cast<hipStream_t>(hip_stream)};
    return run(-1, a, workspace, workspace_bytes);
}

int w4a8_gemm_variant(int variant, int M, int N, int K, int group, const int8_t *X,
                      const float *act_scales, const void *W_packed, const uint8_t *gparams,
                      const float *w_scales, uint16_t *Y, int32_t *ACC, void *workspace,
                      size_t workspace_bytes, void *hip_stream)
{
    if (variant < -1 || variant >= kNumVariants) return fail(LQ_ERR_INVALID, "unknown variant %d", variant);
    const Args a{M, N, K, group, X, act_scales, static_cast<const u32x4 *>(W_packed), gparams, w_scales,
                 reinterpret_cast<__half *>(Y), ACC, static_cast<hipStream_t>(hip_stream)};
    return run(variant, a, workspace, workspace_bytes);
}

int w4a8_variant_count(void) { return kNumVariants; }

const char *w4a8_variant_name(int variant)
{
    return (variant >= 0 && variant < kNumVariants) ? kVariants[variant].name : nullptr;
}

int w4a8_select_variant(int M, int N, int K, int group)
{
    if (M < 0 || !shape_ok(N, K, group)) return fail(LQ_ERR_INVALID, "bad shape");
    return select_variant(M, N, K);
}

int w4a8_dequant_dump(const void *W_packed, const uint8_t *gparams, int N, int K, int group,
                      int8_t *Wd, void *hip_stream)
{
    if (!shape_ok(N, K, group)) return fail(LQ_ERR_INVALID, "bad shape N=%d K=%d group=%d", N, K, group);
    if (!W_packed || !gparams || !Wd) return fail(LQ_ERR_INVALID, "null pointer");
    if (((uintptr_t)W_packed | (uintptr_t)gparams | (uintptr_t)Wd) & 15)
        return fail(LQ_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const dim3 grid((unsigned)((K / 128 + 3) / 4), (unsigned)(N / 16)), block(256);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    if (group == 128)
        hipLaunchKernelGGL(dequant_dump_kernel<true>, grid, block, 0, st,
                           static_cast<const u32x4 *>(W_packed), gparams, N, K, Wd);
    else
        hipLaunchKernelGGL(dequant_dump_kernel<false>, grid, block, 0, st,
                           static_cast<const u32x4 *>(W_packed), gparams, N, K, Wd);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LQ_ERR_HIP, "dequant_dump launch failed: %s", hipGetErrorString(e));
    return LQ_OK;
}

}  // extern "C"
