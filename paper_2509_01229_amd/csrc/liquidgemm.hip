// gfx950 kernels and the C-ABI dispatcher of the LiquidQuant W4A8 GEMM.
//
// Two kernel families share the packed layout of lqq_layout.h and the dequantisation of
// lqq_device.h (paper Sec. 5.3):
//
//   stream  (M <= 64): the memory-bound regime of the paper's cost model (Sec. 3.2,
//           T_LD dominates).  A block owns F tiles of 32 output channels; its NW waves
//           split K between them (in-block split-K), stream the packed weights straight
//           from HBM into registers with one 16-byte load per lane, dequantise, feed the
//           MFMA, and reduce their INT32 partials through LDS -- integer sums, so the
//           result does not depend on the order.  stream16 is the same on the 16-row MFMA
//           shape for M <= 16.  Optional grid-level split-K through a workspace.
//
//   tiled   (larger M): the compute-bound regime (T_DQ + T_MMA dominates).  A block owns
//           128 rows of X and 256 output channels; the X tile is staged in LDS (double
//           buffered) and shared by the waves, each wave keeps its own 64 channels'
//           weights in registers (global -> VGPR, never through LDS: the dequantised
//           operand is consumed by the MFMA of the same wave, which is the point of the
//           paper's implicit fine-grained pipeline, Sec. 5.1) and reuses every dequantised
//           fragment for 4 MFMAs.  Three forms: `duo` (X staged through registers, two k
//           groups per block for grids of at most one block per CU), `duo_dl` (X straight
//           into LDS, deeper pipeline, grids that fill the chip) and `duo_pt` (duo_dl with
//           resident blocks walking several tiles as one stream of stages).
//
// All compute Y = X W^T with the weights on the B operand of the INT8 MFMA, so that a lane
// ends up with 2 adjacent output channels of one row (the tile interleave of the layout)
// and a half-wave writes a full 128-byte line of FP16.
//
// Every kernel here must compile without scratch memory (the build checks it): register
// spills next to the divergent single-thread sections of the split-K protocol are not
// something to rely on.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "lqq_common.h"
#include "lqq_device.h"

namespace lqq {

// Clears the ticket area at the head of a workspace (a fill kernel rather than a memset, so
// that it can be captured in a HIP graph like everything else here).
__global__ __launch_bounds__(256) void workspace_init_kernel(unsigned int *tickets, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) tickets[i] = 0u;
}

// ------------------------------------------------------------------------------------
// Layout hook: packed -> INT8 [N,K] with the kernels' own unpack + Eq. 12 path.
// One wave per 1 KiB chunk (32 channels x 64 k).
// ------------------------------------------------------------------------------------
template <bool G128>
__global__ __launch_bounds__(256) void dequant_dump_kernel(const u32x4 *__restrict__ Wp,
                                                           const uint8_t *__restrict__ gp, int N, int K,
                                                           int8_t *__restrict__ Wd)
{
    const int lane = threadIdx.x & 63;
    const int j = lane & 31, kb = lane >> 5;
    const int chunks_per_tile = K >> 6;
    const int t = blockIdx.y;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= chunks_per_tile) return;
    const u32x4 p = Wp[((size_t)t * chunks_per_tile + c) * 64 + lane];
    UnitParams<G128> up;
    up.load(gp, (size_t)t * (K >> 7) + (c >> 1), j);
    uint32_t s2, a4;
    up.get(c & 1, s2, a4);
    v4i lo, hi;
    dequant_chunk(p, s2, a4, lo, hi);
    int8_t *row = Wd + (size_t)channel_of(t, j) * K + (size_t)c * 64 + 16 * kb;
    *reinterpret_cast<v4i *>(row) = lo;
    *reinterpret_cast<v4i *>(row + 32) = hi;
}

// ------------------------------------------------------------------------------------
// Epilogue of one accumulator element (Sec. 4: first-level dequantisation; Sec. 5.3).
// ------------------------------------------------------------------------------------
__device__ __forceinline__ __half scale_to_half(int acc, float sx, float sw)
{
    return __float2half_rn((float)acc * sx * sw);
}

#include "kernels_common.h"
#include "kernels_stream.h"
#include "kernels_tiled.h"
#include "kernels_tiled_dl.h"
#include "kernels_tiled_pt.h"
#include "kernels_tiled_solo.h"
#include "kernels_tiled_solo16.h"
#include "kernels_reference.h"
#include "kernels_grouped.h"

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
    void *ws;
    size_t ws_bytes;
    size_t *query = nullptr;  // set: store the workspace bytes the launch would use and launch nothing
};

typedef int (*LaunchFn)(const Args &);

// Kernels that need more than the default 48 KiB of dynamic LDS must be told so once per
// device; the grant is remembered, so the launch path of a short kernel pays one map lookup
// instead of a runtime call.
static int allow_lds_once(const void *kernel, size_t bytes)
{
    struct Grant {
        int dev;
        const void *kernel;
        size_t bytes;
    };
    static std::mutex mu;
    static Grant granted[512];  // (device, kernel) pairs seen so far; no heap
    static int count = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(LQ_ERR_HIP, "hipGetDevice failed");
    std::lock_guard<std::mutex> lock(mu);
    Grant *g = nullptr;
    for (int i = 0; i < count && !g; ++i)
        if (granted[i].dev == dev && granted[i].kernel == kernel) g = &granted[i];
    if (g && g->bytes >= bytes) return LQ_OK;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess)
        return fail(LQ_ERR_HIP, "hipFuncSetAttribute(%zu bytes of LDS): %s", bytes, hipGetErrorString(e));
    if (!g && count < 512) g = &granted[count++];
    if (g) *g = Grant{dev, kernel, bytes};  // a full table only means asking again next time
    return LQ_OK;
}
template <class Kernel>
static int allow_lds(Kernel kernel, size_t bytes)
{
    if (bytes <= 48 * 1024) return LQ_OK;
    return allow_lds_once(reinterpret_cast<const void *>(kernel), bytes);
}

// Grid-level split of K for the stream kernels: enough blocks for every CU to hold two
// (about 512), each wave keeping at least two units of 128 k.
static int stream_split(int N, int K, int F, int NW)
{
    const int groups = N / (32 * F), units = K / 128;
    // Measured on MI355X: the exchange of partial tiles through memory costs about 3 us, so
    // K is split across blocks only when N alone leaves most CUs without a block.
    int s = groups > 128 ? 1 : (groups > 64 ? 2 : 4);
    s = std::min(s, units / (2 * NW));
    return std::max(1, s);
}

static size_t stream_ws_bytes(int M, int N, int S, int MF = 1)
{
    if (S <= 1) return 0;
    const int rmax = MF == 1 ? 4 * ((M + 7) / 8) : 16;
    return kTicketBytes + (size_t)S * (N / 32) * MF * rmax * 64 * sizeof(int32_t);
}

// S = requested number of K slices; `named` = the variant names its split (then a missing
// workspace is an error instead of a fall-back to one slice).
template <int F, int NW, int MF, bool XL = false>
static int launch_stream_as(const Args &a, int S, bool named)
{
    if (a.M > 32 * MF) return fail(LQ_ERR_INVALID, "this stream variant handles M <= %d, got %d", 32 * MF, a.M);
    if ((a.N / 32) % F != 0) return fail(LQ_ERR_INVALID, "N/32 not a multiple of F=%d", F);
    const int groups = a.N / (32 * F);
    S = std::max(1, std::min(S, a.K / 128));
    if (S > 1 && groups > kMaxTicketGroups) S = 1;
    size_t need = stream_ws_bytes(a.M, a.N, S, MF);
    if (a.query) return *a.query = need, LQ_OK;
    if (need > 0 && (!a.ws || a.ws_bytes < need)) {
        if (named)
            return fail(LQ_ERR_WORKSPACE, "split-K needs %zu bytes of workspace, got %zu", need,
                        a.ws ? a.ws_bytes : 0);
        S = 1;
        need = 0;
    }
    const dim3 grid(groups, S), block(NW * 64);
    const int rmax = MF == 1 ? 4 * ((a.M + 7) / 8) : 16;
    // reduction buffer; with XL the waves' X regions (32 MF rows x 128 k each) come first in the same memory
    const size_t lds_bytes = std::max((size_t)NW * F * MF * rmax * 64 * sizeof(int), XL ? (size_t)NW * MF * 4096 : 0);
    unsigned int *tickets = static_cast<unsigned int *>(a.ws);
    int32_t *partials = a.ws ? reinterpret_cast<int32_t *>(static_cast<char *>(a.ws) + kTicketBytes) : nullptr;
    if (a.group == 128) {
        if (int rc = allow_lds(&w4a8_stream_kernel<F, NW, MF, true, XL>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_stream_kernel<F, NW, MF, true, XL>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, partials, tickets);
    } else {
        if (int rc = allow_lds(&w4a8_stream_kernel<F, NW, MF, false, XL>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_stream_kernel<F, NW, MF, false, XL>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, partials, tickets);
    }
    return LQ_OK;
}

// SPLIT: 0 = choose with stream_split(), otherwise the fixed number of K slices.
template <int F, int NW, int SPLIT, int MF = 1, bool XL = false>
static int launch_stream(const Args &a)
{
    return launch_stream_as<F, NW, MF, XL>(a, SPLIT ? SPLIT : stream_split(a.N, a.K, F, NW), SPLIT != 0);
}

// 32-row (MF = 1) and 64-row (MF = 2) stream kernels with the block shape chosen from N.
// Measured for both: the best grid is the largest one of at most 256 blocks of 8 waves --
// one tile per block while N / 32 <= 256, else two -- with K split across blocks while
// that still fits and leaves every wave at least four units of 128 k.
template <int MF, bool XL>
static int launch_stream_shaped(const Args &a)
{
    const int tiles = a.N / 32;
    // long K with no room for K slices: two tiles per block share the X fragments and two
    // K slices halve each wave's walk (29 vs 31 us at 32 rows, 39 vs 42 at 64 rows on 8192 x 28672)
    if (tiles > 128 && tiles <= 256 && a.K >= 24576) return launch_stream_as<2, 8, MF, XL>(a, 2, false);
    if (tiles <= 256) {
        const int s_units = std::max(1, a.K / (128 * 8 * 4));
        return launch_stream_as<1, 8, MF, XL>(a, std::min({4, 256 / tiles, s_units}), false);
    }
    return launch_stream_as<2, 8, MF, XL>(a, 1, false);
}

// X through LDS (XL) pays whenever a wave holds two row fragments; with one it is worth
// 4-9 % once most of the 32 rows exist and N is small enough for one tile per block (or, with
// two tiles per block, K is long: 21.5 against 22.8 us at 32 rows on 12288 x 12288), and
// costs a few per cent otherwise (measured at 20..32 rows on 36 weight shapes).
template <int MF>
static int launch_stream_auto(const Args &a)
{
    if (MF == 2) return launch_stream_shaped<2, true>(a);
    const int tiles = a.N / 32;
    const bool xl = a.M > 24 && (tiles <= 256 || (tiles <= 512 && a.K >= 12288));
    return xl ? launch_stream_shaped<1, true>(a) : launch_stream_shaped<1, false>(a);
}

template <int F, int NW, int SPLIT, int UU = 1>
static int launch_stream16(const Args &a)
{
    if (a.M > 16) return fail(LQ_ERR_INVALID, "stream16 variants handle M <= 16, got %d", a.M);
    if ((a.N / 32) % F != 0) return fail(LQ_ERR_INVALID, "N/32 not a multiple of F=%d", F);
    const int groups = a.N / (32 * F);
    int S = SPLIT ? SPLIT : stream_split(a.N, a.K, F, NW);
    // the deep-prefetch form (small shapes) keeps whole K in one block unless N gives very few
    if (!SPLIT && UU == 4) S = groups <= 64 ? 2 : 1;
    if ((a.K / 128) % UU != 0) return fail(LQ_ERR_INVALID, "K/128 not a multiple of UU=%d", UU);
    S = std::min(S, a.K / (128 * UU));
    if (S > 1 && groups > kMaxTicketGroups) S = 1;
    size_t need = S > 1 ? kTicketBytes + (size_t)S * (a.N / 32) * 8 * 64 * sizeof(int32_t) : 0;
    if (a.query) return *a.query = need, LQ_OK;
    if (need > 0 && (!a.ws || a.ws_bytes < need)) {
        if (SPLIT)
            return fail(LQ_ERR_WORKSPACE, "split-K needs %zu bytes of workspace, got %zu", need,
                        a.ws ? a.ws_bytes : 0);
        S = 1;
        need = 0;
    }
    const dim3 grid(groups, S), block(NW * 64);
    const size_t lds_bytes = (size_t)NW * F * 8 * 64 * sizeof(int);
    unsigned int *tickets = static_cast<unsigned int *>(a.ws);
    int32_t *partials = a.ws ? reinterpret_cast<int32_t *>(static_cast<char *>(a.ws) + kTicketBytes) : nullptr;
    if (a.group == 128) {
        if (int rc = allow_lds(&w4a8_stream16_kernel<F, NW, UU, true>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_stream16_kernel<F, NW, UU, true>), grid, block, lds_bytes, a.stream, a.M, a.N,
                           a.K, a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, partials, tickets);
    } else {
        if (int rc = allow_lds(&w4a8_stream16_kernel<F, NW, UU, false>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_stream16_kernel<F, NW, UU, false>), grid, block, lds_bytes, a.stream, a.M, a.N,
                           a.K, a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, partials, tickets);
    }
    return LQ_OK;
}

// Grid-level split of K for the duo kernel with two k groups per block (grids of at most
// one block per CU).  Measured: a slice costs about as much in partial-tile exchange
// (128 KiB per tile and slice, added up by the last block) as half a 256-k unit costs in
// matrix work, which puts the best slice count near 0.75 * sqrt(K / 256); more slices than
// CUs per tile would only queue up.
static int duo_split(int M, int N, int K)
{
    const int tiles = ((M + 127) / 128) * ((N + 255) / 256);
    if (tiles > 128 || tiles > kMaxTicketGroups) return 1;
    const int units = K / 256;
    int s = (int)(0.75 * std::sqrt((double)units) + 0.5);
    s = std::min(std::min(s, 256 / tiles), std::min(units / 2, 8));
    return std::max(1, s);
}
static size_t duo_ws_bytes(int M, int N, int S, int tm = 128)
{
    if (S <= 1) return 0;
    const size_t tiles = (size_t)((M + tm - 1) / tm) * ((N + 255) / 256);
    return kTicketBytes + tiles * S * 4 * 32 * 256 * sizeof(int32_t);  // a tile's slot has the full size whatever its height
}

template <int SPLIT, int KG, int TM = 128>
static int launch_duo_as(const Args &a, int S)
{
    constexpr int WM = TM;
    const int blocks_n = (a.N + 255) / 256, blocks_m = (a.M + WM - 1) / WM;
    if ((long long)a.M * a.K >= (1ll << 32))
        return fail(LQ_ERR_INVALID, "M * K = %lld is beyond the 2^32 - 1 bytes of X one call addresses; split the batch",
                    (long long)a.M * a.K);
    S = std::min(S, a.K / (256 * KG));  // every k group of every slice gets at least one unit
    if (blocks_n * blocks_m * 8 > kMaxTicketGroups || S < 1) S = 1;  // one ticket per (tile, wave of the block)
    size_t need = duo_ws_bytes(a.M, a.N, S, TM);
    if (a.query) return *a.query = need, LQ_OK;
    if (need > 0 && (!a.ws || a.ws_bytes < need)) {
        if (SPLIT)
            return fail(LQ_ERR_WORKSPACE, "split-K needs %zu bytes of workspace, got %zu", need,
                        a.ws ? a.ws_bytes : 0);
        S = 1;
        need = 0;
    }
    // KG groups x 2 stages of X; the in-block reduction reuses them and needs 64 KiB
    const size_t lds_bytes = KG == 1 ? 2 * (size_t)128 * kTilePitch
                                     : std::max<size_t>(KG * 2 * (size_t)128 * kTilePitch, 64 * 1024);
    const dim3 grid((unsigned)(blocks_n * blocks_m), (unsigned)S), block(256 * KG);
    unsigned int *tickets = static_cast<unsigned int *>(a.ws);
    int32_t *partials = a.ws ? reinterpret_cast<int32_t *>(static_cast<char *>(a.ws) + kTicketBytes) : nullptr;
    if constexpr (KG == 2 && TM == 128) {
      // one row tile of 65..96 rows: the kernel that computes three of its four row fragments
      if (a.M > 64 && a.M <= 96) {
        constexpr int KG3 = 2;
        if (a.group == 128) {
            if (int rc = allow_lds(w4a8_duo_kernel<true, KG3, 128, true>, lds_bytes)) return rc;
            hipLaunchKernelGGL((w4a8_duo_kernel<true, KG3, 128, true>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                               a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n, partials, tickets);
        } else {
            if (int rc = allow_lds(w4a8_duo_kernel<false, KG3, 128, true>, lds_bytes)) return rc;
            hipLaunchKernelGGL((w4a8_duo_kernel<false, KG3, 128, true>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                               a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n, partials, tickets);
        }
        return LQ_OK;
      }
    }
    if (a.group == 128) {
        if (int rc = allow_lds(w4a8_duo_kernel<true, KG, TM>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_duo_kernel<true, KG, TM>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K, a.X,
                           a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n, partials, tickets);
    } else {
        if (int rc = allow_lds(w4a8_duo_kernel<false, KG, TM>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_duo_kernel<false, KG, TM>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K, a.X,
                           a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n, partials, tickets);
    }
    return LQ_OK;
}

// KGSEL: 0 = choose from the grid size, 1 / 2 = fixed number of k groups per block.
template <int SPLIT, int KGSEL>
static int launch_duo(const Args &a)
{
    const int tiles = ((a.M + 127) / 128) * ((a.N + 255) / 256);
    int kg = KGSEL, S = SPLIT;
    if (!kg) kg = (tiles * std::max(1, SPLIT) <= 256 && a.K >= 512) ? 2 : 1;
    if (a.K < 512) kg = 1;
    if (!S) S = kg == 2 ? duo_split(a.M, a.N, a.K) : 1;
    return kg == 2 ? launch_duo_as<SPLIT, 2>(a, S) : launch_duo_as<SPLIT, 1>(a, S);
}

// The direct-to-LDS form of the kernel (one k group per block; for grids that fill the chip).
template <int SPLIT>
static int launch_duo_dl(const Args &a)
{
    const int blocks_n = (a.N + 255) / 256, blocks_m = (a.M + 127) / 128;
    if ((long long)a.M * a.K >= (1ll << 32))
        return fail(LQ_ERR_INVALID, "M * K = %lld is beyond the 2^32 - 1 bytes of X one call addresses; split the batch",
                    (long long)a.M * a.K);
    int S = std::min(std::max(1, SPLIT), a.K / 256);
    if (blocks_n * blocks_m > kMaxTicketGroups) S = 1;
    const size_t need = duo_ws_bytes(a.M, a.N, S);
    if (a.query) return *a.query = need, LQ_OK;
    if (need > 0 && (!a.ws || a.ws_bytes < need))
        return fail(LQ_ERR_WORKSPACE, "split-K needs %zu bytes of workspace, got %zu", need, a.ws ? a.ws_bytes : 0);
    const size_t lds_bytes = 4 * (size_t)128 * 128;
    const dim3 grid((unsigned)(blocks_n * blocks_m), (unsigned)S), block(256);
    unsigned int *tickets = static_cast<unsigned int *>(a.ws);
    int32_t *partials = a.ws ? reinterpret_cast<int32_t *>(static_cast<char *>(a.ws) + kTicketBytes) : nullptr;
    if (a.group == 128) {
        if (int rc = allow_lds(w4a8_duo_dl_kernel<true>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_duo_dl_kernel<true>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K, a.X, a.sx,
                           a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n, partials, tickets);
    } else {
        if (int rc = allow_lds(w4a8_duo_dl_kernel<false>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_duo_dl_kernel<false>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K, a.X, a.sx,
                           a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n, partials, tickets);
    }
    return LQ_OK;
}

constexpr long long kAssumedCUs = 256;  // the shape rules of the dispatcher are written for the MI355X
// Compute units of the current device (the grid of the persistent kernels), asked once per device.
static int cu_count()
{
    static std::mutex mu;
    static int cached[64];  // 0 = not asked yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        cached[dev] = cus;
    }
    return cached[dev];
}

// The persistent form of the direct-to-LDS kernel: one block per resident slot (two per CU),
// each walking its share of the tiles as one stream of stages.  Needs K % 512 == 0.
static bool duo_pt_fits(int M, int N, int K)
{
    // (a ragged last row tile of at most 64 rows is better off with the two-fragment path of
    // the one-tile-per-block kernels)
    return K % 512 == 0 && (M % 128 == 0 || M % 128 > 64);
}
static int launch_duo_pt(const Args &a)
{
    if (a.query) return LQ_OK;  // no workspace
    if (a.K % 512 != 0) return fail(LQ_ERR_INVALID, "the persistent tiled variant needs K %% 512 == 0, got %d", a.K);
    const int blocks_n = (a.N + 255) / 256, blocks_m = (a.M + 127) / 128;
    if ((long long)a.M * a.K >= (1ll << 32))
        return fail(LQ_ERR_INVALID, "M * K = %lld is beyond the 2^32 - 1 bytes of X one call addresses; split the batch",
                    (long long)a.M * a.K);
    const int cus = cu_count();
    const int grid = std::min(blocks_m * blocks_n, 2 * std::max(cus, 1));
    const size_t lds_bytes = 4 * (size_t)128 * 128;
    if (a.group == 128) {
        if (int rc = allow_lds(w4a8_duo_pt_kernel<true>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_duo_pt_kernel<true>), dim3((unsigned)grid), dim3(256), lds_bytes, a.stream, a.M, a.N,
                           a.K, a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n);
    } else {
        if (int rc = allow_lds(w4a8_duo_pt_kernel<false>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_duo_pt_kernel<false>), dim3((unsigned)grid), dim3(256), lds_bytes, a.stream, a.M, a.N,
                           a.K, a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n);
    }
    return LQ_OK;
}

// Persistent 256 x 256 tiles, one wave per SIMD (see kernels_tiled_solo.h); KG = 2: 256 x 128
// tiles with the four waves as two k groups.  Needs K % 512 == 0 (the 16x16x64 forms without K
// slices: K % 256 == 0).
// K slices across blocks for outputs with fewer tiles than CUs: every slice a multiple of 512 k,
// tiles * slices at most the CUs (one round), the partial sums of a slice as an INT32 matrix of
// its own in the workspace and a second, streaming kernel that adds them up.  Unlike the ticket
// scheme of the 128-row kernels nothing here is serial -- but the partial matrices are 4 S M N
// bytes written and read once, which is why this pays for long K only.  Returns 1 for no split.
static int solo_split(int tiles, int K, int cus)
{
    const int units = K / 512;
    int best = 1;
    for (int s = 2; s <= 4 && s <= units && tiles * s <= cus; ++s)  // (more than four: measured behind the 128-row tiles)
        if (units % s == 0) best = s;
    return best;
}
static size_t solo_ws_bytes(int M, int N, int S)
{
    return S <= 1 ? 0 : kTicketBytes + (size_t)S * M * N * sizeof(int32_t);
}
// SPLIT: 0 = no K slices, -1 = as many as solo_split gives and the workspace holds, n = exactly n
template <int KG, int SPLIT = 0, bool SHAPE16 = false>
static int launch_solo_pt(const Args &a)
{
    // (the 16x16x64 forms without K slices also take K % 512 == 256: two added stages of zero weights)
    if (a.K % 512 != 0 && !(SHAPE16 && SPLIT <= 0))
        return fail(LQ_ERR_INVALID, "this 256-row tile variant needs K %% 512 == 0, got %d", a.K);
    constexpr int TN = 256 / KG;
    const int blocks_n = (a.N + TN - 1) / TN, blocks_m = (a.M + 255) / 256;
    if ((long long)a.M * a.K >= (1ll << 32))
        return fail(LQ_ERR_INVALID, "M * K = %lld is beyond the 2^32 - 1 bytes of X one call addresses; split the batch",
                    (long long)a.M * a.K);
    if (a.N > (1 << 26))  // (a row's lane offsets are 32-bit byte offsets)
        return fail(LQ_ERR_INVALID, "the 256-row tile variants take N up to 2^26, got %d", a.N);
    const int cus = std::max(cu_count(), 1);
    int S = 1;
    if (SPLIT > 0) {
        S = SPLIT;
        if ((a.K / 512) % S != 0)
            return fail(LQ_ERR_INVALID, "%d K slices need K %% %d == 0, got %d", S, 512 * S, a.K);
    } else if (SPLIT < 0) {
        S = a.K % 512 != 0 ? 1 : solo_split(blocks_m * blocks_n, a.K, a.query ? (int)kAssumedCUs : cus);
        // (a workspace too small for them: the largest number of slices it holds)
        // (a query names its limit, if it has one, in ws_bytes)
        auto too_large = [&](int s) {
            const size_t need = solo_ws_bytes(a.M, a.N, s);
            return a.query ? a.ws_bytes > 0 && a.ws_bytes < need : !a.ws || a.ws_bytes < need;
        };
        while (S > 1 && too_large(S)) {
            do --S; while (S > 1 && (a.K / 512) % S != 0);
        }
    }
    const size_t need = solo_ws_bytes(a.M, a.N, S);
    if (a.query) return *a.query = need, LQ_OK;
    if (need > 0 && (!a.ws || a.ws_bytes < need))
        return fail(LQ_ERR_WORKSPACE, "%d K slices need %zu bytes of workspace, got %zu", S, need, a.ws ? a.ws_bytes : 0);
    int32_t *partials = S > 1 ? reinterpret_cast<int32_t *>(static_cast<char *>(a.ws) + kTicketBytes) : nullptr;
    const int grid = std::min(blocks_m * blocks_n * S, cus);
    const size_t lds_bytes = 4 * (size_t)256 * 128 + 4 * 1024;  // X stages; two copies of both scales
    __half *Y = S > 1 ? nullptr : a.Y;
    int32_t *ACC = S > 1 ? partials : a.ACC;
    if constexpr (SHAPE16) {
        if (a.group == 128) {
            if (int rc = allow_lds(w4a8_solo16_pt_kernel<true, KG>, lds_bytes)) return rc;
            hipLaunchKernelGGL((w4a8_solo16_pt_kernel<true, KG>), dim3((unsigned)grid), dim3(256), lds_bytes, a.stream, a.M,
                               a.N, a.K, a.X, a.sx, a.Wp, a.gp, a.sw, Y, ACC, blocks_m, blocks_n, S);
        } else {
            if (int rc = allow_lds(w4a8_solo16_pt_kernel<false, KG>, lds_bytes)) return rc;
            hipLaunchKernelGGL((w4a8_solo16_pt_kernel<false, KG>), dim3((unsigned)grid), dim3(256), lds_bytes, a.stream, a.M,
                               a.N, a.K, a.X, a.sx, a.Wp, a.gp, a.sw, Y, ACC, blocks_m, blocks_n, S);
        }
    } else if (a.group == 128) {
        if (int rc = allow_lds(w4a8_solo_pt_kernel<true, KG>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_solo_pt_kernel<true, KG>), dim3((unsigned)grid), dim3(256), lds_bytes, a.stream, a.M,
                           a.N, a.K, a.X, a.sx, a.Wp, a.gp, a.sw, Y, ACC, blocks_m, blocks_n, S);
    } else {
        if (int rc = allow_lds(w4a8_solo_pt_kernel<false, KG>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_solo_pt_kernel<false, KG>), dim3((unsigned)grid), dim3(256), lds_bytes, a.stream, a.M,
                           a.N, a.K, a.X, a.sx, a.Wp, a.gp, a.sw, Y, ACC, blocks_m, blocks_n, S);
    }
    if (S > 1) {
        const size_t quads = (size_t)a.M * a.N / 4;
        hipLaunchKernelGGL(splitk_finish_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, a.stream, partials,
                           S, a.M, a.N, a.sx, a.sw, a.Y, a.ACC);
    }
    return LQ_OK;
}

// the explicit producer / consumer form (measured only, never dispatched)
static int launch_excp(const Args &a)
{
    if (a.query) return LQ_OK;  // no workspace
    const int blocks_n = (a.N + 255) / 256, blocks_m = (a.M + 127) / 128;
    if ((long long)a.M * a.K >= (1ll << 32))
        return fail(LQ_ERR_INVALID, "M * K = %lld is beyond the 2^32 - 1 bytes of X one call addresses; split the batch",
                    (long long)a.M * a.K);
    const size_t lds_bytes = 2 * (size_t)128 * kTilePitch + 2 * (size_t)32 * 1024;
    const dim3 grid((unsigned)(blocks_n * blocks_m)), block(512);
    if (a.group == 128) {
        if (int rc = allow_lds(w4a8_excp_kernel<true>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_excp_kernel<true>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K, a.X, a.sx, a.Wp,
                           a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n);
    } else {
        if (int rc = allow_lds(w4a8_excp_kernel<false>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_excp_kernel<false>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K, a.X, a.sx, a.Wp,
                           a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n);
    }
    return LQ_OK;
}

// The tiled kernel with the overflow-safe widened dequantisation in place of LiquidQuant's
// (the dequantisation half of the paper's ablation, Sec. 7.3; measured only, never dispatched).
static int launch_duo_widened(const Args &a)
{
    if (a.query) return LQ_OK;  // no workspace
    const int blocks_n = (a.N + 255) / 256, blocks_m = (a.M + 127) / 128;
    const size_t lds_bytes = 2 * (size_t)128 * kTilePitch;
    const dim3 grid((unsigned)(blocks_n * blocks_m), 1u), block(256);
    if (a.group == 128)
        hipLaunchKernelGGL((w4a8_duo_kernel<true, 1, 128, false, 1>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n, nullptr, nullptr);
    else
        hipLaunchKernelGGL((w4a8_duo_kernel<false, 1, 128, false, 1>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n, nullptr, nullptr);
    return LQ_OK;
}

// The same kernel on a grid of 64-row tiles (two row fragments per wave, two k groups per
// block): twice the tiles for a given M, half the partial-tile volume per slice.
static int duo64_split(int M, int N, int K)
{
    const int tiles = ((M + 63) / 64) * ((N + 255) / 256);
    const int units = K / 256;
    int s = (int)(0.6 * std::sqrt((double)units) + 0.5);  // minimum of the fitted cost below
    // with few tiles the exchange of a slice is cheap (few blocks share the memory system)
    s = std::max(s, tiles <= 40 ? 4 : tiles <= 64 ? 3 : 1);
    s = std::min(std::min(s, 256 / std::max(1, tiles)), std::min(units / 2, 8));
    return std::max(1, s);
}
template <int SPLIT>
static int launch_duo64(const Args &a)
{
    if (a.K < 512) return fail(LQ_ERR_INVALID, "the 64-row tiled variant needs K >= 512");
    return launch_duo_as<SPLIT, 2, 64>(a, SPLIT ? SPLIT : duo64_split(a.M, a.N, a.K));
}

// Which tile height for a problem with few tiles.  Fitted to measurements of both forms with
// two k groups per block (microseconds; u = 256-k units per k group, S = K slices):
//   128-row tiles: 13.9 + 1.95 u + 2.3 (S - 1)       64-row tiles: 8.1 + 1.76 u + c (S - 1),
//   c = 0.8 + 1.6 * blocks / 256 (a slice costs less when few blocks exchange at once)
static bool prefer_64_row_tiles(int M, int N, int K)
{
    const int bn = (N + 255) / 256;
    const int t128 = ((M + 127) / 128) * bn, t64 = ((M + 63) / 64) * bn, units = K / 256;
    if (K < 512 || t64 > 256 || t128 > 256) return false;
    const int s128 = duo_split(M, N, K), s64 = duo64_split(M, N, K);
    const double est128 = 13.9 + 1.95 * units / (2.0 * s128) + 2.3 * (s128 - 1);
    const double est64 = 8.1 + 1.76 * units / (2.0 * s64) + (0.8 + 1.6 * t64 * s64 / 256.0) * (s64 - 1);
    return est64 < est128;
}

struct Variant {
    const char *name;
    LaunchFn fn;
    int max_m;      // 0 = unlimited
    int tiles_div;  // N/32 must be a multiple of this
    int chunks_div; // K/64 must be a multiple of this
    int min_k = 256;
};

// stream*_f<F>_w<NW>[_s<S>]: F tiles per block, NW waves splitting the block's K slice,
// S grid-level K slices (chosen from the shape when not named); _u4 = four 128-k units per
// pipeline step; x = X fragments through LDS; g2 = two k groups per block.
static const Variant kVariants[] = {
    // --- dispatched (select_variant) ---
    {"stream16_f1_w16_s1", &launch_stream16<1, 16, 1>, 16, 1, 1},
    {"stream16_f1_w8_u4", &launch_stream16<1, 8, 0, 4>, 16, 1, 8},
    {"stream16_f1_w8", &launch_stream16<1, 8, 0>, 16, 1, 1},
    {"stream16_f2_w8", &launch_stream16<2, 8, 0>, 16, 2, 1},
    {"stream16_f2_w16_s1", &launch_stream16<2, 16, 1>, 16, 2, 1},
    {"stream16_f2_w4", &launch_stream16<2, 4, 0>, 16, 2, 1},
    {"stream_m32", &launch_stream_auto<1>, 32, 2, 1},
    {"stream_m64", &launch_stream_auto<2>, 64, 2, 1},
    {"duo_m64", &launch_duo64<0>, 0, 1, 1, 512},
    {"duo_m128", &launch_duo<0, 0>, 0, 1, 1},
    {"duo_dl_m128", &launch_duo_dl<0>, 0, 1, 1},
    {"duo_pt_m128", &launch_duo_pt, 0, 1, 8, 512},
    {"solo16_pt_m256", &launch_solo_pt<1, 0, true>, 0, 1, 4},
    {"solo16_g2_m256", &launch_solo_pt<2, 0, true>, 0, 1, 4},
    {"solo16_g2_sk_m256", &launch_solo_pt<2, -1, true>, 0, 1, 8, 512},
    // --- the 256-row tile kernels on the 32x32x32 MFMA (what the 16x16x64 forms are measured against) ---
    {"solo_pt_m256", &launch_solo_pt<1>, 0, 1, 8, 512},
    {"solo_g2_m256", &launch_solo_pt<2>, 0, 1, 8, 512},
    // --- the same kernels with a named number of K slices: the split paths at sizes where the
    //     dispatcher would not split (parity tests) ---
    {"stream16_f2_w8_s2", &launch_stream16<2, 8, 2>, 16, 2, 1},
    {"stream16_f1_w8_u4_s2", &launch_stream16<1, 8, 2, 4>, 16, 1, 8},
    {"stream_f2_w8_s2", &launch_stream<2, 8, 2>, 32, 2, 1},
    {"stream_x_f1_w8_s2", &launch_stream<1, 8, 2, 1, true>, 32, 1, 1},
    {"stream_m64x_f1_w8_s2", &launch_stream<1, 8, 2, 2, true>, 64, 1, 1},
    {"stream_m64x_f2_w8_s4", &launch_stream<2, 8, 4, 2, true>, 64, 2, 1},
    {"duo_m64_s2", &launch_duo64<2>, 0, 1, 1, 512},
    {"duo_m128_s1", &launch_duo<1, 1>, 0, 1, 1},
    {"duo_m128_s2", &launch_duo<2, 1>, 0, 1, 1},
    {"duo_m128_g2_s2", &launch_duo<2, 2>, 0, 1, 1},
    {"duo_dl_m128_s2", &launch_duo_dl<2>, 0, 1, 1},
    {"solo16_pt_m256_s2", &launch_solo_pt<1, 2, true>, 256, 1, 16, 1024},
    {"solo16_g2_m256_s4", &launch_solo_pt<2, 4, true>, 256, 1, 32, 2048},
    // --- ablation forms (Sec. 7.3), measured by the benchmark, never dispatched ---
    {"excp_m128", &launch_excp, 0, 1, 1},
    {"widened_dq_m128", &launch_duo_widened, 0, 1, 1},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

static bool variant_supports(int v, int M, int N, int K)
{
    const Variant &x = kVariants[v];
    return (x.max_m == 0 || M <= x.max_m) && (N / 32) % x.tiles_div == 0 && (K / 64) % x.chunks_div == 0 &&
           K >= x.min_k;
}

static int find_variant(const char *name)
{
    for (int i = 0; i < kNumVariants; ++i)
        if (!strcmp(kVariants[i].name, name)) return i;
    return -1;
}

// The 256-row tiles with one wave per SIMD (solo16_pt_m256: 256 x 256; solo16_g2_m256: 256 x 128
// with two k groups per block) against the 128 x 256 tiles with two waves per SIMD.  Half the
// dequantisation per MFMA makes their stage loop shorter -- per 128 x 256 of output and 1024 k,
// 6.0 us (256 x 256) and 7.0 us (256 x 128) against 7.1 to 7.4 us measured on N = K = 8192 --
// but they run one block per CU, in whole rounds, and rows past M in a 256-row tile are lost.
// Costs in units of one 128 x 256 tile's time on a CU, from the numbers of tiles of each form;
// returns 1 for 256 x 256, 2 for 256 x 128, 0 for neither.
struct TiledCosts {
    double duo, solo, g2;
    double best() const { return std::min(duo, std::min(solo, g2)); }
};
// (pt_ok: the persistent form of the 128-row tiles can run the shape)
static TiledCosts tiled_costs(long long t128, long long t256, long long t2, int K, bool pt_ok)
{
    // (K % 512 == 256: the 16x16x64 forms of the 256-row tiles run two added stages of zero weights,
    // the persistent form of the 128-row tiles does not take the shape -- pt_ok is false then)
    // No form's cost is proportional to its tiles while these leave CUs idle or half occupied (a
    // partly filled chip clocks higher).  Fitted to measurements on K = 8192 (us / 64, so that a
    // round of 256 128-row tiles, one per CU, costs about 1):
    //   128-row tiles, K slices across blocks up to 128 tiles:  29.6 / 38.7 / 44 us at 64 / 96 / 128
    //   ... 129..256 tiles, persistent form (one block per CU): 50.6 / 57.3 / 63.5 at 160 / 192 / 256
    //       (one tile per block: 56 / 60 / 67)
    //   ... 257..512 tiles (a second resident block on some CUs): 85 / 95 / 102 / 111 / 116 at 270 / 320 / 384 / 448 / 512
    //   ... beyond: whole rounds of 512 at 2 each, the rest as above
    //   256 x 256 tiles, one round: 84 / 93 / 107 at 160 / 192 / 256 tiles; more: whole rounds at 2 * 0.86
    //   256 x 128 tiles, one round of more than half the CUs: 45.8 / 49 / 56 / 61.5 at 144 / 160 / 192 / 256
    //       (at 128 tiles equal to the 128-row tiles; their tiles are separate, a second round costs a tenth more)
    // one round of up to 512 tiles (or the rest after whole rounds of 512: 4096 + 40 rows on 8192 x 8192,
    // 1056 tiles, took 259 us against 235 us of 4096 rows)
    auto part = [](long long t) {
        const double fill = (double)t / kAssumedCUs;
        return t == 0 ? 0.0 : 2 * t <= kAssumedCUs ? 0.24 + 0.90 * fill : t <= kAssumedCUs ? 0.47 + 0.52 * fill : 0.80 + 0.51 * fill;
    };
    const double fill = (double)t128 / kAssumedCUs;
    const double duo = t128 <= kAssumedCUs && 2 * t128 > kAssumedCUs && !pt_ok
                           ? 0.60 + 0.45 * fill
                           : 2.0 * (t128 / (2 * kAssumedCUs)) + part(t128 % (2 * kAssumedCUs));
    const double short_k = K >= 4096 ? 1.0 : 1.06;  // (their longer epilogue weighs more)
    // (those were measured with the 32x32x32 MFMA; on the 16x16x64 one the 256 x 256 tiles take 8 % less)
    const double solo = (t256 <= kAssumedCUs ? 0.734 + 0.94 * t256 / kAssumedCUs
                                             : 2.0 * ((t256 + kAssumedCUs - 1) / kAssumedCUs) * 0.86) * short_k * 0.92;
    // (... and the 256 x 128 tiles 1 to 5 % less, most on a full round: 57.4 against 60.4 us at 256 tiles,
    // 48.8 against 50.5 at 192, 28.3 against 28.5 at 172 tiles with K = 4096)
    const double g2 = 16 * t2 > 8.5 * kAssumedCUs && t2 <= kAssumedCUs
                          ? (0.406 + 0.56 * t2 / kAssumedCUs) * short_k * (1.0 - 0.05 * t2 / kAssumedCUs)
                          : 1e30;
    return TiledCosts{duo, solo, g2};
}
static TiledCosts tiled_costs(int M, int N, int K)
{
    const long long bm256 = (M + 255) / 256;
    return tiled_costs((long long)((M + 127) / 128) * ((N + 255) / 256), bm256 * ((N + 255) / 256),
                       bm256 * ((N + 127) / 128), K, K % 512 == 0);
}
static int solo_form_of(const TiledCosts &c)
{
    if (c.solo < c.duo && c.solo <= c.g2) return 1;
    if (c.g2 < c.duo) return 2;
    return 0;
}
static int solo_form_for(long long t128, long long t256, long long t2, int K)
{
    return solo_form_of(tiled_costs(t128, t256, t2, K, false));
}
static int solo_form_that_pays(int M, int N, int K) { return solo_form_of(tiled_costs(M, N, K)); }

// Shape -> kernel.  Up to 32 rows the weights are streamed once with X fragments in
// registers (16-row MFMA shape up to 16 rows); anything larger runs the 128 x 256 tiles of
// the duo kernel, whose launcher adds in-block and grid-level split-K while the output
// alone gives at most one tile per CU.
static int select_variant(int M, int N, int K)
{
    if (M <= 16) {
        // Measured over 36 weight shapes (N, K from 2048 to 28672) at 1, 8 and 16 rows.
        const int tiles = N / 32;
        if (tiles <= 256) {
            // one tile per block.  Short K is bound by launch and first-load latency: sixteen
            // waves per block take one or two units of 128 k each ...
            if (K <= 4096) return find_variant("stream16_f1_w16_s1");
            if (K <= 8192 && K % 512 == 0) {
                // ... up to 8192, all of a wave's loads (512 k) in flight at once; from 9 rows
                // K slices across blocks while N leaves room for them, else sixteen waves again
                if (M <= 8) return find_variant("stream16_f1_w8_u4");
                return find_variant(tiles <= 128 ? "stream16_f1_w8" : "stream16_f1_w16_s1");
            }
            // 129..256 tiles and long K (no room for K slices across blocks): up to 8 rows, sixteen
            // waves per block split K (21.5 instead of 26 us on 8192 x 28672, 12.4 / 17.8 on
            // 6144 x 16384); above, two tiles per block and two K slices (23.3 / 25.9, 14.8 / 15.7)
            if (tiles > 128 && M <= 8 && K >= 12288) return find_variant("stream16_f1_w16_s1");
            if (tiles > 128 && M > 8 && K >= 16384) return find_variant("stream16_f2_w8");
            // otherwise 2 or 4 K slices across blocks
            return find_variant("stream16_f1_w8");
        }
        // up to 512 tiles with short K: sixteen waves again (8.1 instead of 9.1 us on 16384 x 4096)
        if (tiles <= 512 && K <= 4096) return find_variant(M <= 8 ? "stream16_f1_w16_s1" : "stream16_f2_w16_s1");
        if (N / 64 >= 384) return find_variant(K <= 2048 ? "stream16_f2_w8" : "stream16_f2_w4");
        return find_variant("stream16_f2_w8");
    }
    if (M <= 32) return find_variant("stream_m32");
    // up to 64 rows the weights are still best streamed once per block column (X through LDS)
    // unless N alone fills the chip with 128 x 256 tiles
    // (except 129..256 tiles with very long K from 48 rows on: no room for K slices across blocks,
    // and the tiles' split-K grid is 8-16 % ahead, 32.8 against 38.1 us at 64 rows on 6144 x 28672)
    if (M <= 64 && N / 32 <= 512 && !(M >= 48 && N / 32 > 128 && N / 32 <= 256 && K >= 24576))
        return find_variant("stream_m64");
    // 256-row tiles with one wave per SIMD where their whole rounds come out ahead
    if (const int form = solo_form_that_pays(M, N, K)) return find_variant(form == 1 ? "solo16_pt_m256" : "solo16_g2_m256");
    // ... and, with very long K and row tiles that are nearly full, their 256 x 128 form with K
    // slices across blocks where tiles x slices come to one round of at least three quarters of the
    // CUs (256 x 8192 x 28672: 65 against 70 us; 512 rows: 114 against 121; 256 x 6144 x 16384: 37
    // against 40; shorter K or emptier rounds: equal or behind -- the partial sums are a matrix per slice)
    if (K >= 16384 && K % 512 == 0 && (M % 256 == 0 || M % 256 > 192)) {
        const long long t2 = (long long)((M + 255) / 256) * ((N + 127) / 128);
        if (t2 <= kAssumedCUs / 2) {
            const int slices = solo_split((int)t2, K, (int)kAssumedCUs);
            if (slices > 1 && 4 * t2 * slices >= 3 * kAssumedCUs) return find_variant("solo16_g2_sk_m256");
        }
    }
    // more 128 x 256 tiles than CUs (blocks of one k group): the deeper memory pipeline of the
    // direct-to-LDS form pays (3 to 6 % measured from 320 tiles up, 1 to 5 % at 264..288); with
    // one tile per CU or fewer, the two k groups per block of the other form do
    // (from two tiles per resident slot on and with whole 512-k units, its persistent form:
    // one pipeline fill per block instead of per tile, 1 to 2 % measured)
    const int tiles128 = ((M + 127) / 128) * ((N + 255) / 256);
    if (tiles128 > 256) return find_variant(duo_pt_fits(M, N, K) ? "duo_pt_m128" : "duo_dl_m128");
    // more than half a round of them (no room for K slices across blocks): the persistent form again,
    // one block per CU -- 50.6 against 56.1 us on 640 x 8192 x 8192, 28.0 against 31.1 on 384 x 11008 x 4096
    // (also with a ragged last row tile of at most 64 rows: 47.8 against 50.9 us on 576 x 8192 x 8192)
    if (tiles128 > 128 && K % 512 == 0) return find_variant("duo_pt_m128");
    // few tiles: a grid of 64-row tiles can fill the chip with half the split-K exchange
    return find_variant(prefer_64_row_tiles(M, N, K) ? "duo_m64" : "duo_m128");
}

// A batch whose 256 x 256 tiles are whole rounds plus a few rows (4096 + 40 rows on 8192 x 8192)
// is better run as two launches over consecutive rows: the row blocks that fill whole rounds with
// the 256 x 256 tiles, and the rest with whatever the dispatcher picks for it -- 226 us against
// 259 us of the best single kernel there.  Also with a larger rest, unless the rest would run on
// 256 x 256 tiles itself (then the one persistent launch over all tiles is 1 to 5 % ahead of two):
// 1536 + 512 rows on the 70B qkv projection 143 against 150 us, 2048 + 1024 on 8192 x 8192 157
// against 162, 1024 + 256 on 28672 x 8192 240 against 255, 2048 + 512 on 8192 x 8192 143 against
// 156 and on 8192 x 28672 423 against 513, 3072 + 512 on 5120 x 13824 201 against 245, 4096 + 1024
// on 4096 x 4096 78 against 84 (4096 + 1904 on 4096 x 4096 and 4096 + 1024 on 8192 x 8192: equal).
// Same cost units as solo_form_for; a second launch is charged 5 us
// (2048 + 100 rows on 8192 x 4096: 55.7 + 16.2 us against 78.4 us of the best single kernel; 1024 + 30 rows on
// 16384 x 4096: 56 + 11.3 against 79.7).  Returns
// the rows of the first piece (M if the batch stays whole).
static int rows_of_first_launch(int M, int N, int K)
{
    if (M <= 256) return M;
    const int bm = (M + 255) / 256, bn = (N + 255) / 256;
    double best = tiled_costs(M, N, K).best() * 0.97;  // (a split has to win by 3 %)
    const double second_launch = 5.0 / (8.0 * K / 1024.0);  // (a unit is 64 us at K = 8192)
    const double short_k = K >= 4096 ? 1.0 : 1.06;
    int rows = M;
    for (int rounds = 1; rounds <= 8; ++rounds) {
        const int rb = (int)(kAssumedCUs * rounds / bn);  // row blocks whose tiles fill `rounds` rounds
        if (rb >= bm) break;
        if (rb < 1) continue;
        const TiledCosts rest = tiled_costs(M - 256 * rb, N, K);
        // (a larger rest not where it would be 256 x 256 tiles again: the one persistent launch
        // over all of them is 1 to 5 % ahead of two)
        if (M - 256 * rb > 256 && solo_form_of(rest) == 1) continue;
        const double c = rounds * 2.0 * 0.86 * 0.92 * short_k + rest.best() + second_launch;
        if (c < best) best = c, rows = 256 * rb;
    }
    return rows;
}

static int check_device_args(const Args &a)
{
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

static int run_rows(int variant, const Args &a)
{
    if (variant < 0) variant = select_variant(a.M, a.N, a.K);
    if (variant < 0 || variant >= kNumVariants) return fail(LQ_ERR_INVALID, "unknown variant %d", variant);
    if (!variant_supports(variant, a.M, a.N, a.K))
        return fail(LQ_ERR_INVALID, "variant %s cannot run M=%d N=%d K=%d", kVariants[variant].name, a.M, a.N,
                    a.K);
    (void)hipGetLastError();
    // The tiled kernels address X with 32-bit byte offsets.  A batch with M * K >= 2^32 is
    // run as consecutive row chunks (multiples of 256 rows, so every chunk keeps the
    // alignment and the tile grid of a call of its own) on the same stream; rows are
    // independent, so the result is that of one launch.
    const long long rows_max = ((1ll << 32) - 1) / a.K / 256 * 256;
    size_t need_max = 0;
    for (long long r0 = 0; r0 < a.M; r0 += rows_max) {
        Args c = a;
        size_t need = 0;
        if (a.query) c.query = &need;
        c.M = (int)std::min<long long>(rows_max, a.M - r0);
        c.X = a.X + r0 * a.K;
        if (a.sx) c.sx = a.sx + r0;
        if (a.Y) c.Y = a.Y + r0 * a.N;
        if (a.ACC) c.ACC = a.ACC + r0 * a.N;
        if (int rc = kVariants[variant].fn(c)) return rc;
        need_max = std::max(need_max, need);
    }
    if (a.query) return *a.query = need_max, LQ_OK;
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(LQ_ERR_HIP, "launch of %s failed: %s", kVariants[variant].name, hipGetErrorString(e));
    return LQ_OK;
}

static int run(int variant, const Args &a)
{
    if (int rc = check_device_args(a)) return rc;
    if (a.M == 0) return LQ_OK;
    const int first = variant < 0 ? rows_of_first_launch(a.M, a.N, a.K) : a.M;
    if (first == a.M) return run_rows(variant, a);
    // two launches on the same stream (rows are independent); a workspace serves both in turn
    Args head = a, rest = a;
    size_t need_head = 0, need_rest = 0;
    if (a.query) head.query = &need_head, rest.query = &need_rest;
    head.M = first;
    rest.M = a.M - first;
    rest.X = a.X + (size_t)first * a.K;
    if (a.sx) rest.sx = a.sx + first;
    if (a.Y) rest.Y = a.Y + (size_t)first * a.N;
    if (a.ACC) rest.ACC = a.ACC + (size_t)first * a.N;
    if (int rc = run_rows(find_variant("solo16_pt_m256"), head)) return rc;
    if (int rc = run_rows(-1, rest)) return rc;
    if (a.query) *a.query = std::max(need_head, need_rest);
    return LQ_OK;
}

// ------------------------------------------------------------------------------------
// Grouped GEMM: experts are sorted by their number of rows into the three kernel families
// (<= 16 rows: 16-row stream kernel, <= 32: 32-row stream kernel, more: 128 x 256 tiles),
// and each family that is not empty gets one launch over all of its experts.
// ------------------------------------------------------------------------------------
struct GroupedArgs {
    int E, N, K, group;
    const int *row_offsets;  // host, E + 1
    GroupedPtrs p;
    hipStream_t stream;
};

template <class Kernel, class... A>
static int launch_checked(const char *what, Kernel kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st,
                          A... args)
{
    if (int rc = allow_lds(kernel, lds)) return rc;
    (void)hipGetLastError();
    hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LQ_ERR_HIP, "launch of %s failed: %s", what, hipGetErrorString(e));
    return LQ_OK;
}

// The experts of more than 32 rows (or row ranges of them) as 128- or 64-row tiles: one launch.
static int grouped_tiles_run(const GroupedArgs &a, GroupTable &big)
{
    const bool g128 = a.group == 128;
    const int blocks_n = (a.N + 255) / 256;
    long long big_blocks = 0, big_blocks64 = 0;
    for (int i = 0; i < big.count; ++i) {
        big_blocks += (long long)((big.rows[i] + 127) / 128) * blocks_n;
        big_blocks64 += (long long)((big.rows[i] + 63) / 64) * blocks_n;
        if (big_blocks > 0x7fffffff) return fail(LQ_ERR_INVALID, "grouped GEMM too large for one launch");
        big.block_end[i] = (int)big_blocks;
    }
    if (big_blocks64 <= 256 && big_blocks64 > big_blocks && a.K >= 512) {
        // few blocks and experts of more than 64 rows: a grid of 64-row tiles has up to twice the
        // blocks, still at most one per CU (8 experts of 72 rows on 4096 x 14336: 128 -> 256 blocks)
        long long end = 0;
        for (int i = 0; i < big.count; ++i) {
            end += (long long)((big.rows[i] + 63) / 64) * blocks_n;
            big.block_end[i] = (int)end;
        }
        const dim3 grid((unsigned)big_blocks64);
        const size_t lds2 = std::max<size_t>(4 * (size_t)128 * kTilePitch, 64 * 1024);
        return g128 ? launch_checked("grouped duo", w4a8_duo_grouped_kernel<true, 2, 64>, grid, dim3(512), lds2, a.stream,
                                     big, a.p, a.N, a.K)
                    : launch_checked("grouped duo", w4a8_duo_grouped_kernel<false, 2, 64>, grid, dim3(512), lds2, a.stream,
                                     big, a.p, a.N, a.K);
    }
    const dim3 grid((unsigned)big_blocks);
    // as for single GEMMs: two k groups per block while the grid gives at most one block per CU
    const bool kg2 = big_blocks <= 256 && a.K >= 512;
    const size_t lds1 = 2 * (size_t)128 * kTilePitch;
    const size_t lds2 = std::max<size_t>(2 * lds1, 64 * 1024);
    // more blocks than CUs: the direct-to-LDS form, as for single GEMMs (its X offsets have 32
    // bits) -- unless the experts are so small that most tiles have two row fragments, which
    // the other form runs with a deeper W pipeline (8 experts of 58..71 rows: 63 against 67 us;
    // of 128 rows: 91 against 79; of about 1000: 531 against 513)
    bool dl = !kg2 && a.K >= 512;
    long long big_rows = 0;
    for (int i = 0; i < big.count; ++i) {
        dl = dl && (long long)big.rows[i] * a.K < (1ll << 32);
        big_rows += big.rows[i];
    }
    dl = dl && big_rows > 96ll * big.count;
    if (dl)
        return g128 ? launch_checked("grouped duo", w4a8_duo_dl_grouped_kernel<true>, grid, dim3(256),
                                     4 * (size_t)128 * 128, a.stream, big, a.p, a.N, a.K)
                    : launch_checked("grouped duo", w4a8_duo_dl_grouped_kernel<false>, grid, dim3(256),
                                     4 * (size_t)128 * 128, a.stream, big, a.p, a.N, a.K);
    if (kg2)
        return g128 ? launch_checked("grouped duo", w4a8_duo_grouped_kernel<true, 2>, grid, dim3(512), lds2, a.stream, big,
                                     a.p, a.N, a.K)
                    : launch_checked("grouped duo", w4a8_duo_grouped_kernel<false, 2>, grid, dim3(512), lds2, a.stream, big,
                                     a.p, a.N, a.K);
    return g128 ? launch_checked("grouped duo", w4a8_duo_grouped_kernel<true, 1>, grid, dim3(256), lds1, a.stream, big,
                                 a.p, a.N, a.K)
                : launch_checked("grouped duo", w4a8_duo_grouped_kernel<false, 1>, grid, dim3(256), lds1, a.stream, big,
                                 a.p, a.N, a.K);
}

static int grouped_run(const GroupedArgs &a)
{
    GroupTable small{}, mid{}, big{};
    for (int e = 0; e < a.E; ++e) {
        const int r0 = a.row_offsets[e], rows = a.row_offsets[e + 1] - r0;
        if (rows == 0) continue;
        GroupTable &t = rows <= 16 ? small : (rows <= 32 ? mid : big);
        const int i = t.count++;
        t.expert[i] = e, t.row_off[i] = r0, t.rows[i] = rows;
    }
    const bool g128 = a.group == 128;
    const int groups = a.N / 64;  // stream kernels: two tiles of 32 channels per block
    if (small.count) {
        const dim3 grid((unsigned)(small.count * groups));
        // four waves per block once the grid alone gives every CU several blocks
        const bool w4 = (long long)small.count * groups >= 384 * 2;
        const size_t lds = (size_t)(w4 ? 4 : 8) * 2 * 8 * 64 * sizeof(int);
        int rc;
        if (w4)
            rc = g128 ? launch_checked("grouped stream16", w4a8_stream16_grouped_kernel<4, 1, true>, grid, dim3(256),
                                       lds, a.stream, small, a.p, a.N, a.K, groups)
                      : launch_checked("grouped stream16", w4a8_stream16_grouped_kernel<4, 1, false>, grid, dim3(256),
                                       lds, a.stream, small, a.p, a.N, a.K, groups);
        else
            rc = g128 ? launch_checked("grouped stream16", w4a8_stream16_grouped_kernel<8, 1, true>, grid, dim3(512),
                                       lds, a.stream, small, a.p, a.N, a.K, groups)
                      : launch_checked("grouped stream16", w4a8_stream16_grouped_kernel<8, 1, false>, grid, dim3(512),
                                       lds, a.stream, small, a.p, a.N, a.K, groups);
        if (rc) return rc;
    }
    if (mid.count) {
        const dim3 grid((unsigned)(mid.count * groups));
        const size_t lds = (size_t)8 * 2 * 16 * 64 * sizeof(int);
        const int rc = g128 ? launch_checked("grouped stream", w4a8_stream_grouped_kernel<8, true>, grid, dim3(512), lds,
                                             a.stream, mid, a.p, a.N, a.K, groups)
                            : launch_checked("grouped stream", w4a8_stream_grouped_kernel<8, false>, grid, dim3(512),
                                             lds, a.stream, mid, a.p, a.N, a.K, groups);
        if (rc) return rc;
    }
    if (!big.count) return LQ_OK;
    // The larger experts: whole 256-row blocks of them (and a last block of more than 128 rows) as
    // 256 x 256 tiles of the one-wave-per-SIMD kernel, one persistent launch over all experts, where
    // those tiles pay; what is left of each expert (at most 128 rows) and everything else as 128- or
    // 64-row tiles in a launch of their own.
    const int blocks_n = (a.N + 255) / 256;
    GroupTable main{}, rest{};
    long long main_t128 = 0, main_t256 = 0;
    bool fits = a.N <= (1 << 26);
    for (int i = 0; i < big.count; ++i) {
        const int rows = big.rows[i], tail = rows % 256;
        const int rows_rest = tail > 0 && tail <= 128 ? tail : 0, rows_main = rows - rows_rest;
        fits = fits && (long long)rows * a.K < (1ll << 32);
        if (rows_main) {
            const int k = main.count++;
            main.expert[k] = big.expert[i], main.row_off[k] = big.row_off[i], main.rows[k] = rows_main;
            main_t128 += (long long)((rows_main + 127) / 128) * blocks_n;
            main_t256 += (long long)((rows_main + 255) / 256) * blocks_n;
            if (main_t256 > 0x7fffffff) return fail(LQ_ERR_INVALID, "grouped GEMM too large for one launch");
            main.block_end[k] = (int)main_t256;
        }
        if (rows_rest) {
            const int k = rest.count++;
            rest.expert[k] = big.expert[i], rest.row_off[k] = big.row_off[i] + rows_main, rest.rows[k] = rows_rest;
        }
    }
    if (main.count && fits && solo_form_for(main_t128, main_t256, 0, a.K) == 1) {
        const int cus = cu_count();
        const dim3 grid((unsigned)std::min<long long>(main_t256, std::max(cus, 1)));
        const size_t lds = 4 * (size_t)256 * 128 + 4 * 1024;
        const int rc = g128 ? launch_checked("grouped solo", w4a8_solo_grouped_kernel<true>, grid, dim3(256), lds,
                                             a.stream, main, a.p, a.N, a.K)
                            : launch_checked("grouped solo", w4a8_solo_grouped_kernel<false>, grid, dim3(256), lds,
                                             a.stream, main, a.p, a.N, a.K);
        if (rc) return rc;
        return rest.count ? grouped_tiles_run(a, rest) : LQ_OK;
    }
    return grouped_tiles_run(a, big);
}

// ------------------------------------------------------------------------------------
// Built-in split-K workspace for callers that cannot allocate (w4a8_gemm_static): tickets
// followed by partial tiles, laid out exactly like a caller's workspace.  Zero when the code
// object is loaded; the kernels leave the tickets zero after every call.  The array's name
// is only a host-side handle: its address on the current device comes from the runtime.
// ------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = kTicketBytes + ((size_t)32 << 20);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;

static int static_scratch_ptr(void **out)
{
    static std::mutex mu;
    static void *addr[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(LQ_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(LQ_ERR_INVALID, "device %d out of range", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(LQ_ERR_HIP, "hipGetSymbolAddress(built-in workspace): %s", hipGetErrorString(e));
        addr[dev] = p;
    }
    *out = addr[dev];
    return LQ_OK;
}

}  // namespace lqq

using namespace lqq;

extern "C" {

size_t w4a8_gemm_workspace_size(int M, int N, int K, int group)
{
    if (M <= 0 || !shape_ok(N, K, group)) return 0;
    // Enough for any variant that can run the shape.  Tiled kernels split K only while the
    // output has fewer tiles than CUs (at most 8 slices); stream kernels take at most 16
    // slices (the 16-row kernels always exchange 8 values per lane and tile).
    const int tiles = ((M + 127) / 128) * ((N + 255) / 256);
    size_t need = tiles >= 192 ? 0 : std::max(duo_ws_bytes(M, N, 8), duo_ws_bytes(M, N, 8, 64));
    if (M <= 32) need = std::max(need, stream_ws_bytes(M, N, 16));
    if (M <= 64) need = std::max(need, stream_ws_bytes(M, N, 16, 2));
    if (M <= 16) need = std::max(need, kTicketBytes + (size_t)16 * (N / 32) * 8 * 64 * sizeof(int32_t));
    if (K % 512 == 0) {
        // the 256-row tiles with K slices: a whole INT32 matrix per slice, at most one round of blocks
        // (up to 256 rows also the variants with a named number of slices)
        const long long t256 = (long long)((M + 255) / 256) * ((N + 255) / 256);
        const int s = M <= 256 ? 4 : (int)std::min<long long>(4, kAssumedCUs / t256);
        need = std::max(need, solo_ws_bytes(M, N, s));
    }
    return need;
}

int w4a8_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!workspace || workspace_bytes == 0) return LQ_OK;
    if ((uintptr_t)workspace & 15) return fail(LQ_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const int n = (int)(std::min(workspace_bytes, kTicketBytes) / sizeof(unsigned int));
    if (n == 0) return LQ_OK;
    (void)hipGetLastError();
    hipLaunchKernelGGL(workspace_init_kernel, dim3((n + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<unsigned int *>(workspace), n);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LQ_ERR_HIP, "workspace init launch failed: %s", hipGetErrorString(e));
    return LQ_OK;
}

int w4a8_gemm(int M, int N, int K, int group, const int8_t *X, const float *act_scales,
              const void *W_packed, const uint8_t *gparams, const float *w_scales, uint16_t *Y,
              void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!Y && M != 0) return fail(LQ_ERR_INVALID, "null Y");
    const Args a{M, N, K, group, X, act_scales, static_cast<const u32x4 *>(W_packed), gparams, w_scales,
                 reinterpret_cast<__half *>(Y), nullptr, static_cast<hipStream_t>(hip_stream), workspace, workspace_bytes};
    return run(-1, a);
}

int w4a8_gemm_static(int M, int N, int K, int group, const int8_t *X, const float *act_scales,
                     const void *W_packed, const uint8_t *gparams, const float *w_scales, uint16_t *Y,
                     void *hip_stream)
{
    if (!Y && M != 0) return fail(LQ_ERR_INVALID, "null Y");
    Args a{M, N, K, group, X, act_scales, static_cast<const u32x4 *>(W_packed), gparams, w_scales,
           reinterpret_cast<__half *>(Y), nullptr, static_cast<hipStream_t>(hip_stream), nullptr, 0};
    // what the dispatcher's kernel for this shape would use of a workspace (nothing is launched;
    // a launcher that can make do with fewer K slices is told how much there is)
    size_t need = 0;
    a.query = &need;
    a.ws_bytes = kStaticScratchBytes;
    if (int rc = run(-1, a)) return rc;
    a.query = nullptr;
    a.ws_bytes = 0;
    if (M == 0) return LQ_OK;
    if (need > kStaticScratchBytes)
        return fail(LQ_ERR_WORKSPACE,
                    "M=%d N=%d K=%d needs %zu bytes of split-K workspace, the built-in one holds %zu: "
                    "use w4a8_gemm with a workspace of the caller",
                    M, N, K, need, kStaticScratchBytes);
    if (need > 0) {
        if (int rc = static_scratch_ptr(&a.ws)) return rc;
        a.ws_bytes = kStaticScratchBytes;
    }
    return run(-1, a);
}

int w4a8_gemm_i32(int M, int N, int K, int group, const int8_t *X, const void *W_packed,
                  const uint8_t *gparams, int32_t *ACC, void *workspace, size_t workspace_bytes,
                  void *hip_stream)
{
    if (!ACC && M != 0) return fail(LQ_ERR_INVALID, "null ACC");
    const Args a{M, N, K, group, X, nullptr, static_cast<const u32x4 *>(W_packed), gparams, nullptr,
                 nullptr, ACC, static_cast<hipStream_t>(hip_stream), workspace, workspace_bytes};
    return run(-1, a);
}

int w4a8_gemm_variant(int variant, int M, int N, int K, int group, const int8_t *X,
                      const float *act_scales, const void *W_packed, const uint8_t *gparams,
                      const float *w_scales, uint16_t *Y, int32_t *ACC, void *workspace,
                      size_t workspace_bytes, void *hip_stream)
{
    if (variant < -1 || variant >= kNumVariants) return fail(LQ_ERR_INVALID, "unknown variant %d", variant);
    const Args a{M, N, K, group, X, act_scales, static_cast<const u32x4 *>(W_packed), gparams, w_scales,
                 reinterpret_cast<__half *>(Y), ACC, static_cast<hipStream_t>(hip_stream), workspace, workspace_bytes};
    return run(variant, a);
}

int w4a8_variant_count(void) { return kNumVariants; }

const char *w4a8_variant_name(int variant)
{
    return (variant >= 0 && variant < kNumVariants) ? kVariants[variant].name : nullptr;
}

int w4a8_variant_supports(int variant, int M, int N, int K, int group)
{
    if (variant < 0 || variant >= kNumVariants || M < 0 || !shape_ok(N, K, group)) return 0;
    return variant_supports(variant, M, N, K) ? 1 : 0;
}

int w4a8_select_variant(int M, int N, int K, int group)
{
    if (M < 0 || !shape_ok(N, K, group)) return fail(LQ_ERR_INVALID, "bad shape");
    return select_variant(M, N, K);
}

int w4a8_select_plan(int M, int N, int K, int group, int *rows_first, int *variant_rest)
{
    if (M < 0 || !shape_ok(N, K, group) || !rows_first || !variant_rest) return fail(LQ_ERR_INVALID, "bad shape");
    const int first = M > 0 ? rows_of_first_launch(M, N, K) : M;
    *rows_first = first;
    *variant_rest = first == M ? -1 : select_variant(M - first, N, K);
    return first == M ? select_variant(M, N, K) : find_variant("solo16_pt_m256");
}

int w4a8_dequant_dump(const void *W_packed, const uint8_t *gparams, int N, int K, int group,
                      int8_t *Wd, void *hip_stream)
{
    if (!shape_ok(N, K, group)) return fail(LQ_ERR_INVALID, "bad shape N=%d K=%d group=%d", N, K, group);
    if (!W_packed || !gparams || !Wd) return fail(LQ_ERR_INVALID, "null pointer");
    if (((uintptr_t)W_packed | (uintptr_t)gparams | (uintptr_t)Wd) & 15)
        return fail(LQ_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const dim3 grid((unsigned)((K / 64 + 3) / 4), (unsigned)(N / 32)), block(256);
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

int w4a8_grouped_gemm(int E, const int *row_offsets, int N, int K, int group, const int8_t *X,
                      const float *act_scales, const void *W_packed, const uint8_t *gparams,
                      const float *w_scales, uint16_t *Y, int32_t *ACC, void *hip_stream)
{
    if (E < 1 || E > kMaxExperts) return fail(LQ_ERR_INVALID, "E=%d out of range (1..%d)", E, kMaxExperts);
    if (!shape_ok(N, K, group))
        return fail(LQ_ERR_INVALID, "bad shape N=%d K=%d group=%d (need N%%64==0, K%%256==0, group 64|128, K<=131072)",
                    N, K, group);
    if (!row_offsets || row_offsets[0] != 0) return fail(LQ_ERR_INVALID, "row_offsets must start at 0");
    for (int e = 0; e < E; ++e) {
        if (row_offsets[e + 1] < row_offsets[e]) return fail(LQ_ERR_INVALID, "row_offsets must not decrease");
        // the kernels address an expert's rows of X with 32-bit byte offsets
        if ((long long)(row_offsets[e + 1] - row_offsets[e]) * K >= (1ll << 32))
            return fail(LQ_ERR_INVALID, "expert %d has rows * K >= 2^32 bytes of X; split it into two experts", e);
    }
    if (row_offsets[E] == 0) return LQ_OK;
    if (!Y && !ACC) return fail(LQ_ERR_INVALID, "no output pointer");
    if (!X || !W_packed || !gparams) return fail(LQ_ERR_INVALID, "null input pointer");
    if (Y && (!act_scales || !w_scales)) return fail(LQ_ERR_INVALID, "null scale pointer");
    const uintptr_t bits = (uintptr_t)X | (uintptr_t)W_packed | (uintptr_t)gparams | (uintptr_t)act_scales |
                           (uintptr_t)w_scales | (uintptr_t)Y | (uintptr_t)ACC;
    if (bits & 15) return fail(LQ_ERR_ALIGN, "device pointers must be 16-byte aligned");
    GroupedArgs a{};
    a.E = E, a.N = N, a.K = K, a.group = group, a.row_offsets = row_offsets;
    a.p = GroupedPtrs{X, act_scales, static_cast<const u32x4 *>(W_packed), gparams, w_scales,
                      reinterpret_cast<__half *>(Y), ACC, (size_t)N * K / 32, (size_t)2 * N * K / group};
    a.stream = static_cast<hipStream_t>(hip_stream);
    return grouped_run(a);
}

int w8a8_gemm(int M, int N, int K, const int8_t *X, const float *act_scales, const void *W8_packed,
              const float *w_scales, uint16_t *Y, int32_t *ACC, void *hip_stream)
{
    if (M < 0 || !shape_ok(N, K, 64))
        return fail(LQ_ERR_INVALID, "bad shape M=%d N=%d K=%d (need M>=0, N%%64==0, K%%256==0, K<=131072)", M, N, K);
    if (M == 0) return LQ_OK;
    if (!Y && !ACC) return fail(LQ_ERR_INVALID, "no output pointer");
    if (!X || !W8_packed) return fail(LQ_ERR_INVALID, "null input pointer");
    if (Y && (!act_scales || !w_scales)) return fail(LQ_ERR_INVALID, "null scale pointer");
    if (((uintptr_t)X | (uintptr_t)W8_packed | (uintptr_t)act_scales | (uintptr_t)w_scales | (uintptr_t)Y |
         (uintptr_t)ACC) & 15)
        return fail(LQ_ERR_ALIGN, "device pointers must be 16-byte aligned");
    if ((long long)M * K >= (1ll << 32))
        return fail(LQ_ERR_INVALID, "M * K = %lld is beyond the 2^32 - 1 bytes of X one call addresses; split the batch",
                    (long long)M * K);
    const int blocks_n = (N + 255) / 256, blocks_m = (M + 127) / 128;
    const size_t lds_bytes = 4 * (size_t)128 * 128;
    if (int rc = allow_lds(w8a8_kernel, lds_bytes)) return rc;
    (void)hipGetLastError();
    hipLaunchKernelGGL(w8a8_kernel, dim3((unsigned)(blocks_n * blocks_m)), dim3(256), lds_bytes,
                       static_cast<hipStream_t>(hip_stream), M, N, K, X, act_scales,
                       static_cast<const u32x4 *>(W8_packed), w_scales, reinterpret_cast<__half *>(Y), ACC,
                       blocks_m, blocks_n);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LQ_ERR_HIP, "w8a8 launch failed: %s", hipGetErrorString(e));
    return LQ_OK;
}

}  // extern "C"
