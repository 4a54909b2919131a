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
//           fragment for 4 MFMAs.  `duo` is the kernel that is dispatched (two waves per
//           SIMD); `tile` is its plain predecessor, kept as a named variant.
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

// ------------------------------------------------------------------------------------
// stream kernel.  A unit is 128 k (two chunks per tile).  grid = (N / (32 F), S): block
// (bx, ks) owns F tiles and the ks-th of S slices of K; its NW waves take the slice's
// units round-robin.  S > 1 (grid-level split-K) is used when N alone gives too few blocks
// to keep every HBM channel busy; the S partial tiles meet in a workspace and the last
// block to arrive (a ticket per tile group) adds them up and runs the epilogue.  All sums
// are INT32, so neither level of split-K changes the result.
// ------------------------------------------------------------------------------------
#ifndef LQ_DUO_ABL
#define LQ_DUO_ABL 0
#endif
#ifdef LQ_ABLATE
// experiments only: per-wave wall-clock stamps (start, first unit done, loop done, end)
__device__ long long g_dbg_stamps[4 * 16384];
#define LQ_STAMP(slot)                                                                          \
    do {                                                                                        \
        const unsigned w_ = (blockIdx.y * gridDim.x + blockIdx.x) * NW + wave;                  \
        if (lane == 0 && w_ < 16384) g_dbg_stamps[4 * w_ + (slot)] = wall_clock64();            \
    } while (0)
// same for the duo kernel: 8 slots per wave
#define LQ_DSTAMP(slot)                                                                         \
    do {                                                                                        \
        const unsigned w_ = (blockIdx.y * gridDim.x + blockIdx.x) * (4 * KG) + (threadIdx.x >> 6); \
        if ((threadIdx.x & 63) == 0 && w_ < 8192) g_dbg_stamps[8 * w_ + (slot)] = wall_clock64(); \
    } while (0)
#else
#define LQ_STAMP(slot) \
    do {               \
    } while (0)
#define LQ_DSTAMP(slot) \
    do {                \
    } while (0)
#endif

// Arrival tickets of the grid-level split-K, one per tile group, live at the head of the
// caller's workspace (kTicketBytes, zeroed once by the caller or by w4a8_workspace_init).
// The last block of a group resets its ticket, so every call finds zeros again; calls that
// overlap in time are independent as long as they use different workspaces.
constexpr int kMaxTicketGroups = 8192;
constexpr size_t kTicketBytes = kMaxTicketGroups * sizeof(unsigned int);

// Device-scope (write-through / cache-bypassing) 16-byte accesses for the exchange of
// split-K partial tiles between blocks that may sit on different XCDs: the sc1 forms of
// the plain global load and store, which is what a relaxed agent-scope atomic compiles to.
// OFF = constant byte offset (0 .. 4095) folded into the instruction, so that the four
// accesses of one accumulator fragment share one address register pair.
template <int OFF = 0>
__device__ __forceinline__ void store_sc1_x4(int32_t *p, const v4i v)
{
    asm volatile("global_store_dwordx4 %0, %1, off offset:%2 sc1" ::"v"(p), "v"(v), "n"(OFF) : "memory");
}
template <int OFF = 0>
__device__ __forceinline__ v4i load_sc1_x4(const int32_t *p)
{
    v4i v;
    asm volatile("global_load_dwordx4 %0, %1, off offset:%2 sc1" : "=v"(v) : "v"(p), "n"(OFF) : "memory");
    return v;
}
__device__ __forceinline__ void wait_vmcnt0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// at most N vector memory loads of this wave still in flight (they complete in order)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// the same wait, tied to the registers that the loads above are filling
__device__ __forceinline__ void wait_vmcnt0(v4i &a, v4i &b, v4i &c, v4i &d)
{
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d)::"memory");
}

// Where a block works: gx = its tile group (or output tile) among gnx, ks = its slice of S
// K slices.  Plain launches take these from the grid (blockIdx.x, gridDim.x, blockIdx.y,
// gridDim.y); grouped launches compute them per expert.
struct Place {
    int gx, gnx, ks, S;
    unsigned int *tickets;  // arrival tickets of the split-K groups (unused when S == 1)
};
__device__ __forceinline__ Place grid_place(unsigned int *tickets)
{
    return Place{(int)blockIdx.x, (int)gridDim.x, (int)blockIdx.y, (int)gridDim.y, tickets};
}

template <int F, int MF, bool G128>
struct StreamRegs {
    u32x4 w[F][2];
    UnitParams<G128> p[F];
    u32x4 x[MF][4];
};

// MF = row fragments of 32 per wave: 1 for M <= 32, 2 for M <= 64 (the weights are still
// streamed once; the dequantised operand of a chunk feeds MF MFMAs).  Four fragments were
// measured too: the X fragments, which every block reads for itself from L2, then outweigh
// the weights four to one and the 128 x 256 tiles with X shared through LDS are faster.
template <int F, int NW, int MF, bool G128>
__device__ __forceinline__ void stream_block(
    const Place pl, int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int32_t *__restrict__ partials)
{
    extern __shared__ __attribute__((aligned(16))) int red[];  // [NW][F * MF * rmax][64]
    __shared__ int s_last;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 31, kb = lane >> 5;
    const int t0 = pl.gx * F;
    const int units = K >> 7;
    const int chunks_per_tile = K >> 6;
    const int S = pl.S, ks = pl.ks;
    const int u_begin = (int)((long long)units * ks / S), u_end = (int)((long long)units * (ks + 1) / S);

    v16i acc[F][MF];
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][mf][r] = 0;

    // X fragments come straight from global memory (L2): lane (j, kb) needs 16 bytes of row
    // j (+ 32 per further fragment) per k-step.  Lanes past M read row M-1 (one more hit on
    // a line that is fetched anyway); an output row depends only on its own X row and rows
    // past M are not stored.
    const int8_t *xrow[MF];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) xrow[mf] = X + (size_t)min(j + 32 * mf, M - 1) * K + 16 * kb;

    auto load_unit = [&](int u, StreamRegs<F, MF, G128> &r) {
#pragma unroll
        for (int f = 0; f < F; ++f) {
            const u32x4 *base = Wp + ((size_t)(t0 + f) * chunks_per_tile + 2 * (size_t)u) * 64 + lane;
            r.w[f][0] = __builtin_nontemporal_load(base);
            r.w[f][1] = __builtin_nontemporal_load(base + 64);
            r.p[f].load(gp, (size_t)(t0 + f) * units + u, j);
        }
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int ks4 = 0; ks4 < 4; ++ks4)
                r.x[mf][ks4] = *reinterpret_cast<const u32x4 *>(xrow[mf] + (size_t)u * 128 + 32 * ks4);
    };
    auto compute_unit = [&](const StreamRegs<F, MF, G128> &r) {
#pragma unroll
        for (int f = 0; f < F; ++f)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                uint32_t s2, a4;
                r.p[f].get(c, s2, a4);
                v4i lo, hi;
                dequant_chunk(r.w[f][c], s2, a4, lo, hi);
#pragma unroll
                for (int mf = 0; mf < MF; ++mf) {
                    acc[f][mf] = mfma_i8(__builtin_bit_cast(v4i, r.x[mf][2 * c]), lo, acc[f][mf]);
                    acc[f][mf] = mfma_i8(__builtin_bit_cast(v4i, r.x[mf][2 * c + 1]), hi, acc[f][mf]);
                }
            }
    };

    // Register double buffering: the loads of the next unit are in flight while the
    // current one is dequantised and multiplied.
    LQ_STAMP(0);
    StreamRegs<F, MF, G128> cur, nxt;
    int u = u_begin + wave;
    if (u < u_end) load_unit(u, cur);
    for (; u < u_end; u += NW) {
        const bool more = (u + NW) < u_end;
        if (more) load_unit(u + NW, nxt);
        compute_unit(cur);
        if (more) cur = nxt;
    }
    LQ_STAMP(2);

    // In-block split-K reduction (integer, order independent).  With one row fragment only
    // the accumulator elements that hold rows < M take part: rows of element r lie in
    // [8*(r/4), 8*(r/4)+8).  Value v = (f * MF + mf) * rmax + r of lane l is row
    // 32*mf + acc_row(r, l), slot l%32 of tile t0 + f.
    const int rmax = MF == 1 ? 4 * ((M + 7) >> 3) : 16;
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (r < rmax) red[((wave * F * MF + f * MF + mf) * rmax + r) * 64 + lane] = acc[f][mf][r];
    __syncthreads();
    const int vals = F * MF * rmax;
    auto block_sum = [&](int idx) {
        int sum = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red[(w * vals + (idx >> 6)) * 64 + (idx & 63)];
        return sum;
    };
    auto finish = [&](int idx, int sum) {  // epilogue of one output (Sec. 4, Sec. 5.3)
        const int v = idx >> 6, l = idx & 63;
        const int fm = v / rmax;
        const int m = 32 * (fm % MF) + acc_row(v % rmax, l);
        if (m < M) {
            const int n = channel_of(t0 + fm / MF, l & 31);
            if (ACC) ACC[(size_t)m * N + n] = sum;
            if (Y) Y[(size_t)m * N + n] = scale_to_half(sum, sx[m], sw[n]);
        }
    };
    if (S == 1) {
        for (int idx = threadIdx.x; idx < vals * 64; idx += NW * 64) finish(idx, block_sum(idx));
    } else {
        // Partial tile of this slice: [ks][blockIdx.x][vals * 64], coalesced.  The tiles are
        // written and read with device-scope atomics, which act at the memory side common to
        // all XCDs, so no cache has to be flushed or invalidated; the barrier's wait for
        // outstanding memory operations orders them before the ticket.
        int32_t *mine = partials + ((size_t)ks * pl.gnx + pl.gx) * (size_t)(vals * 64);
        for (int idx = threadIdx.x; idx < vals * 64; idx += NW * 64)
            __hip_atomic_store(mine + idx, block_sum(idx), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();  // includes s_waitcnt vmcnt(0): every store above has been acknowledged
        if (threadIdx.x == 0) {
            const unsigned t = __hip_atomic_fetch_add(&pl.tickets[pl.gx], 1u, __ATOMIC_RELAXED,
                                                      __HIP_MEMORY_SCOPE_AGENT);
            s_last = (t == (unsigned)(S - 1));
        }
        __syncthreads();
        if (s_last) {
            for (int idx = threadIdx.x; idx < vals * 64; idx += NW * 64) {
                int sum = 0;
                for (int k2 = 0; k2 < S; ++k2)
                    sum += __hip_atomic_load(
                        partials + ((size_t)k2 * pl.gnx + pl.gx) * (size_t)(vals * 64) + idx,
                        __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                finish(idx, sum);
            }
            if (threadIdx.x == 0)  // ready for the next call
                __hip_atomic_store(&pl.tickets[pl.gx], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    LQ_STAMP(3);
}

template <int F, int NW, int MF, bool G128>
__global__ __launch_bounds__(NW * 64) void w4a8_stream_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int32_t *__restrict__ partials,
    unsigned int *__restrict__ tickets)
{
    stream_block<F, NW, MF, G128>(grid_place(tickets), M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
}

// ------------------------------------------------------------------------------------
// stream16 kernel: the stream kernel for M <= 16 on v_mfma_i32_16x16x64_i8.
//
// A 32-row MFMA wastes half of its rows on a decode batch, and in this regime the per-CU
// arithmetic (dequantisation + MFMA) is not far below what the HBM stream demands.  The
// packed layout is unchanged: after the usual dequantisation one v_permlane16_swap per
// register turns the chunk's two 32x32x32 operands into the operands of two 16x16x64
// MFMAs (see regroup_16x16), which take half the matrix-pipe time, a quarter of the
// accumulator registers and half of the X registers.
// ------------------------------------------------------------------------------------
// UU = 128-k units per pipeline step (1 or 2): bytes in flight per wave = F * UU * 2 KiB.
template <int F, int UU, bool G128>
struct Stream16Regs {
    u32x4 w[F][2 * UU];
    UnitParams<G128> p[F][UU];
    u32x4 x[2 * UU];
};

// ABL (experiments only, 0 in shipped variants): 1 = no X loads, 2 = no parameter loads,
// 4 = no dequantisation, 8 = no reduction / epilogue.  Results are wrong for ABL != 0.
template <int F, int NW, int UU, bool G128, int ABL = 0>
__device__ __forceinline__ void stream16_block(
    const Place pl, int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int32_t *__restrict__ partials)
{
    constexpr int VALS = F * 8;  // accumulator registers per lane
    extern __shared__ __attribute__((aligned(16))) int red[];  // [NW][VALS][64]
    __shared__ int s_last;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 31;
    const int t0 = pl.gx * F;
    const int units = K >> 7;                   // 128-k units (parameter granularity)
    const int steps = units / UU;               // pipeline steps of UU units
    const int chunks_per_tile = K >> 6;
    const int S = pl.S, ks = pl.ks;
    const int u_begin = (int)((long long)steps * ks / S), u_end = (int)((long long)steps * (ks + 1) / S);

    v4i acc[F][2];
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
        for (int h = 0; h < 2; ++h) acc[f][h] = v4i{0, 0, 0, 0};

    // X operand of a 16x16x64 MFMA: lane l supplies row l%16, k-block l/16 of a chunk, in
    // the k-block order that regroup_16x16 produces.  Lanes past M read row M-1.
    const int8_t *xrow = X + (size_t)min(lane & 15, M - 1) * K + kstep16_offset(lane >> 4);

    // The outputs this thread will finish (idx = threadIdx.x + i * blockDim.x) are known
    // now: fetch their scales here, so that the epilogue does not end on a cold load.
    constexpr int OUTS = (VALS * 64 + NW * 64 - 1) / (NW * 64);
    float pre_sx[OUTS], pre_sw[OUTS];
    if (Y) {
#pragma unroll
        for (int i = 0; i < OUTS; ++i) {
            const int idx = threadIdx.x + i * NW * 64;
            const int v = min(idx >> 6, VALS - 1), l = idx & 63;
            pre_sx[i] = sx[min(4 * (l >> 4) + (v & 3), M - 1)];
            pre_sw[i] = sw[channel_of(t0 + (v >> 3), 16 * ((v >> 2) & 1) + (l & 15))];
        }
    }

    auto load_unit = [&](int u, Stream16Regs<F, UU, G128> &r) {
#pragma unroll
        for (int f = 0; f < F; ++f) {
            const u32x4 *base = Wp + ((size_t)(t0 + f) * chunks_per_tile + 2 * UU * (size_t)u) * 64 + lane;
#pragma unroll
            for (int c = 0; c < 2 * UU; ++c) r.w[f][c] = __builtin_nontemporal_load(base + 64 * c);
#pragma unroll
            for (int q = 0; q < UU; ++q) {
                if (ABL & 2)
                    r.p[f][q].raw = 0x01800180u;
                else
                    r.p[f][q].load(gp, (size_t)(t0 + f) * units + (size_t)u * UU + q, j);
            }
        }
#pragma unroll
        for (int c = 0; c < 2 * UU; ++c)
            r.x[c] = (ABL & 1) ? u32x4{1u, 2u, 3u, (unsigned)u}
                               : *reinterpret_cast<const u32x4 *>(xrow + (size_t)u * (128 * UU) + 64 * c);
    };
    auto compute_unit = [&](const Stream16Regs<F, UU, G128> &r) {
#pragma unroll
        for (int f = 0; f < F; ++f)
#pragma unroll
            for (int c = 0; c < 2 * UU; ++c) {
                uint32_t s2, a4;
                r.p[f][c >> 1].get(c & 1, s2, a4);
                v4i lo, hi, b1, b2;
                if (ABL & 4) {
                    lo = __builtin_bit_cast(v4i, r.w[f][c]);
                    hi = lo + (int)s2;
                } else {
                    dequant_chunk(r.w[f][c], s2, a4, lo, hi);
                }
                regroup_16x16(lo, hi, b1, b2);
                const v4i xa = __builtin_bit_cast(v4i, r.x[c]);
                acc[f][0] = mfma16_i8(xa, b1, acc[f][0]);
                acc[f][1] = mfma16_i8(xa, b2, acc[f][1]);
            }
    };

    Stream16Regs<F, UU, G128> cur, nxt;
    int u = u_begin + wave;
    if (u < u_end) load_unit(u, cur);
    for (; u < u_end; u += NW) {
        const bool more = (u + NW) < u_end;
        if (more) load_unit(u + NW, nxt);
        compute_unit(cur);
        if (more) cur = nxt;
    }

    if (ABL & 8) {
        int sum = 0;
#pragma unroll
        for (int f = 0; f < F; ++f) sum += acc[f][0][0] + acc[f][1][1] + acc[f][0][2] + acc[f][1][3];
        if (sum == 0x12345678) ACC[0] = sum;
        return;
    }
    // in-block split-K reduction: value v = (f*2 + h)*4 + r of lane l is row 4*(l/16) + r,
    // slot 16*h + l%16 of tile t0 + f
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[(wave * VALS + (f * 2 + h) * 4 + r) * 64 + lane] = acc[f][h][r];
    __syncthreads();
    auto block_sum = [&](int idx) {
        int sum = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red[(w * VALS + (idx >> 6)) * 64 + (idx & 63)];
        return sum;
    };
    auto finish = [&](int i, int idx, int sum) {
        const int v = idx >> 6, l = idx & 63;
        const int m = 4 * (l >> 4) + (v & 3);
        if (m < M) {
            const int n = channel_of(t0 + (v >> 3), 16 * ((v >> 2) & 1) + (l & 15));
            if (ACC) ACC[(size_t)m * N + n] = sum;
            if (Y) Y[(size_t)m * N + n] = scale_to_half(sum, pre_sx[i], pre_sw[i]);
        }
    };
    if (S == 1) {
#pragma unroll
        for (int i = 0; i < OUTS; ++i) {
            const int idx = threadIdx.x + i * NW * 64;
            if (idx < VALS * 64) finish(i, idx, block_sum(idx));
        }
    } else {
        // grid-level split-K: same protocol as w4a8_stream_kernel
        int32_t *mine = partials + ((size_t)ks * pl.gnx + pl.gx) * (size_t)(VALS * 64);
        for (int idx = threadIdx.x; idx < VALS * 64; idx += NW * 64)
            __hip_atomic_store(mine + idx, block_sum(idx), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned t = __hip_atomic_fetch_add(&pl.tickets[pl.gx], 1u, __ATOMIC_RELAXED,
                                                      __HIP_MEMORY_SCOPE_AGENT);
            s_last = (t == (unsigned)(S - 1));
        }
        __syncthreads();
        if (s_last) {
#pragma unroll
            for (int i = 0; i < OUTS; ++i) {
                const int idx = threadIdx.x + i * NW * 64;
                if (idx >= VALS * 64) break;
                int sum = 0;
                for (int k2 = 0; k2 < S; ++k2)
                    sum += __hip_atomic_load(
                        partials + ((size_t)k2 * pl.gnx + pl.gx) * (size_t)(VALS * 64) + idx,
                        __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                finish(i, idx, sum);
            }
            if (threadIdx.x == 0)
                __hip_atomic_store(&pl.tickets[pl.gx], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <int F, int NW, int UU, bool G128, int ABL = 0>
__global__ __launch_bounds__(NW * 64) void w4a8_stream16_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int32_t *__restrict__ partials,
    unsigned int *__restrict__ tickets)
{
    stream16_block<F, NW, UU, G128, ABL>(grid_place(tickets), M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
}

// ------------------------------------------------------------------------------------
// Epilogue shared by the tiled kernels.  Element r of acc[mf][t] is row
// m0 + 32*mf + acc_row(r, lane) and channel n + t (n = 64*group + 2*slot): the two tiles
// give 2 adjacent channels per lane, so each store is 4 bytes of FP16 (8 of INT32) and a
// half-wave writes a full 128-byte line.  Scales are fetched up front, four consecutive
// rows at a time (rows past M read s_x[M-1]; only the stores are predicated), so no
// load sits behind a branch.
// ------------------------------------------------------------------------------------
template <int MF>
__device__ __forceinline__ void store_tile(const v16i (&acc)[MF][2], int M, int N, int m0, int n, int lane,
                                           const float *__restrict__ sx, const float *__restrict__ sw,
                                           __half *__restrict__ Y, int32_t *__restrict__ ACC)
{
    const int kb = lane >> 5;
    if (ACC) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + 32 * mf + 8 * (r >> 2) + 4 * kb + (r & 3);
                if (m < M) *reinterpret_cast<int2 *>(ACC + (size_t)m * N + n) = int2{acc[mf][0][r], acc[mf][1][r]};
            }
    }
    if (Y) {
        const float2 swv = *reinterpret_cast<const float2 *>(sw + n);
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) {
            float sxv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) sxv[r] = sx[min(m0 + 32 * mf + 8 * (r >> 2) + 4 * kb + (r & 3), M - 1)];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + 32 * mf + 8 * (r >> 2) + 4 * kb + (r & 3);
                union {
                    __half h[2];
                    uint32_t u;
                } o;
                o.h[0] = scale_to_half(acc[mf][0][r], sxv[r], swv.x);
                o.h[1] = scale_to_half(acc[mf][1][r], sxv[r], swv.y);
                if (m < M) *reinterpret_cast<uint32_t *>(Y + (size_t)m * N + n) = o.u;
            }
        }
    }
}

// ------------------------------------------------------------------------------------
// tile kernel.  MF = 32-row fragments per wave; block tile = (32*MF) x 256.
// ------------------------------------------------------------------------------------
constexpr int kTilePitch = 128 + 16;  // LDS row pitch in bytes: rows shift by 9 x 16 B

// Block id -> (bm, bn).  Consecutive hardware ids go to different XCDs (8 of them, each
// with its own L2), so ids are first regrouped so that each XCD owns a contiguous range
// of logical ids, then walked in groups of 4 row-blocks so that blocks resident together
// on one XCD share X rows and W columns in its L2.
__device__ __forceinline__ void block_coords(int blocks_m, int blocks_n, int &bm, int &bn)
{
    const int total = blocks_m * blocks_n;
    int lid = blockIdx.x;
    if ((total & 7) == 0) lid = (lid & 7) * (total >> 3) + (lid >> 3);
#ifndef LQ_GM
#define LQ_GM 4
#endif
    constexpr int GM = LQ_GM;
    const int per_group = GM * blocks_n;
    const int first = (lid / per_group) * GM;
    const int gsz = min(blocks_m - first, GM);
    const int in_group = lid % per_group;
    bm = first + in_group % gsz;
    bn = in_group / gsz;
}

template <int MF, bool G128>
__global__ __launch_bounds__(256, 2) void w4a8_tile_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int blocks_m, int blocks_n)
{
    constexpr int WM = 32 * MF;
    constexpr int XP = MF;  // 16-byte X pieces per thread per stage of 128 k
    constexpr int STAGE = WM * kTilePitch;
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, kb = lane >> 5;
    int bm, bn;
    block_coords(blocks_m, blocks_n, bm, bn);
    const int m0 = bm * WM;
    const int ng = bn * 4 + wave;  // 64-channel group of this wave
    const bool active = ng < (N >> 6);
    // A wave past the last group recomputes the last one and stores nothing, so that the
    // main loop has no divergent path around its barriers.
    const int t0 = 2 * (active ? ng : (N >> 6) - 1);
    const int stages = K >> 7;
    const int chunks_per_tile = K >> 6;

    v16i acc[MF][2];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mf][t][r] = 0;

    u32x4 xr[XP];
    u32x4 wc[2][2], wn[2][2];
    UnitParams<G128> pc[2], pn[2];

    // Rows past M read row M-1: an output row depends only on its own X row, and rows
    // past M are never stored.
    auto load_x = [&](int s) {
#pragma unroll
        for (int i = 0; i < XP; ++i) {
            const int q = tid + 256 * i;
            const int row = q >> 3, col = q & 7;
            const int m = min(m0 + row, M - 1);
            xr[i] = *reinterpret_cast<const u32x4 *>(X + (size_t)m * K + (size_t)s * 128 + 16 * col);
        }
    };
    auto store_x = [&](int buf) {
        int8_t *base = lds + buf * STAGE;
#pragma unroll
        for (int i = 0; i < XP; ++i) {
            const int q = tid + 256 * i;
            const int row = q >> 3, col = q & 7;
            *reinterpret_cast<u32x4 *>(base + row * kTilePitch + 16 * col) = xr[i];
        }
    };
    auto load_w = [&](int s, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const u32x4 *base = Wp + ((size_t)(t0 + t) * chunks_per_tile + 2 * (size_t)s) * 64 + lane;
            w[t][0] = base[0];
            w[t][1] = base[64];
            p[t].load(gp, (size_t)(t0 + t) * stages + s, j);
        }
    };
    auto compute = [&](int buf) {
        const int8_t *xs = lds + buf * STAGE + j * kTilePitch + 16 * kb;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            v4i blo[2], bhi[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                uint32_t s2, a4;
                pc[t].get(c, s2, a4);
                dequant_chunk(wc[t][c], s2, a4, blo[t], bhi[t]);
            }
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) {
                const v4i a0 = *reinterpret_cast<const v4i *>(xs + mf * 32 * kTilePitch + 64 * c);
                const v4i a1 = *reinterpret_cast<const v4i *>(xs + mf * 32 * kTilePitch + 64 * c + 32);
#pragma unroll
                for (int t = 0; t < 2; ++t) acc[mf][t] = mfma_i8(a0, blo[t], acc[mf][t]);
#pragma unroll
                for (int t = 0; t < 2; ++t) acc[mf][t] = mfma_i8(a1, bhi[t], acc[mf][t]);
            }
        }
    };

    load_x(0);
    load_w(0, wc, pc);
    store_x(0);
    __syncthreads();

    // Steady state: the global loads of stage s+1 are issued before the MFMAs of stage s
    // and land in LDS / registers after them.
    for (int s = 0; s + 1 < stages; ++s) {
        load_x(s + 1);
        load_w(s + 1, wn, pn);
        __builtin_amdgcn_sched_barrier(0);  // keep the prefetch ahead of the MFMAs
        compute(s & 1);
        __builtin_amdgcn_sched_barrier(0);
        store_x((s + 1) & 1);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            wc[t][0] = wn[t][0];
            wc[t][1] = wn[t][1];
            pc[t] = pn[t];
        }
    }
    compute((stages - 1) & 1);

    if (!active) return;
    // Epilogue: element r of acc[mf][t] is row m0 + 32*mf + acc_row(r), channel
    // 64*ng + 2*j + t: the two tiles give 2 adjacent channels per lane.
    store_tile<MF>(acc, M, N, m0, 64 * ng + 2 * j, lane, sx, sw, Y, ACC);
}

// Block barrier that orders LDS traffic only: __syncthreads() would also wait for every
// outstanding global load (vmcnt(0)), which is exactly what the prefetches must not do.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ------------------------------------------------------------------------------------
// duo kernel: two waves per SIMD.
//
// On CDNA a wave issues in order and an MFMA holds the SIMD's vector issue for part of its
// duration (8 to 16 of the 32 cycles of a 32x32x32 INT8 MFMA, measured), so the VALU work of
// the dequantisation overlaps best with matrix work of ANOTHER wave on the same SIMD --
// the observation behind the paper's implicit fine-grained pipeline (Sec. 5.1:
// dequantisation in one compute group overlaps MMA in another, with the hardware
// arbitrating).  This kernel therefore keeps every wave at <= 256 registers
// (wave tile 128 x 64, block tile 128 x 256, two blocks per CU) and software-pipelines each
// wave at the granularity of one k-step (32 k): while the 8 MFMAs of a k-step run, the
// B operand of the next k-step is dequantised and its X fragments are read from LDS.
// ------------------------------------------------------------------------------------
//
// KG = 2 is the variant for grids of at most one block per CU: the block then holds two
// groups of four waves that work on the same 128 x 256 tile, each on its own half of the
// block's k range with its own LDS stages, and exchange halves of their accumulators
// through LDS at the end (in-block split-K).  Every SIMD again has two waves, which a
// single 4-wave block per CU would not give.
// MF = row fragments of 32 that the block computes (4, or 2 for a row tile with at most 64
// rows below M: a ragged last tile, an expert with few tokens): such a tile pays for half
// the MFMAs, X staging and fragment reads.  The tile grid is that of 128-row tiles either way.
template <bool G128, int KG, int MF, int TM = 128>
__device__ __forceinline__ void duo_tile(
    const Place pl, const int bm, const int bn, int M, int N, int K, const int8_t *__restrict__ X,
    const float *__restrict__ sx, const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp,
    const float *__restrict__ sw, __half *__restrict__ Y, int32_t *__restrict__ ACC,
    int32_t *__restrict__ partials)
{
    constexpr int WM = TM, XP = MF;  // TM = rows between consecutive row tiles (128, or 64 with MF = 2)
    static_assert(32 * MF <= TM, "a tile cannot hold more row fragments than its height");
    constexpr int STAGE = 128 * kTilePitch;
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    __shared__ int s_last;

    const int tid = threadIdx.x & 255;  // thread within its k group
    const int grp = KG == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it in an SGPR
    const int j = lane & 31, kb = lane >> 5;
    const int m0 = bm * WM;
    const int ng = bn * 4 + wave;
    const bool active = ng < (N >> 6);
    const int t0 = 2 * (active ? ng : (N >> 6) - 1);
    // grid-level split-K: slice ks of S covers whole units of 256 k ...
    const int S = pl.S, ks = pl.ks;
    const int u_begin = (int)((long long)(K >> 8) * ks / S), u_end = (int)((long long)(K >> 8) * (ks + 1) / S);
    // ... and the in-block split gives group 0 the first ceil(half) of them.  All groups run
    // the loop of group 0 (the barriers are block-wide); a group with one unit less feeds
    // zeros as X in its last pass.
    const int u_first = (u_end - u_begin + KG - 1) / KG;
    const int s_begin = 2 * (u_begin + (grp ? u_first : 0));
    const int my_stages = 2 * (grp ? u_end - u_begin - u_first : u_first);
    const int stages = 2 * u_first;  // loop length in stages of 128 k (even)
    const int stages_total = K >> 7;
    const int chunks_per_tile = K >> 6;

    LQ_DSTAMP(0);
    v16i acc[MF][2];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mf][t][r] = 0;

    // X piece i of this thread: row (tid>>3) + 32*i, 16-byte column tid&7
    const int xrow = tid >> 3, xcol = tid & 7;
    // 32-bit offsets from block-uniform bases instead of one 64-bit pointer per piece: the
    // kernel runs at the 256-register limit and X has fewer than 2^32 bytes (K <= 131072 and
    // the host rejects M * K >= 2^32).
    const int8_t *xbase = X + (size_t)s_begin * 128;
    uint32_t xg[XP];
#pragma unroll
    for (int i = 0; i < XP; ++i) xg[i] = (uint32_t)min(m0 + xrow + 32 * i, M - 1) * (uint32_t)K + 16 * xcol;
    const int xl = xrow * kTilePitch + 16 * xcol;
    // tile t0 + 1 lies one tile stream behind t0 (block-uniform strides)
    const u32x4 *wg0 = Wp + ((size_t)t0 * chunks_per_tile + 2 * (size_t)s_begin) * 64 + lane;
    const uint8_t *pg0 = gp + (((size_t)t0 * stages_total + s_begin) * 32 + j) * (G128 ? 2 : 4);
    const size_t wg_stride = (size_t)chunks_per_tile * 64;
    const size_t pg_stride = (size_t)stages_total * 32 * (G128 ? 2 : 4);
    int8_t *lds_g = lds + grp * (2 * STAGE);  // the two X stages of this k group
    const int8_t *xs = lds_g + j * kTilePitch + 16 * kb;

    u32x4 xr[XP];
    u32x4 wr[2][2][2];  // [stage parity][tile][chunk]
    UnitParams<G128> pr[2][2];
    v4i bf[2][2];       // [ping-pong][tile]
    v4i af[2][MF];      // [ping-pong][m fragment]

    auto load_x = [&](int s) {
        if (KG > 1 && s >= my_stages) {  // past this group's slice: contributes nothing
#pragma unroll
            for (int i = 0; i < XP; ++i) xr[i] = u32x4{0, 0, 0, 0};
            return;
        }
        s = min(s, my_stages - 1);
#pragma unroll
        for (int i = 0; i < XP; ++i)
            xr[i] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)s * 128 + xg[i]);
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XP; ++i)
            *reinterpret_cast<u32x4 *>(lds_g + buf * STAGE + xl + i * 32 * kTilePitch) = xr[i];
    };
    auto load_w = [&](int s, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
        s = min(s, my_stages - 1);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const u32x4 *wg = wg0 + t * wg_stride;
            const uint8_t *pg = pg0 + t * pg_stride;
            w[t][0] = wg[(size_t)s * 128];
            w[t][1] = wg[(size_t)s * 128 + 64];
            if (G128)
                p[t].raw = *reinterpret_cast<const uint16_t *>(pg + (size_t)s * 64);
            else
                p[t].raw = *reinterpret_cast<const uint32_t *>(pg + (size_t)s * 128);
        }
    };
    // B operand of k-step (c, h) for both tiles
    auto build_b = [&](const u32x4 (&w)[2][2], const UnitParams<G128> (&p)[2], int c, int h, v4i (&b)[2]) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#if defined(LQ_ABLATE) && (LQ_DUO_ABL & 1)  // experiments only: raw bytes instead of the dequantised operand
            b[t] = __builtin_bit_cast(v4i, w[t][c]) + h + (int)p[t].raw;
#elif defined(LQ_ABLATE) && (LQ_DUO_ABL & 4)
            // experiments only: the overflow-safe dequantisation that LiquidQuant avoids --
            // code * s + min in signed 16-bit lanes (two codes per register), low bytes
            // gathered with a byte permute: about twice the instructions, same result
            uint32_t s2, a4;
            p[t].get(c, s2, a4);
            const uint32_t mn2 = (((a4 & 0xffu) - 128u) & 0xffffu) * 0x00010001u;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t q = w[t][c][d] >> (4 * h);
                const uint32_t ra = q & 0x000F000Fu, rb = (q >> 8) & 0x000F000Fu;
                const uint32_t ma = pk_mad_u16(ra, s2, mn2), mb = pk_mad_u16(rb, s2, mn2);
                b[t][d] = (int)__builtin_amdgcn_perm(mb, ma, 0x06020400u);
            }
#else
            uint32_t s2, a4;
            p[t].get(c, s2, a4);
            dequant_half(w[t][c], s2, a4, h, b[t]);
#endif
        }
    };
    auto read_a = [&](int buf, int c, int h, v4i (&a)[MF]) {
#if defined(LQ_ABLATE) && (LQ_DUO_ABL & 2)  // experiments only: no X fragment reads from LDS
        if (buf + c + h == -1)
#endif
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
            a[mf] = *reinterpret_cast<const v4i *>(xs + buf * STAGE + mf * 32 * kTilePitch + 64 * c + 32 * h);
    };
    auto mma = [&](const v4i (&a)[MF], const v4i (&b)[2]) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int t = 0; t < 2; ++t) acc[mf][t] = mfma_i8(a[mf], b[t], acc[mf][t]);
    };

    // One stage: w_cur = W(s) on entry and W(s+2) on exit, w_nxt = W(s+1); af[0], bf[0] hold
    // k-step (0,0) of this stage on entry and of the next stage on exit; xr holds X(s+1).
    auto stage = [&](int s, u32x4 (&w_cur)[2][2], UnitParams<G128> (&p_cur)[2], u32x4 (&w_nxt)[2][2],
                     UnitParams<G128> (&p_nxt)[2], int buf) {
        // k-step (0,0)
        store_x(buf ^ 1);  // X(s+1); that buffer was released by the previous barrier
        read_a(buf, 0, 1, af[1]);
        build_b(w_cur, p_cur, 0, 1, bf[1]);
        mma(af[0], bf[0]);
        __builtin_amdgcn_sched_barrier(0);
        // k-step (0,1)
        load_x(s + 2);
        read_a(buf, 1, 0, af[0]);
        build_b(w_cur, p_cur, 1, 0, bf[0]);
        mma(af[1], bf[1]);
        __builtin_amdgcn_sched_barrier(0);
        // k-step (1,0)
        read_a(buf, 1, 1, af[1]);
        build_b(w_cur, p_cur, 1, 1, bf[1]);
        mma(af[0], bf[0]);
        __builtin_amdgcn_sched_barrier(0);
        // k-step (1,1): W(s) is fully consumed, the next stage's X is complete after the barrier
        lds_barrier();
        read_a(buf ^ 1, 0, 0, af[0]);
        build_b(w_nxt, p_nxt, 0, 0, bf[0]);
        load_w(s + 2, w_cur, p_cur);
        mma(af[1], bf[1]);
        __builtin_amdgcn_sched_barrier(0);
    };

    // prologue (the W loads are issued after X(1) so that, as in the steady state, the
    // only loads younger than an X stage are one stage of W)
    load_x(0);
    store_x(0);
    load_x(1);
    __builtin_amdgcn_sched_barrier(0);
    load_w(0, wr[0], pr[0]);
    load_w(1, wr[1], pr[1]);
    __builtin_amdgcn_sched_barrier(0);
    build_b(wr[0], pr[0], 0, 0, bf[0]);
    lds_barrier();
    read_a(0, 0, 0, af[0]);
    __builtin_amdgcn_sched_barrier(0);

    LQ_DSTAMP(1);
    for (int s = 0; s < stages; s += 2) {
        stage(s, wr[0], pr[0], wr[1], pr[1], 0);
        stage(s + 1, wr[1], pr[1], wr[0], pr[0], 1);
    }
    LQ_DSTAMP(2);

    // What is left is written once per k group with compile-time fragment indices: group G
    // finishes the MFK = MF / KG row fragments starting at MF0 = G * MFK.
    auto finish = [&](auto group_tag) {
        constexpr int G = decltype(group_tag)::value;
        constexpr int MFK = MF / KG, MF0 = G * MFK, GIVE0 = (KG - 1 - G) * MFK;
        if (KG > 1) {
            // In-block reduction through LDS (the X stages are dead by now), one column tile
            // at a time so that 64 KiB suffice: every wave hands the fragments it does not
            // finish to the wave of the other group that owns the same 128 x 64 sub-tile.
            v4i *ex = reinterpret_cast<v4i *>(lds);
            lds_barrier();
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int i = 0; i < MFK; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        ex[(((G * 4 + wave) * MFK + i) * 4 + q) * 64 + lane] =
                            v4i{acc[GIVE0 + i][t][4 * q], acc[GIVE0 + i][t][4 * q + 1],
                                acc[GIVE0 + i][t][4 * q + 2], acc[GIVE0 + i][t][4 * q + 3]};
                lds_barrier();
#pragma unroll
                for (int i = 0; i < MFK; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v4i v = ex[((((KG - 1 - G) * 4 + wave) * MFK + i) * 4 + q) * 64 + lane];
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[MF0 + i][t][4 * q + e] += v[e];
                    }
                if (t == 0) lds_barrier();
            }
        }
        LQ_DSTAMP(3);
        if (S > 1) {
            // Grid-level split-K (same protocol as the stream kernels): every block publishes its
            // INT32 partial tile with device-scope write-through stores, takes a ticket, and the
            // last one of the S slices adds the others to its registers and runs the epilogue.
            // Layout: [tile][slice][wave of the block][MFK*8 x (64 lanes x 16 B)], fully coalesced.
            constexpr int EPW = (4 / KG) * 8;  // slots of a full 4-fragment tile, whatever MF is
            const size_t tile = pl.gx;
            const int bw = G * 4 + wave;
            int32_t *mine = partials + (((tile * S + ks) * (4 * KG) + bw) * EPW) * 256 + lane * 4;
            // row fragments that lie wholly past M are neither published nor read back
            auto live = [&](int i) { return m0 + 32 * (MF0 + i) < M; };
#pragma unroll
            for (int i = 0; i < MFK; ++i) {
                if (!live(i)) continue;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    int32_t *frag = mine + (i * 2 + t) * 4 * 256;
                    auto part = [&](int q) {
                        return v4i{acc[MF0 + i][t][4 * q], acc[MF0 + i][t][4 * q + 1], acc[MF0 + i][t][4 * q + 2],
                                   acc[MF0 + i][t][4 * q + 3]};
                    };
                    store_sc1_x4<0>(frag, part(0));
                    store_sc1_x4<1024>(frag, part(1));
                    store_sc1_x4<2048>(frag, part(2));
                    store_sc1_x4<3072>(frag, part(3));
                }
            }
            wait_vmcnt0();
            LQ_DSTAMP(4);
            __syncthreads();
            if (threadIdx.x == 0) {
                const unsigned tk = __hip_atomic_fetch_add(&pl.tickets[tile], 1u, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
                s_last = (tk == (unsigned)(S - 1));
            }
            __syncthreads();
            LQ_DSTAMP(5);
            if (!s_last) return;
            // The 8 loads of one row fragment (2 column tiles x 4 pieces of 16 bytes per lane)
            // are in flight before the first is waited for: the latency of these device-scope
            // reads, not their volume, is what this tail costs.
            for (int k2 = 0; k2 < S; ++k2) {
                if (k2 == ks) continue;
                const int32_t *other = partials + (((tile * S + k2) * (4 * KG) + bw) * EPW) * 256 + lane * 4;
#pragma unroll
                for (int i = 0; i < MFK; ++i) {
                    if (!live(i)) continue;
                    v4i v[2][4];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const int32_t *frag = other + (i * 2 + t) * 4 * 256;
                        v[t][0] = load_sc1_x4<0>(frag);
                        v[t][1] = load_sc1_x4<1024>(frag);
                        v[t][2] = load_sc1_x4<2048>(frag);
                        v[t][3] = load_sc1_x4<3072>(frag);
                    }
                    wait_vmcnt0(v[0][0], v[0][1], v[0][2], v[0][3]);
                    wait_vmcnt0(v[1][0], v[1][1], v[1][2], v[1][3]);
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[MF0 + i][t][4 * q + e] += v[t][q][e];
                }
            }
            LQ_DSTAMP(6);
            if (threadIdx.x == 0)
                __hip_atomic_store(&pl.tickets[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (!active) return;
        store_tile<MFK>(*reinterpret_cast<const v16i(*)[MFK][2]>(&acc[MF0]), M, N, m0 + 32 * MF0,
                        64 * ng + 2 * j, lane, sx, sw, Y, ACC);
        LQ_DSTAMP(7);
    };
    if (KG == 1 || grp == 0)
        finish(std::integral_constant<int, 0>{});
    else
        finish(std::integral_constant<int, KG - 1>{});
}

template <bool G128, int KG, int TM = 128>
__device__ __forceinline__ void duo_block(
    const Place pl, const int bm, const int bn, int M, int N, int K, const int8_t *__restrict__ X,
    const float *__restrict__ sx, const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp,
    const float *__restrict__ sw, __half *__restrict__ Y, int32_t *__restrict__ ACC,
    int32_t *__restrict__ partials)
{
    if (TM == 64)
        duo_tile<G128, KG, 2, 64>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
    else if (M - 128 * bm <= 64)  // block-uniform
        duo_tile<G128, KG, 2>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
    else
        duo_tile<G128, KG, 4>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
}

template <bool G128, int KG, int TM = 128>
__global__ __launch_bounds__(256 * KG, KG == 1 ? 2 : 1) void w4a8_duo_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int blocks_m, int blocks_n,
    int32_t *__restrict__ partials, unsigned int *__restrict__ tickets)
{
    int bm, bn;
    block_coords(blocks_m, blocks_n, bm, bn);
    duo_block<G128, KG, TM>(grid_place(tickets), bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
}

// The same barrier for code that waits for its loads itself: a fence would also wait for
// every asynchronous load into LDS that is still in flight.
__device__ __forceinline__ void lds_barrier_raw()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ------------------------------------------------------------------------------------
// duo kernel, direct-to-LDS form (one k group per block, large grids).
//
// Same tiles, wave layout and k-step pipeline as duo_tile, but a deeper memory pipeline: the
// X stages go from global memory straight into LDS (global_load_lds, no staging registers,
// no LDS stores), four stages deep, and the registers this frees hold a third stage of W.
// Every load is then issued two full stages (64 MFMAs of this wave plus as many of the wave
// it shares the SIMD with) before its data is needed, instead of three to four k-steps.
//
// LDS stage: 128 rows x 128 bytes without padding.  One load instruction of a wave fills
// 1 KiB in lane order, which holds 8 rows; lane p of wave w carries, in load i, row
// 32 i + 8 w + r and 16-byte column c with r = (p >> 3) ^ (w & 1), c = (p & 7) ^ r.  Read
// back by fragments (lane = row), 16 consecutive rows of one column then fall on 16
// different 16-byte bank groups.
// ------------------------------------------------------------------------------------
template <bool G128, int MF>
__device__ __forceinline__ void duo_dl_tile(
    const Place pl, const int bm, const int bn, int M, int N, int K, const int8_t *__restrict__ X,
    const float *__restrict__ sx, const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp,
    const float *__restrict__ sw, __half *__restrict__ Y, int32_t *__restrict__ ACC,
    int32_t *__restrict__ partials)
{
    constexpr int KG = 1;  // (for the stamps of the experiments build)
    constexpr int XP = MF;
    constexpr int STAGE = 128 * 128;
    constexpr int PER_STAGE = XP + 6;  // loads of one stage: XP of X, 4 of codes, 2 of parameters
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    __shared__ int s_last;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = lane & 31, kb = lane >> 5;
    const int m0 = bm * 128;
    const int ng = bn * 4 + wave;
    const bool active = ng < (N >> 6);
    const int t0 = 2 * (active ? ng : (N >> 6) - 1);
    const int S = pl.S, ks = pl.ks;
    const int u_begin = (int)((long long)(K >> 8) * ks / S), u_end = (int)((long long)(K >> 8) * (ks + 1) / S);
    const int s_begin = 2 * u_begin;
    const int stages = 2 * (u_end - u_begin);
    const int stages_total = K >> 7;
    const int chunks_per_tile = K >> 6;

    LQ_DSTAMP(0);
#ifdef LQ_ABLATE  // experiments only: where the wave runs (XCC id, hardware id register)
    {
        const unsigned w_ = (blockIdx.y * gridDim.x + blockIdx.x) * (4 * KG) + (threadIdx.x >> 6);
        if ((threadIdx.x & 63) == 0 && w_ < 8192) {
            g_dbg_stamps[8 * w_ + 3] = __builtin_amdgcn_s_getreg(0xF814);
            g_dbg_stamps[8 * w_ + 4] = __builtin_amdgcn_s_getreg(0xF804);
        }
    }
#endif
    v16i acc[MF][2];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mf][t][r] = 0;

    const int8_t *xbase = X + (size_t)s_begin * 128;
    const int ld_r = (lane >> 3) ^ (wave & 1), ld_c = (lane & 7) ^ ld_r;
    uint32_t xg[XP];
#pragma unroll
    for (int i = 0; i < XP; ++i)
        xg[i] = (uint32_t)min(m0 + 32 * i + 8 * wave + ld_r, M - 1) * (uint32_t)K + 16 * ld_c;
    // wave-uniform bases plus 32-bit lane offsets: one address register serves all loads of a kind
    const char *wbase = reinterpret_cast<const char *>(Wp + ((size_t)t0 * chunks_per_tile + 2 * (size_t)s_begin) * 64);
    const char *pbase = reinterpret_cast<const char *>(gp) + ((size_t)t0 * stages_total + s_begin) * 32 * (G128 ? 2 : 4);
    const size_t wg_stride = (size_t)chunks_per_tile * 1024;
    const size_t pg_stride = (size_t)stages_total * 32 * (G128 ? 2 : 4);
    uint32_t wl = lane * 16;  // (not const: see issue_x)
    const uint32_t pl_off = j * (G128 ? 2 : 4);
    // fragment row j sits in 1 KiB piece j >> 3 at position 8 (r ^ (piece & 1)) + (c ^ r), r = j & 7
    const int8_t *xs = lds + (j >> 3) * 1024 + 128 * ((j & 7) ^ ((j >> 3) & 1));
    const int jr = j & 7;

    u32x4 wr[3][2][2];  // [stage mod 3][tile][chunk]
    UnitParams<G128> pr[3][2];
    v4i bf[2][2];
    v4i af[2][MF];

    // The asynchronous loads are written in assembly so that the compiler's own wait-count
    // bookkeeping does not see them (it would otherwise drain every load in flight before
    // each LDS read); this code waits for them itself, see stage().
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) void *)lds;
    auto issue_x = [&](int s, int buf) {
        s = min(s, stages - 1);
#if defined(LQ_ABLATE) && (LQ_DUO_ABL & 8)  // experiments only: every stage re-reads stage 0 (cache hits)
        s = 0;
#endif
        const uint32_t so = (uint32_t)s * 128;
#pragma unroll
        for (int i = 0; i < XP; ++i)
            asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         : "+v"(wl)  // untouched; makes the W loads that follow depend on this statement
                         : "v"(xg[i] + so), "s"(xbase), "s"(lds0 + buf * STAGE + (4 * i + wave) * 1024)
                         : "memory", "m0");
    };
    auto load_w = [&](int s, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
        s = min(s, stages - 1);
#if defined(LQ_ABLATE) && (LQ_DUO_ABL & 16)  // experiments only: every stage re-reads stage 0 (cache hits)
        s = 0;
#endif
        const uint32_t wo = wl + (uint32_t)s * 2048, po = pl_off + (uint32_t)s * (G128 ? 64 : 128);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const char *wb = wbase + t * wg_stride;
            const char *pb = pbase + t * pg_stride;
            w[t][0] = *reinterpret_cast<const u32x4 *>(wb + wo);
            w[t][1] = *reinterpret_cast<const u32x4 *>(wb + wo + 1024);
            if (G128)
                p[t].raw = *reinterpret_cast<const uint16_t *>(pb + po);
            else
                p[t].raw = *reinterpret_cast<const uint32_t *>(pb + po);
        }
    };
    auto build_b = [&](const u32x4 (&w)[2][2], const UnitParams<G128> (&p)[2], int c, int h, v4i (&b)[2]) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            uint32_t s2, a4;
            p[t].get(c, s2, a4);
            dequant_half(w[t][c], s2, a4, h, b[t]);
        }
    };
    auto read_a = [&](int buf, int c, int h, v4i (&a)[MF]) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
            a[mf] = *reinterpret_cast<const v4i *>(xs + 16 * ((4 * c + 2 * h + kb) ^ jr) + buf * STAGE + mf * 4096);
    };
    auto mma = [&](const v4i (&a)[MF], const v4i (&b)[2]) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int t = 0; t < 2; ++t) acc[mf][t] = mfma_i8(a[mf], b[t], acc[mf][t]);
    };
    // One stage: w_cur = W(s) on entry and W(s+3) on exit, w_nxt = W(s+1).  Loads in flight
    // when the stage reaches its barrier, oldest first: X(s+1), W(s+1), X(s+2), W(s+2); "at
    // most PER_STAGE in flight" therefore means that this wave's part of X(s+1) is in LDS.
    // That count holds as long as the compiler leaves the W loads where they are written.  It
    // may issue them later (never earlier than the X loads of their stage, see issue_x), so
    // the first use of W(s+1) also sits above the barrier: loads complete in order, and the
    // wait that the compiler puts in front of that use covers the older X(s+1) whatever it
    // did with the W loads.
    auto stage = [&](int s, u32x4 (&w_cur)[2][2], UnitParams<G128> (&p_cur)[2], u32x4 (&w_nxt)[2][2],
                     UnitParams<G128> (&p_nxt)[2], auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;  // one of the last stages: nothing left to prefetch
        const int buf = s & 3;
        read_a(buf, 0, 1, af[1]);
        build_b(w_cur, p_cur, 0, 1, bf[1]);
        mma(af[0], bf[0]);
        __builtin_amdgcn_sched_barrier(0);
        read_a(buf, 1, 0, af[0]);
        build_b(w_cur, p_cur, 1, 0, bf[0]);
        mma(af[1], bf[1]);
        __builtin_amdgcn_sched_barrier(0);
        read_a(buf, 1, 1, af[1]);
        build_b(w_cur, p_cur, 1, 1, bf[1]);
        mma(af[0], bf[0]);
        __builtin_amdgcn_sched_barrier(0);
        build_b(w_nxt, p_nxt, 0, 0, bf[0]);
        asm volatile("" : "+v"(bf[0][0]), "+v"(bf[0][1]));  // (keeps that use above the barrier)
        if (TAIL)
            wait_vmcnt0();
        else
            wait_vmcnt<PER_STAGE>();
        lds_barrier_raw();  // X(s+1) is complete and visible; every wave is done reading X(s-1)
        __builtin_amdgcn_sched_barrier(0);
        read_a((s + 1) & 3, 0, 0, af[0]);
        __builtin_amdgcn_sched_barrier(0);
        if (!TAIL) issue_x(s + 3, (s + 3) & 3);  // into the stage that held X(s-1)
        if (!TAIL) load_w(s + 3, w_cur, p_cur);
        mma(af[1], bf[1]);
        __builtin_amdgcn_sched_barrier(0);
    };
    const std::false_type body{};
    const std::true_type tail{};

    issue_x(0, 0);
    load_w(0, wr[0], pr[0]);
    __builtin_amdgcn_sched_barrier(0);
    issue_x(1, 1);
    load_w(1, wr[1], pr[1]);
    __builtin_amdgcn_sched_barrier(0);
    issue_x(2, 2);
    load_w(2, wr[2], pr[2]);
    __builtin_amdgcn_sched_barrier(0);
    build_b(wr[0], pr[0], 0, 0, bf[0]);
    asm volatile("" : "+v"(bf[0][0]), "+v"(bf[0][1]));
    wait_vmcnt<2 * PER_STAGE>();
    lds_barrier_raw();
    read_a(0, 0, 0, af[0]);
    __builtin_amdgcn_sched_barrier(0);

    LQ_DSTAMP(1);
    // Three stages per trip (one turn of the W registers) without branches inside, so that
    // every load stays where the in-flight count above expects it; the one or two stages
    // that may be left over run after the loop, waiting for everything still in flight.
    int s = 0;
    for (; s + 3 <= stages; s += 3) {
        stage(s, wr[0], pr[0], wr[1], pr[1], body);
        stage(s + 1, wr[1], pr[1], wr[2], pr[2], body);
        stage(s + 2, wr[2], pr[2], wr[0], pr[0], body);
    }
    if (s < stages) stage(s, wr[0], pr[0], wr[1], pr[1], tail);
    if (s + 1 < stages) stage(s + 1, wr[1], pr[1], wr[2], pr[2], tail);
    // the (clamped) prefetches past the last stage write LDS too: they must have landed
    // before the block ends and its LDS goes to another block
    wait_vmcnt0();
    LQ_DSTAMP(2);

    if (S > 1) {
        // grid-level split-K: same protocol and workspace layout as duo_tile with one k group
        constexpr int EPW = 4 * 8;
        const size_t tile = pl.gx;
        int32_t *mine = partials + (((tile * S + ks) * 4 + wave) * EPW) * 256 + lane * 4;
        auto live = [&](int i) { return m0 + 32 * i < M; };
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            if (!live(i)) continue;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                int32_t *frag = mine + (i * 2 + t) * 4 * 256;
                auto part = [&](int q) {
                    return v4i{acc[i][t][4 * q], acc[i][t][4 * q + 1], acc[i][t][4 * q + 2], acc[i][t][4 * q + 3]};
                };
                store_sc1_x4<0>(frag, part(0));
                store_sc1_x4<1024>(frag, part(1));
                store_sc1_x4<2048>(frag, part(2));
                store_sc1_x4<3072>(frag, part(3));
            }
        }
        wait_vmcnt0();
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned tk = __hip_atomic_fetch_add(&pl.tickets[tile], 1u, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
            s_last = (tk == (unsigned)(S - 1));
        }
        __syncthreads();
        if (!s_last) return;
        for (int k2 = 0; k2 < S; ++k2) {
            if (k2 == ks) continue;
            const int32_t *other = partials + (((tile * S + k2) * 4 + wave) * EPW) * 256 + lane * 4;
#pragma unroll
            for (int i = 0; i < MF; ++i) {
                if (!live(i)) continue;
                v4i v[2][4];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int32_t *frag = other + (i * 2 + t) * 4 * 256;
                    v[t][0] = load_sc1_x4<0>(frag);
                    v[t][1] = load_sc1_x4<1024>(frag);
                    v[t][2] = load_sc1_x4<2048>(frag);
                    v[t][3] = load_sc1_x4<3072>(frag);
                }
                wait_vmcnt0(v[0][0], v[0][1], v[0][2], v[0][3]);
                wait_vmcnt0(v[1][0], v[1][1], v[1][2], v[1][3]);
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[i][t][4 * q + e] += v[t][q][e];
            }
        }
        if (threadIdx.x == 0)
            __hip_atomic_store(&pl.tickets[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!active) return;
    store_tile<MF>(acc, M, N, m0, 64 * ng + 2 * j, lane, sx, sw, Y, ACC);
    LQ_DSTAMP(7);
}

template <bool G128>
__global__ __launch_bounds__(256, 2) void w4a8_duo_dl_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int blocks_m, int blocks_n,
    int32_t *__restrict__ partials, unsigned int *__restrict__ tickets)
{
    int bm, bn;
    block_coords(blocks_m, blocks_n, bm, bn);
    const Place pl = grid_place(tickets);
    if (M - 128 * bm <= 64)  // block-uniform
        duo_dl_tile<G128, 2>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
    else
        duo_dl_tile<G128, 4>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
}

// ------------------------------------------------------------------------------------
// W8A8 reference kernel (Sec. 3.2 / 7.3: the baseline without dequantisation that the paper
// measures W4A8 against), on the skeleton of the direct-to-LDS tiled kernel: same tiles,
// wave layout, X pipeline and epilogue; the B operand is the loaded INT8 register itself.
// A stage of W is 32 registers per wave (8 loads of 16 bytes per lane), so two stages are
// held instead of three and every load is issued one stage ahead.  No split-K: a reference
// for grids that fill the chip.
// ------------------------------------------------------------------------------------
template <int MF>
__device__ __forceinline__ void w8a8_tile(const int bm, const int bn, int M, int N, int K,
                                          const int8_t *__restrict__ X, const float *__restrict__ sx,
                                          const u32x4 *__restrict__ W8, const float *__restrict__ sw,
                                          __half *__restrict__ Y, int32_t *__restrict__ ACC)
{
    constexpr int XP = MF;
    constexpr int STAGE = 128 * 128;
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = lane & 31, kb = lane >> 5;
    const int m0 = bm * 128;
    const int ng = bn * 4 + wave;
    const bool active = ng < (N >> 6);
    const int t0 = 2 * (active ? ng : (N >> 6) - 1);
    const int stages = K >> 7;

    v16i acc[MF][2];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mf][t][r] = 0;

    const int ld_r = (lane >> 3) ^ (wave & 1), ld_c = (lane & 7) ^ ld_r;
    uint32_t xg[XP];
#pragma unroll
    for (int i = 0; i < XP; ++i)
        xg[i] = (uint32_t)min(m0 + 32 * i + 8 * wave + ld_r, M - 1) * (uint32_t)K + 16 * ld_c;
    // tile t0 + t: K / 32 k-steps of 1 KiB each
    const char *wbase = reinterpret_cast<const char *>(W8) + (size_t)t0 * K * 32;
    const size_t w_stride = (size_t)K * 32;
    const uint32_t wl = lane * 16;
    const int8_t *xs = lds + (j >> 3) * 1024 + 128 * ((j & 7) ^ ((j >> 3) & 1));
    const int jr = j & 7;

    u32x4 wr[2][2][4];  // [stage parity][tile][k-step of the stage]
    v4i af[2][MF];

    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) void *)lds;
    auto issue_x = [&](int s, int buf) {
        s = min(s, stages - 1);
        const uint32_t so = (uint32_t)s * 128;
#pragma unroll
        for (int i = 0; i < XP; ++i)
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                         :
                         : "v"(xg[i] + so), "s"(X), "s"(lds0 + buf * STAGE + (4 * i + wave) * 1024)
                         : "memory", "m0");
    };
    auto load_w = [&](int s, u32x4 (&w)[2][4]) {
        s = min(s, stages - 1);
        const uint32_t wo = wl + (uint32_t)s * 4096;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const char *wb = wbase + t * w_stride;
#pragma unroll
            for (int q = 0; q < 4; ++q) w[t][q] = *reinterpret_cast<const u32x4 *>(wb + wo + q * 1024);
        }
    };
    auto read_a = [&](int buf, int q, v4i (&a)[MF]) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
            a[mf] = *reinterpret_cast<const v4i *>(xs + 16 * ((2 * q + kb) ^ jr) + buf * STAGE + mf * 4096);
    };
    auto mma = [&](const v4i (&a)[MF], const u32x4 (&w)[2][4], int q) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int t = 0; t < 2; ++t)
                acc[mf][t] = mfma_i8(a[mf], __builtin_bit_cast(v4i, w[t][q]), acc[mf][t]);
    };
    // One stage; loads in flight at its barrier: X(s+1), W(s+1) -- waited for completely.
    auto stage = [&](int s, u32x4 (&w_cur)[2][4], auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        const int buf = s & 3;
        read_a(buf, 1, af[1]);
        mma(af[0], w_cur, 0);
        __builtin_amdgcn_sched_barrier(0);
        read_a(buf, 2, af[0]);
        mma(af[1], w_cur, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_a(buf, 3, af[1]);
        mma(af[0], w_cur, 2);
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt0();
        lds_barrier_raw();
        __builtin_amdgcn_sched_barrier(0);
        read_a((s + 1) & 3, 0, af[0]);
        mma(af[1], w_cur, 3);
        __builtin_amdgcn_sched_barrier(0);
        if (!TAIL) issue_x(s + 2, (s + 2) & 3);
        if (!TAIL) load_w(s + 2, w_cur);
        __builtin_amdgcn_sched_barrier(0);
    };
    const std::false_type body{};
    const std::true_type tail{};

    issue_x(0, 0);
    load_w(0, wr[0]);
    __builtin_amdgcn_sched_barrier(0);
    issue_x(1, 1);
    load_w(1, wr[1]);
    __builtin_amdgcn_sched_barrier(0);
    // (everything, not a count: the compiler is free to issue the W loads above later than
    // written, which would shift a count)
    wait_vmcnt0();
    lds_barrier_raw();
    read_a(0, 0, af[0]);
    __builtin_amdgcn_sched_barrier(0);
    int s = 0;
    for (; s + 2 <= stages; s += 2) {  // stages is even (K % 256 == 0)
        stage(s, wr[0], body);
        stage(s + 1, wr[1], body);
    }
    (void)tail;
    wait_vmcnt0();  // the clamped prefetches past the end write LDS too

    if (!active) return;
    store_tile<MF>(acc, M, N, m0, 64 * ng + 2 * j, lane, sx, sw, Y, ACC);
}

__global__ __launch_bounds__(256, 2) void w8a8_kernel(int M, int N, int K, const int8_t *__restrict__ X,
                                                      const float *__restrict__ sx,
                                                      const u32x4 *__restrict__ W8,
                                                      const float *__restrict__ sw, __half *__restrict__ Y,
                                                      int32_t *__restrict__ ACC, int blocks_m, int blocks_n)
{
    int bm, bn;
    block_coords(blocks_m, blocks_n, bm, bn);
    if (M - 128 * bm <= 64)  // block-uniform
        w8a8_tile<2>(bm, bn, M, N, K, X, sx, W8, sw, Y, ACC);
    else
        w8a8_tile<4>(bm, bn, M, N, K, X, sx, W8, sw, Y, ACC);
}

// ------------------------------------------------------------------------------------
// Explicit coarse-grained pipeline (the ExCP of Sec. 5.1 that the paper argues against),
// built only to be measured against the kernels above: the waves of a block are
// specialised.  Waves 4..7 load W, dequantise it and write the INT8 operands to LDS; waves
// 0..3 read both operands from LDS and run the MFMAs; a block barrier per stage of 128 k
// hands a stage over.  Wave i and wave 4 + i share a SIMD, so dequantisation and matrix
// work overlap as in the other kernels -- what this form adds is the round trip of the
// dequantised weights through LDS (8 stores and 8 more loads of 16 bytes per lane and
// stage) and the coupling of all eight waves at every stage.  128 x 256 tiles, no
// split-K, every load handled by the compiler (X staged through registers).
// ------------------------------------------------------------------------------------
template <bool G128>
__global__ __launch_bounds__(512, 1) void w4a8_excp_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int blocks_m, int blocks_n)
{
    constexpr int XSTAGE = 128 * kTilePitch;  // X stage (padded rows, as in duo_tile)
    constexpr int BSTAGE = 4 * 2 * 4 * 1024;  // B stage: 4 waves x 2 tiles x 4 k-steps x (64 lanes x 16 B)
    constexpr int BOFF = 2 * XSTAGE;
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    int bm, bn;
    block_coords(blocks_m, blocks_n, bm, bn);
    const int tid = threadIdx.x & 255;
    const bool producer = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8)) != 0;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, kb = lane >> 5;
    const int m0 = bm * 128;
    const int ng = bn * 4 + wave;
    const bool active = ng < (N >> 6);
    const int t0 = 2 * (active ? ng : (N >> 6) - 1);
    const int stages = K >> 7;
    const int chunks_per_tile = K >> 6;
    int8_t *bmine = lds + BOFF + wave * (2 * 4 * 1024) + lane * 16;  // + buf * BSTAGE + (t * 4 + q) * 1024

    if (producer) {
        const int xrow = tid >> 3, xcol = tid & 7;
        uint32_t xg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) xg[i] = (uint32_t)min(m0 + xrow + 32 * i, M - 1) * (uint32_t)K + 16 * xcol;
        const int xl = xrow * kTilePitch + 16 * xcol;
        const u32x4 *wg0 = Wp + (size_t)t0 * chunks_per_tile * 64 + lane;
        const uint8_t *pg0 = gp + ((size_t)t0 * stages * 32 + j) * (G128 ? 2 : 4);
        const size_t wg_stride = (size_t)chunks_per_tile * 64;
        const size_t pg_stride = (size_t)stages * 32 * (G128 ? 2 : 4);
        u32x4 xr[4];
        u32x4 wr[2][2][2];
        UnitParams<G128> pr[2][2];
        auto load_x = [&](int s) {
            s = min(s, stages - 1);
#pragma unroll
            for (int i = 0; i < 4; ++i) xr[i] = *reinterpret_cast<const u32x4 *>(X + (size_t)s * 128 + xg[i]);
        };
        auto store_x = [&](int buf) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *reinterpret_cast<u32x4 *>(lds + buf * XSTAGE + xl + i * 32 * kTilePitch) = xr[i];
        };
        auto load_w = [&](int s, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
            s = min(s, stages - 1);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const u32x4 *wg = wg0 + t * wg_stride;
                const uint8_t *pg = pg0 + t * pg_stride;
                w[t][0] = wg[(size_t)s * 128];
                w[t][1] = wg[(size_t)s * 128 + 64];
                if (G128)
                    p[t].raw = *reinterpret_cast<const uint16_t *>(pg + (size_t)s * 64);
                else
                    p[t].raw = *reinterpret_cast<const uint32_t *>(pg + (size_t)s * 128);
            }
        };
        // dequantise one stage of this wave's two tiles into B stage `buf`
        auto produce = [&](const u32x4 (&w)[2][2], const UnitParams<G128> (&p)[2], int buf) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    uint32_t s2, a4;
                    p[t].get(c, s2, a4);
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        v4i b;
                        dequant_half(w[t][c], s2, a4, h, b);
                        *reinterpret_cast<v4i *>(bmine + buf * BSTAGE + (t * 4 + 2 * c + h) * 1024) = b;
                    }
                }
        };
        load_x(0);
        load_w(0, wr[0], pr[0]);
        load_w(1, wr[1], pr[1]);
        produce(wr[0], pr[0], 0);
        store_x(0);
        load_w(2, wr[0], pr[0]);
        lds_barrier();  // stage 0 is ready
        // during stage s the consumers work on stage s and this half produces stage s + 1
        auto stage = [&](int s, u32x4 (&w_nxt)[2][2], UnitParams<G128> (&p_nxt)[2]) {
            load_x(s + 1);
            produce(w_nxt, p_nxt, (s + 1) & 1);
            load_w(s + 3, w_nxt, p_nxt);
            store_x((s + 1) & 1);
            lds_barrier();
        };
        for (int s = 0; s < stages; s += 2) {  // stages is even
            stage(s, wr[1], pr[1]);
            stage(s + 1, wr[0], pr[0]);
        }
        return;
    }

    // consumers
    v16i acc[4][2];
#pragma unroll
    for (int mf = 0; mf < 4; ++mf)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mf][t][r] = 0;
    const int8_t *xs = lds + j * kTilePitch + 16 * kb;
    v4i af[2][4], bq[2][2];
    auto read_ab = [&](int s, int q, v4i (&a)[4], v4i (&b)[2]) {
        const int buf = s & 1;
#pragma unroll
        for (int mf = 0; mf < 4; ++mf)
            a[mf] = *reinterpret_cast<const v4i *>(xs + buf * XSTAGE + mf * 32 * kTilePitch + 32 * q);
#pragma unroll
        for (int t = 0; t < 2; ++t)
            b[t] = *reinterpret_cast<const v4i *>(bmine + buf * BSTAGE + (t * 4 + q) * 1024);
    };
    auto mma = [&](const v4i (&a)[4], const v4i (&b)[2]) {
#pragma unroll
        for (int mf = 0; mf < 4; ++mf)
#pragma unroll
            for (int t = 0; t < 2; ++t) acc[mf][t] = mfma_i8(a[mf], b[t], acc[mf][t]);
    };
    lds_barrier();  // stage 0 is ready
    read_ab(0, 0, af[0], bq[0]);
    for (int s = 0; s < stages; ++s) {
        read_ab(s, 1, af[1], bq[1]);
        mma(af[0], bq[0]);
        __builtin_amdgcn_sched_barrier(0);
        read_ab(s, 2, af[0], bq[0]);
        mma(af[1], bq[1]);
        __builtin_amdgcn_sched_barrier(0);
        read_ab(s, 3, af[1], bq[1]);
        mma(af[0], bq[0]);
        __builtin_amdgcn_sched_barrier(0);
        lds_barrier();  // stage s + 1 is ready, and the producers may overwrite stage s
        read_ab(s + 1, 0, af[0], bq[0]);
        mma(af[1], bq[1]);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (!active) return;
    store_tile<4>(acc, M, N, m0, 64 * ng + 2 * j, lane, sx, sw, Y, ACC);
}

// ------------------------------------------------------------------------------------
// Grouped launches (mixture-of-experts layers, Sec. 7.3): one launch runs the same per-block
// code over several experts that share N, K and the group size.  Expert i of the launch
// owns rows row_off[i] .. row_off[i] + rows[i] - 1 of X / Y and the expert[i]-th weight
// blob.  The table travels by value in the kernel arguments (no device copy, nothing to
// allocate), which bounds a call to 64 experts.
// ------------------------------------------------------------------------------------
constexpr int kMaxExperts = 64;
struct GroupTable {
    int count;
    int block_end[kMaxExperts];  // running total of blocks up to and including entry i
    int expert[kMaxExperts];
    int row_off[kMaxExperts];
    int rows[kMaxExperts];
};
struct GroupedPtrs {
    const int8_t *X;
    const float *sx;
    const u32x4 *Wp;
    const uint8_t *gp;
    const float *sw;
    __half *Y;
    int32_t *ACC;
    size_t w_stride;   // u32x4 elements between the packed codes of consecutive experts
    size_t gp_stride;  // bytes between their group parameters
};

template <int NW, int UU, bool G128>
__global__ __launch_bounds__(NW * 64) void w4a8_stream16_grouped_kernel(const GroupTable g, const GroupedPtrs p,
                                                                        int N, int K, int groups)
{
    const int i = blockIdx.x / groups, gx = blockIdx.x % groups;
    const int e = g.expert[i], r0 = g.row_off[i];
    stream16_block<2, NW, UU, G128>(Place{gx, groups, 0, 1, nullptr}, g.rows[i], N, K, p.X + (size_t)r0 * K, p.sx + r0,
                                    p.Wp + e * p.w_stride, p.gp + e * p.gp_stride, p.sw + (size_t)e * N,
                                    p.Y ? p.Y + (size_t)r0 * N : nullptr, p.ACC ? p.ACC + (size_t)r0 * N : nullptr,
                                    nullptr);
}

template <int NW, bool G128>
__global__ __launch_bounds__(NW * 64) void w4a8_stream_grouped_kernel(const GroupTable g, const GroupedPtrs p,
                                                                      int N, int K, int groups)
{
    const int i = blockIdx.x / groups, gx = blockIdx.x % groups;
    const int e = g.expert[i], r0 = g.row_off[i];
    stream_block<2, NW, 1, G128>(Place{gx, groups, 0, 1, nullptr}, g.rows[i], N, K, p.X + (size_t)r0 * K, p.sx + r0,
                              p.Wp + e * p.w_stride, p.gp + e * p.gp_stride, p.sw + (size_t)e * N,
                              p.Y ? p.Y + (size_t)r0 * N : nullptr, p.ACC ? p.ACC + (size_t)r0 * N : nullptr,
                              nullptr);
}

template <bool G128, int KG>
__global__ __launch_bounds__(256 * KG, KG == 1 ? 2 : 1) void w4a8_duo_grouped_kernel(const GroupTable g,
                                                                                     const GroupedPtrs p, int N,
                                                                                     int K)
{
    int i = 0;
    while (i < g.count - 1 && (int)blockIdx.x >= g.block_end[i]) ++i;
    const int local = (int)blockIdx.x - (i ? g.block_end[i - 1] : 0);
    const int M = g.rows[i], e = g.expert[i], r0 = g.row_off[i];
    // row tiles of one column block are neighbours, so they meet on the expert's W columns
    const int blocks_m = (M + 127) >> 7;
    const int bm = local % blocks_m, bn = local / blocks_m;
    duo_block<G128, KG>(Place{0, 1, 0, 1, nullptr}, bm, bn, M, N, K, p.X + (size_t)r0 * K, p.sx + r0,
                        p.Wp + e * p.w_stride, p.gp + e * p.gp_stride, p.sw + (size_t)e * N,
                        p.Y ? p.Y + (size_t)r0 * N : nullptr, p.ACC ? p.ACC + (size_t)r0 * N : nullptr, nullptr);
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
    void *ws;
    size_t ws_bytes;
};

typedef int (*LaunchFn)(const Args &);

template <class Kernel>
static int allow_lds(Kernel kernel, size_t bytes)
{
    if (bytes <= 48 * 1024) return LQ_OK;
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess)
        return fail(LQ_ERR_HIP, "hipFuncSetAttribute(%zu bytes of LDS): %s", bytes, hipGetErrorString(e));
    return LQ_OK;
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
template <int F, int NW, int MF>
static int launch_stream_as(const Args &a, int S, bool named)
{
    if (a.M > 32 * MF) return fail(LQ_ERR_INVALID, "this stream variant handles M <= %d, got %d", 32 * MF, a.M);
    if ((a.N / 32) % F != 0) return fail(LQ_ERR_INVALID, "N/32 not a multiple of F=%d", F);
    const int groups = a.N / (32 * F);
    S = std::max(1, std::min(S, a.K / 128));
    if (S > 1 && groups > kMaxTicketGroups) S = 1;
    size_t need = stream_ws_bytes(a.M, a.N, S, MF);
    if (need > 0 && (!a.ws || a.ws_bytes < need)) {
        if (named)
            return fail(LQ_ERR_WORKSPACE, "split-K needs %zu bytes of workspace, got %zu", need,
                        a.ws ? a.ws_bytes : 0);
        S = 1;
        need = 0;
    }
    const dim3 grid(groups, S), block(NW * 64);
    const int rmax = MF == 1 ? 4 * ((a.M + 7) / 8) : 16;
    const size_t lds_bytes = (size_t)NW * F * MF * rmax * 64 * sizeof(int);
    unsigned int *tickets = static_cast<unsigned int *>(a.ws);
    int32_t *partials = a.ws ? reinterpret_cast<int32_t *>(static_cast<char *>(a.ws) + kTicketBytes) : nullptr;
    if (a.group == 128) {
        if (int rc = allow_lds(&w4a8_stream_kernel<F, NW, MF, true>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_stream_kernel<F, NW, MF, true>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, partials, tickets);
    } else {
        if (int rc = allow_lds(&w4a8_stream_kernel<F, NW, MF, false>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_stream_kernel<F, NW, MF, false>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, partials, tickets);
    }
    return LQ_OK;
}

// SPLIT: 0 = choose with stream_split(), otherwise the fixed number of K slices.
template <int F, int NW, int SPLIT, int MF = 1>
static int launch_stream(const Args &a)
{
    return launch_stream_as<F, NW, MF>(a, SPLIT ? SPLIT : stream_split(a.N, a.K, F, NW), SPLIT != 0);
}

// 32-row (MF = 1) and 64-row (MF = 2) stream kernels with the block shape chosen from N.
// Measured for both: the best grid is the largest one of at most 256 blocks of 8 waves --
// one tile per block while N / 32 <= 256, else two -- with K split across blocks while
// that still fits.
template <int MF>
static int launch_stream_auto(const Args &a)
{
    const int tiles = a.N / 32;
    // long K with no room for K slices: two tiles per block share the X fragments and two
    // K slices halve each wave's walk (27 vs 31 us at 24 rows on 8192 x 28672)
    if (tiles > 128 && tiles <= 256 && a.K >= 16384) return launch_stream_as<2, 8, MF>(a, 2, false);
    if (tiles <= 256) return launch_stream_as<1, 8, MF>(a, std::min(4, 256 / tiles), false);
    return launch_stream_as<2, 8, MF>(a, std::min(4, 512 / tiles), false);
}

template <int F, int NW, int SPLIT, int ABL = 0, int UU = 1>
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
        if (int rc = allow_lds(&w4a8_stream16_kernel<F, NW, UU, true, ABL>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_stream16_kernel<F, NW, UU, true, ABL>), grid, block, lds_bytes, a.stream, a.M, a.N,
                           a.K, a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, partials, tickets);
    } else {
        if (int rc = allow_lds(&w4a8_stream16_kernel<F, NW, UU, false, ABL>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_stream16_kernel<F, NW, UU, false, ABL>), grid, block, lds_bytes, a.stream, a.M, a.N,
                           a.K, a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, partials, tickets);
    }
    return LQ_OK;
}

template <int MF>
static int launch_tile(const Args &a)
{
    constexpr int WM = 32 * MF;
    const int blocks_n = (a.N + 255) / 256, blocks_m = (a.M + WM - 1) / WM;
    const size_t lds_bytes = 2 * (size_t)WM * kTilePitch;
    const dim3 grid((unsigned)(blocks_n * blocks_m)), block(256);
    if (a.group == 128) {
        if (int rc = allow_lds(&w4a8_tile_kernel<MF, true>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_tile_kernel<MF, true>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n);
    } else {
        if (int rc = allow_lds(&w4a8_tile_kernel<MF, false>, lds_bytes)) return rc;
        hipLaunchKernelGGL((w4a8_tile_kernel<MF, false>), grid, block, lds_bytes, a.stream, a.M, a.N, a.K,
                           a.X, a.sx, a.Wp, a.gp, a.sw, a.Y, a.ACC, blocks_m, blocks_n);
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
    if (blocks_n * blocks_m > kMaxTicketGroups || S < 1) S = 1;
    size_t need = duo_ws_bytes(a.M, a.N, S, TM);
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

// the explicit producer / consumer form (measured only, never dispatched)
static int launch_excp(const Args &a)
{
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

// stream_f<F>_w<NW>[_s<S>]: F tiles per block, NW waves splitting the block's K slice,
// S grid-level K slices (chosen from the shape when not named).
static const Variant kVariants[] = {
    {"stream_f2_w8", &launch_stream<2, 8, 0>, 32, 2, 1},
    {"stream_f2_w8_s1", &launch_stream<2, 8, 1>, 32, 2, 1},
    {"stream_f2_w8_s2", &launch_stream<2, 8, 2>, 32, 2, 1},
    {"stream_f2_w8_s4", &launch_stream<2, 8, 4>, 32, 2, 1},
    {"stream_f1_w8_s1", &launch_stream<1, 8, 1>, 32, 1, 1},
    {"stream_f1_w8_s2", &launch_stream<1, 8, 2>, 32, 1, 1},
    {"stream_f1_w8_s4", &launch_stream<1, 8, 4>, 32, 1, 1},
    {"stream_m32", &launch_stream_auto<1>, 32, 2, 1},
    {"stream_m64", &launch_stream_auto<2>, 64, 2, 1},
    {"stream_m64_f2_w8", &launch_stream<2, 8, 0, 2>, 64, 2, 1},
    {"stream_m64_f2_w8_s1", &launch_stream<2, 8, 1, 2>, 64, 2, 1},
    {"stream_m64_f2_w8_s2", &launch_stream<2, 8, 2, 2>, 64, 2, 1},
    {"stream_m64_f2_w8_s4", &launch_stream<2, 8, 4, 2>, 64, 2, 1},
    {"stream_m64_f1_w8_s1", &launch_stream<1, 8, 1, 2>, 64, 1, 1},
    {"stream_m64_f1_w8_s2", &launch_stream<1, 8, 2, 2>, 64, 1, 1},
    {"stream16_f2_w8", &launch_stream16<2, 8, 0>, 16, 2, 1},
    {"stream16_f2_w4", &launch_stream16<2, 4, 0>, 16, 2, 1},
    {"stream16_f2_w8_s1", &launch_stream16<2, 8, 1>, 16, 2, 1},
    {"stream16_f2_w8_s2", &launch_stream16<2, 8, 2>, 16, 2, 1},
    {"stream16_f2_w8_s4", &launch_stream16<2, 8, 4>, 16, 2, 1},
    {"stream16_f1_w8", &launch_stream16<1, 8, 0>, 16, 1, 1},
    {"stream16_f1_w8_s1", &launch_stream16<1, 8, 1>, 16, 1, 1},
    {"stream16_f2_w16_s1", &launch_stream16<2, 16, 1>, 16, 2, 1},
    {"stream16_f1_w16_s1", &launch_stream16<1, 16, 1>, 16, 1, 1},
    {"stream16_f1_w8_u4", &launch_stream16<1, 8, 0, 0, 4>, 16, 1, 8},
    {"stream16_f1_w8_u4_s1", &launch_stream16<1, 8, 1, 0, 4>, 16, 1, 8},
    {"stream16_f1_w8_u4_s2", &launch_stream16<1, 8, 2, 0, 4>, 16, 1, 8},
    {"tile_m32", &launch_tile<1>, 0, 1, 1},
    {"tile_m64", &launch_tile<2>, 0, 1, 1},
    {"tile_m128", &launch_tile<4>, 0, 1, 1},
    {"duo_m128", &launch_duo<0, 0>, 0, 1, 1},
    {"duo_m128_s1", &launch_duo<1, 1>, 0, 1, 1},
    {"duo_m128_s2", &launch_duo<2, 1>, 0, 1, 1},
    {"duo_m128_s4", &launch_duo<4, 1>, 0, 1, 1},
    {"duo_m128_s8", &launch_duo<8, 1>, 0, 1, 1},
    {"duo_dl_m128", &launch_duo_dl<0>, 0, 1, 1},
    {"duo_dl_m128_s2", &launch_duo_dl<2>, 0, 1, 1},
    {"duo_dl_m128_s3", &launch_duo_dl<3>, 0, 1, 1},
    {"excp_m128", &launch_excp, 0, 1, 1},
    {"duo_m64", &launch_duo64<0>, 0, 1, 1, 512},
    {"duo_m64_s1", &launch_duo64<1>, 0, 1, 1, 512},
    {"duo_m64_s2", &launch_duo64<2>, 0, 1, 1, 512},
    {"duo_m64_s3", &launch_duo64<3>, 0, 1, 1, 512},
    {"duo_m64_s4", &launch_duo64<4>, 0, 1, 1, 512},
    {"duo_m128_g2", &launch_duo<0, 2>, 0, 1, 1},
    {"duo_m128_g2_s1", &launch_duo<1, 2>, 0, 1, 1},
    {"duo_m128_g2_s2", &launch_duo<2, 2>, 0, 1, 1},
    {"duo_m128_g2_s3", &launch_duo<3, 2>, 0, 1, 1},
    {"duo_m128_g2_s4", &launch_duo<4, 2>, 0, 1, 1},
    {"duo_m128_g2_s6", &launch_duo<6, 2>, 0, 1, 1},
#ifdef LQ_ABLATE
    {"abl_s16_noX", &launch_stream16<2, 4, 1, 1>, 16, 2, 1},
    {"abl_s16_noP", &launch_stream16<2, 4, 1, 2>, 16, 2, 1},
    {"abl_s16_noDq", &launch_stream16<2, 4, 1, 4>, 16, 2, 1},
    {"abl_s16_noRed", &launch_stream16<2, 4, 1, 8>, 16, 2, 1},
    {"abl_s16_noXP", &launch_stream16<2, 4, 1, 3>, 16, 2, 1},
    {"abl_s16_noXPDq", &launch_stream16<2, 4, 1, 7>, 16, 2, 1},
    {"abl_s16_onlyW", &launch_stream16<2, 4, 1, 15>, 16, 2, 1},
#endif
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

// Shape -> kernel.  Up to 32 rows the weights are streamed once with X fragments in
// registers (16-row MFMA shape up to 16 rows); anything larger runs the 128 x 256 tiles of
// the duo kernel, whose launcher adds in-block and grid-level split-K while the output
// alone gives at most one tile per CU.
static int select_variant(int M, int N, int K)
{
    if (M <= 16) {
        // small weight matrices are bound by launch and first-load latency: one tile per
        // block and all of a wave's loads (512 k) in flight at once
        if (K % 512 == 0 && K <= 8192 && N / 32 <= 256)
            return find_variant(M > 8 && K >= 4096 ? "stream16_f1_w16_s1" : "stream16_f1_w8_u4");
        // other matrices of up to 256 tiles: still one tile per block, and K slices across blocks
        if (N / 32 <= 256) return find_variant("stream16_f1_w8");
        return find_variant(N / 64 >= 384 ? "stream16_f2_w4" : "stream16_f2_w8");
    }
    if (M <= 32) return find_variant("stream_m32");
    // up to 64 rows the weights are still best streamed once per block column unless N alone
    // fills the chip with 128 x 256 tiles
    if (M <= 64 && N / 32 <= 512) {
        // ... except when N alone gives the stream kernel its 256 blocks (no K slices) and K is
        // long: each wave then walks K / 1024 units of 128 k at about 0.027 us per row, against
        // the tiled kernel's split-K grid (fits of measured times, microseconds)
        if (N / 32 >= 256 && K >= 8192) {
            const double est_stream = 7.5 + 0.027 * M * (K / 1024) * (N / 32 > 256 ? 1.15 : 1.0);
            const int S = duo_split(M, N, K);
            const double est_tiled = 0.85 * (8.1 + 1.76 * (K / 256) / (2.0 * S) + 2.4 * (S - 1));
            if (est_tiled < est_stream) return find_variant("duo_m128");
        }
        return find_variant("stream_m64");
    }
    // clearly more 128 x 256 tiles than CUs: the deeper memory pipeline of the direct-to-LDS
    // form pays (3 to 6 % measured from 320 tiles up); with one tile per CU or fewer, the two k
    // groups per block of the other form do
    if (((M + 127) / 128) * ((N + 255) / 256) >= 320 && (long long)M * K < (1ll << 32))
        return find_variant("duo_dl_m128");
    // few tiles: a grid of 64-row tiles can fill the chip with half the split-K exchange
    return find_variant(prefer_64_row_tiles(M, N, K) ? "duo_m64" : "duo_m128");
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

static int run(int variant, const Args &a)
{
    if (int rc = check_device_args(a)) return rc;
    if (a.M == 0) return LQ_OK;
    if (variant < 0) variant = select_variant(a.M, a.N, a.K);
    if (variant < 0 || variant >= kNumVariants) return fail(LQ_ERR_INVALID, "unknown variant %d", variant);
    if (!variant_supports(variant, a.M, a.N, a.K))
        return fail(LQ_ERR_INVALID, "variant %s cannot run M=%d N=%d K=%d", kVariants[variant].name, a.M, a.N,
                    a.K);
    (void)hipGetLastError();
    if (int rc = kVariants[variant].fn(a)) return rc;
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(LQ_ERR_HIP, "launch of %s failed: %s", kVariants[variant].name, hipGetErrorString(e));
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

static int grouped_run(const GroupedArgs &a)
{
    GroupTable small{}, mid{}, big{};
    long long big_blocks = 0;
    const int blocks_n = (a.N + 255) / 256;
    for (int e = 0; e < a.E; ++e) {
        const int r0 = a.row_offsets[e], rows = a.row_offsets[e + 1] - r0;
        if (rows == 0) continue;
        GroupTable &t = rows <= 16 ? small : (rows <= 32 ? mid : big);
        const int i = t.count++;
        t.expert[i] = e, t.row_off[i] = r0, t.rows[i] = rows;
        if (&t == &big) {
            big_blocks += (long long)((rows + 127) / 128) * blocks_n;
            if (big_blocks > 0x7fffffff) return fail(LQ_ERR_INVALID, "grouped GEMM too large for one launch");
            t.block_end[i] = (int)big_blocks;
        }
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
    if (big.count) {
        const dim3 grid((unsigned)big_blocks);
        // as for single GEMMs: two k groups per block while the grid gives at most one block per CU
        const bool kg2 = big_blocks <= 256 && a.K >= 512;
        const size_t lds1 = 2 * (size_t)128 * kTilePitch;
        const size_t lds2 = std::max<size_t>(2 * lds1, 64 * 1024);
        int rc;
        if (kg2)
            rc = g128 ? launch_checked("grouped duo", w4a8_duo_grouped_kernel<true, 2>, grid, dim3(512), lds2, a.stream,
                                       big, a.p, a.N, a.K)
                      : launch_checked("grouped duo", w4a8_duo_grouped_kernel<false, 2>, grid, dim3(512), lds2, a.stream,
                                       big, a.p, a.N, a.K);
        else
            rc = g128 ? launch_checked("grouped duo", w4a8_duo_grouped_kernel<true, 1>, grid, dim3(256), lds1, a.stream,
                                       big, a.p, a.N, a.K)
                      : launch_checked("grouped duo", w4a8_duo_grouped_kernel<false, 1>, grid, dim3(256), lds1, a.stream,
                                       big, a.p, a.N, a.K);
        if (rc) return rc;
    }
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

#ifdef LQ_ABLATE
int w4a8_debug_stamps(long long *host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_dbg_stamps), sizeof(long long) * n);
}
#endif

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
    for (int e = 0; e < E; ++e)
        if (row_offsets[e + 1] < row_offsets[e]) return fail(LQ_ERR_INVALID, "row_offsets must not decrease");
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
