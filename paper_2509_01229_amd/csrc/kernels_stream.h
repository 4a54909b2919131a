// stream and stream16 kernels (M <= 64): weights streamed once, K split between the waves of a block.
// (part of liquidgemm.hip: included there, inside namespace lqq)
#pragma once

// ------------------------------------------------------------------------------------
// stream kernel.  A unit is 128 k (two chunks per tile).  grid = (N / (32 F), S): block
// (bx, ks) owns F tiles and the ks-th of S slices of K; its NW waves take the slice's
// units round-robin.  S > 1 (grid-level split-K) is used when N alone gives too few blocks
// to keep every HBM channel busy; the S partial tiles meet in a workspace and the last
// block to arrive (a ticket per tile group) adds them up and runs the epilogue.  All sums
// are INT32, so neither level of split-K changes the result.
// ------------------------------------------------------------------------------------
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
//
// XL = the X fragments pass through LDS.  Read straight from global memory, one fragment
// load touches 32 rows, 16 bytes of each (32 cache lines for 1 KiB); with two row fragments
// these loads, not the weights, set the pace.  With XL a wave fetches its 32 MF rows x 128 k
// of a unit with loads that cover 8 whole rows each (8 lines per KiB), stores them to a
// region of LDS of its own and reads the fragments back from there.  The region is laid out
// like a stage of the direct-to-LDS tile kernel (1 KiB pieces of 8 rows, the 16-byte columns
// of a row rotated by an XOR with the row) so that neither the stores nor the fragment reads
// meet bank conflicts.
template <int F, int NW, int MF, bool G128, bool XL = false>
__device__ __forceinline__ void stream_block(
    const Place pl, int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int32_t *__restrict__ partials)
{
    extern __shared__ __attribute__((aligned(16))) int red[];  // [NW][F * MF * rmax][64]; XL: first the X regions
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
    // XL: load i of a unit (i = 0 .. 4 MF - 1) fills the 1 KiB piece i of the wave's region in
    // lane order; lane p brings row 8 i + r, 16-byte column c with r = (p >> 3) ^ (i & 1),
    // c = (p & 7) ^ r.  Fragment row j' = 32 mf + j is then found in piece j' >> 3 at
    // 128 ((j & 7) ^ (piece & 1)) + 16 (column ^ (j & 7)).
    int8_t *const xregion = reinterpret_cast<int8_t *>(red) + wave * (MF * 4096);
    const int8_t *const xfrag = xregion + (j >> 3) * 1024 + 128 * ((j & 7) ^ ((j >> 3) & 1));
    uint32_t xoff[XL ? 4 * MF : 1];
    if (XL) {
#pragma unroll
        for (int i = 0; i < 4 * MF; ++i) {
            const int r = (lane >> 3) ^ (i & 1), c = (lane & 7) ^ r;
            xoff[i] = (uint32_t)min(8 * i + r, M - 1) * (uint32_t)K + 16 * c;
        }
    }

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
                r.x[mf][ks4] = XL ? *reinterpret_cast<const u32x4 *>(X + ((size_t)xoff[XL ? 4 * mf + ks4 : 0] + (size_t)u * 128))
                                  : *reinterpret_cast<const u32x4 *>(xrow[mf] + (size_t)u * 128 + 32 * ks4);
    };
    auto compute_unit = [&](const StreamRegs<F, MF, G128> &r) {
        if (XL) {
#pragma unroll
            for (int mf = 0; mf < MF; ++mf)
#pragma unroll
                for (int ks4 = 0; ks4 < 4; ++ks4)
                    *reinterpret_cast<u32x4 *>(xregion + (4 * mf + ks4) * 1024 + 16 * lane) = r.x[mf][ks4];
        }
        auto frag = [&](int mf, int ks4) {
            return XL ? *reinterpret_cast<const v4i *>(xfrag + mf * 4096 + 16 * ((2 * ks4 + kb) ^ (j & 7)))
                      : __builtin_bit_cast(v4i, r.x[mf][ks4]);
        };
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
                    acc[f][mf] = mfma_i8(frag(mf, 2 * c), lo, acc[f][mf]);
                    acc[f][mf] = mfma_i8(frag(mf, 2 * c + 1), hi, acc[f][mf]);
                }
            }
    };

    // Register double buffering: the loads of the next unit are in flight while the
    // current one is dequantised and multiplied.
    StreamRegs<F, MF, G128> cur, nxt;
    int u = u_begin + wave;
    if (u < u_end) load_unit(u, cur);
    for (; u < u_end; u += NW) {
        const bool more = (u + NW) < u_end;
        if (more) load_unit(u + NW, nxt);
        compute_unit(cur);
        if (more) cur = nxt;
    }

    // In-block split-K reduction (integer, order independent).  With one row fragment only
    // the accumulator elements that hold rows < M take part: rows of element r lie in
    // [8*(r/4), 8*(r/4)+8).  Value v = (f * MF + mf) * rmax + r of lane l is row
    // 32*mf + acc_row(r, l), slot l%32 of tile t0 + f.
    const int rmax = MF == 1 ? 4 * ((M + 7) >> 3) : 16;
    if (XL) __syncthreads();  // the X regions are done with: the reduction takes the same LDS
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
        // all XCDs, so no cache has to be flushed or invalidated.  Every wave waits for the
        // acknowledgement of its own stores (a block barrier alone does not: it orders LDS
        // traffic only) before the barrier that precedes the ticket, so a block that sees
        // the last ticket also sees every partial tile.
        int32_t *mine = partials + ((size_t)ks * pl.gnx + pl.gx) * (size_t)(vals * 64);
        for (int idx = threadIdx.x; idx < vals * 64; idx += NW * 64)
            __hip_atomic_store(mine + idx, block_sum(idx), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        wait_vmcnt0();
        __syncthreads();
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
}

template <int F, int NW, int MF, bool G128, bool XL = false>
__global__ __launch_bounds__(NW * 64) void w4a8_stream_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int32_t *__restrict__ partials,
    unsigned int *__restrict__ tickets)
{
    stream_block<F, NW, MF, G128, XL>(grid_place(tickets), M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
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

template <int F, int NW, int UU, bool G128>
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
                r.p[f][q].load(gp, (size_t)(t0 + f) * units + (size_t)u * UU + q, j);
            }
        }
#pragma unroll
        for (int c = 0; c < 2 * UU; ++c)
            r.x[c] = *reinterpret_cast<const u32x4 *>(xrow + (size_t)u * (128 * UU) + 64 * c);
    };
    auto compute_unit = [&](const Stream16Regs<F, UU, G128> &r) {
#pragma unroll
        for (int f = 0; f < F; ++f)
#pragma unroll
            for (int c = 0; c < 2 * UU; ++c) {
                uint32_t s2, a4;
                r.p[f][c >> 1].get(c & 1, s2, a4);
                v4i lo, hi, b1, b2;
                dequant_chunk(r.w[f][c], s2, a4, lo, hi);
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
        // grid-level split-K: same protocol as w4a8_stream_kernel (stores acknowledged, then
        // the barrier, then the ticket)
        int32_t *mine = partials + ((size_t)ks * pl.gnx + pl.gx) * (size_t)(VALS * 64);
        for (int idx = threadIdx.x; idx < VALS * 64; idx += NW * 64)
            __hip_atomic_store(mine + idx, block_sum(idx), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        wait_vmcnt0();
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

template <int F, int NW, int UU, bool G128>
__global__ __launch_bounds__(NW * 64) void w4a8_stream16_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int32_t *__restrict__ partials,
    unsigned int *__restrict__ tickets)
{
    stream16_block<F, NW, UU, G128>(grid_place(tickets), M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
}

