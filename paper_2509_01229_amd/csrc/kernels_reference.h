// Measuring sticks: the W8A8 reference kernel and the explicit producer / consumer pipeline.
// (part of liquidgemm.hip: included there, inside namespace lqq)
#pragma once

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

