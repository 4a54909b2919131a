// solo16 kernel: the persistent 256 x 256 tiles of the solo kernel on the 16x16x64 MFMA.
// (part of liquidgemm.hip: included there, inside namespace lqq, after kernels_tiled_solo.h)
#pragma once

// ------------------------------------------------------------------------------------
// Under operands that change from one MFMA to the next this chip is bound by its power, not by
// its matrix pipes, and the two INT8 MFMA shapes differ there: a loop of v_mfma_i32_16x16x64_i8
// on random bytes sustains 4.2 POP/s where v_mfma_i32_32x32x32_i8 sustains 3.5 (the small shape
// moves half the accumulator registers per operation).  This is the solo kernel (one wave per
// SIMD, wave tile 256 x 64, 256 accumulator registers, every dequantised operand reused by all
// 256 rows; paper Sec. 3.2, Eq. 6: T_DQ per MMA shrinks with that reuse) with the small shape:
//   * a k-step is one chunk of 64 k: 64 MFMAs, token fragment i / 4 (16 rows) times channel
//     fragment i % 4 (16 channels);
//   * the channel operands of a chunk come from the same two 16-byte lane loads as before: the
//     low and the high nibbles are dequantised as for the 32x32x32 order (Sec. 5.3, 7
//     instructions per 8 codes) and one v_permlane16_swap per register regroups them into the
//     operands of two 16-channel fragments (regroup_16x16), k blocks in the order 0, 2, 1, 3,
//     which the token fragments are read in as well (kstep16_offset);
//   * the weights are the MFMA's first operand, so that a lane receives four consecutive slots
//     of a tile for one token: with the even and the odd channels of the two tiles of a
//     64-channel group, 8 consecutive channels, stored as one 16-byte piece of FP16.
// Load side, LDS ring, scale staging and tile walk are those of solo_body.
//
// KG = 2 (tile 256 x 128 for outputs with fewer 256 x 256 tiles than CUs, as in solo_body): the
// four waves are two k groups of two, group g computes chunk g of every stage, so a stage is one
// k-step per wave: its slot 0 waits for the next stage's loads, slot 1 meets the other waves,
// and the 12 loads of the stage three ahead follow in the same k-step.  After the tile's last
// stage the groups exchange half of their accumulators through the drained LDS ring and each
// finishes eight of the sixteen token fragments.  Tiles are separate there (fill per tile).
// ------------------------------------------------------------------------------------
// f(integral_constant<int, B>), ..., f(integral_constant<int, E - 1>): the 64 slots of a k-step are
// written out this way -- a loop of that size is past what the compiler unrolls on request, and
// accumulators indexed by a loop counter would live in memory
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

template <bool G128, int KG, class Src>
__device__ __forceinline__ void solo16_body(const Src &src, const int N, const int K)
{
    constexpr int TF = 16;  // token fragments of 16 rows per wave
    constexpr int STAGE = 256 * 128;
    constexpr int PER_STAGE = 8 + (KG == 1 ? 6 : 4);  // loads of one stage: 8 of X, 4 / KG of codes, 2 of parameters
    constexpr int WPB = 4 / KG;                       // 64-channel groups per block
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = lane & 31;
    const int j16 = lane & 15, kq = lane >> 4;
    const int grp = KG == 2 ? wave >> 1 : 0;       // KG = 2: the chunk of every stage this wave computes
    const int colw = KG == 2 ? (wave & 1) : wave;  // which 64 channels of the block's 256 / KG
    // Stages of 128 k of a tile's K slice.  The stage loop runs them four at a time: where their
    // number is 2 mod 4 (K % 512 == 256, one slice), two stages are added whose loads re-read the
    // last real stage and whose group parameters are replaced, as they arrive, by those of an
    // all-zero group (s = 0, a = 128: (code * 0 + 128) XOR 0x80 = 0) -- they add nothing.
    const int stages_real = (K >> 7) / src.slices();
    const int stages = (stages_real + 3) & ~3;
    const bool has_pad = stages != stages_real;
    constexpr uint32_t kZeroGroup = G128 ? 0x8000u : 0x80008000u;
    const int chunks_per_tile = K >> 6;
    const int tiles = src.tiles(), G = (int)gridDim.x;

    // ---- load side (as in solo_body): the tile whose stages are being prefetched ------------
    const int ld_r = (lane >> 3) ^ (wave & 1), ld_c = (lane & 7) ^ ld_r;
    int ld_row = 8 * wave + ld_r;
    const size_t wg_stride = (size_t)chunks_per_tile * 1024;
    const size_t pg_stride = (size_t)(K >> 7) * 32 * (G128 ? 2 : 4);
    uint32_t wl = lane * 16;  // (not const: the X loads name it as an operand, see issue_x1)
    const uint32_t pl_off = j * (G128 ? 2 : 4);
    // lane offsets of the two channel tiles of a wave's 64 channels (a tile's codes and parameters
    // span less than 4 GiB: K < 2^22 here)
    uint32_t wl_t[2] = {wl, wl + (uint32_t)wg_stride}, pl_t[2] = {pl_off, pl_off + (uint32_t)pg_stride};
    asm volatile("" : "+v"(wl_t[0]), "+v"(wl_t[1]), "+v"(pl_t[0]), "+v"(pl_t[1]));
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) void *)lds;
    int l_lid = (int)blockIdx.x, l_s = 0;  // tile and stage the next prefetch takes
    int l_e = 0;                           // the stage it reads: l_s, or the last real one for an added stage
    uint32_t xg[8];
    const char *wbase, *pbase;
    const int8_t *ld_X;
    auto load_side_tile = [&](int lid) {
        const SoloTile t = src.tile(lid, G);
        const int bm = t.bm, M = t.M;
        const int ng = t.bn * WPB + colw;
        const int t0 = 2 * min(ng, (N >> 6) - 1);
        asm volatile("" : "+v"(ld_row));
#pragma unroll
        for (int i = 0; i < 8; ++i)
            xg[i] = (uint32_t)min(bm * 256 + 32 * i + ld_row, M - 1) * (uint32_t)K + 16 * ld_c;
        const size_t s0 = (size_t)t.ks * stages_real;  // first stage of the K slice
        ld_X = t.X + s0 * 128;
        wbase = reinterpret_cast<const char *>(t.Wp + (size_t)t0 * chunks_per_tile * 64) + s0 * 2048;
        pbase = reinterpret_cast<const char *>(t.gp) + (size_t)t0 * pg_stride + s0 * (G128 ? 64 : 128);
    };
    // The load side runs three stages ahead of the compute side and a tile's stages are a
    // multiple of four, so it reaches the end of a tile only behind a stage with q = 1 (KG = 2:
    // q = 0): the other stages advance without a test.  After the block's last tile (KG = 2: of
    // every tile) it falls back four stages and re-reads stages of that tile into LDS stages and
    // registers nobody reads any more.
    auto load_side_step = [&] {
        ++l_s;
        l_e = min(l_s, stages_real - 1);
    };
    auto load_side_advance = [&] {
        if (++l_s == stages) {
            asm volatile("" ::: "memory");
            if (KG == 1 && l_lid + G < tiles) {
                l_lid += G;
                l_s = 0;
                load_side_tile(l_lid);
            } else {
                l_s = stages - 4;
            }
        }
        l_e = min(l_s, stages_real - 1);
    };
    auto issue_x1 = [&](int buf, int i) {
        asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     : "+v"(wl)
                     : "v"(xg[i]), "s"(ld_X + (size_t)l_e * 128), "s"(lds0 + buf * STAGE + (4 * i + wave) * 1024)
                     : "memory", "m0");
    };
    // piece 0, 1 = the codes of the stage's chunk 0, 1 of channel tile t (KG = 2: piece 0 = the
    // wave's own chunk, there is no piece 1), piece 2 = its group parameters
    auto load_w_piece = [&](int t, int piece, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
        // (one scalar base per stage for the codes and one for the parameters: the tile is in
        // the lane offset, the chunk in the instruction's immediate)
        if (piece < 2) {
            const char *wb = wbase + (size_t)l_e * 2048 + (KG == 2 ? grp * 1024 : 0);
            if (piece == 0)
                asm volatile("global_load_dwordx4 %0, %1, %2" : "=&v"(w[t][piece]) : "v"(wl_t[t]), "s"(wb) : "memory");
            else
                asm volatile("global_load_dwordx4 %0, %1, %2 offset:1024" : "=&v"(w[t][piece]) : "v"(wl_t[t]), "s"(wb) : "memory");
        } else {
            const char *pb = pbase + (size_t)l_e * (G128 ? 64 : 128);
            if (G128)
                asm volatile("global_load_ushort %0, %1, %2" : "=&v"(p[t].raw) : "v"(pl_t[t]), "s"(pb) : "memory");
            else
                asm volatile("global_load_dword %0, %1, %2" : "=&v"(p[t].raw) : "v"(pl_t[t]), "s"(pb) : "memory");
        }
    };
    auto arrive_w = [&](auto pending_tag, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
        if (KG == 2)
            asm volatile("s_waitcnt vmcnt(%4)"
                         : "+v"(w[0][0]), "+v"(w[1][0]), "+v"(p[0].raw), "+v"(p[1].raw)
                         : "n"(decltype(pending_tag)::value)
                         : "memory");
        else
        asm volatile("s_waitcnt vmcnt(%6)"
                     : "+v"(w[0][0]), "+v"(w[0][1]), "+v"(w[1][0]), "+v"(w[1][1]), "+v"(p[0].raw), "+v"(p[1].raw)
                     : "n"(decltype(pending_tag)::value)
                     : "memory");
    };

    // ---- compute side ------------------------------------------------------------------------
    // acc[tf][2 t + h]: tokens 16 tf .. + 15 x slots 16 h .. + 15 of channel tile t; element v of
    // lane l = slot 16 h + 4 (l / 16) + v, token 16 tf + l % 16
    v4i acc[TF][4];
    auto clear_acc = [&] {
        static_for<0, 4 * TF>([&](auto i_tag) {
            constexpr int i = decltype(i_tag)::value;
            acc[i >> 2][i & 3] = v4i{0, 0, 0, 0};
            // (each in its own registers from the start: one zero shared by all of them would need
            // registers beyond the 256 the accumulators fill)
            asm volatile("" : "+a"(acc[i >> 2][i & 3]));
        });
    };
    clear_acc();
    asm volatile("s_nop 3" ::: "memory");  // (accumulation registers written by moves: wait states before an MFMA reads them)
    auto acc_elem = [&](int tf, int f, int v) {
        int x;
        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(acc[tf][f][v]));
        return x;
    };
    u32x4 wr[4][2][2];  // [stage mod 4][tile][chunk]
    UnitParams<G128> pr[4][2];
    v4i bw[2][4];  // channel operands of the running and of the next k-step
    v4i ax[8];     // token fragments: fragment tf in ax[tf % 8]
    uint32_t s2v, a4v;
    uint32_t lo[4], hi[4];  // one tile's registers on their way through the dequantisation
    // token row 16 tf + j16 of a stage: 1 KiB piece 2 tf + (j16 >> 3), row slot (j16 & 7) ^ (piece & 1),
    // 16-byte column (4 c + k block of this lane group) ^ (j16 & 7)
    const int8_t *xs = lds + (j16 >> 3) * 1024 + 128 * ((j16 & 7) ^ (j16 >> 3));
    const int8_t *xs_c[2][2];  // [LDS half][chunk] (KG = 2: entry 0 is the wave's own chunk)
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int c = 0; c < 2; ++c)
            xs_c[u][c] = xs + u * (2 * STAGE) + 16 * ((4 * (KG == 2 ? grp : c) + (kstep16_offset(kq) >> 4)) ^ (j16 & 7));

    auto SB = [] { __builtin_amdgcn_sched_barrier(0); };
    // (written out: the compiler's own choice for this shape is the form whose result may lie in
    // other registers than its addend, and with all 256 accumulation registers taken it then
    // moves accumulators through vector registers and memory.  Nothing here reads an accumulator
    // sooner than 63 MFMAs after it was written; the epilogue waits by itself.)
    auto mm = [&](int i, const v4i (&b)[4]) {
        asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+a"(acc[i >> 2][i & 3]) : "v"(b[i & 3]), "v"(ax[(i >> 2) & 7]));
    };
    // The same with piece xi of LDS stage buf of the X prefetch behind it: the MFMA is the wait
    // state the load needs after the write of m0.
    auto mm_x = [&](int i, const v4i (&b)[4], int buf, int xi) {
        asm volatile("s_mov_b32 m0, %4\n\tv_mfma_i32_16x16x64_i8 %0, %5, %6, %0\n\tglobal_load_lds_dwordx4 %2, %3"
                     : "+a"(acc[i >> 2][i & 3]), "+v"(wl)
                     : "v"(xg[xi]), "s"(ld_X + (size_t)l_e * 128), "s"(lds0 + buf * STAGE + (4 * xi + wave) * 1024),
                       "v"(b[i & 3]), "v"(ax[(i >> 2) & 7])
                     : "memory", "m0");
    };
    auto rd = [&](int buf, int c, int tf) {
        ax[tf & 7] = *reinterpret_cast<const v4i *>(xs_c[buf >> 1][c] + (buf & 1) * STAGE + tf * 2048);
    };
    // slot i (0..63) of a k-step that builds bn = the operands of chunk c of (w, p): per tile 32
    // slots -- parameters, 4 x and, 4 x shift, 4 x and, 8 x multiply-add, 8 x XOR, 4 x regroup
    // (KG = 2: the wave's chunk is the only one in its registers, entry 0)
    auto build = [&](int i, const u32x4 (&w)[2][2], const UnitParams<G128> (&p)[2], int c, v4i (&bn)[4]) {
        const int t = i >> 5, k = i & 31;
        const u32x4 &wc = w[t][KG == 2 ? 0 : c];
        auto regroup = [&](int d) {
            const auto r = __builtin_amdgcn_permlane16_swap(lo[d], hi[d], false, false);
            bn[2 * t][d] = (int)r[0];
            bn[2 * t + 1][d] = (int)r[1];
        };
        if (k == 0)
            p[t].get(c, s2v, a4v);
        else if (k <= 4)
            lo[k - 1] = wc[k - 1] & 0x0F0F0F0Fu;
        else if (k <= 8)
            hi[k - 5] = wc[k - 5] >> 4;
        else if (k <= 12)
            hi[k - 9] &= 0x0F0F0F0Fu;
        else if (k <= 16)
            lo[k - 13] = pk_mad_u16(lo[k - 13], s2v, a4v);
        else if (k <= 20)
            hi[k - 17] = pk_mad_u16(hi[k - 17], s2v, a4v);
        else if (k <= 24)
            lo[k - 21] ^= 0x80808080u;
        else if (k <= 28)
            hi[k - 25] ^= 0x80808080u;
        else if (k == 29)
            regroup(0);
        else if (k == 30)
            regroup(1);
        else {
            regroup(2);
            regroup(3);
        }
    };
    // Token fragment tf is used by slots 4 tf .. 4 tf + 3 and its register set is refilled in the
    // slot after with the fragment eight further on (28 MFMAs ahead of its use): slot 0 reads
    // fragment 7 of the running k-step, slots 4 .. 32 its fragments 8 .. 15, slots 36 .. 60
    // fragments 0 .. 6 of the next k-step.
    // (cb, cc) = LDS stage and chunk of the running k-step, (nb, nc) of the next.
    // ex(i): what else slot i carries (a piece of the W prefetch, the stage's wait and barrier);
    // xsl(i): 8 * LDS stage + piece of the X prefetch that slot i issues with its MFMA, or -1
    auto kstep = [&](const v4i (&bc)[4], v4i (&bn)[4], const u32x4 (&w)[2][2], const UnitParams<G128> (&p)[2], int c,
                     int cb, int cc, int nb, int nc, auto ex, auto xsl) {
        static_for<0, 64>([&](auto i_tag) {
            constexpr int i = decltype(i_tag)::value;
            if (xsl(i) >= 0)
                mm_x(i, bc, xsl(i) >> 3, xsl(i) & 7);
            else
                mm(i, bc);
            if (i == 0)
                rd(cb, cc, 7);
            else if (!(i & 3) && i <= 32)
                rd(cb, cc, i / 4 + 7);
            else if (!(i & 3))
                rd(nb, nc, i / 4 - 9);
            if (i == 0) ex(-1);  // (before the slot's phase: the wait for the registers it expands)
            build(i, w, p, c, bn);
            ex(i);
            SB();
        });
    };
    auto first_operands = [&](int q) {
        static_for<0, 64>([&](auto i_tag) { build(decltype(i_tag)::value, wr[q], pr[q], grp, bw[0]); });
        static_for<0, 7>([&](auto t_tag) { rd(q, 0, decltype(t_tag)::value); });
    };
    // One stage q (= stage mod 4: LDS stage and W register set; bw[0] holds the operands of its
    // chunk 0, ax its fragments 0..6 on entry): two k-steps.  The second first waits for X and W
    // of the next stage, then meets the other waves and starts the prefetch of the stage three
    // ahead; the 14 loads of a prefetch are spread over the 128 slots up to the next stage's barrier.
    bool tail_pad = false;  // this trip of the stage loop ends with the two added stages
    auto stage = [&](auto q_tag) {
        constexpr int q = decltype(q_tag)::value, nq = (q + 1) & 3, gq = (q + 2) & 3, fq = (q + 3) & 3;
        // the parameters that arrive in this stage are those of stage q + 1: an added stage's become
        // those of an all-zero group
        auto zero_added = [&] {
            if constexpr (q == 1 || q == 2) {
                if (tail_pad) pr[nq][0].raw = kZeroGroup, pr[nq][1].raw = kZeroGroup;
            }
        };
        if constexpr (KG == 2) {
            // one k-step: the wave's chunk of stage q, the operands of its chunk of the next stage
            // built beside it, and all 12 loads of the stage three ahead
            kstep(bw[q & 1], bw[~q & 1], wr[nq], pr[nq], grp, q, 0, nq, 0, [&](int i) {
                if (i == -1) arrive_w(std::integral_constant<int, PER_STAGE>{}, wr[nq], pr[nq]), zero_added();
                if (i == 1) asm volatile("s_barrier" ::: "memory");
                if (i == 50) load_w_piece(0, 0, wr[fq], pr[fq]);
                if (i == 53) load_w_piece(0, 2, wr[fq], pr[fq]);
                if (i == 57) load_w_piece(1, 0, wr[fq], pr[fq]);
                if (i == 61) load_w_piece(1, 2, wr[fq], pr[fq]);
            }, [&](int i) { return i >= 5 && i <= 47 && (i - 5) % 6 == 0 ? fq * 8 + (i - 5) / 6 : -1; });
            if (q == 0)
                load_side_advance();
            else
                load_side_step();
#pragma unroll
            for (int f = 0; f < 4; ++f)
#pragma unroll
                for (int d = 0; d < 4; ++d) asm volatile("" : "+v"(bw[~q & 1][f][d]));
            SB();
        } else {
        kstep(bw[0], bw[1], wr[q], pr[q], 1, q, 0, q, 1, [&](int i) {
            if (i == 27) load_w_piece(0, 0, wr[gq], pr[gq]);
            if (i == 33) load_w_piece(0, 1, wr[gq], pr[gq]);
            if (i == 39) load_w_piece(0, 2, wr[gq], pr[gq]);
            if (i == 45) load_w_piece(1, 0, wr[gq], pr[gq]);
            if (i == 51) load_w_piece(1, 1, wr[gq], pr[gq]);
            if (i == 57) load_w_piece(1, 2, wr[gq], pr[gq]);
        }, [&](int i) { return i == 3 ? gq * 8 + 4 : i == 9 ? gq * 8 + 5 : i == 15 ? gq * 8 + 6 : i == 21 ? gq * 8 + 7 : -1; });
        if (q == 1)
            load_side_advance();
        else
            load_side_step();
        SB();
        kstep(bw[1], bw[0], wr[nq], pr[nq], 0, q, 1, nq, 0, [&](int i) {
            if (i == -1) arrive_w(std::integral_constant<int, PER_STAGE>{}, wr[nq], pr[nq]), zero_added();
            if (i == 1) asm volatile("s_barrier" ::: "memory");
        }, [&](int i) { return i == 7 ? fq * 8 + 0 : i == 21 ? fq * 8 + 1 : i == 35 ? fq * 8 + 2 : i == 49 ? fq * 8 + 3 : -1; });
        // (the next stage's first operands are complete here, also where the next stage is the
        // next trip of a loop: nothing of them may sink into the loop's latch)
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int d = 0; d < 4; ++d) asm volatile("" : "+v"(bw[0][f][d]));
        SB();
        }
    };
    const std::integral_constant<int, 0> q0{};
    const std::integral_constant<int, 1> q1{};
    const std::integral_constant<int, 2> q2{};
    const std::integral_constant<int, 3> q3{};

    // ---- epilogue of one tile (Sec. 4, first-level dequantisation: acc * s_x[row] * s_w[channel]) ----
    // Of token 16 tf + j16 a lane holds, for h = 0, 1, the 8 consecutive channels
    // 64 ng + 32 h + 8 kq .. + 7: slot 16 h + 4 kq + v of the even (t = 0) and of the odd tile.
    int M = 0;
    __half *Y = nullptr;
    int32_t *ACC = nullptr;
    // KG = 1: all sixteen token fragments.  KG = 2: the eight from TF0 on, each element the sum of
    // this wave's and of the other k group's, which lies in LDS at `other` ([fragment][4 channel
    // fragments] x 64 lanes x 16 bytes).
    // The FP16 outputs and the INT32 sums are two passes over the accumulators (a call usually asks
    // for one of them): no test per fragment, the activation scales of all fragments read from LDS
    // up front, the row base moved by additions, the other group's sums fetched one fragment ahead.
    auto epilogue = [&](auto full_tag, auto tf0_tag, int bm, int ng, const float *sx_tile, const float *sw_wave,
                        const int8_t *other) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr int TF0 = decltype(tf0_tag)::value;
        constexpr int NF = TF / KG;
        const uint32_t lane_off = (uint32_t)j16 * (uint32_t)N + (uint32_t)(64 * ng + 8 * kq);  // in elements
        const int row_first = bm * 256 + 16 * TF0;  // wave-uniform
        v4i add[2][4];
        auto fetch_other = [&](int i) {
            if constexpr (KG == 2) {
#pragma unroll
                for (int f = 0; f < 4; ++f)
                    add[i & 1][f] = *reinterpret_cast<const v4i *>(other + (i * 4 + f) * 1024 + lane * 16);
            }
        };
        auto element = [&](int i, int f, int v) {
            if constexpr (KG == 2)
                return acc_elem(TF0 + i, f, v) + add[i & 1][f][v];
            else
                return acc_elem(TF0 + i, f, v);
        };
        if (Y) {
            float swv[2][8], sxv[NF];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int e4 = 0; e4 < 2; ++e4) {
                    const float4 v = *reinterpret_cast<const float4 *>(sw_wave + 32 * h + 8 * kq + 4 * e4);
                    swv[h][4 * e4 + 0] = v.x, swv[h][4 * e4 + 1] = v.y, swv[h][4 * e4 + 2] = v.z, swv[h][4 * e4 + 3] = v.w;
                }
#pragma unroll
            for (int i = 0; i < NF; ++i) sxv[i] = sx_tile[16 * (TF0 + i) + j16];
            const size_t step = (size_t)N * 32;  // bytes from one token fragment to the next
            const char *row = reinterpret_cast<const char *>(Y) + (size_t)row_first * ((size_t)N * 2);
            fetch_other(0);
            static_for<0, NF>([&](auto i_tag) {
                constexpr int i = decltype(i_tag)::value;
                if (i + 1 < NF) fetch_other(i + 1);
                const bool live = FULL || row_first + 16 * i + j16 < M;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    v4i out;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float x0 = (float)element(i, h, v) * sxv[i], x1 = (float)element(i, 2 + h, v) * sxv[i];
                        out[v] = (int)scale_pair_to_half2(x0, swv[h][2 * v], x1, swv[h][2 * v + 1]);
                    }
                    if (live) {
                        if (h == 0)
                            asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" : : "v"(lane_off * 2), "v"(out), "s"(row) : "memory");
                        else
                            asm volatile("global_store_dwordx4 %0, %1, %2 offset:64\n\ts_nop 1" : : "v"(lane_off * 2), "v"(out), "s"(row) : "memory");
                    }
                }
                row += step;
                asm volatile("" : "+s"(row));
                __builtin_amdgcn_sched_barrier(0);
            });
        }
        if (ACC) {
            const size_t step = (size_t)N * 64;
            const char *row = reinterpret_cast<const char *>(ACC) + (size_t)row_first * ((size_t)N * 4);
            fetch_other(0);
            static_for<0, NF>([&](auto i_tag) {
                constexpr int i = decltype(i_tag)::value;
                if (i + 1 < NF) fetch_other(i + 1);
                const bool live = FULL || row_first + 16 * i + j16 < M;
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int e4 = 0; e4 < 2; ++e4) {
                        const v4i out{element(i, h, 2 * e4), element(i, 2 + h, 2 * e4), element(i, h, 2 * e4 + 1),
                                      element(i, 2 + h, 2 * e4 + 1)};
                        if (live) {
                            if (h == 0 && e4 == 0)
                                asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" : : "v"(lane_off * 4), "v"(out), "s"(row) : "memory");
                            else if (h == 0)
                                asm volatile("global_store_dwordx4 %0, %1, %2 offset:16\n\ts_nop 1" : : "v"(lane_off * 4), "v"(out), "s"(row) : "memory");
                            else if (e4 == 0)
                                asm volatile("global_store_dwordx4 %0, %1, %2 offset:128\n\ts_nop 1" : : "v"(lane_off * 4), "v"(out), "s"(row) : "memory");
                            else
                                asm volatile("global_store_dwordx4 %0, %1, %2 offset:144\n\ts_nop 1" : : "v"(lane_off * 4), "v"(out), "s"(row) : "memory");
                        }
                    }
                row += step;
                asm volatile("" : "+s"(row));
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    };

    // KG = 2: the eight fragments from TF0 on go to this wave's 32 KiB of the LDS ring
    auto send_fragments = [&](auto tf0_tag) {
        constexpr int TF0 = decltype(tf0_tag)::value;
        int8_t *mine = lds + wave * STAGE + lane * 16;
        static_for<0, 32>([&](auto i_tag) {
            constexpr int i = decltype(i_tag)::value;
            *reinterpret_cast<v4i *>(mine + i * 1024) = v4i{acc_elem(TF0 + i / 4, i % 4, 0), acc_elem(TF0 + i / 4, i % 4, 1),
                                                            acc_elem(TF0 + i / 4, i % 4, 2), acc_elem(TF0 + i / 4, i % 4, 3)};
        });
    };

    // ---- pipeline fill: stages 0 and 1 of a tile and the first four loads of stage 2 (KG = 2:
    // stages 0, 1 and 2) ---------------------------------------------------------------------------
    auto fill = [&] {
        load_side_tile(l_lid);
#pragma unroll
        for (int q = 0; q < (KG == 2 ? 3 : 2); ++q) {
#pragma unroll
            for (int i = 0; i < 8; ++i) issue_x1(q, i);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                load_w_piece(t, 0, wr[q], pr[q]);
                if (KG == 1) load_w_piece(t, 1, wr[q], pr[q]);
                load_w_piece(t, 2, wr[q], pr[q]);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (KG == 2)
                load_side_step();
            else
                load_side_advance();
        }
        if (KG == 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i) issue_x1(2, i);
        }
        // X(0) of this wave is in LDS, W(0) in its registers
        arrive_w(std::integral_constant<int, KG == 2 ? 2 * PER_STAGE : PER_STAGE + 4>{}, wr[0], pr[0]);
        asm volatile("s_barrier" ::: "memory");
        first_operands(0);
        __builtin_amdgcn_sched_barrier(0);
    };
    if (KG == 1) fill();

    // ---- the block's tiles ---------------------------------------------------------------------
    uint32_t sx_par = 0;  // which of the two copies of the tile's scales is this tile's
    for (int lid = (int)blockIdx.x; lid < tiles; lid += G) {
        const SoloTile cur = src.tile(lid, G);
        const int bm = cur.bm, ng = cur.bn * WPB + colw;
        M = cur.M, Y = cur.Y, ACC = cur.ACC;
        if (KG == 2) {
            l_lid = lid;
            l_s = l_e = 0;
            fill();
        }
        // the tile's 256 activation scales and the wave's 64 channel scales go to LDS now (see solo_body)
        if (Y) {
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                         :
                         : "v"((uint32_t)min(bm * 256 + 64 * wave + lane, M - 1) * 4u), "s"(cur.sx),
                           "s"(lds0 + 4 * STAGE + sx_par * 1024 + wave * 256)
                         : "memory", "m0");
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                         :
                         : "v"((uint32_t)(64 * min(ng, (N >> 6) - 1) + lane) * 4u), "s"(cur.sw),
                           "s"(lds0 + 4 * STAGE + 2048 + sx_par * 1024 + wave * 256)
                         : "memory", "m0");
        }
        for (int it = 0; it < stages; it += 4) {
            tail_pad = has_pad && it + 4 >= stages;
            stage(q0);
            stage(q1);
            stage(q2);
            stage(q3);
        }
        const float *sx_tile = reinterpret_cast<const float *>(lds + 4 * STAGE + sx_par * 1024);
        const float *sw_wave = reinterpret_cast<const float *>(lds + 4 * STAGE + 2048 + sx_par * 1024 + wave * 256);
        sx_par ^= 1;
        // (the accumulators are read inside inline assembly, where the compiler does not count the
        // wait states an MFMA result needs before it is read)
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
        const bool full = bm * 256 + 256 <= M;
        const std::integral_constant<int, 0> f0{};
        if constexpr (KG == 1) {
            if (ng < (N >> 6)) {
                if (full)
                    epilogue(std::true_type{}, f0, bm, ng, sx_tile, sw_wave, nullptr);
                else
                    epilogue(std::false_type{}, f0, bm, ng, sx_tile, sw_wave, nullptr);
            }
        } else {
            // every load of this tile has landed (those past its end too) and every wave is past
            // its last read of the ring: the ring is free for the exchange.  Group 0 finishes
            // fragments 0..7 and sends 8..15, group 1 the other way round.
            const std::integral_constant<int, 8> f8{};
            wait_vmcnt0();
            __syncthreads();
            if (grp == 0)
                send_fragments(f8);
            else
                send_fragments(f0);
            __syncthreads();
            const int8_t *other = lds + (wave ^ 2) * STAGE;
            if (ng < (N >> 6)) {
                if (grp == 0) {
                    if (full)
                        epilogue(std::true_type{}, f0, bm, ng, sx_tile, sw_wave, other);
                    else
                        epilogue(std::false_type{}, f0, bm, ng, sx_tile, sw_wave, other);
                } else {
                    if (full)
                        epilogue(std::true_type{}, f8, bm, ng, sx_tile, sw_wave, other);
                    else
                        epilogue(std::false_type{}, f8, bm, ng, sx_tile, sw_wave, other);
                }
            }
            __syncthreads();  // the ring is read; the next tile's fill may overwrite it
        }
        clear_acc();
        asm volatile("s_nop 3" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    }
    // the prefetches past the last stage write LDS too: they must have landed before the block ends
    wait_vmcnt0();
}

template <bool G128, int KG = 1>
__global__ __launch_bounds__(256, 1) void w4a8_solo16_pt_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int blocks_m, int blocks_n, int S)
{
    solo16_body<G128, KG>(SoloDense{M, N, X, sx, Wp, gp, sw, Y, ACC, blocks_m, blocks_n, S}, N, K);
}
