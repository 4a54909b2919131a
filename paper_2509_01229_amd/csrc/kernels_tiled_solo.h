// solo kernel: persistent tiles of 256 x 256, one wave per SIMD, 256 x 64 per wave.
// (part of liquidgemm.hip: included there, inside namespace lqq)
#pragma once

// ------------------------------------------------------------------------------------
// With two waves per SIMD and 128 x 64 per wave the tiled kernels issue 3.5 dequantisation
// instructions per MFMA, and measured without them the same kernel needs a sixth fewer cycles:
// an 8-pass MFMA leaves the SIMD's vector issue free for about four other instructions, and
// dequantisation plus addressing use all of them (paper Sec. 3.2: T_DQ per MMA shrinks with
// the rows that reuse a dequantised fragment; Eq. 6).  This kernel doubles that reuse instead
// of the waves: one wave per SIMD owns 256 rows x 64 channels, its 256 accumulator registers
// live in the accumulation half of the register file, and every dequantised B operand feeds
// eight MFMAs (1.75 dequantisation instructions per MFMA).  A single wave has nobody to cover
// its stalls, so everything is software-pipelined in one pinned instruction stream: per MFMA
// one half phase of the dequantisation (two instructions) and every second MFMA one fragment
// read, fragments refreshed in place 14 MFMAs ahead of their use, X and W prefetched three
// stages ahead, and -- as in duo_pt -- the block is persistent, so that the stream of stages
// continues across tile boundaries.
//
// Block = 4 waves (one per SIMD), tile 256 x 256, one block per CU; LDS = 4 stages of
// 256 rows x 128 bytes in the layout of duo_dl_tile (1 KiB pieces of 8 rows, 16-byte columns
// rotated by the row) plus two copies of a tile's 256 activation and 256 channel scales; four
// register stages of W.  K % 512 == 0.
//
// KG = 2 is the form for outputs with fewer 256 x 256 tiles than CUs: tile 256 x 128, the four
// waves are two k groups of two; both groups walk every stage, group g computing the stage's
// chunk g (64 of its 128 k) -- so the ring of four LDS stages still runs three stages ahead --
// and after the tile's last stage the groups exchange half of their accumulators through the
// (drained) LDS ring and each finishes four of the eight row fragments.  Tiles are separate
// there: the pipeline drains and refills between them.
// ------------------------------------------------------------------------------------
// One tile of a launch: rows bm * 256 .. of a matrix of M rows, channels bn * (256 / KG) ..,
// and of K slice ks (0 where K is not split across blocks)
struct SoloTile {
    int M, bm, bn, ks;
    const int8_t *X;
    const float *sx;
    const u32x4 *Wp;
    const uint8_t *gp;
    const float *sw;
    __half *Y;
    int32_t *ACC;
};
// Logical tile id of a persistent launch of G blocks -> position in a grid of blocks_m x blocks_n:
// the ids of one XCD (hardware block id mod 8; b + i G keeps it) form a contiguous range,
// walked four row blocks at a time (see block_coords).
__device__ __forceinline__ int solo_xcd_order(int lid, int tiles, int G)
{
    return (tiles & 7) == 0 && (G & 7) == 0 ? (lid & 7) * (tiles >> 3) + (lid >> 3) : lid;
}
__device__ __forceinline__ void solo_coords(int lid, int blocks_m, int blocks_n, int &bm, int &bn)
{
    constexpr int GM = 4;
    const int per_group = GM * blocks_n;
    const int first = (lid / per_group) * GM;
    const int gsz = min(blocks_m - first, GM);
    const int in_group = lid % per_group;
    bm = first + in_group % gsz;
    bn = in_group / gsz;
}
// The tiles of one GEMM.  With S > 1 every tile is computed in S equal K slices by S blocks,
// slice ks writing its INT32 partial sums to matrix ks of ACC ([S][M][N]; Y is null then) for
// splitk_finish_kernel to add up: the form for outputs with too few tiles for the chip
// (Sec. 3.2: the batch sizes between the memory-bound and the compute-bound regime).
struct SoloDense {
    int M, N;
    const int8_t *X;
    const float *sx;
    const u32x4 *Wp;
    const uint8_t *gp;
    const float *sw;
    __half *Y;
    int32_t *ACC;
    int blocks_m, blocks_n, S;
    __device__ __forceinline__ int slices() const { return S; }
    __device__ __forceinline__ int tiles() const { return blocks_m * blocks_n * S; }
    __device__ __forceinline__ SoloTile tile(int lid, int G) const
    {
        int bm, bn;
        const int per_slice = blocks_m * blocks_n;
        const int item = solo_xcd_order(lid, tiles(), G);  // an XCD's items: one slice (or part of one) of all tiles
        const int ks = item / per_slice;
        solo_coords(item - ks * per_slice, blocks_m, blocks_n, bm, bn);
        return SoloTile{M, bm, bn, ks, X, sx, Wp, gp, sw, Y, ACC + (size_t)ks * M * N};
    }
};

template <bool G128, int KG, class Src>
__device__ __forceinline__ void solo_body(const Src &src, const int N, const int K)
{
    constexpr int MF = 8;
    constexpr int STAGE = 256 * 128;
    constexpr int PER_STAGE = 8 + (KG == 1 ? 6 : 4);  // loads of one stage: 8 of X, 4 / KG of codes, 2 of parameters
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = lane & 31, kb = lane >> 5, jr = j & 7;
    const int grp = KG == 2 ? wave >> 1 : 0;          // KG = 2: the chunk of every stage this wave computes
    const int colw = KG == 2 ? (wave & 1) : wave;     // which 64 channels of the block's 256 / KG
    constexpr int WPB = 4 / KG;                       // 64-channel groups per block
    const int stages = (K >> 7) / src.slices();  // of a tile's K slice, a multiple of four
    const int chunks_per_tile = K >> 6;
    const int tiles = src.tiles(), G = (int)gridDim.x;

    // ---- load side: the tile whose stages are being prefetched ------------------------------
    const int ld_r = (lane >> 3) ^ (wave & 1), ld_c = (lane & 7) ^ ld_r;
    int ld_row = 8 * wave + ld_r;
    const size_t wg_stride = (size_t)chunks_per_tile * 1024;
    const size_t pg_stride = (size_t)(K >> 7) * 32 * (G128 ? 2 : 4);
    uint32_t wl = lane * 16;  // (not const: the X loads name it as an operand, see issue_x1)
    const uint32_t pl_off = j * (G128 ? 2 : 4);
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) void *)lds;
    int l_lid = (int)blockIdx.x, l_s = 0;  // tile and stage the next prefetch takes
    uint32_t xg[8];
    const char *wbase, *pbase;
    const int8_t *ld_X;
    auto load_side_tile = [&](int lid) {
        const SoloTile t = src.tile(lid, G);
        const int bm = t.bm, M = t.M;
        const int ng = t.bn * WPB + colw;
        const int t0 = 2 * min(ng, (N >> 6) - 1);
        // (recomputed from one register per tile: eight row numbers kept across the tile loop
        // would not fit beside the epilogue)
        asm volatile("" : "+v"(ld_row));
#pragma unroll
        for (int i = 0; i < 8; ++i)
            xg[i] = (uint32_t)min(bm * 256 + 32 * i + ld_row, M - 1) * (uint32_t)K + 16 * ld_c;
        const size_t s0 = (size_t)t.ks * stages;  // first stage of the K slice
        ld_X = t.X + s0 * 128;
        wbase = reinterpret_cast<const char *>(t.Wp + (size_t)t0 * chunks_per_tile * 64) + s0 * 2048;
        pbase = reinterpret_cast<const char *>(t.gp) + (size_t)t0 * pg_stride + s0 * (G128 ? 64 : 128);
    };
    // after the last stage of the block's last tile (KG = 2: of every tile) the load side stays
    // on that stage (the prefetches past the end re-read it; nothing consumes them)
    auto load_side_advance = [&] {
        if (++l_s == stages) {
            asm volatile("" ::: "memory");  // (a real branch: none of this is worth computing speculatively in every stage)
            if (KG == 1 && l_lid + G < tiles) {
                l_lid += G;
                l_s = 0;
                load_side_tile(l_lid);
            } else {
                l_s = stages - 1;
            }
        }
    };
    // piece i of a stage: rows 32 i + 8 wave .. + 7, into 1 KiB piece 4 i + wave of LDS stage buf
    auto issue_x1 = [&](int buf, int i) {
        asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     : "+v"(wl)  // untouched; makes the W loads that follow depend on this statement
                     : "v"(xg[i]), "s"(ld_X + (size_t)l_s * 128), "s"(lds0 + buf * STAGE + (4 * i + wave) * 1024)
                     : "memory", "m0");
    };
    // The W loads are written out as well, so that every wait of the stage loop is one that is
    // written here: the compiler does not see the X loads, and its own wait for a W register
    // would count only the W loads behind it -- far fewer than are in flight -- and so would
    // also wait for the X of the stage issued last.  With one wave per SIMD that wait is not
    // covered by anybody.  The registers must not be touched between load_w1 and arrive_w (the
    // compiler takes them for complete): no kernel here may spill, and wr and pr are written and
    // read in place.
    // piece 0, 1 = the codes of the stage's chunk 0, 1 of channel tile t (KG = 2: piece 0 = the
    // wave's own chunk, there is no piece 1), piece 2 = the tile's group parameters
    auto load_w_piece = [&](int t, int piece, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
        // (the stage's offset goes into the scalar base: the lane offsets stay what they are)
        if (piece < 2) {
            const char *wb = wbase + t * wg_stride + (size_t)l_s * 2048 + (KG == 2 ? grp * 1024 : piece * 1024);
            asm volatile("global_load_dwordx4 %0, %1, %2" : "=&v"(w[t][piece]) : "v"(wl), "s"(wb) : "memory");
        } else {
            const char *pb = pbase + t * pg_stride + (size_t)l_s * (G128 ? 64 : 128);
            if (G128)
                asm volatile("global_load_ushort %0, %1, %2" : "=&v"(p[t].raw) : "v"(pl_off), "s"(pb) : "memory");
            else
                asm volatile("global_load_dword %0, %1, %2" : "=&v"(p[t].raw) : "v"(pl_off), "s"(pb) : "memory");
        }
    };
    auto load_w1 = [&](int t, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
        load_w_piece(t, 0, w, p);
        if (KG == 1) load_w_piece(t, 1, w, p);
        load_w_piece(t, 2, w, p);
    };
    // waits until at most PENDING loads of this wave are in flight; every use of (w, p) behind it
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
    v16i acc[MF][2];
    auto clear_acc = [&] {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mf][t][r] = 0;
    };
    clear_acc();
    // one accumulator element, read where it sits (a copy of a whole 16-register fragment into
    // vector registers needs 16 contiguous free ones, which the allocator does not find here)
    auto acc_elem = [&](int mf, int t, int r) {
        int v;
        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[mf][t][r]));
        return v;
    };
    u32x4 wr[4][2][2];  // [stage mod 4][tile][chunk]
    UnitParams<G128> pr[4][2];
    v4i bf[2][2];
    v4i a1[MF];
    uint32_t s2v[2], a4v[2];  // broadcast parameters of the chunk whose B operands are being built
    uint32_t tq[4];           // the four registers of one tile in flight through the dequantisation
    // fragment row j of fragment mf sits in 1 KiB piece 4 mf + (j >> 3) at position
    // 8 (r ^ (piece & 1)) + (c ^ r), r = j & 7: one base per 16-byte column pair (c, h) and
    // half of the LDS (the offset field of an LDS read has 16 bits), the rest is an immediate
    const int8_t *xs = lds + (j >> 3) * 1024 + 128 * ((j & 7) ^ ((j >> 3) & 1));
    const int8_t *xs_ch[2][2][2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int h = 0; h < 2; ++h)  // (KG = 2: entry 0 is the wave's own chunk)
                xs_ch[u][c][h] = xs + u * (2 * STAGE) + 16 * ((4 * (KG == 2 ? grp : c) + 2 * h + kb) ^ jr);

    auto SB = [] { __builtin_amdgcn_sched_barrier(0); };
    auto mm = [&](int i, const v4i (&b)[2]) {
        acc[i >> 1][i & 1] = mfma_i8(a1[i >> 1], b[i & 1], acc[i >> 1][i & 1]);
    };
    auto rd = [&](int buf, int c, int h, int mf) {
        a1[mf] = *reinterpret_cast<const v4i *>(xs_ch[buf >> 1][c][h] + (buf & 1) * STAGE + mf * 4096);
    };
    // one half phase (registers 2 half, 2 half + 1 of a tile's four) of the dequantisation:
    // step 0 shift (high nibbles only), 1 mask, 2 multiply-add, 3 XOR
    auto dq_half = [&](int step, int half, int t, const u32x4 &w, v4i &b, bool hi) {
#pragma unroll
        for (int d = 2 * half; d < 2 * half + 2; ++d) {
            if (step == 0)
                tq[d] = w[d] >> 4;
            else if (step == 1)
                tq[d] = (hi ? tq[d] : w[d]) & 0x0F0F0F0Fu;
            else if (step == 2)
                tq[d] = pk_mad_u16(tq[d], s2v[t], a4v[t]);
            else
                b[d] = (int)(tq[d] ^ 0x80808080u);
        }
    };
    // slot i (0..15) of a k-step that builds bn = B(c, 1) of w: 16 half phases
    auto build_hi = [&](int i, const u32x4 (&w)[2][2], int c, v4i (&bn)[2]) {
        const int t = i >> 3, k = i & 7;
        dq_half(k >> 1, k & 1, t, w[t][c], bn[t], true);
    };
    // slot i of a k-step that builds bn = B(c, 0) of (w, p): parameters, then 12 half phases
    // (c = which of the stage's chunk registers, pc = which chunk's parameters: the same but for KG = 2)
    auto build_lo = [&](int i, const u32x4 (&w)[2][2], const UnitParams<G128> (&p)[2], int c, int pc, v4i (&bn)[2]) {
        if (i < 2) {
            p[i].get(pc, s2v[i], a4v[i]);
        } else if (i < 14) {
            const int t = (i - 2) / 6, k = (i - 2) % 6;
            dq_half(1 + (k >> 1), k & 1, t, w[t][c], bn[t], false);
        }
    };
    // Fragment mf is used by slots 2 mf and 2 mf + 1; fragment 7 of the running k-step is read
    // in its slot 0 and fragment mf of the next k-step in slot 2 mf + 2 (14 MFMAs ahead).
    // (cb, cc, ch) = LDS stage, chunk and half of the running k-step, (nb, nc, nh) of the next.
    // ex(i): what else slot i carries (a piece of the prefetch, the stage's wait and barrier)
    auto kstep_hi = [&](const v4i (&bc)[2], v4i (&bn)[2], const u32x4 (&w)[2][2], int c, int cb, int cc, int ch,
                        int nb, int nc, int nh, auto ex) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            mm(i, bc);
            if (i == 0)
                rd(cb, cc, ch, 7);
            else if (!(i & 1))
                rd(nb, nc, nh, i / 2 - 1);
            build_hi(i, w, c, bn);
            ex(i);
            SB();
        }
    };
    auto kstep_lo = [&](const v4i (&bc)[2], v4i (&bn)[2], const u32x4 (&w)[2][2], const UnitParams<G128> (&p)[2],
                        int c, int pc, int cb, int cc, int ch, int nb, int nc, int nh, auto ex) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            mm(i, bc);
            if (i == 0)
                rd(cb, cc, ch, 7);
            else if (!(i & 1))
                rd(nb, nc, nh, i / 2 - 1);
            if (i == 0) ex(-1);  // (before the slot's phase: the wait for the registers it expands)
            build_lo(i, w, p, c, pc, bn);
            ex(i);
            SB();
        }
    };
    // builds bf[0] = B(first chunk, 0) of stage set q and reads fragments 0..6 of its first k-step
    auto first_operands = [&](int q) {
#pragma unroll
        for (int i = 0; i < 14; ++i) build_lo(i, wr[q], pr[q], 0, grp, bf[0]);
#pragma unroll
        for (int mf = 0; mf < 7; ++mf) rd(q, 0, 0, mf);
    };
    // One stage q (= stage mod 4: LDS stage and W register set; bf[0] holds its B(0, 0), a1 its
    // fragments 0..6 on entry).  Its last k-step first waits for X and W of the next stage, then
    // meets the other waves (their parts of that X are visible; the LDS stage of the stage before
    // this one is released) and starts the prefetch of the stage three ahead into that LDS stage
    // and the free register set.  The 14 loads of a prefetch are spread over the 62 slots up to
    // the next stage's barrier -- four in the last k-step, ten in the first three of the next
    // stage: the four waves of a CU share one path from the L1, and all of a stage's loads
    // within one k-step ask twice what it delivers, which stalls the issue of every wave.  They
    // sit in odd slots, one load each: the even slots carry the fragment reads from LDS.
    // The next stage may belong to the block's next tile: its operands then wait in registers
    // while the epilogue runs (after the last tile they are those of a re-read stage, unused).
    auto stage = [&](auto q_tag) {
        constexpr int q = decltype(q_tag)::value, nq = (q + 1) & 3, gq = (q + 2) & 3, fq = (q + 3) & 3;
        if constexpr (KG == 2) {
            // two k-steps: the wave's chunk; the ten later loads of the running prefetch in the first
            kstep_hi(bf[0], bf[1], wr[q], 0, q, 0, 0, q, 0, 1, [&](int i) {
                if (i == 1) issue_x1(gq, 4);
                if (i == 3) issue_x1(gq, 5);
                if (i == 5) issue_x1(gq, 6);
                if (i == 7) issue_x1(gq, 7);
                if (i == 9) load_w_piece(0, 0, wr[gq], pr[gq]);
                if (i == 11) load_w_piece(0, 2, wr[gq], pr[gq]);
                if (i == 13) load_w_piece(1, 0, wr[gq], pr[gq]);
                if (i == 15) load_w_piece(1, 2, wr[gq], pr[gq]);
            });
            load_side_advance();
            SB();
            kstep_lo(bf[1], bf[0], wr[nq], pr[nq], 0, grp, q, 0, 1, nq, 0, 0, [&](int i) {
                if (i == -1) arrive_w(std::integral_constant<int, PER_STAGE>{}, wr[nq], pr[nq]);
                if (i == 1) asm volatile("s_barrier" ::: "memory");
                if (i == 3) issue_x1(fq, 0);
                if (i == 7) issue_x1(fq, 1);
                if (i == 11) issue_x1(fq, 2);
                if (i == 15) issue_x1(fq, 3);
            });
        } else {
        kstep_hi(bf[0], bf[1], wr[q], 0, q, 0, 0, q, 0, 1, [&](int i) {
            if (i == 3) issue_x1(gq, 4);
            if (i == 9) issue_x1(gq, 5);
            if (i == 15) issue_x1(gq, 6);
        });
        kstep_lo(bf[1], bf[0], wr[q], pr[q], 1, 1, q, 0, 1, q, 1, 0, [&](int i) {
            if (i == 5) issue_x1(gq, 7);
            if (i == 9) load_w_piece(0, 0, wr[gq], pr[gq]);
            if (i == 13) load_w_piece(0, 1, wr[gq], pr[gq]);
        });
        kstep_hi(bf[0], bf[1], wr[q], 1, q, 1, 0, q, 1, 1, [&](int i) {
            if (i == 1) load_w_piece(0, 2, wr[gq], pr[gq]);
            if (i == 5) load_w_piece(1, 0, wr[gq], pr[gq]);
            if (i == 9) load_w_piece(1, 1, wr[gq], pr[gq]);
            if (i == 13) load_w_piece(1, 2, wr[gq], pr[gq]);
        });
        load_side_advance();
        SB();
        kstep_lo(bf[1], bf[0], wr[nq], pr[nq], 0, 0, q, 1, 1, nq, 0, 0, [&](int i) {
            if (i == -1) arrive_w(std::integral_constant<int, PER_STAGE>{}, wr[nq], pr[nq]);
            if (i == 1) asm volatile("s_barrier" ::: "memory");
            if (i == 3) issue_x1(fq, 0);
            if (i == 7) issue_x1(fq, 1);
            if (i == 11) issue_x1(fq, 2);
            if (i == 15) issue_x1(fq, 3);
        });
        }
        // (the next stage's first B operand is complete here, also where the next stage is the
        // next trip of a loop: nothing of it may sink into the loop's latch)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int d = 0; d < 4; ++d) asm volatile("" : "+v"(bf[0][t][d]));
        SB();
    };
    const std::integral_constant<int, 0> q0{};
    const std::integral_constant<int, 1> q1{};
    const std::integral_constant<int, 2> q2{};
    const std::integral_constant<int, 3> q3{};

    // ---- epilogue of one tile (Sec. 4, first-level dequantisation: acc * s_x[row] * s_w[channel]) ----
    auto store_y = [&](uint32_t byte_off, uint32_t two_halves, const char *row) {
        asm volatile("global_store_dword %0, %1, %2" : : "v"(byte_off), "v"(two_halves), "s"(row) : "memory");
    };
    auto store_acc = [&](uint32_t byte_off, int a, int b, const char *row) {
        const uint64_t two = (uint32_t)a | ((uint64_t)(uint32_t)b << 32);
        asm volatile("global_store_dwordx2 %0, %1, %2" : : "v"(byte_off), "v"(two), "s"(row) : "memory");
    };
    // KG = 1: all eight fragments.  KG = 2: the four from MF0 on, each element the sum of this
    // wave's and of the other k group's, which lies in LDS at `other` ([fragment][channel tile]
    // [4 registers] x 64 lanes x 16 bytes).
    int M = 0;  // of the tile in its epilogue
    __half *Y = nullptr;
    int32_t *ACC = nullptr;
    auto epilogue = [&](auto full_tag, auto mf0_tag, int bm, int ng, const float *sx_tile, const float2 swv,
                        const int8_t *other) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr int MF0 = decltype(mf0_tag)::value;
        const uint32_t lane_off = (uint32_t)(4 * kb) * (uint32_t)N + (uint32_t)(64 * ng + 2 * j);  // in elements
#pragma unroll
        for (int mf = MF0; mf < MF0 + MF / KG; ++mf) {
            const int row0 = bm * 256 + 32 * mf;  // wave-uniform
            v4i add[2][4];
            if constexpr (KG == 2) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4)
                        add[t][q4] = *reinterpret_cast<const v4i *>(other + (((mf - MF0) * 2 + t) * 4 + q4) * 1024 + lane * 16);
            }
            auto element = [&](int t, int r) {
                if constexpr (KG == 2)
                    return acc_elem(mf, t, r) + add[t][r >> 2][r & 3];
                else
                    return acc_elem(mf, t, r);
            };
            if (Y) {
                float sxv[16];
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const float4 v = *reinterpret_cast<const float4 *>(sx_tile + 32 * mf + 8 * q4 + 4 * kb);
                    sxv[4 * q4 + 0] = v.x;
                    sxv[4 * q4 + 1] = v.y;
                    sxv[4 * q4 + 2] = v.z;
                    sxv[4 * q4 + 3] = v.w;
                }
                // (the two halves of a store go straight into one register -- low half, then high half
                // -- and the row base moves by additions: a lone wave pays for every instruction here)
                const size_t pitch = (size_t)N * 2;
                const char *row = reinterpret_cast<const char *>(Y) + (size_t)row0 * pitch;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ur = row0 + 8 * (r >> 2) + (r & 3);
                    const float x0 = (float)element(0, r) * sxv[r], x1 = (float)element(1, r) * sxv[r];
                    uint32_t two;  // fp16(x0 * s_w[n]) | fp16(x1 * s_w[n + 1]) << 16, each product rounded to FP32 first
                    asm("v_fma_mixlo_f16 %0, %1, %2, 0\n\tv_fma_mixhi_f16 %0, %3, %4, 0"
                        : "=&v"(two)
                        : "v"(x0), "v"(swv.x), "v"(x1), "v"(swv.y));
                    if (FULL || ur + 4 * kb < M) store_y(lane_off * 2, two, row);
                    row += (r & 3) == 3 ? 5 * pitch : pitch;
                }
            }
            if (ACC) {
                const size_t pitch = (size_t)N * 4;
                const char *row = reinterpret_cast<const char *>(ACC) + (size_t)row0 * pitch;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ur = row0 + 8 * (r >> 2) + (r & 3);
                    if (FULL || ur + 4 * kb < M) store_acc(lane_off * 4, element(0, r), element(1, r), row);
                    row += (r & 3) == 3 ? 5 * pitch : pitch;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // KG = 2: the four fragments from MF0 on go to this wave's 32 KiB of the LDS ring
    auto send_fragments = [&](auto mf0_tag) {
        constexpr int MF0 = decltype(mf0_tag)::value;
        int8_t *mine = lds + wave * STAGE + lane * 16;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *reinterpret_cast<v4i *>(mine + ((i * 2 + t) * 4 + q4) * 1024) =
                        v4i{acc_elem(MF0 + i, t, 4 * q4), acc_elem(MF0 + i, t, 4 * q4 + 1),
                            acc_elem(MF0 + i, t, 4 * q4 + 2), acc_elem(MF0 + i, t, 4 * q4 + 3)};
    };

    // ---- pipeline fill: stages 0 and 1 of a tile and the first four loads of stage 2 ----------
    auto fill = [&] {
        load_side_tile(l_lid);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
#pragma unroll
            for (int i = 0; i < 8; ++i) issue_x1(q, i);
            load_w1(0, wr[q], pr[q]);
            load_w1(1, wr[q], pr[q]);
            __builtin_amdgcn_sched_barrier(0);
            load_side_advance();
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) issue_x1(2, i);
        arrive_w(std::integral_constant<int, PER_STAGE + 4>{}, wr[0], pr[0]);  // and X(0) of this wave is in LDS
        asm volatile("s_barrier" ::: "memory");
        first_operands(0);
        __builtin_amdgcn_sched_barrier(0);
    };
    if (KG == 1) fill();

    // ---- the block's tiles ---------------------------------------------------------------------
    uint32_t sx_par = 0;  // which of the two copies of the tile's activation scales is this tile's
    for (int lid = (int)blockIdx.x; lid < tiles; lid += G) {
        const SoloTile cur = src.tile(lid, G);
        const int bm = cur.bm, ng = cur.bn * WPB + colw;
        M = cur.M, Y = cur.Y, ACC = cur.ACC;
        if (KG == 2) {
            l_lid = lid;
            l_s = 0;
            fill();
        }
        // The tile's 256 activation scales go to LDS now (64 per wave, rows past M take the last
        // row's): the epilogue of a single wave per SIMD would otherwise sit through the latency
        // of its scale loads once per fragment.  Complete and visible after the waits and
        // barriers of the first stages; two copies, so that a wave still in its epilogue is not
        // overtaken by the next tile's load.
        // (A call for the INT32 accumulators alone passes no scales.)
        if (Y) {
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                         :
                         : "v"((uint32_t)min(bm * 256 + 64 * wave + lane, M - 1) * 4u), "s"(cur.sx),
                           "s"(lds0 + 4 * STAGE + sx_par * 1024 + wave * 256)
                         : "memory", "m0");
            // (and the wave's 64 channel scales, for the same reason)
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                         :
                         : "v"((uint32_t)(64 * min(ng, (N >> 6) - 1) + lane) * 4u), "s"(cur.sw),
                           "s"(lds0 + 4 * STAGE + 2048 + sx_par * 1024 + wave * 256)
                         : "memory", "m0");
        }
        for (int it = 0; it < stages; it += 4) {
            stage(q0);
            stage(q1);
            stage(q2);
            stage(q3);
        }
        // epilogue of the tile (the prefetches of the next tile's first stages are in flight)
        const float *sx_tile = reinterpret_cast<const float *>(lds + 4 * STAGE + sx_par * 1024);
        const float2 swv = *reinterpret_cast<const float2 *>(lds + 4 * STAGE + 2048 + sx_par * 1024 + wave * 256 + 8 * j);
        sx_par ^= 1;
        // One fragment at a time, fenced: the accumulators sit in the accumulation registers, and
        // an epilogue free to read all 256 of them at once does not fit beside the prefetched W.
        // Element r of a fragment is row 8 (r >> 2) + 4 kb + (r & 3); a row's address is a
        // wave-uniform base (scalar registers) plus one 32-bit lane offset, which is the form
        // written out in store_y / store_acc.  A tile with all of its 256 rows inside M stores
        // without a test per row.
        // (acc_elem reads inside inline assembly, where the compiler does not count the wait
        // states an MFMA result needs before it is read: the last MFMA is further back than that
        // anyway, and this says so)
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
        const bool full = bm * 256 + 256 <= M;
        if constexpr (KG == 1) {
            const std::integral_constant<int, 0> f0{};
            if (ng < (N >> 6)) {
                if (full)
                    epilogue(std::true_type{}, f0, bm, ng, sx_tile, swv, nullptr);
                else
                    epilogue(std::false_type{}, f0, bm, ng, sx_tile, swv, nullptr);
            }
        } else {
            // every load of this tile has landed (those past its end too) and every wave is past
            // its last read of the ring: the ring is free for the exchange.  Group 0 finishes
            // fragments 0..3 and sends 4..7, group 1 the other way round.
            const std::integral_constant<int, 0> f0{};
            const std::integral_constant<int, 4> f4{};
            wait_vmcnt0();
            __syncthreads();
            if (grp == 0)
                send_fragments(f4);
            else
                send_fragments(f0);
            __syncthreads();
            const int8_t *other = lds + (wave ^ 2) * STAGE;
            if (ng < (N >> 6)) {
                if (grp == 0) {
                    if (full)
                        epilogue(std::true_type{}, f0, bm, ng, sx_tile, swv, other);
                    else
                        epilogue(std::false_type{}, f0, bm, ng, sx_tile, swv, other);
                } else {
                    if (full)
                        epilogue(std::true_type{}, f4, bm, ng, sx_tile, swv, other);
                    else
                        epilogue(std::false_type{}, f4, bm, ng, sx_tile, swv, other);
                }
            }
            __syncthreads();  // the ring is read; the next tile's fill may overwrite it
        }
        clear_acc();
        __builtin_amdgcn_sched_barrier(0);
    }
    // the prefetches past the last stage write LDS too: they must have landed before the block
    // ends and its LDS goes to another block
    wait_vmcnt0();
}

template <bool G128, int KG = 1>
__global__ __launch_bounds__(256, 1) void w4a8_solo_pt_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int blocks_m, int blocks_n, int S)
{
    solo_body<G128, KG>(SoloDense{M, N, X, sx, Wp, gp, sw, Y, ACC, blocks_m, blocks_n, S}, N, K);
}

// Adds up the S partial matrices of a launch with K slices and finishes the outputs like the
// tile epilogue does (Sec. 4: acc * s_x[row] * s_w[channel]).  Four channels per thread.
__global__ __launch_bounds__(256) void splitk_finish_kernel(
    const int32_t *__restrict__ part, int S, int M, int N, const float *__restrict__ sx,
    const float *__restrict__ sw, __half *__restrict__ Y, int32_t *__restrict__ ACC)
{
    const size_t quads = (size_t)M * N / 4, MN = (size_t)M * N;
    const size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= quads) return;
    v4i sum = *reinterpret_cast<const v4i *>(part + 4 * q);
#pragma unroll 4
    for (int s = 1; s < S; ++s) {
        const v4i v = *reinterpret_cast<const v4i *>(part + (size_t)s * MN + 4 * q);
        sum[0] += v[0], sum[1] += v[1], sum[2] += v[2], sum[3] += v[3];
    }
    if (ACC) *reinterpret_cast<v4i *>(ACC + 4 * q) = sum;
    if (Y) {
        const int m = (int)(4 * q / N), n = (int)(4 * q - (size_t)m * N);
        const float a = sx[m];
        const float4 w = *reinterpret_cast<const float4 *>(sw + n);
        uint2 out;
        out.x = scale_pair_to_half2((float)sum[0] * a, w.x, (float)sum[1] * a, w.y);
        out.y = scale_pair_to_half2((float)sum[2] * a, w.z, (float)sum[3] * a, w.w);
        *reinterpret_cast<uint2 *>(Y + 4 * q) = out;
    }
}
