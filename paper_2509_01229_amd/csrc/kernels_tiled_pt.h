// duo kernel, persistent form: resident blocks walk a list of output tiles.
// (part of liquidgemm.hip: included there, inside namespace lqq)
#pragma once

// ------------------------------------------------------------------------------------
// Persistent tiles (Sec. 5.4 of the paper: persistent kernel with a tile scheduler).
//
// The direct-to-LDS tile kernel spends a seventh of a wave's life outside its K loop: every
// tile starts with loads that nothing overlaps and ends with an epilogue that nothing
// follows.  Here the grid is one block per resident slot (two per CU) and block b computes
// tiles b, b + G, b + 2 G, ... as ONE stream of 128-k stages: the prefetches of the last
// stages of a tile already fetch the first stages of the next one (the load side runs three
// stages ahead of the compute side and has tile coordinates of its own), the four LDS stages
// and the W registers keep rotating across the tile boundary, and only the accumulators are
// drained in between.  So a block pays for one pipeline fill, however many tiles it computes.
//
// Same tile (128 x 256, wave tile 128 x 64), same LDS layout and the same pinned k-step as
// duo_dl_tile.  Differences: four register stages of W instead of three, so that the loop
// is unrolled by four and the LDS stage of every read is a compile-time constant (the
// fragment addresses are four lane-dependent bases plus immediates); a tile has a multiple of
// four stages (K % 512 == 0: the launcher sends other shapes to duo_dl_tile); every tile runs
// the four-fragment path (rows past M are computed on clamped loads and not stored).  The last
// stage of a tile leaves the first operands of the next stage unbuilt, so that the epilogue
// finds their registers free; they are built right after it.
// ------------------------------------------------------------------------------------
template <bool G128>
__global__ __launch_bounds__(256, 2) void w4a8_duo_pt_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int blocks_m, int blocks_n)
{
    constexpr int MF = 4;
    constexpr int STAGE = 128 * 128;
    constexpr int PER_STAGE = 4 + 6;  // loads of one stage: 4 of X, 4 of codes, 2 of parameters
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = lane & 31, kb = lane >> 5, jr = j & 7;
    const int stages = K >> 7;  // per tile, a multiple of four
    const int chunks_per_tile = K >> 6;
    const int tiles = blocks_m * blocks_n, G = (int)gridDim.x;

    // logical tile id -> (bm, bn): the ids of one XCD (hardware block id mod 8; b + i G keeps
    // it) form a contiguous range, walked four row blocks at a time (see block_coords)
    auto coords = [&](int lid, int &bm, int &bn) {
        if ((tiles & 7) == 0 && (G & 7) == 0) lid = (lid & 7) * (tiles >> 3) + (lid >> 3);
        constexpr int GM = 4;
        const int per_group = GM * blocks_n;
        const int first = (lid / per_group) * GM;
        const int gsz = min(blocks_m - first, GM);
        const int in_group = lid % per_group;
        bm = first + in_group % gsz;
        bn = in_group / gsz;
    };

    // ---- load side: the tile whose stages are being prefetched ------------------------------
    const int ld_r = (lane >> 3) ^ (wave & 1), ld_c = (lane & 7) ^ ld_r;
    const size_t wg_stride = (size_t)chunks_per_tile * 1024;
    const size_t pg_stride = (size_t)stages * 32 * (G128 ? 2 : 4);
    uint32_t wl = lane * 16;  // (not const: the X loads name it as an operand, see issue_x1)
    const uint32_t pl_off = j * (G128 ? 2 : 4);
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) void *)lds;
    int l_lid = (int)blockIdx.x, l_s = 0;  // tile and stage the next prefetch takes
    uint32_t xg[4];
    const char *wbase, *pbase;
    auto load_side_tile = [&](int lid) {
        int bm, bn;
        coords(lid, bm, bn);
        const int ng = bn * 4 + wave;
        const int t0 = 2 * min(ng, (N >> 6) - 1);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            xg[i] = (uint32_t)min(bm * 128 + 32 * i + 8 * wave + ld_r, M - 1) * (uint32_t)K + 16 * ld_c;
        wbase = reinterpret_cast<const char *>(Wp + (size_t)t0 * chunks_per_tile * 64);
        pbase = reinterpret_cast<const char *>(gp) + (size_t)t0 * stages * 32 * (G128 ? 2 : 4);
    };
    // after the last stage of the block's last tile the load side stays on that stage (the
    // prefetches past the end re-read it; nothing consumes them)
    auto load_side_advance = [&] {
        if (++l_s == stages) {
            asm volatile("" ::: "memory");  // (a real branch: none of this is worth computing speculatively in every stage)
            if (l_lid + G < tiles) {
                l_lid += G;
                l_s = 0;
                load_side_tile(l_lid);
            } else {
                l_s = stages - 1;
            }
        }
    };
    auto issue_x1 = [&](int buf, int i) {
        asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     : "+v"(wl)  // untouched; makes the W loads that follow depend on this statement
                     : "v"(xg[i]), "s"(X + (size_t)l_s * 128), "s"(lds0 + buf * STAGE + (4 * i + wave) * 1024)
                     : "memory", "m0");
    };
    // The W loads are written out like the X loads, so that the one wait of the stage loop is the
    // one written here (see w4a8_solo_pt_kernel: the compiler does not see the X loads, and its
    // own wait for a W register would also drain the X loads of the youngest stage, which keeps
    // a stage's loads from being spread over the stage).  The registers must not be touched
    // between a load and arrive_w: no kernel here may spill, and wr and pr are used in place.
    // piece 0, 1 = the codes of the stage's chunk 0, 1 of channel tile t, piece 2 = its group
    // parameters; the stage's offset goes into the scalar base.
    auto load_w_piece = [&](int t, int piece, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
        if (piece < 2) {
            const char *wb = wbase + t * wg_stride + (size_t)l_s * 2048 + piece * 1024;
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
        load_w_piece(t, 1, w, p);
        load_w_piece(t, 2, w, p);
    };
    // waits until at most PENDING loads of this wave are in flight; every use of (w, p) behind it
    auto arrive_w = [&](auto pending_tag, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
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
    u32x4 wr[4][2][2];  // [stage mod 4][tile][chunk]
    UnitParams<G128> pr[4][2];
    v4i bf[2][2];
    v4i a1[MF];
    uint32_t s2v[2], a4v[2];  // broadcast parameters of the chunk whose B operands are being built
    uint32_t tq[4];           // the four registers in flight through the phases of the dequantisation
    // fragment row j sits in 1 KiB piece j >> 3 at position 8 (r ^ (piece & 1)) + (c ^ r), r = j & 7;
    // one base per 16-byte column pair (c, h) of a stage, everything else is an immediate
    const int8_t *xs = lds + (j >> 3) * 1024 + 128 * ((j & 7) ^ ((j >> 3) & 1));
    const int8_t *xs_ch[2][2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int h = 0; h < 2; ++h) xs_ch[c][h] = xs + 16 * ((4 * c + 2 * h + kb) ^ jr);

    auto SB = [] { __builtin_amdgcn_sched_barrier(0); };
    auto mm = [&](int i, const v4i (&b)[2]) {
        acc[i >> 1][i & 1] = mfma_i8(a1[i >> 1], b[i & 1], acc[i >> 1][i & 1]);
    };
    auto rd = [&](int buf, int c, int h, int mf) {
        a1[mf] = *reinterpret_cast<const v4i *>(xs_ch[c][h] + buf * STAGE + mf * 4096);
    };
    auto ph_par = [&](const UnitParams<G128> (&p)[2], int c) {
        p[0].get(c, s2v[0], a4v[0]);
        p[1].get(c, s2v[1], a4v[1]);
    };
    auto ph_shr = [&](const u32x4 &w) {
#pragma unroll
        for (int d = 0; d < 4; ++d) tq[d] = w[d] >> 4;
    };
    auto ph_and_hi = [&] {
#pragma unroll
        for (int d = 0; d < 4; ++d) tq[d] &= 0x0F0F0F0Fu;
    };
    auto ph_and_lo = [&](const u32x4 &w) {
#pragma unroll
        for (int d = 0; d < 4; ++d) tq[d] = w[d] & 0x0F0F0F0Fu;
    };
    auto ph_mad = [&](int t) {
#pragma unroll
        for (int d = 0; d < 4; ++d) tq[d] = pk_mad_u16(tq[d], s2v[t], a4v[t]);
    };
    auto ph_xor = [&](v4i &b) {
#pragma unroll
        for (int d = 0; d < 4; ++d) b[d] = (int)(tq[d] ^ 0x80808080u);
    };
    // k-step that multiplies (a1, bc) and builds bn = B(c, 1) of w; (cb, cc, ch) = LDS stage,
    // chunk and half of the running k-step, (nb, nc, nh) of the next one (see duo_dl_tile)
    // ex(i): what else slot i carries (a piece of the prefetch: odd slots, the even ones read LDS)
    auto kstep_hi = [&](const v4i (&bc)[2], v4i (&bn)[2], const u32x4 (&w)[2][2], int c, int cb, int cc, int ch,
                        int nb, int nc, int nh, auto ex) {
        mm(0, bc); rd(cb, cc, ch, 3); ph_shr(w[0][c]); SB();
        mm(1, bc); ph_and_hi(); ex(1); SB();
        mm(2, bc); rd(nb, nc, nh, 0); ph_mad(0); SB();
        mm(3, bc); ph_xor(bn[0]); ex(3); SB();
        mm(4, bc); rd(nb, nc, nh, 1); ph_shr(w[1][c]); SB();
        mm(5, bc); ph_and_hi(); ex(5); SB();
        mm(6, bc); rd(nb, nc, nh, 2); ph_mad(1); SB();
        mm(7, bc); ph_xor(bn[1]); ex(7); SB();
    };
    auto kstep_lo = [&](const v4i (&bc)[2], v4i (&bn)[2], const u32x4 (&w)[2][2], const UnitParams<G128> (&p)[2],
                        int c, int cb, int cc, int ch, int nb, int nc, int nh, auto ex) {
        mm(0, bc); rd(cb, cc, ch, 3); ph_par(p, c); SB();
        mm(1, bc); ph_and_lo(w[0][c]); ex(1); SB();
        mm(2, bc); rd(nb, nc, nh, 0); ph_mad(0); SB();
        mm(3, bc); ph_xor(bn[0]); ex(3); SB();
        mm(4, bc); rd(nb, nc, nh, 1); ph_and_lo(w[1][c]); SB();
        mm(5, bc); ph_mad(1); ex(5); SB();
        mm(6, bc); rd(nb, nc, nh, 2); ph_xor(bn[1]); SB();
        mm(7, bc); ex(7); SB();
    };
    // builds bf[0] = B(0, 0) of stage set q and reads fragments 0..2 of its first k-step
    auto first_operands = [&](int q) {
        ph_par(pr[q], 0);
        ph_and_lo(wr[q][0][0]); ph_mad(0); ph_xor(bf[0][0]);
        ph_and_lo(wr[q][1][0]); ph_mad(1); ph_xor(bf[0][1]);
        rd(q, 0, 0, 0), rd(q, 0, 0, 1), rd(q, 0, 0, 2);
    };
    // One stage q (= stage mod 4: LDS stage and W register set; bf[0] holds its B(0, 0), a1 its
    // fragments 0..2 on entry).  In its last k-step: the stage barrier behind the second MFMA
    // (X of the next stage complete and visible; the LDS stage of the stage before released),
    // then the prefetch of the stage three ahead into that LDS stage and the free register set.
    // LAST = last stage of a tile: the first operands of the next stage are left to the caller.
    auto stage = [&](auto q_tag, auto last_tag) {
        constexpr int q = decltype(q_tag)::value, nq = (q + 1) & 3, gq = (q + 2) & 3, fq = (q + 3) & 3;
        constexpr bool LAST = decltype(last_tag)::value;
        // the seven later loads of the prefetch that the stage before began (into set gq)
        kstep_hi(bf[0], bf[1], wr[q], 0, q, 0, 0, q, 0, 1, [&](int i) {
            if (i == 1) issue_x1(gq, 3);
            if (i == 5) load_w_piece(0, 0, wr[gq], pr[gq]);
        });
        kstep_lo(bf[1], bf[0], wr[q], pr[q], 1, q, 0, 1, q, 1, 0, [&](int i) {
            if (i == 1) load_w_piece(0, 1, wr[gq], pr[gq]);
            if (i == 5) load_w_piece(0, 2, wr[gq], pr[gq]);
        });
        kstep_hi(bf[0], bf[1], wr[q], 1, q, 1, 0, q, 1, 1, [&](int i) {
            if (i == 1) load_w_piece(1, 0, wr[gq], pr[gq]);
            if (i == 3) load_w_piece(1, 1, wr[gq], pr[gq]);
            if (i == 5) load_w_piece(1, 2, wr[gq], pr[gq]);
        });
        load_side_advance();
        SB();
        // last k-step: X and W of the next stage have landed (the stage behind it may be in
        // flight), then the barrier (every wave's part of that X is visible, the LDS stage of the
        // stage before this one is released), then the first three loads of the prefetch of the
        // stage three ahead
        mm(0, bf[1]); rd(q, 1, 1, 3);
        arrive_w(std::integral_constant<int, PER_STAGE>{}, wr[nq], pr[nq]);
        if (!LAST) ph_par(pr[nq], 0);
        SB();
        mm(1, bf[1]); if (!LAST) ph_and_lo(wr[nq][0][0]);
        asm volatile("s_barrier" ::: "memory");
        SB();
        mm(2, bf[1]); if (!LAST) { rd(nq, 0, 0, 0); ph_mad(0); } SB();
        mm(3, bf[1]); if (!LAST) ph_xor(bf[0][0]); issue_x1(fq, 0); SB();
        mm(4, bf[1]); if (!LAST) { rd(nq, 0, 0, 1); ph_and_lo(wr[nq][1][0]); } SB();
        mm(5, bf[1]); if (!LAST) ph_mad(1); issue_x1(fq, 1); SB();
        mm(6, bf[1]); if (!LAST) { rd(nq, 0, 0, 2); ph_xor(bf[0][1]); } SB();
        mm(7, bf[1]); issue_x1(fq, 2); SB();
    };
    const std::integral_constant<int, 0> q0{};
    const std::integral_constant<int, 1> q1{};
    const std::integral_constant<int, 2> q2{};
    const std::integral_constant<int, 3> q3{};
    const std::false_type inner{};
    const std::true_type last{};

    // ---- pipeline fill: stages 0 and 1 of the first tile and the first three loads of stage 2 ----
    load_side_tile(l_lid);
#pragma unroll
    for (int q = 0; q < 2; ++q) {
#pragma unroll
        for (int i = 0; i < 4; ++i) issue_x1(q, i);
        load_w1(0, wr[q], pr[q]);
        load_w1(1, wr[q], pr[q]);
        __builtin_amdgcn_sched_barrier(0);
        load_side_advance();
    }
#pragma unroll
    for (int i = 0; i < 3; ++i) issue_x1(2, i);  // (the rest of stage 2 in the first three k-steps of stage 0)
    arrive_w(std::integral_constant<int, PER_STAGE + 3>{}, wr[0], pr[0]);  // and X(0) of this wave is in LDS
    asm volatile("s_barrier" ::: "memory");
    first_operands(0);
    __builtin_amdgcn_sched_barrier(0);

    // ---- the block's tiles ---------------------------------------------------------------------
    for (int lid = (int)blockIdx.x; lid < tiles; lid += G) {
        for (int it = 4; it < stages; it += 4) {
            stage(q0, inner);
            stage(q1, inner);
            stage(q2, inner);
            stage(q3, inner);
        }
        stage(q0, inner);
        stage(q1, inner);
        stage(q2, inner);
        stage(q3, last);
        // epilogue of the tile (the prefetches of the next tile's first stages are in flight)
        int bm, bn;
        coords(lid, bm, bn);
        const int ng = bn * 4 + wave;
        if (ng < (N >> 6)) store_tile<MF>(acc, M, N, bm * 128, 64 * ng + 2 * j, lane, sx, sw, Y, ACC);
        clear_acc();
        __builtin_amdgcn_sched_barrier(0);
        first_operands(0);  // of the next tile's first stage (harmless after the last tile)
        __builtin_amdgcn_sched_barrier(0);
    }
    // the prefetches past the last stage write LDS too: they must have landed before the block
    // ends and its LDS goes to another block
    wait_vmcnt0();
}
