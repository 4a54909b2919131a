// duo kernel, direct-to-LDS form.
// (part of liquidgemm.hip: included there, inside namespace lqq)
#pragma once

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
    // the same loads one piece / one tile at a time (for the pinned instruction order below)
    auto issue_x1 = [&](int s, int buf, int i) {
        s = min(s, stages - 1);
        asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     : "+v"(wl)
                     : "v"(xg[i % XP] + (uint32_t)s * 128), "s"(xbase), "s"(lds0 + buf * STAGE + (4 * i + wave) * 1024)
                     : "memory", "m0");
    };
    auto load_w1 = [&](int s, int t, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
        s = min(s, stages - 1);
        const uint32_t wo = wl + (uint32_t)s * 2048, po = pl_off + (uint32_t)s * (G128 ? 64 : 128);
        const char *wb = wbase + t * wg_stride;
        const char *pb = pbase + t * pg_stride;
        w[t][0] = *reinterpret_cast<const u32x4 *>(wb + wo);
        w[t][1] = *reinterpret_cast<const u32x4 *>(wb + wo + 1024);
        if (G128)
            p[t].raw = *reinterpret_cast<const uint16_t *>(pb + po);
        else
            p[t].raw = *reinterpret_cast<const uint32_t *>(pb + po);
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
    // ---- the four-fragment tile: the same stage with its instruction order pinned ----------
    // Left to itself the compiler emits the 8 MFMAs of a k-step in pairs and the dequantisation
    // in runs of 20 to 30 vector instructions (serialised through one temporary, with a wait
    // state between each packed multiply-add and its XOR), so the two waves of a SIMD often
    // have no matrix instruction to offer at the same time.  Here every MFMA is followed by one
    // phase of the dequantisation of one tile's four registers (shift, mask, multiply-add or
    // XOR: four independent instructions) and, in the first half of the k-step, one fragment
    // read from LDS; scheduling barriers keep that order.  An 8-pass MFMA leaves room for about
    // four other vector instructions, so this is the densest order the k-step allows.
    uint32_t s2v[2], a4v[2];  // broadcast parameters of the chunk whose B operands are being built
    uint32_t tq[4];           // the four registers in flight through the phases
    auto SB = [] { __builtin_amdgcn_sched_barrier(0); };
    auto mm = [&](int i, const v4i (&a)[MF], const v4i (&b)[2]) {
        acc[(i >> 1) % MF][i & 1] = mfma_i8(a[(i >> 1) % MF], b[i & 1], acc[(i >> 1) % MF][i & 1]);
    };
    auto rd = [&](int buf, int c, int h, int mf, v4i (&a)[MF]) {
        a[mf % MF] = *reinterpret_cast<const v4i *>(xs + 16 * ((4 * c + 2 * h + kb) ^ jr) + buf * STAGE + (mf % MF) * 4096);
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
    // A fragments are single-buffered and refreshed in place: fragment 3 of the running k-step
    // is read in its slot 0 (its registers were last used by slot 7 of the k-step before) and
    // fragments 0..2 of the next k-step in slots 2, 4 and 6, right behind their last use;
    // every read is six MFMAs ahead of its first use.  (cb, cc, ch) = LDS stage, chunk and half
    // of the running k-step, (nb, nc, nh) of the next one.
    v4i (&a1)[MF] = af[0];
    // k-step that multiplies (a1, bc) and builds bn = B(c, 1) of w
    auto kstep_hi = [&](const v4i (&bc)[2], v4i (&bn)[2], const u32x4 (&w)[2][2], int c, int cb, int cc, int ch,
                        int nb, int nc, int nh) {
        mm(0, a1, bc); rd(cb, cc, ch, 3, a1); ph_shr(w[0][c]); SB();
        mm(1, a1, bc); ph_and_hi(); SB();
        mm(2, a1, bc); rd(nb, nc, nh, 0, a1); ph_mad(0); SB();
        mm(3, a1, bc); ph_xor(bn[0]); SB();
        mm(4, a1, bc); rd(nb, nc, nh, 1, a1); ph_shr(w[1][c]); SB();
        mm(5, a1, bc); ph_and_hi(); SB();
        mm(6, a1, bc); rd(nb, nc, nh, 2, a1); ph_mad(1); SB();
        mm(7, a1, bc); ph_xor(bn[1]); SB();
    };
    // k-step that multiplies (a1, bc) and builds bn = B(c, 0) of (w, p)
    auto kstep_lo = [&](const v4i (&bc)[2], v4i (&bn)[2], const u32x4 (&w)[2][2], const UnitParams<G128> (&p)[2],
                        int c, int cb, int cc, int ch, int nb, int nc, int nh) {
        mm(0, a1, bc); rd(cb, cc, ch, 3, a1); ph_par(p, c); SB();
        mm(1, a1, bc); ph_and_lo(w[0][c]); SB();
        mm(2, a1, bc); rd(nb, nc, nh, 0, a1); ph_mad(0); SB();
        mm(3, a1, bc); ph_xor(bn[0]); SB();
        mm(4, a1, bc); rd(nb, nc, nh, 1, a1); ph_and_lo(w[1][c]); SB();
        mm(5, a1, bc); ph_mad(1); SB();
        mm(6, a1, bc); rd(nb, nc, nh, 2, a1); ph_xor(bn[1]); SB();
        mm(7, a1, bc); SB();
    };
    // One stage, same contract as stage() above (bf[0] holds B(0, 0) of the stage on entry and
    // of the next stage on exit).  The last k-step builds that next B(0, 0); the stage barrier
    // sits behind its second MFMA, before the first fragment read of the next stage, and the
    // prefetches follow the last MFMA.
    auto stage_pinned = [&](int s, u32x4 (&w_cur)[2][2], UnitParams<G128> (&p_cur)[2], u32x4 (&w_nxt)[2][2],
                            UnitParams<G128> (&p_nxt)[2], auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        const int buf = s & 3, nbuf = (s + 1) & 3;
        kstep_hi(bf[0], bf[1], w_cur, 0, buf, 0, 0, buf, 0, 1);
        kstep_lo(bf[1], bf[0], w_cur, p_cur, 1, buf, 0, 1, buf, 1, 0);
        kstep_hi(bf[0], bf[1], w_cur, 1, buf, 1, 0, buf, 1, 1);
        mm(0, a1, bf[1]); rd(buf, 1, 1, 3, a1); ph_par(p_nxt, 0); SB();
        mm(1, a1, bf[1]); ph_and_lo(w_nxt[0][0]);
        asm volatile("" : "+v"(tq[0]), "+v"(tq[1]), "+v"(tq[2]), "+v"(tq[3]));  // (that use of W(s+1) stays above the barrier, see stage())
        if (TAIL)
            wait_vmcnt0();
        else
            wait_vmcnt<PER_STAGE>();
        // X(s+1) is complete and visible and every wave is done reading X(s-1), whose LDS stage
        // the prefetches below refill.  No wait for this wave's own fragment reads still in
        // flight: they are of stage s, which nothing overwrites before the next barrier.
        asm volatile("s_barrier" ::: "memory");
        SB();
        mm(2, a1, bf[1]); rd(nbuf, 0, 0, 0, a1); ph_mad(0); if (!TAIL) issue_x1(s + 3, (s + 3) & 3, 0); SB();
        mm(3, a1, bf[1]); ph_xor(bf[0][0]); if (!TAIL) issue_x1(s + 3, (s + 3) & 3, 1); SB();
        mm(4, a1, bf[1]); rd(nbuf, 0, 0, 1, a1); ph_and_lo(w_nxt[1][0]); if (!TAIL) issue_x1(s + 3, (s + 3) & 3, 2); SB();
        mm(5, a1, bf[1]); ph_mad(1); if (!TAIL) issue_x1(s + 3, (s + 3) & 3, 3); SB();
        mm(6, a1, bf[1]); rd(nbuf, 0, 0, 2, a1); ph_xor(bf[0][1]); if (!TAIL) load_w1(s + 3, 0, w_cur, p_cur); SB();
        mm(7, a1, bf[1]); if (!TAIL) load_w1(s + 3, 1, w_cur, p_cur); SB();
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
    ph_par(pr[0], 0);
    asm volatile("" : "+v"(bf[0][0]), "+v"(bf[0][1]));
    wait_vmcnt<2 * PER_STAGE>();
    lds_barrier_raw();
    if constexpr (MF == 4) {
        rd(0, 0, 0, 0, af[0]), rd(0, 0, 0, 1, af[0]), rd(0, 0, 0, 2, af[0]);  // the first k-step reads fragment 3 itself
    } else {
        read_a(0, 0, 0, af[0]);
    }
    __builtin_amdgcn_sched_barrier(0);

    // Three stages per trip (one turn of the W registers) without branches inside, so that
    // every load stays where the in-flight count above expects it; the one or two stages
    // that may be left over run after the loop, waiting for everything still in flight.
    int s = 0;
    if constexpr (MF == 4) {
        for (; s + 3 <= stages; s += 3) {
            stage_pinned(s, wr[0], pr[0], wr[1], pr[1], body);
            stage_pinned(s + 1, wr[1], pr[1], wr[2], pr[2], body);
            stage_pinned(s + 2, wr[2], pr[2], wr[0], pr[0], body);
        }
        // the one or two stages that may remain run in the compiler's own order (same contract,
        // fragment 3 of their first k-step read here)
        if (s < stages) {
            rd(s & 3, 0, 0, 3, af[0]);
            stage(s, wr[0], pr[0], wr[1], pr[1], tail);
        }
        if (s + 1 < stages) stage(s + 1, wr[1], pr[1], wr[2], pr[2], tail);
    } else {
        for (; s + 3 <= stages; s += 3) {
            stage(s, wr[0], pr[0], wr[1], pr[1], body);
            stage(s + 1, wr[1], pr[1], wr[2], pr[2], body);
            stage(s + 2, wr[2], pr[2], wr[0], pr[0], body);
        }
        if (s < stages) stage(s, wr[0], pr[0], wr[1], pr[1], tail);
        if (s + 1 < stages) stage(s + 1, wr[1], pr[1], wr[2], pr[2], tail);
    }
    // the (clamped) prefetches past the last stage write LDS too: they must have landed
    // before the block ends and its LDS goes to another block
    wait_vmcnt0();

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

