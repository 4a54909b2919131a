// Tiled kernel (larger M): the duo kernel (two waves per SIMD), X staged through registers.
// (part of liquidgemm.hip: included there, inside namespace lqq)
#pragma once

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
// With one k group a tile of 65..96 rows takes 3 fragments (8 experts of 58..71 tokens on
// 14336 x 4096: 65 instead of 72 us).
// DQ = how the B operand is dequantised: 0 = LiquidQuant (Eq. 12, the product path), 1 = the
// overflow-safe widened form it replaces (ablation variant only, never dispatched).
template <bool G128, int KG, int MF, int TM = 128, int MFC = MF, int DQ = 0>
__device__ __forceinline__ void duo_tile(
    const Place pl, const int bm, const int bn, int M, int N, int K, const int8_t *__restrict__ X,
    const float *__restrict__ sx, const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp,
    const float *__restrict__ sw, __half *__restrict__ Y, int32_t *__restrict__ ACC,
    int32_t *__restrict__ partials)
{
    // MFC = fragments the K loop computes: MF, or 3 of 4 for a tile of 65..96 rows where two k
    // groups must share out an even number (the fourth stays zero through the exchange)
    constexpr int WM = TM, XP = MFC;  // TM = rows between consecutive row tiles (128, or 64 with MF = 2)
    static_assert(32 * MF <= TM, "a tile cannot hold more row fragments than its height");
    constexpr int STAGE = 128 * kTilePitch;
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

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

    v16i acc[MF][2];
#pragma unroll
    for (int mf = 0; mf < MFC; ++mf)
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
    // W register stages: two, or three where the accumulators leave room (two row fragments):
    // the loads of a stage are then in flight for two stages instead of one
    constexpr int WS = MF <= 2 ? 3 : 2;
    u32x4 wr[WS][2][2];  // [stage mod WS][tile][chunk]
    UnitParams<G128> pr[WS][2];
    v4i bf[2][2];       // [ping-pong][tile]
    v4i af[2][MFC];     // [ping-pong][m fragment]

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
            uint32_t s2, a4;
            p[t].get(c, s2, a4);
            if constexpr (DQ == 0) {
                dequant_half(w[t][c], s2, a4, h, b[t]);
            } else {
                // The overflow-safe form that LiquidQuant avoids (Sec. 4 "Dequantization",
                // Sec. 7.3 ablation): code * s + min in signed 16-bit lanes, two codes per
                // register, low bytes gathered with a byte permute -- the same integers for
                // about twice the instructions.
                const uint32_t mn2 = (((a4 & 0xffu) - 128u) & 0xffffu) * 0x00010001u;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const uint32_t q = w[t][c][d] >> (4 * h);
                    const uint32_t ra = q & 0x000F000Fu, rb = (q >> 8) & 0x000F000Fu;
                    const uint32_t ma = pk_mad_u16(ra, s2, mn2), mb = pk_mad_u16(rb, s2, mn2);
                    b[t][d] = (int)__builtin_amdgcn_perm(mb, ma, 0x06020400u);
                    // one register at a time: the kernel has no registers to spare for four
                    // chains of temporaries in flight at once
                    asm volatile("" : "+v"(b[t][d]));
                }
            }
        }
    };
    auto read_a = [&](int buf, int c, int h, v4i (&a)[MFC]) {
#pragma unroll
        for (int mf = 0; mf < MFC; ++mf)
            a[mf] = *reinterpret_cast<const v4i *>(xs + buf * STAGE + mf * 32 * kTilePitch + 64 * c + 32 * h);
    };
    auto mma = [&](const v4i (&a)[MFC], const v4i (&b)[2]) {
#pragma unroll
        for (int mf = 0; mf < MFC; ++mf)
#pragma unroll
            for (int t = 0; t < 2; ++t) acc[mf][t] = mfma_i8(a[mf], b[t], acc[mf][t]);
    };

    // One stage: w_cur = W(s) on entry and W(s+WS) on exit, w_nxt = W(s+1); af[0], bf[0] hold
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
        load_w(s + WS, w_cur, p_cur);
        mma(af[1], bf[1]);
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- the four-fragment tile: the same stage with its instruction order pinned ----------
    // (see duo_dl_tile: one phase of the dequantisation of one tile's four registers behind
    // every MFMA, fragment reads in the first half of a k-step, the X stores, X loads and W
    // loads of the stage one piece per MFMA; scheduling barriers keep the order)
    uint32_t s2v[2], a4v[2];  // broadcast parameters of the chunk whose B operands are being built
    uint32_t tq[4];           // the four registers in flight through the phases
    auto SB = [] { __builtin_amdgcn_sched_barrier(0); };
    auto mm = [&](int i, const v4i (&a)[MFC], const v4i (&b)[2]) {
        acc[(i >> 1) % MFC][i & 1] = mfma_i8(a[(i >> 1) % MFC], b[i & 1], acc[(i >> 1) % MFC][i & 1]);
    };
    auto rd = [&](int buf, int c, int h, int mf, v4i (&a)[MFC]) {
        a[mf % MFC] = *reinterpret_cast<const v4i *>(xs + buf * STAGE + (mf % MFC) * 32 * kTilePitch + 64 * c + 32 * h);
    };
    auto load_x1 = [&](int s, int i) {
        if (KG > 1 && s >= my_stages) {
            xr[i % XP] = u32x4{0, 0, 0, 0};
            return;
        }
        s = min(s, my_stages - 1);
        xr[i % XP] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)s * 128 + xg[i % XP]);
    };
    auto store_x1 = [&](int buf, int i) {
        *reinterpret_cast<u32x4 *>(lds_g + buf * STAGE + xl + (i % XP) * 32 * kTilePitch) = xr[i % XP];
    };
    // (wave-uniform bases plus 32-bit lane offsets: no 64-bit address arithmetic per load)
    const char *wbase_u = reinterpret_cast<const char *>(Wp + ((size_t)t0 * chunks_per_tile + 2 * (size_t)s_begin) * 64);
    const char *pbase_u = reinterpret_cast<const char *>(gp) + ((size_t)t0 * stages_total + s_begin) * 32 * (G128 ? 2 : 4);
    const uint32_t wl_off = lane * 16, pl_off = j * (G128 ? 2 : 4);
    auto load_w1 = [&](int s, int t, u32x4 (&w)[2][2], UnitParams<G128> (&p)[2]) {
        s = min(s, my_stages - 1);
        const uint32_t wo = wl_off + (uint32_t)s * 2048, po = pl_off + (uint32_t)s * (G128 ? 64 : 128);
        const char *wb = wbase_u + t * (wg_stride * 16);
        const char *pb = pbase_u + t * pg_stride;
        w[t][0] = *reinterpret_cast<const u32x4 *>(wb + wo);
        w[t][1] = *reinterpret_cast<const u32x4 *>(wb + wo + 1024);
        if (G128)
            p[t].raw = *reinterpret_cast<const uint16_t *>(pb + po);
        else
            p[t].raw = *reinterpret_cast<const uint32_t *>(pb + po);
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
    // A fragments are single-buffered and refreshed in place (fragment 3 of the running k-step
    // in its slot 0, fragments 0..2 of the next k-step in slots 2, 4 and 6, behind their last
    // use).  With two LDS stages the stage barrier must find no read of the running stage in
    // flight (the fence in lds_barrier() waits for them), so in the last k-step it sits behind
    // the fourth MFMA, three slots after the last such read, and the first fragments of the
    // next stage are read in slots 4 to 6.
    auto stage_pinned = [&](int s, u32x4 (&w_cur)[2][2], UnitParams<G128> (&p_cur)[2], u32x4 (&w_nxt)[2][2],
                            UnitParams<G128> (&p_nxt)[2], int buf) {
        v4i (&a1)[MFC] = af[0];
        // k-step (0,0): builds B(0,1), stores X(s+1) into the other LDS stage
        mm(0, a1, bf[0]); rd(buf, 0, 0, 3, a1); ph_shr(w_cur[0][0]); SB();
        mm(1, a1, bf[0]); store_x1(buf ^ 1, 0); ph_and_hi(); SB();
        mm(2, a1, bf[0]); rd(buf, 0, 1, 0, a1); ph_mad(0); SB();
        mm(3, a1, bf[0]); store_x1(buf ^ 1, 1); ph_xor(bf[1][0]); SB();
        mm(4, a1, bf[0]); rd(buf, 0, 1, 1, a1); ph_shr(w_cur[1][0]); SB();
        mm(5, a1, bf[0]); store_x1(buf ^ 1, 2); ph_and_hi(); SB();
        mm(6, a1, bf[0]); rd(buf, 0, 1, 2, a1); ph_mad(1); SB();
        mm(7, a1, bf[0]); store_x1(buf ^ 1, 3); ph_xor(bf[1][1]); SB();
        // k-step (0,1): builds B(1,0), loads X(s+2)
        mm(0, a1, bf[1]); rd(buf, 0, 1, 3, a1); ph_par(p_cur, 1); SB();
        mm(1, a1, bf[1]); load_x1(s + 2, 0); ph_and_lo(w_cur[0][1]); SB();
        mm(2, a1, bf[1]); rd(buf, 1, 0, 0, a1); ph_mad(0); SB();
        mm(3, a1, bf[1]); load_x1(s + 2, 1); ph_xor(bf[0][0]); SB();
        mm(4, a1, bf[1]); rd(buf, 1, 0, 1, a1); ph_and_lo(w_cur[1][1]); SB();
        mm(5, a1, bf[1]); load_x1(s + 2, 2); ph_mad(1); SB();
        mm(6, a1, bf[1]); rd(buf, 1, 0, 2, a1); ph_xor(bf[0][1]); SB();
        mm(7, a1, bf[1]); load_x1(s + 2, 3); SB();
        // k-step (1,0): builds B(1,1)
        mm(0, a1, bf[0]); rd(buf, 1, 0, 3, a1); ph_shr(w_cur[0][1]); SB();
        mm(1, a1, bf[0]); ph_and_hi(); SB();
        mm(2, a1, bf[0]); rd(buf, 1, 1, 0, a1); ph_mad(0); SB();
        mm(3, a1, bf[0]); ph_xor(bf[1][0]); SB();
        mm(4, a1, bf[0]); rd(buf, 1, 1, 1, a1); ph_shr(w_cur[1][1]); SB();
        mm(5, a1, bf[0]); ph_and_hi(); SB();
        mm(6, a1, bf[0]); rd(buf, 1, 1, 2, a1); ph_mad(1); SB();
        mm(7, a1, bf[0]); ph_xor(bf[1][1]); SB();
        // k-step (1,1): builds B(0,0) of the next stage, loads W(s+WS)
        mm(0, a1, bf[1]); rd(buf, 1, 1, 3, a1); ph_par(p_nxt, 0); SB();
        mm(1, a1, bf[1]); ph_and_lo(w_nxt[0][0]); SB();
        mm(2, a1, bf[1]); ph_mad(0); SB();
        mm(3, a1, bf[1]); ph_xor(bf[0][0]); SB();
        lds_barrier();  // X(s+1) is complete; every wave is done reading this stage
        SB();
        mm(4, a1, bf[1]); rd(buf ^ 1, 0, 0, 0, a1); ph_and_lo(w_nxt[1][0]); SB();
        mm(5, a1, bf[1]); rd(buf ^ 1, 0, 0, 1, a1); ph_mad(1); load_w1(s + WS, 0, w_cur, p_cur); SB();
        mm(6, a1, bf[1]); rd(buf ^ 1, 0, 0, 2, a1); ph_xor(bf[0][1]); SB();
        mm(7, a1, bf[1]); load_w1(s + WS, 1, w_cur, p_cur); SB();
    };
    // The two-fragment tile (64-row tiles, ragged last tiles): 4 MFMAs per k-step against 28
    // to 32 dequantisation instructions, so the vector port sets the pace and the order only has
    // to keep it full: two phases (eight independent instructions) behind every MFMA, no
    // dependent instruction next to its producer (a packed multiply-add followed directly by its
    // XOR costs a wait state), fragments double-buffered.
    auto stage_pinned2 = [&](int s, u32x4 (&w_cur)[2][2], UnitParams<G128> (&p_cur)[2], u32x4 (&w_nxt)[2][2],
                             UnitParams<G128> (&p_nxt)[2], int buf) {
        // k-step (0,0): builds B(0,1), reads A(0,1), stores X(s+1) into the other LDS stage
        mm(0, af[0], bf[0]); rd(buf, 0, 1, 0, af[1]); ph_shr(w_cur[0][0]); ph_and_hi(); SB();
        mm(1, af[0], bf[0]); rd(buf, 0, 1, 1, af[1]); ph_mad(0); ph_xor(bf[1][0]); SB();
        mm(2, af[0], bf[0]); store_x1(buf ^ 1, 0); ph_shr(w_cur[1][0]); ph_and_hi(); SB();
        mm(3, af[0], bf[0]); store_x1(buf ^ 1, 1); ph_mad(1); ph_xor(bf[1][1]); SB();
        // k-step (0,1): builds B(1,0), reads A(1,0), loads X(s+2)
        mm(0, af[1], bf[1]); rd(buf, 1, 0, 0, af[0]); ph_par(p_cur, 1); ph_and_lo(w_cur[0][1]); SB();
        mm(1, af[1], bf[1]); rd(buf, 1, 0, 1, af[0]); ph_mad(0); ph_xor(bf[0][0]); SB();
        mm(2, af[1], bf[1]); load_x1(s + 2, 0); ph_and_lo(w_cur[1][1]); ph_mad(1); SB();
        mm(3, af[1], bf[1]); load_x1(s + 2, 1); ph_xor(bf[0][1]); SB();
        // k-step (1,0): builds B(1,1), reads A(1,1)
        mm(0, af[0], bf[0]); rd(buf, 1, 1, 0, af[1]); ph_shr(w_cur[0][1]); ph_and_hi(); SB();
        mm(1, af[0], bf[0]); rd(buf, 1, 1, 1, af[1]); ph_mad(0); ph_xor(bf[1][0]); SB();
        mm(2, af[0], bf[0]); ph_shr(w_cur[1][1]); ph_and_hi(); SB();
        mm(3, af[0], bf[0]); ph_mad(1); ph_xor(bf[1][1]); SB();
        // k-step (1,1): builds B(0,0) of the next stage; barrier; fragments of the next stage;
        // loads of W(s+WS)
        mm(0, af[1], bf[1]); ph_par(p_nxt, 0); ph_and_lo(w_nxt[0][0]); SB();
        mm(1, af[1], bf[1]); ph_mad(0); ph_xor(bf[0][0]); SB();
        lds_barrier();  // X(s+1) is complete; every wave is done reading this stage
        SB();
        mm(2, af[1], bf[1]); rd(buf ^ 1, 0, 0, 0, af[0]); rd(buf ^ 1, 0, 0, 1, af[0]); ph_and_lo(w_nxt[1][0]); ph_mad(1); SB();
        mm(3, af[1], bf[1]); ph_xor(bf[0][1]); load_w1(s + WS, 0, w_cur, p_cur); load_w1(s + WS, 1, w_cur, p_cur); SB();
    };
    constexpr bool PINNED = MF == 4 && MFC == 4 && DQ == 0;
    constexpr bool PINNED2 = MF == 2 && MFC == 2 && DQ == 0;

    // prologue (the W loads are issued after X(1) so that, as in the steady state, the
    // only loads younger than an X stage are one stage of W)
    load_x(0);
    store_x(0);
    load_x(1);
    __builtin_amdgcn_sched_barrier(0);
    load_w(0, wr[0], pr[0]);
    load_w(1, wr[1], pr[1]);
    if (WS == 3) load_w(2, wr[WS - 1], pr[WS - 1]);
    __builtin_amdgcn_sched_barrier(0);
    build_b(wr[0], pr[0], 0, 0, bf[0]);
    if (PINNED || PINNED2) ph_par(pr[0], 0);
    lds_barrier();
    if constexpr (PINNED) {
        rd(0, 0, 0, 0, af[0]), rd(0, 0, 0, 1, af[0]), rd(0, 0, 0, 2, af[0]);  // the first k-step reads fragment 3 itself
    } else {
        read_a(0, 0, 0, af[0]);
    }
    __builtin_amdgcn_sched_barrier(0);

    if constexpr (PINNED) {
        for (int s = 0; s < stages; s += 2) {
            stage_pinned(s, wr[0], pr[0], wr[1], pr[1], 0);
            stage_pinned(s + 1, wr[1], pr[1], wr[0], pr[0], 1);
        }
    } else if (WS == 2) {
        for (int s = 0; s < stages; s += 2) {
            stage(s, wr[0], pr[0], wr[1], pr[1], 0);
            stage(s + 1, wr[1], pr[1], wr[0], pr[0], 1);
        }
    } else {
        // three W stages against two X stages: the pattern repeats every six stages.  The
        // loop has one exit (with more the register allocator spills); the two or four
        // stages that may remain (the number of stages is even) follow it.
        auto ST = [&](int s_, u32x4 (&wc)[2][2], UnitParams<G128> (&pc)[2], u32x4 (&wn)[2][2], UnitParams<G128> (&pn)[2],
                      int buf) {
            if constexpr (PINNED2)
                stage_pinned2(s_, wc, pc, wn, pn, buf);
            else
                stage(s_, wc, pc, wn, pn, buf);
        };
        int s = 0;
        for (; s + 6 <= stages; s += 6) {
            ST(s, wr[0], pr[0], wr[1], pr[1], 0);
            ST(s + 1, wr[1], pr[1], wr[WS - 1], pr[WS - 1], 1);
            ST(s + 2, wr[WS - 1], pr[WS - 1], wr[0], pr[0], 0);
            ST(s + 3, wr[0], pr[0], wr[1], pr[1], 1);
            ST(s + 4, wr[1], pr[1], wr[WS - 1], pr[WS - 1], 0);
            ST(s + 5, wr[WS - 1], pr[WS - 1], wr[0], pr[0], 1);
        }
        if (s < stages) {
            ST(s, wr[0], pr[0], wr[1], pr[1], 0);
            ST(s + 1, wr[1], pr[1], wr[WS - 1], pr[WS - 1], 1);
            if (s + 2 < stages) {
                ST(s + 2, wr[WS - 1], pr[WS - 1], wr[0], pr[0], 0);
                ST(s + 3, wr[0], pr[0], wr[1], pr[1], 1);
            }
        }
    }
    // fragments that the loop did not compute come into being only here (no registers before)
#pragma unroll
    for (int mf = MFC; mf < MF; ++mf)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mf][t][r] = 0;

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
        // the fragments this group finishes, in registers of their own: the rest of acc is dead
        v16i fin[MFK][2];
#pragma unroll
        for (int i = 0; i < MFK; ++i)
#pragma unroll
            for (int t = 0; t < 2; ++t) fin[i][t] = acc[MF0 + i][t];
        if (S > 1) {
            // Grid-level split-K: every wave publishes its part of the block's INT32 partial tile
            // with device-scope write-through stores and takes a ticket; the last one of the S
            // slices adds the others to its registers and runs the epilogue.
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
                        return v4i{fin[i][t][4 * q], fin[i][t][4 * q + 1], fin[i][t][4 * q + 2],
                                   fin[i][t][4 * q + 3]};
                    };
                    store_sc1_x4<0>(frag, part(0));
                    store_sc1_x4<1024>(frag, part(1));
                    store_sc1_x4<2048>(frag, part(2));
                    store_sc1_x4<3072>(frag, part(3));
                }
            }
            // Every wave owns its 64 channels of the tile in every slice, so the protocol runs per
            // wave, without block barriers: stores acknowledged, then a ticket of this (tile, wave);
            // the wave that draws the last of the S tickets adds the other slices and finishes.
            wait_vmcnt0();
            unsigned int *ticket = pl.tickets + tile * 8 + bw;
            unsigned tk = 0;
            if (lane == 0) tk = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            tk = (unsigned)__builtin_amdgcn_readfirstlane((int)tk);
            if (tk != (unsigned)(S - 1)) return;
            // The loads of up to two row fragments (2 x 2 column tiles x 4 pieces of 16 bytes per
            // lane) are in flight before the first is waited for: the latency of these
            // device-scope reads, not their volume, is what this tail costs.
            constexpr int FB = 1;  // (two at a time would not fit the registers of the two-k-group kernel)
            for (int k2 = 0; k2 < S; ++k2) {
                if (k2 == ks) continue;
                const int32_t *other = partials + (((tile * S + k2) * (4 * KG) + bw) * EPW) * 256 + lane * 4;
#pragma unroll
                for (int i0 = 0; i0 < MFK; i0 += FB) {
                    v4i v[FB][2][4];
#pragma unroll
                    for (int f = 0; f < FB; ++f) {
                        if (!live(i0 + f)) continue;
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            const int32_t *frag = other + ((i0 + f) * 2 + t) * 4 * 256;
                            v[f][t][0] = load_sc1_x4<0>(frag);
                            v[f][t][1] = load_sc1_x4<1024>(frag);
                            v[f][t][2] = load_sc1_x4<2048>(frag);
                            v[f][t][3] = load_sc1_x4<3072>(frag);
                        }
                    }
#pragma unroll
                    for (int f = 0; f < FB; ++f) {
                        if (!live(i0 + f)) continue;
                        wait_vmcnt0(v[f][0][0], v[f][0][1], v[f][0][2], v[f][0][3]);
                        wait_vmcnt0(v[f][1][0], v[f][1][1], v[f][1][2], v[f][1][3]);
#pragma unroll
                        for (int t = 0; t < 2; ++t)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
#pragma unroll
                                for (int e = 0; e < 4; ++e) fin[i0 + f][t][4 * q + e] += v[f][t][q][e];
                    }
                }
            }
            if (lane == 0)  // ready for the next call
                __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (!active) return;
        store_tile<MFK>(fin, M, N, m0 + 32 * MF0,
                        64 * ng + 2 * j, lane, sx, sw, Y, ACC);
    };
    if (KG == 1 || grp == 0)
        finish(std::integral_constant<int, 0>{});
    else
        finish(std::integral_constant<int, KG - 1>{});
}

// ALL3 = every row tile of the launch has 65..96 rows (M itself has): the kernel holds that
// path only.  (Inside the general two-k-group kernel it would be a third copy of the tile code,
// and the register allocation of the four-fragment copy, which has none to spare, then spills.)
template <bool G128, int KG, int TM = 128, bool ALL3 = false, int DQ = 0>
__device__ __forceinline__ void duo_block(
    const Place pl, const int bm, const int bn, int M, int N, int K, const int8_t *__restrict__ X,
    const float *__restrict__ sx, const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp,
    const float *__restrict__ sw, __half *__restrict__ Y, int32_t *__restrict__ ACC,
    int32_t *__restrict__ partials)
{
    if (DQ != 0)  // ablation variant: the four-fragment path only (rows past M are computed and not stored)
        duo_tile<G128, KG, 4, 128, 4, DQ>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
    else if (ALL3)
        duo_tile<G128, KG, 4, 128, 3, DQ>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
    else if (TM == 64)
        duo_tile<G128, KG, 2, 64, 2, DQ>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
    else if (M - 128 * bm <= 64)  // block-uniform
        duo_tile<G128, KG, 2, 128, 2, DQ>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
    else {
        if constexpr (KG == 1) {
            if (M - 128 * bm <= 96) {
                duo_tile<G128, KG, 3, 128, 3, DQ>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
                return;
            }
        }
        duo_tile<G128, KG, 4, 128, 4, DQ>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
    }
}

template <bool G128, int KG, int TM = 128, bool ALL3 = false, int DQ = 0>
__global__ __launch_bounds__(256 * KG, KG == 1 ? 2 : 1) void w4a8_duo_kernel(
    int M, int N, int K, const int8_t *__restrict__ X, const float *__restrict__ sx,
    const u32x4 *__restrict__ Wp, const uint8_t *__restrict__ gp, const float *__restrict__ sw,
    __half *__restrict__ Y, int32_t *__restrict__ ACC, int blocks_m, int blocks_n,
    int32_t *__restrict__ partials, unsigned int *__restrict__ tickets)
{
    int bm, bn;
    block_coords(blocks_m, blocks_n, bm, bn);
    duo_block<G128, KG, TM, ALL3, DQ>(grid_place(tickets), bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, partials);
}

// The same barrier for code that waits for its loads itself: a fence would also wait for
// every asynchronous load into LDS that is still in flight.
__device__ __forceinline__ void lds_barrier_raw()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

