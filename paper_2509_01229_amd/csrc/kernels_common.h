// Pieces shared by the GEMM kernels: split-K tickets and device-scope accesses, block placement, epilogue of the tiled kernels.
// (part of liquidgemm.hip: included there, inside namespace lqq)
#pragma once

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
// (A store of more than 8 bytes reads its data registers for two more cycles; the compiler counts
// those wait states for its own instructions but does not look into assembly statements, and the
// next statement may be one that overwrites the registers -- hence the s_nop.)
template <int OFF = 0>
__device__ __forceinline__ void store_sc1_x4(int32_t *p, const v4i v)
{
    asm volatile("global_store_dwordx4 %0, %1, off offset:%2 sc1\n\ts_nop 1" ::"v"(p), "v"(v), "n"(OFF) : "memory");
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


// ------------------------------------------------------------------------------------
// Epilogue shared by the tiled kernels.  Element r of acc[mf][t] is row
// m0 + 32*mf + acc_row(r, lane) and channel n + t (n = 64*group + 2*slot): the two tiles
// give 2 adjacent channels per lane, so each store is 4 bytes of FP16 (8 of INT32) and a
// half-wave writes a full 128-byte line.  Scales are fetched up front, four consecutive
// rows at a time (rows past M read s_x[M-1]; only the stores are predicated), so no
// load sits behind a branch.
// ------------------------------------------------------------------------------------
// A row's address is a wave-uniform base (scalar registers, moved from row to row by additions)
// plus one 32-bit lane offset, the stores are written in that form; the two halves of an FP16
// store go straight into one register (low half, then high half).  m0 must be wave-uniform.
__device__ __forceinline__ void store_row_u32(uint32_t byte_off, uint32_t v, const char *row)
{
    asm volatile("global_store_dword %0, %1, %2" : : "v"(byte_off), "v"(v), "s"(row) : "memory");
}
__device__ __forceinline__ void store_row_i32x2(uint32_t byte_off, int a, int b, const char *row)
{
    const uint64_t two = (uint32_t)a | ((uint64_t)(uint32_t)b << 32);
    asm volatile("global_store_dwordx2 %0, %1, %2" : : "v"(byte_off), "v"(two), "s"(row) : "memory");
}
// fp16(x0 * s0) | fp16(x1 * s1) << 16, each product rounded to FP32 first (as scale_to_half does)
__device__ __forceinline__ uint32_t scale_pair_to_half2(float x0, float s0, float x1, float s1)
{
    uint32_t two;
    asm("v_fma_mixlo_f16 %0, %1, %2, 0\n\tv_fma_mixhi_f16 %0, %3, %4, 0" : "=&v"(two) : "v"(x0), "v"(s0), "v"(x1), "v"(s1));
    return two;
}
template <int MF>
__device__ __forceinline__ void store_tile(const v16i (&acc)[MF][2], int M, int N, int m0, int n, int lane,
                                           const float *__restrict__ sx, const float *__restrict__ sw,
                                           __half *__restrict__ Y, int32_t *__restrict__ ACC)
{
    const int kb = lane >> 5;
    const uint32_t lane_off = (uint32_t)(4 * kb) * (uint32_t)N + (uint32_t)n;  // in elements (N <= 2^26)
    m0 = __builtin_amdgcn_readfirstlane(m0);
    if (ACC) {
        const size_t pitch = (size_t)N * 4;
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) {
            const char *row = reinterpret_cast<const char *>(ACC) + (size_t)(m0 + 32 * mf) * pitch;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + 32 * mf + 8 * (r >> 2) + 4 * kb + (r & 3);
                if (m < M) store_row_i32x2(lane_off * 4, acc[mf][0][r], acc[mf][1][r], row);
                row += (r & 3) == 3 ? 5 * pitch : pitch;
            }
        }
    }
    if (Y) {
        const float2 swv = *reinterpret_cast<const float2 *>(sw + n);
        const size_t pitch = (size_t)N * 2;
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) {
            float sxv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) sxv[r] = sx[min(m0 + 32 * mf + 8 * (r >> 2) + 4 * kb + (r & 3), M - 1)];
            const char *row = reinterpret_cast<const char *>(Y) + (size_t)(m0 + 32 * mf) * pitch;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + 32 * mf + 8 * (r >> 2) + 4 * kb + (r & 3);
                const uint32_t two = scale_pair_to_half2((float)acc[mf][0][r] * sxv[r], swv.x, (float)acc[mf][1][r] * sxv[r], swv.y);
                if (m < M) store_row_u32(lane_off * 2, two, row);
                row += (r & 3) == 3 ? 5 * pitch : pitch;
            }
        }
    }
}


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
    constexpr int GM = 4;
    const int per_group = GM * blocks_n;
    const int first = (lid / per_group) * GM;
    const int gsz = min(blocks_m - first, GM);
    const int in_group = lid % per_group;
    bm = first + in_group % gsz;
    bn = in_group / gsz;
}

