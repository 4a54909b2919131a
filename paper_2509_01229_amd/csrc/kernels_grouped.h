// Grouped (mixture-of-experts) launches of the per-block device functions.
// (part of liquidgemm.hip: included there, inside namespace lqq)
#pragma once

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
    if (g.rows[i] > 24) {  // block-uniform: X through LDS once most of the 32 rows exist (57 -> 51 us for 8 x 32 rows on 4096 x 14336)
        stream_block<2, NW, 1, G128, true>(Place{gx, groups, 0, 1, nullptr}, g.rows[i], N, K, p.X + (size_t)r0 * K,
                                           p.sx + r0, p.Wp + e * p.w_stride, p.gp + e * p.gp_stride,
                                           p.sw + (size_t)e * N, p.Y ? p.Y + (size_t)r0 * N : nullptr,
                                           p.ACC ? p.ACC + (size_t)r0 * N : nullptr, nullptr);
        return;
    }
    stream_block<2, NW, 1, G128>(Place{gx, groups, 0, 1, nullptr}, g.rows[i], N, K, p.X + (size_t)r0 * K, p.sx + r0,
                              p.Wp + e * p.w_stride, p.gp + e * p.gp_stride, p.sw + (size_t)e * N,
                              p.Y ? p.Y + (size_t)r0 * N : nullptr, p.ACC ? p.ACC + (size_t)r0 * N : nullptr,
                              nullptr);
}

// TM = rows per row tile (128, or 64: twice the blocks for launches that would leave CUs idle)
template <bool G128, int KG, int TM = 128>
__global__ __launch_bounds__(256 * KG, KG == 1 ? 2 : 1) void w4a8_duo_grouped_kernel(const GroupTable g,
                                                                                     const GroupedPtrs p, int N,
                                                                                     int K)
{
    int i = 0;
    while (i < g.count - 1 && (int)blockIdx.x >= g.block_end[i]) ++i;
    const int local = (int)blockIdx.x - (i ? g.block_end[i - 1] : 0);
    const int M = g.rows[i], e = g.expert[i], r0 = g.row_off[i];
    // row tiles of one column block are neighbours, so they meet on the expert's W columns
    const int blocks_m = (M + TM - 1) / TM;
    const int bm = local % blocks_m, bn = local / blocks_m;
    duo_block<G128, KG, TM>(Place{0, 1, 0, 1, nullptr}, bm, bn, M, N, K, p.X + (size_t)r0 * K, p.sx + r0,
                            p.Wp + e * p.w_stride, p.gp + e * p.gp_stride, p.sw + (size_t)e * N,
                            p.Y ? p.Y + (size_t)r0 * N : nullptr, p.ACC ? p.ACC + (size_t)r0 * N : nullptr,
                            nullptr);
}

// The direct-to-LDS form of the tiles for launches with more blocks than CUs (one k group per
// block, two blocks per CU).
template <bool G128>
__global__ __launch_bounds__(256, 2) void w4a8_duo_dl_grouped_kernel(const GroupTable g, const GroupedPtrs p, int N,
                                                                     int K)
{
    int i = 0;
    while (i < g.count - 1 && (int)blockIdx.x >= g.block_end[i]) ++i;
    const int local = (int)blockIdx.x - (i ? g.block_end[i - 1] : 0);
    const int M = g.rows[i], e = g.expert[i], r0 = g.row_off[i];
    const int blocks_m = (M + 127) >> 7;
    const int bm = local % blocks_m, bn = local / blocks_m;
    const Place pl{0, 1, 0, 1, nullptr};
    const int8_t *X = p.X + (size_t)r0 * K;
    const float *sx = p.sx + r0, *sw = p.sw + (size_t)e * N;
    const u32x4 *Wp = p.Wp + e * p.w_stride;
    const uint8_t *gp = p.gp + e * p.gp_stride;
    __half *Y = p.Y ? p.Y + (size_t)r0 * N : nullptr;
    int32_t *ACC = p.ACC ? p.ACC + (size_t)r0 * N : nullptr;
    const int left = M - 128 * bm;  // block-uniform
    if (left <= 64)
        duo_dl_tile<G128, 2>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, nullptr);
    else if (left <= 96)
        duo_dl_tile<G128, 3>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, nullptr);
    else
        duo_dl_tile<G128, 4>(pl, bm, bn, M, N, K, X, sx, Wp, gp, sw, Y, ACC, nullptr);
}

// The 256 x 256 tiles (one wave per SIMD, see kernels_tiled_solo.h) of all experts of a launch as
// one persistent stream: resident blocks walk the tiles of every expert, prefetching across the
// boundaries between them.  block_end counts 256 x 256 tiles here.
struct SoloGrouped {
    const GroupTable &g;
    const GroupedPtrs &p;
    int N, K, blocks_n;
    __device__ __forceinline__ int slices() const { return 1; }
    __device__ __forceinline__ int tiles() const { return g.block_end[g.count - 1]; }
    __device__ __forceinline__ SoloTile tile(int lid, int G) const
    {
        lid = solo_xcd_order(lid, tiles(), G);
        int i = 0;
        while (i < g.count - 1 && lid >= g.block_end[i]) ++i;
        const int local = lid - (i ? g.block_end[i - 1] : 0);
        const int M = g.rows[i], e = g.expert[i], r0 = g.row_off[i];
        int bm, bn;
        solo_coords(local, (M + 255) / 256, blocks_n, bm, bn);
        return SoloTile{M,
                        bm,
                        bn,
                        0,
                        p.X + (size_t)r0 * K,
                        p.sx + r0,
                        p.Wp + e * p.w_stride,
                        p.gp + e * p.gp_stride,
                        p.sw + (size_t)e * N,
                        p.Y ? p.Y + (size_t)r0 * N : nullptr,
                        p.ACC ? p.ACC + (size_t)r0 * N : nullptr};
    }
};
template <bool G128>
__global__ __launch_bounds__(256, 1) void w4a8_solo_grouped_kernel(const GroupTable g, const GroupedPtrs p, int N, int K)
{
    solo16_body<G128, 1>(SoloGrouped{g, p, N, K, (N + 255) / 256}, N, K);
}
