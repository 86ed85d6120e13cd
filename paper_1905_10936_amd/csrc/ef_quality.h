// Compressor-quality diagnostics of libef (Section 3.2 of arxiv 1905.10936): see ef_tile.h for the tile scheme.
#pragma once
#include "ef_tile.h"

namespace ef {

// ------------------------------------------------- compressor quality ---
//
// phi(v) = min_b ||v_Gb||_1^2 / (d_b ||v_Gb||_2^2) (Proposition 1) and
// delta(v) = ||v||_1^2 / (d ||v||_2^2) (non-block compressor, Eq. (1)), in
// fp64.  Three small kernels: out[2i] = 1 (the ratio of an all-zero block,
// which the compressor reproduces exactly); per tile (a pass of its own over v, or
// inside the worker kernel on the p it has in registers anyway) the sums of |v| and v^2
// of the tile and of its open segments, and the ratios of the segments that
// close inside the tile; per crossing block the sums of its tiles' partials in
// a fixed order.  The minimum is taken with an integer atomic on the bits of
// the (non-negative) ratio, which does not depend on the order of arrival.

struct QualityArgs {
    const float *v;             // [n][stride]
    int64_t stride;
    double *tile_sums;          // [n][ntiles][2]   (sum |v|, sum v^2) of each tile
    double *part_sums;          // [n][2*ntiles][2] the same for each open segment (slot as in part_index)
    double *out;                // [n][2]           phi, delta
};

__device__ __forceinline__ void ratio_min(unsigned long long *phi_bits, double l1, double l2, int64_t db)
{
    if (l2 > 0.0) {
        const double ratio = l1 * l1 / ((double)db * l2);
        atomicMin(phi_bits, (unsigned long long)__double_as_longlong(ratio));
    }
}

__global__ __launch_bounds__(THREADS) void k_quality_init(double *out, int n)
{
    for (int i = threadIdx.x; i < n; i += THREADS) {
        out[2 * i] = 1.0;
        out[2 * i + 1] = 1.0;
    }
}

// The share of one tile of vector `vec` in phi and delta: a holds the tile's values (any sign; past
// the end of the vector 0).  Called by every thread of the workgroup; uses S.red, and for a tile
// where several blocks meet S.val and S.long_list as well (free again on return).
__device__ __forceinline__ void quality_of_tile(float4 (&a)[SUBROWS], const Layout &L, const QualityArgs &Q, int32_t tile,
                                                int vec, int n_valid, TileShared &S)
{
    __shared__ double seg_sum[2][2];            // [head, tail][l1, l2] of the open segments
    __shared__ unsigned long long tile_min;
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    unsigned long long *phi_bits = reinterpret_cast<unsigned long long *>(Q.out + 2 * (int64_t)vec);
    double l1 = 0.0, l2 = 0.0;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        a[k] = make_float4(fabsf(a[k].x), fabsf(a[k].y), fabsf(a[k].z), fabsf(a[k].w));
        const double x = a[k].x, y = a[k].y, z = a[k].z, w = a[k].w;
        l1 += (x + y) + (z + w);
        l2 += (x * x + y * y) + (z * z + w * w);
    }
    l1 = block_sum(l1, S.red);
    l2 = block_sum(l2, S.red);
    double *ts = Q.tile_sums + ((int64_t)vec * L.ntiles + tile) * 2;
    double *ps = Q.part_sums + ((int64_t)vec * 2 * L.ntiles + 2 * (int64_t)tile) * 2;
    if (threadIdx.x == 0) {
        ts[0] = l1;
        ts[1] = l2;
    }
    if (fb == lb) {
        const int64_t bs = L.offs[fb], be = L.offs[fb + 1];
        if (threadIdx.x == 0) {
            if (bs >= tile_start && be <= tile_start + TILE) {
                ratio_min(phi_bits, l1, l2, be - bs);
            } else {
                ps[0] = l1;         // first (and only) segment of the tile: slot 0
                ps[1] = l2;
            }
        }
        return;
    }
    // several blocks meet in this tile: segmented sums through LDS; the smallest ratio of the
    // segments that close here is collected in LDS first, one global atomic per tile
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) *reinterpret_cast<float4 *>(&S.val[local_base(k)]) = a[k];
    if (threadIdx.x == 0) {
        S.n_long = 0;
        tile_min = (unsigned long long)__double_as_longlong(1.0);
    }
    __syncthreads();
    const int nseg = lb - fb + 1;
    const bool head_open = L.offs[fb] < tile_start;
    const bool tail_open = L.offs[lb + 1] > tile_start + TILE;
    for (int sg = threadIdx.x; sg < nseg; sg += THREADS) {
        const int64_t b = fb + sg;
        const int64_t bs = L.offs[b], be = L.offs[b + 1];
        const int lo = (int)max(bs - tile_start, (int64_t)0);
        const int hi = (int)min(be - tile_start, (int64_t)n_valid);
        if (hi - lo > SMALL_SEG) {
            S.long_list[atomicAdd(&S.n_long, 1)] = sg;
            continue;
        }
        double s1 = 0.0, s2 = 0.0;
        for (int j = lo; j < hi; ++j) {
            const double x = S.val[j];
            s1 += x;
            s2 += x * x;
        }
        const bool open = (sg == 0 && head_open) || (sg == nseg - 1 && tail_open);
        if (open) {
            seg_sum[sg == 0 ? 0 : 1][0] = s1;
            seg_sum[sg == 0 ? 0 : 1][1] = s2;
        } else {
            ratio_min(&tile_min, s1, s2, be - bs);
        }
    }
    __syncthreads();
    const int n_long = S.n_long;
    for (int q = wave_id(); q < n_long; q += NWAVES) {
        const int sg = S.long_list[q];
        const int64_t b = fb + sg;
        const int64_t bs = L.offs[b], be = L.offs[b + 1];
        const int lo = (int)max(bs - tile_start, (int64_t)0);
        const int hi = (int)min(be - tile_start, (int64_t)n_valid);
        double s1 = 0.0, s2 = 0.0;
        for (int j = lo + lane_id(); j < hi; j += 64) {
            const double x = S.val[j];
            s1 += x;
            s2 += x * x;
        }
        s1 = wave_sum(s1);
        s2 = wave_sum(s2);
        const bool open = (sg == 0 && head_open) || (sg == nseg - 1 && tail_open);
        if (lane_id() == 0) {
            if (open) {
                seg_sum[sg == 0 ? 0 : 1][0] = s1;
                seg_sum[sg == 0 ? 0 : 1][1] = s2;
            } else {
                ratio_min(&tile_min, s1, s2, be - bs);
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (tile_min != (unsigned long long)__double_as_longlong(1.0)) atomicMin(phi_bits, tile_min);
        if (head_open) {
            ps[0] = seg_sum[0][0];
            ps[1] = seg_sum[0][1];
        }
        if (tail_open) {
            ps[2] = seg_sum[1][0];
            ps[3] = seg_sum[1][1];
        }
    }
    __syncthreads();            // S.val and seg_sum are free again
}

__global__ __launch_bounds__(THREADS) void k_quality_tiles(Layout L, QualityArgs Q)
{
    __shared__ TileShared S;
    const int32_t tile = blockIdx.x;
    const int vec = blockIdx.y;
    const int n_valid = tile_valid(L, tile);
    float4 a[SUBROWS];
    load_tile(Q.v + (int64_t)vec * Q.stride + (int64_t)tile * TILE, a, n_valid);     // elements past d read as 0
    quality_of_tile(a, L, Q, tile, vec, n_valid, S);
}

// Workgroups 0 .. n_cross-1: one block that spans several tiles each.  The last
// workgroup of each vector: delta from the tile sums.
__global__ __launch_bounds__(THREADS) void k_quality_blocks(Layout L, QualityArgs Q, const int32_t *cross_blocks,
                                                            int n_cross)
{
    __shared__ double red[NWAVES];
    const int vec = blockIdx.y;
    double s1 = 0.0, s2 = 0.0;
    if ((int)blockIdx.x < n_cross) {
        const int64_t b = cross_blocks[blockIdx.x];
        const BlockSpan sp = block_span(L, b);
        const double *ps = Q.part_sums + (int64_t)vec * 2 * L.ntiles * 2;
        for (int64_t i = threadIdx.x; i < sp.n; i += THREADS) {
            const int64_t w = part_index(sp.t0 + i, sp);
            s1 += ps[2 * w];
            s2 += ps[2 * w + 1];
        }
        s1 = block_sum(s1, red);
        s2 = block_sum(s2, red);
        if (threadIdx.x == 0)
            ratio_min(reinterpret_cast<unsigned long long *>(Q.out + 2 * (int64_t)vec), s1, s2, sp.be - sp.bs);
        return;
    }
    const double *ts = Q.tile_sums + (int64_t)vec * L.ntiles * 2;
    for (int64_t t = threadIdx.x; t < L.ntiles; t += THREADS) {
        s1 += ts[2 * t];
        s2 += ts[2 * t + 1];
    }
    s1 = block_sum(s1, red);
    s2 = block_sum(s2, red);
    if (threadIdx.x == 0) Q.out[2 * (int64_t)vec + 1] = s2 > 0.0 ? s1 * s1 / ((double)L.d * s2) : 1.0;
}

}  // namespace ef
