// Server kernels of libef (Algorithm 4 of arxiv 1905.10936): see ef_tile.h for the tile scheme.
#pragma once
#include "ef_tile.h"

namespace ef {

// -------------------------------------------------------- server kernels ---

// (1/M) * acc as Algorithm 4 writes it: one correctly rounded fp32 division, or,
// when M is a power of two, the product with the exact reciprocal, which is the
// same real number and therefore rounds to the same bits.
__device__ __forceinline__ float mean_of(float acc, float Mf, float Minv)
{
    return Minv != 0.0f ? acc * Minv : acc / Mf;
}

constexpr int SERVER_CHUNK = 8;     // workers whose sign words are in flight together
constexpr int SCALE_GROUP = 4;      // mixed tiles: workers whose scales are staged in LDS together ...
constexpr int SCALE_STAGE = 2048;   // ... in this many floats

// p~ of a tile that lies inside one block b (Algorithm 4, server: decode and add the M payloads
// in worker order, divide by M, add the rescaled server residual tv).  The sign words of
// SERVER_CHUNK workers are loaded together (one 32-bit word per worker and sub-row holds this
// lane's 4 bits), the block's M scales come through scalar loads.  Decoding goes through a
// small table in LDS: entry (u, nibble) holds the four values +-s_u that the nibble stands for,
// so a lane gets its four addends of worker u with one bit-field extract and one 128-bit LDS
// read (16 entries of 16 bytes cover the 64 banks once: no conflicts) instead of shifting and
// selecting bit by bit (measured 0.57 -> 0.55 ms at M = 8, 0.70 -> 0.64 ms at M = 16 on 2^28
// elements).  Called by every thread of the workgroup; S.val is free again on return.
__device__ __forceinline__ void server_values_whole(const ServerArgs &A, int64_t tile_start, int32_t b,
                                                    const float4 (&tv)[SUBROWS], float4 (&p)[SUBROWS], TileShared &S)
{
    float acc[SUBROWS][4];
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[k][c] = 0.0f;

    const uint32_t *s32 = reinterpret_cast<const uint32_t *>(A.signs_in);
    const int64_t in_hw = 2 * A.in_signs_stride;
    const unsigned sh = (unsigned)(lane_id() & 7) * 4u;
    // half-word index of sub-row k for this lane: consecutive sub-rows are 8 half-words apart
    const int64_t hw0 = (tile_start + local_base(0)) >> 5;

    for (int i0 = 0; i0 < A.M; i0 += SERVER_CHUNK) {
        uint32_t word[SERVER_CHUNK][SUBROWS];
        float sc[SERVER_CHUNK];
#pragma unroll
        for (int u = 0; u < SERVER_CHUNK; ++u) {
            const int i = min(i0 + u, A.M - 1);          // past M: a valid address whose value is not used
            sc[u] = A.scales_in[(int64_t)i * A.in_scales_stride + b];
#pragma unroll
            for (int k = 0; k < SUBROWS; ++k) word[u][k] = s32[(int64_t)i * in_hw + hw0 + 8 * k];
        }
        // table[u][nibble] = the four values (+-s_u) a nibble of worker u's sign bits stands for
        float4 *table = reinterpret_cast<float4 *>(S.val);
        if (i0 > 0) __syncthreads();
        if (threadIdx.x < SERVER_CHUNK * 16) {
            const int u = threadIdx.x >> 4, nib = threadIdx.x & 15;
            float su = sc[0];
#pragma unroll
            for (int q = 1; q < SERVER_CHUNK; ++q) su = (u == q) ? sc[q] : su;
            table[threadIdx.x] = make_float4(signed_scale(su, nib & 1), signed_scale(su, nib & 2),
                                             signed_scale(su, nib & 4), signed_scale(su, nib & 8));
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < SERVER_CHUNK; ++u) {
            if (i0 + u < A.M) {
#pragma unroll
                for (int k = 0; k < SUBROWS; ++k) {
                    const float4 dv = table[u * 16 + ((word[u][k] >> sh) & 15u)];
                    acc[k][0] = acc[k][0] + dv.x;
                    acc[k][1] = acc[k][1] + dv.y;
                    acc[k][2] = acc[k][2] + dv.z;
                    acc[k][3] = acc[k][3] + dv.w;
                }
            }
        }
    }
    __syncthreads();            // the table's space is free again
    const float r = A.r, Mf = A.Mf, Minv = A.Minv;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        p[k].x = mean_of(acc[k][0], Mf, Minv) + r * tv[k].x;
        p[k].y = mean_of(acc[k][1], Mf, Minv) + r * tv[k].y;
        p[k].z = mean_of(acc[k][2], Mf, Minv) + r * tv[k].z;
        p[k].w = mean_of(acc[k][3], Mf, Minv) + r * tv[k].w;
    }
}

// The same for a tile where several blocks meet (or the ragged end of the vector): a
// per-element segment index in LDS selects each worker's scale.  te: the tile of the server residual.
__device__ __forceinline__ void server_values_mixed(const Layout &L, const ServerArgs &A, int32_t tile, int n_valid,
                                                    const float *te, float4 (&p)[SUBROWS], TileShared &S)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    float acc[SUBROWS][4];
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[k][c] = 0.0f;

    // this lane's 4 sign bits of sub-row k live in the 32-bit half-word hw0 + 8k
    const uint32_t *s32 = reinterpret_cast<const uint32_t *>(A.signs_in);
    const int64_t hw0 = (tile_start + local_base(0)) >> 5;
    const unsigned sh = (unsigned)(lane_id() & 7) * 4u;
    const int64_t n_hw = 2 * L.W;
    const int64_t in_hw = 2 * A.in_signs_stride;

    const int nseg = lb - fb + 1;
    build_segment_index(L, tile, n_valid, fb, nseg, S);
    const int4 *seg4 = reinterpret_cast<const int4 *>(S.val);
    // The scales of the tile's segments are staged in LDS, SCALE_GROUP workers at a time where
    // they fit (one coalesced read per worker instead of a gather per element), and looked up
    // there; a tile with more segments than the stage holds gathers them from global memory.
    __shared__ float seg_scale[SCALE_STAGE];
    const int group = nseg * SCALE_GROUP <= SCALE_STAGE ? SCALE_GROUP : nseg <= SCALE_STAGE ? 1 : 0;
    if (group) {
        for (int i0 = 0; i0 < A.M; i0 += group) {
            uint32_t word[SCALE_GROUP][SUBROWS];
#pragma unroll
            for (int u = 0; u < SCALE_GROUP; ++u) {
                const int i = min(i0 + u, A.M - 1);      // past the group or M: loaded, not used
#pragma unroll
                for (int k = 0; k < SUBROWS; ++k) {
                    const int64_t hw = hw0 + 8 * k;
                    word[u][k] = (hw < n_hw) ? s32[(int64_t)i * in_hw + hw] : 0u;
                }
            }
            if (i0 > 0) __syncthreads();                 // the stage is read no more
            for (int u = 0; u < group && i0 + u < A.M; ++u) {
                const float *sc_i = A.scales_in + (int64_t)(i0 + u) * A.in_scales_stride + fb;
                for (int j = threadIdx.x; j < nseg; j += THREADS) seg_scale[u * nseg + j] = sc_i[j];
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < SCALE_GROUP; ++u) {
                if (u < group && i0 + u < A.M) {
                    const float *sc_u = seg_scale + u * nseg;
#pragma unroll
                    for (int k = 0; k < SUBROWS; ++k) {
                        const unsigned nibble = (word[u][k] >> sh) & 0xFu;
                        const int4 sg = seg4[local_base(k) >> 2];
                        acc[k][0] = acc[k][0] + signed_scale(sc_u[sg.x], nibble & 1u);
                        acc[k][1] = acc[k][1] + signed_scale(sc_u[sg.y], nibble & 2u);
                        acc[k][2] = acc[k][2] + signed_scale(sc_u[sg.z], nibble & 4u);
                        acc[k][3] = acc[k][3] + signed_scale(sc_u[sg.w], nibble & 8u);
                    }
                }
            }
        }
    } else {
        for (int i = 0; i < A.M; ++i) {
            const float *sc_i = A.scales_in + (int64_t)i * A.in_scales_stride + fb;
#pragma unroll
            for (int k = 0; k < SUBROWS; ++k) {
                const int64_t hw = hw0 + 8 * k;
                const uint32_t word = (hw < n_hw) ? s32[(int64_t)i * in_hw + hw] : 0u;
                const unsigned nibble = (word >> sh) & 0xFu;
                const int4 sg = seg4[local_base(k) >> 2];
                acc[k][0] = acc[k][0] + signed_scale(sc_i[sg.x], nibble & 1u);
                acc[k][1] = acc[k][1] + signed_scale(sc_i[sg.y], nibble & 2u);
                acc[k][2] = acc[k][2] + signed_scale(sc_i[sg.z], nibble & 4u);
                acc[k][3] = acc[k][3] + signed_scale(sc_i[sg.w], nibble & 8u);
            }
        }
    }
    __syncthreads();            // S.val is free again
    float4 tv[SUBROWS];
    load_tile(te, tv, n_valid);
    const float r = A.r, Mf = A.Mf, Minv = A.Minv;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        p[k].x = mean_of(acc[k][0], Mf, Minv) + r * tv[k].x;
        p[k].y = mean_of(acc[k][1], Mf, Minv) + r * tv[k].y;
        p[k].z = mean_of(acc[k][2], Mf, Minv) + r * tv[k].z;
        p[k].w = mean_of(acc[k][3], Mf, Minv) + r * tv[k].w;
    }
}

// One mixed tile of the server.  The residual tile is loaded after the payloads have been added up,
// and the segment indices stay in LDS: both keep the registers of this path within what the whole
// tiles, which are nearly all of the work, need anyway.
__device__ __forceinline__ void server_mixed_tile(const Layout &L, const Scratch &X, const ServerArgs &A, int32_t tile,
                                               int set, int n_valid, TileShared &S)
{
    float *te = A.err + (int64_t)tile * TILE;
    float4 p[SUBROWS];
    server_values_mixed(L, A, tile, n_valid, te, p, S);
    compress_mixed(p, L, tile, n_valid, A.signs, A.scales, te, X, set, S);
}

// Server part of Algorithm 4, all tiles in one launch, one workgroup per tile: the mixed tiles
// first, then the whole tiles in ascending order (see k_worker_tiles).  p~ as above, then
// compressed like a worker's p; the workgroup of a whole tile waits in the kernel for its
// block's scale.
// MIXED = false: the layout has only whole tiles, and the code for the others is left out.
// Six workgroups per CU (80 VGPRs): measured 0.58 ms against 0.63 ms at five and 0.73 ms at eight
// (where a third of the tile spills) on 2^28 elements and 8 workers.
template <bool MIXED>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(6, 8)))
void k_server_tiles(Layout L, ScratchRef R, ServerArgs A, int set)
{
    const Scratch X = open_call(R);
    __shared__ TileShared S;
    const bool whole = !MIXED || (int)blockIdx.x >= L.n_mixed;
    // without mixed tiles the list of whole tiles is 0, 1, 2, ...: one dependent load less
    const int32_t tile = !MIXED ? (int32_t)blockIdx.x : whole ? L.uniform_tiles[blockIdx.x - L.n_mixed] : L.mixed_tiles[blockIdx.x];
    const int n_valid = whole ? TILE : tile_valid(L, tile);
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t b = L.tile_fb[tile];
    float *te = A.err + tile_start;
    float4 tv[SUBROWS], p[SUBROWS];
    if (whole) {
        Posted P;
        const LoadedCorrection corr = loaded_correction(L, tile, X, set);
        load_tile(te, tv, TILE);
        correct_loaded_residual(tv, corr);
        server_values_whole(A, tile_start, b, tv, p, S);
        const int kind = compress_uniform(p, L, tile, TILE, A.signs, A.scales, te, X, set, S, P);
        resolve_posted(P, L, X, set, A.scales, S);
        if (kind == UNI_PENDING) finish_uniform(p, tile, TILE, b, 0ull, te, L, X, set, S);
    } else if constexpr (MIXED) {
        server_mixed_tile(L, X, A, tile, set, n_valid, S);
    }
}

}  // namespace ef
