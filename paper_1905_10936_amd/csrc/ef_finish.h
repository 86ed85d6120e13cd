// Kernels that run after the main kernel of a call, and the parameter update: see ef_tile.h for the tile scheme.
#pragma once
#include "ef_tile.h"

namespace ef {

// ---------------------------------------------------- second-pass kernels ---

// e <- p - Delta on one open segment of a tile whose p was parked in the
// residual buffer (e_{t+1} = p_t - Delta_t of Algorithm 4), now that every scale
// exists.  The sign is taken from p itself.  which: 0 = first (or only)
// segment of the tile, 1 = last segment.
__device__ __forceinline__ void residual_segment(const Layout &L, int32_t tile, int which, float *err_set,
                                                 const float *scales)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const int n_valid = tile_valid(L, tile);
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    float *err_tile = err_set + tile_start;
    if (fb == lb && n_valid == TILE) {
        // a whole tile of one block (a block beyond fuse_limit, or a tile whose wait ran out):
        // streamed like the first pass streams it
        float4 v[SUBROWS];
        load_tile(err_tile, v, TILE);
        const float sb = scales[fb];
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) residual4(v[k], sb);
        store_tile(err_tile, v, TILE);
        return;
    }
    int lo, hi;
    float s;
    if (which == 0) {
        lo = 0;
        hi = (int)min(L.offs[fb + 1] - tile_start, (int64_t)n_valid);
        s = scales[fb];
    } else {
        lo = (int)(L.offs[lb] - tile_start);
        hi = n_valid;
        s = scales[lb];
    }
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        const int lb0 = local_base(k);
        if (lb0 >= hi || lb0 + 4 <= lo) continue;
        if (lb0 >= lo && lb0 + 4 <= hi) {
            float4 v = *reinterpret_cast<const float4 *>(err_tile + lb0);
            residual4(v, s);
            *reinterpret_cast<float4 *>(err_tile + lb0) = v;
        } else {
            // the other elements of this float4 belong to another segment, which
            // another workgroup may be updating right now: touch only our own
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int j = lb0 + c;
                if (j >= lo && j < hi) err_tile[j] = residual(err_tile[j], s);
            }
        }
    }
}

// Scales the first kernels of a call did not write: those of the blocks on the
// per-layout list (crossing blocks without a uniform tile, blocks larger than
// fuse_limit: workgroups 0 .. n_late*nsets-1) and those whose gatherer gave
// up gathering (list filled at run time: the last DEFER_WGS workgroups).
__global__ __launch_bounds__(THREADS) void k_finalize_scales(Layout L, ScratchRef R, const int32_t *late_blocks,
                                                             int n_late, int nsets, float *scales,
                                                             int64_t scales_stride)
{
    const Scratch X = open_call(R);
    __shared__ double red[NWAVES];
    const int n_static = n_late * nsets;
    if ((int)blockIdx.x < n_static) {
        const int64_t b = late_blocks[blockIdx.x % n_late];
        const int w = blockIdx.x / n_late;
        const double total = sum_block_partials(L, b, set_part(X, L, X.set_base + w), red);
        if (threadIdx.x == 0) {
            const float sc = (float)(total / (double)(L.offs[b + 1] - L.offs[b]));
            scales[(int64_t)w * scales_stride + b] = sc;
            // remembered for the deferred correction of the block's residual
            if (L.lazy && L.late_index[b] >= 0)
                X.lazy_scales[(int64_t)(X.set_base + w) * X.lazy_stride + L.late_index[b]] = sc;
        }
        return;
    }
    const unsigned n = *X.fin_cnt;
    for (unsigned i = blockIdx.x - n_static; i < n; i += DEFER_WGS) {
        const unsigned long long it = X.fin_list[i];
        const int set = (int)(it >> 32);
        const int64_t b = (int64_t)(it & 0xffffffffull);
        const double total = sum_block_partials(L, b, set_part(X, L, set), red);
        if (threadIdx.x == 0)
            scales[(int64_t)(set - X.set_base) * scales_stride + b] = (float)(total / (double)(L.offs[b + 1] - L.offs[b]));
    }
}

// e <- p - Delta wherever the first kernels parked p: the segments on the
// per-layout list (open segments of mixed tiles, tiles of blocks larger than
// fuse_limit: workgroups 0 .. n_items*nsets-1) and the tiles whose wait ran out
// (list filled at run time: the last DEFER_WGS workgroups).  Also clears the
// list counters the next call will use.
__global__ __launch_bounds__(THREADS) void k_residual_parked(Layout L, ScratchRef R, const uint32_t *items,
                                                             int n_items, int nsets, float *err, int64_t err_stride,
                                                             const float *scales, int64_t scales_stride)
{
    const Scratch X = open_call(R);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        X.next_cnt[0] = 0u;
        X.next_cnt[2] = 0u;
        X.next_cnt[4] = 0u;
    }
    const int n_static = n_items * nsets;
    if ((int)blockIdx.x < n_static) {
        const uint32_t it = items[blockIdx.x % n_items];
        const int w = blockIdx.x / n_items;
        residual_segment(L, (int32_t)(it >> 1), (int)(it & 1u), err + (int64_t)w * err_stride,
                         scales + (int64_t)w * scales_stride);
        return;
    }
    const unsigned n = *X.defer_cnt;
    for (unsigned i = blockIdx.x - n_static; i < n; i += DEFER_WGS) {
        const unsigned long long it = X.defer_list[i];
        const int w = (int)(it >> 33) - X.set_base;
        const int32_t tile = (int32_t)((it >> 1) & 0xffffffffull);
        residual_segment(L, tile, (int)(it & 1ull), err + (int64_t)w * err_stride, scales + (int64_t)w * scales_stride);
    }
}

// The call is over: count it and flip the tags of the sets it used (one thread).
__global__ void k_advance(CallState *state, int set_base, int nsets, int lazy)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const unsigned long long used = nsets >= 64 ? ~0ull : ((1ull << nsets) - 1ull);
        state->calls = state->calls + 1u;
        if (set_base == 0) {
            state->worker_tags ^= used;
            // with the deferred correction on, the large blocks of these sets now hold p
            state->worker_pending = lazy ? (state->worker_pending | used) : (state->worker_pending & ~used);
        } else {
            state->server_tag ^= 1u;
            state->server_pending = lazy ? 1u : 0u;
        }
    }
}

// Deferred correction made now (ef_flush): e <- p - Delta on the whole tiles of the blocks larger
// than fuse_limit, for the sets whose buffers still hold p.  One workgroup per (tile, set).
__global__ __launch_bounds__(THREADS) void k_flush(Layout L, ScratchRef R, const int32_t *tiles, int n_tiles,
                                                   float *err, int64_t err_stride)
{
    const Scratch X = open_call(R);
    const int32_t tile = tiles[blockIdx.x];
    const int set = X.set_base + blockIdx.y;
    float *e = err + (int64_t)blockIdx.y * err_stride + (int64_t)tile * TILE;
    float4 v[SUBROWS];
    if (!((X.pending >> blockIdx.y) & 1ull)) return;
    load_tile(e, v, TILE);
    correct_loaded_residual(v, loaded_correction(L, tile, X, set));
    store_tile(e, v, TILE);
}

__global__ void k_flush_done(CallState *state, int set_base, int nsets)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const unsigned long long used = nsets >= 64 ? ~0ull : ((1ull << nsets) - 1ull);
        if (set_base == 0)
            state->worker_pending &= ~used;
        else
            state->server_pending = 0u;
    }
}

// ----------------------------------------------------------- apply kernel ---

// Parameter update.  WD = false: x <- x - eta * Delta~ (Algorithm 4).
// WD = true: weight decay kept outside the compressed signal (Appendix A),
//   mt <- mu*mt + lambda*x ;  x <- x - eta*((Delta~ + mu*mt) + lambda*x),
// one fp32 rounding per operation in the order written.
template <bool WD>
__device__ __forceinline__ void apply_tile(const Layout &L, float *x, float *mt, const uint64_t *signs,
                                           const float *scales, float eta, float mu, float lambda, TileShared &S)
{
    const int32_t tile = blockIdx.x;
    const int n_valid = tile_valid(L, tile);
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    float *xt = x + tile_start;
    float *mtt = WD ? mt + tile_start : nullptr;
    const uint32_t *s32 = reinterpret_cast<const uint32_t *>(signs);
    const unsigned sh = (unsigned)(lane_id() & 7) * 4u;
    const int64_t n_hw = 2 * L.W;
    const int *seg = reinterpret_cast<const int *>(S.val);
    float4 xv4[SUBROWS], mv4[SUBROWS];
    load_tile(xt, xv4, n_valid);
    if (WD) load_tile(mtt, mv4, n_valid);
    if (fb != lb) build_segment_index(L, tile, n_valid, fb, lb - fb + 1, S);
    const float s_uniform = scales[fb];
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        const int lb0 = local_base(k);
        const int64_t hw = (tile_start + lb0) >> 5;
        const uint32_t word = (hw < n_hw) ? s32[hw] : 0u;
        const unsigned nibble = (word >> sh) & 0xFu;
        float xv[4] = {xv4[k].x, xv4[k].y, xv4[k].z, xv4[k].w};
        float mv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (WD) {
            mv[0] = mv4[k].x;
            mv[1] = mv4[k].y;
            mv[2] = mv4[k].z;
            mv[3] = mv4[k].w;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = lb0 + c;
            float s = s_uniform;
            if (fb != lb) s = scales[fb + ((j < n_valid) ? seg[j] : 0)];
            const float delta = signed_scale(s, (nibble >> c) & 1u);
            if (WD) {
                const float lx = lambda * xv[c];
                const float a = mu * mv[c];
                mv[c] = a + lx;
                const float b = mu * mv[c];
                const float u1 = delta + b;
                const float u = u1 + lx;
                const float step = eta * u;
                xv[c] = xv[c] - step;
            } else {
                const float u = eta * delta;
                xv[c] = xv[c] - u;
            }
        }
        xv4[k] = make_float4(xv[0], xv[1], xv[2], xv[3]);
        if (WD) mv4[k] = make_float4(mv[0], mv[1], mv[2], mv[3]);
    }
    store_tile(xt, xv4, n_valid);
    if (WD) store_tile(mtt, mv4, n_valid);
}

__global__ __launch_bounds__(THREADS) void k_apply(Layout L, float *x, const uint64_t *signs,
                                                   const float *scales, float eta)
{
    __shared__ TileShared S;
    apply_tile<false>(L, x, nullptr, signs, scales, eta, 0.0f, 0.0f, S);
}

__global__ __launch_bounds__(THREADS) void k_apply_wd(Layout L, float *x, float *mt, const uint64_t *signs,
                                                      const float *scales, float eta, float mu, float lambda)
{
    __shared__ TileShared S;
    apply_tile<true>(L, x, mt, signs, scales, eta, mu, lambda, S);
}

}  // namespace ef
