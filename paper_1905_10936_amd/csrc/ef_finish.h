// Kernels that run after the main kernel of a call, and the parameter update: see ef_tile.h for the tile scheme.
#pragma once
#include "ef_tile.h"

namespace ef {

// ------------------------------------------- the kernel that ends a call ---

// e <- p - Delta on one open segment of a tile whose p was parked in the
// residual buffer (e_{t+1} = p_t - Delta_t of Algorithm 4), now that its block's
// scale s exists.  The sign is taken from p itself.  which: 0 = first (or only)
// segment of the tile, 1 = last segment.
__device__ __forceinline__ void residual_segment(const Layout &L, int32_t tile, int which, float *err_set, float s)
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
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) residual4(v[k], s);
        store_tile(err_tile, v, TILE);
        return;
    }
    int lo, hi;
    if (which == 0) {
        lo = 0;
        hi = (int)min(L.offs[fb + 1] - tile_start, (int64_t)n_valid);
    } else {
        lo = (int)(L.offs[lb] - tile_start);
        hi = n_valid;
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

// What the kernel that ends a call works through.
struct TailArgs {
    const int32_t *late_blocks;     // [n_late] blocks larger than fuse_limit: their scales are formed here
    int n_late;
    const uint32_t *items;          // [n_items] (tile << 1) | which: segments whose p the main kernels always park
    int n_items;
    int nsets;
    float *err;                     // residual buffers of the call's sets, err_stride apart
    int64_t err_stride;
    float *scales;                  // scale arrays of the call's sets, scales_stride apart
    int64_t scales_stride;
    int fin_wgs, res_wgs;           // workgroups given to the two lists above
    CallState *state;
    int lazy;
};

// Scale of block b of `set` inside the kernel that ends a call.  Every partial of the call has
// been posted by then, so the scale can always be formed on the spot from the partials (the
// same sum in the same order, hence the same bits, whoever forms it); for a block of many tiles
// that is worth avoiding, so the ready word is looked at first (bounded), where the main kernels
// and this kernel's own workgroups post every scale they form.  Called by every thread of the
// workgroup; same answer to all.
__device__ __forceinline__ float tail_scale(const Layout &L, const Scratch &X, int set, int64_t b, SyncShared &S)
{
    const BlockSpan sp = block_span(L, b);
    float s = 0.f;
    if (sp.n > 2 * THREADS && wait_ready(b, 0ull, L, X, set, S, &s)) return s;
    const double total = sum_block_partials(L, b, set_part(X, L, set), S.red);
    return (float)(total / (double)(sp.be - sp.bs));
}

// The call is over: count it, flip the tags of the sets it used, clear the counters the next
// call will use (one thread).
__device__ __forceinline__ void advance_call(CallState *state, const Scratch &X, int nsets, int lazy)
{
    const unsigned long long used = nsets >= 64 ? ~0ull : ((1ull << nsets) - 1ull);
    X.next_cnt[0] = 0u;
    X.next_cnt[2] = 0u;
    X.next_cnt[4] = 0u;
    *X.done = 0u;
    state->calls = state->calls + 1u;
    if (X.set_base == 0) {
        state->worker_tags ^= used;
        // with the deferred correction on, the large blocks of these sets now hold p
        state->worker_pending = lazy ? (state->worker_pending | used) : (state->worker_pending & ~used);
    } else {
        state->server_tag ^= 1u;
        state->server_pending = lazy ? 1u : 0u;
    }
}

// Ends a worker or server call.  In this order of workgroups:
//   fin_wgs workgroups   form the scales of the blocks larger than fuse_limit (per-layout list),
//                        write them out and post them in the blocks' ready words;
//   res_wgs workgroups   e <- p - Delta on the segments whose p is always parked (per-layout
//                        list: the open segments of those blocks, and the segments that
//                        blocks with whole tiles have in mixed tiles);
//   DEFER_WGS workgroups the same two jobs for what the main kernels gave up on at run time
//                        (a gather or a wait that ran out): normally nothing.
// Each workgroup strides over its list.  The last workgroup to finish steps the plan's call
// state to the next call (no workgroup reads it after its first instructions).
__global__ __launch_bounds__(THREADS) void k_tail(Layout L, ScratchRef R, TailArgs T)
{
    const Scratch X = open_call(R);
    __shared__ SyncShared S;
    const int wg = blockIdx.x;
    if (wg < T.fin_wgs) {
        const int n = T.n_late * T.nsets;
        for (int i = wg; i < n; i += T.fin_wgs) {
            const int64_t b = T.late_blocks[i % T.n_late];
            const int w = i / T.n_late;
            const int set = X.set_base + w;
            const double total = sum_block_partials(L, b, set_part(X, L, set), S.red);
            if (threadIdx.x == 0) {
                const float sc = (float)(total / (double)(L.offs[b + 1] - L.offs[b]));
                T.scales[(int64_t)w * T.scales_stride + b] = sc;
                __hip_atomic_store(ready_word(X, L, set, b),
                                   ((unsigned long long)X.epoch << 32) | (unsigned long long)__float_as_uint(sc),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // remembered for the deferred correction of the block's residual
                if (L.lazy && L.late_index[b] >= 0)
                    X.lazy_scales[(int64_t)set * X.lazy_stride + L.late_index[b]] = sc;
            }
        }
    } else if (wg < T.fin_wgs + T.res_wgs) {
        const int64_t n = (int64_t)T.n_items * T.nsets;
        int64_t have_b = -1;
        int have_w = -1;
        float s = 0.f;
        for (int64_t i = wg - T.fin_wgs; i < n; i += T.res_wgs) {
            const uint32_t it = T.items[i % T.n_items];
            const int w = (int)(i / T.n_items);
            const int32_t tile = (int32_t)(it >> 1);
            const int which = (int)(it & 1u);
            const int64_t b = which ? L.tile_lb[tile] : L.tile_fb[tile];
            if (b != have_b || w != have_w) {       // consecutive items of a workgroup mostly share the block
                s = tail_scale(L, X, X.set_base + w, b, S);
                have_b = b;
                have_w = w;
            }
            residual_segment(L, tile, which, T.err + (int64_t)w * T.err_stride, s);
        }
    } else {
        const int q = wg - T.fin_wgs - T.res_wgs;
        const unsigned n_fin = *X.fin_cnt;
        for (unsigned i = q; i < n_fin; i += DEFER_WGS) {
            const unsigned long long it = X.fin_list[i];
            const int set = (int)(it >> 32);
            const int64_t b = (int64_t)(it & 0xffffffffull);
            const double total = sum_block_partials(L, b, set_part(X, L, set), S.red);
            if (threadIdx.x == 0) {
                const float sc = (float)(total / (double)(L.offs[b + 1] - L.offs[b]));
                T.scales[(int64_t)(set - X.set_base) * T.scales_stride + b] = sc;
                __hip_atomic_store(ready_word(X, L, set, b),
                                   ((unsigned long long)X.epoch << 32) | (unsigned long long)__float_as_uint(sc),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        const unsigned n_def = *X.defer_cnt;
        for (unsigned i = q; i < n_def; i += DEFER_WGS) {
            const unsigned long long it = X.defer_list[i];
            const int set = (int)(it >> 33);
            const int32_t tile = (int32_t)((it >> 1) & 0xffffffffull);
            const int which = (int)(it & 1ull);
            const int64_t b = which ? L.tile_lb[tile] : L.tile_fb[tile];
            const float s = tail_scale(L, X, set, b, S);
            residual_segment(L, tile, which, T.err + (int64_t)(set - X.set_base) * T.err_stride, s);
        }
    }
    // last one out steps the call state
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned before = atomicAdd(X.done, 1u);
        if (before + 1u == gridDim.x) advance_call(T.state, X, T.nsets, T.lazy);
    }
}

// A long per-layout list of parked segments (the whole tiles of blocks larger than fuse_limit when
// the correction is not deferred) streams faster with one workgroup per item, dispatched in list
// order, than through the strided loop of k_tail, and a grid of that size is too large for that
// kernel's count of finished workgroups.  So this kernel runs after k_tail, with the scales taken
// from the call's finished scale arrays.  One workgroup per (item, set).
__global__ __launch_bounds__(THREADS) void k_residual_static(Layout L, const uint32_t *items, int n_items, float *err,
                                                             int64_t err_stride, const float *scales,
                                                             int64_t scales_stride)
{
    const uint32_t it = items[blockIdx.x];
    const int w = blockIdx.y;
    const int32_t tile = (int32_t)(it >> 1);
    const int which = (int)(it & 1u);
    const int64_t b = which ? L.tile_lb[tile] : L.tile_fb[tile];
    residual_segment(L, tile, which, err + (int64_t)w * err_stride, scales[(int64_t)w * scales_stride + b]);
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
