// Worker kernels of libef (Algorithm 4 and Algorithm 3 of arxiv 1905.10936): see ef_tile.h for the tile scheme.
#pragma once
#include "ef_tile.h"
#include "ef_quality.h"

namespace ef {

// --------------------------------------------------------- worker kernels ---

// The worker's corrected gradient, one rounding per operation, left to right.
// MOM (Algorithm 4): m <- mu*m + g and p = mu*m + g + r*e; m is overwritten
// with the new momentum, e with p.  !MOM (Algorithm 3, no momentum buffer):
// p = g + r*e; m is not touched.
template <bool MOM>
__device__ __forceinline__ void worker_values(const float4 (&g)[SUBROWS], float4 (&m)[SUBROWS], float4 (&e)[SUBROWS],
                                              float mu, float r)
{
    if (!MOM) {
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) {
            e[k].x = g[k].x + r * e[k].x;
            e[k].y = g[k].y + r * e[k].y;
            e[k].z = g[k].z + r * e[k].z;
            e[k].w = g[k].w + r * e[k].w;
        }
        return;
    }
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        m[k].x = mu * m[k].x + g[k].x;
        m[k].y = mu * m[k].y + g[k].y;
        m[k].z = mu * m[k].z + g[k].z;
        m[k].w = mu * m[k].w + g[k].w;
        e[k].x = (mu * m[k].x + g[k].x) + r * e[k].x;
        e[k].y = (mu * m[k].y + g[k].y) + r * e[k].y;
        e[k].z = (mu * m[k].z + g[k].z) + r * e[k].z;
        e[k].w = (mu * m[k].w + g[k].w) + r * e[k].w;
    }
}

// Mixed tiles of all workers, one workgroup per (tile, worker).  Runs before
// the uniform-tile kernel of the same call.
template <bool MOM>
__global__ __launch_bounds__(THREADS) void k_worker_mixed(Layout L, ScratchRef R, WorkerArgs A)
{
    const Scratch X = open_call(R);
    __shared__ TileShared S;
    const int32_t tile = L.mixed_tiles[blockIdx.x];
    const int worker = blockIdx.y;
    const int n_valid = tile_valid(L, tile);
    const int64_t tile_start = (int64_t)tile * TILE;
    const float *g = A.grad + (int64_t)worker * A.grad_stride + tile_start;
    float *m = MOM ? A.mom + (int64_t)worker * A.state_stride + tile_start : nullptr;
    float *e = A.err + (int64_t)worker * A.state_stride + tile_start;
    float4 gv[SUBROWS], mv[SUBROWS], pv[SUBROWS];
    load_tile(g, gv, n_valid);
    if (MOM) load_tile(m, mv, n_valid);
    load_tile(e, pv, n_valid);
    worker_values<MOM>(gv, mv, pv, A.mu, A.r);
    if (MOM) store_tile(m, mv, n_valid);
    float *scales_out = A.scales + (int64_t)worker * A.scales_stride;
    compress_mixed(pv, L, tile, n_valid, A.signs + (int64_t)worker * A.signs_stride, scales_out, e, X, worker, S);
}

// Uniform tiles of the worker as a persistent kernel.
//
// Every workgroup loops: take the next tile, issue its loads, and while they
// are in flight write out the oldest of the tiles it holds: the last
// PIPE_DEPTH in registers and, behind them, STAGE_DEPTH more in LDS (a tile
// leaving the registers is not written out yet but moved to LDS and written
// out STAGE_DEPTH tiles later; one LDS round trip per element doubles the
// number of tiles in flight, hence the size of the blocks that finish in one
// pass).  By then its block's scale has had six tile-times to form, so the
// wait is normally over before it starts.  Then the workgroup computes the new
// tile, posts its partial sum and keeps it in turn.  Tiles are handed out one
// by one through a ticket counter, so at any moment the resident workgroups
// work on one compact, advancing window of the fp32 streams (best DRAM page
// locality, no dependence on dispatch order).  A workgroup never waits for a
// block of which it still holds an unposted tile, so a wait only ever depends
// on workgroups that wait for strictly older blocks; it could starve only if
// one block had more than (resident workgroups x 6) uniform tiles, which
// fuse_limit rules out, and it is bounded by spin_limit in any case.
//
// What is streamed comes from a producer (Algorithm 4 or Algorithm 3 worker):
//   issue(L, idx, tile)        start the tile's loads (idx: which worker)
//   produce(L, idx, tile, p)   the corrected values p of Algorithm 4 (and the role's other stores)
//   signs(L, idx), scales(L, idx), err_tile(idx, tile)   where that participant's outputs go
struct HeldTile {
    float4 p[SUBROWS];
    int32_t tile;
    int idx;
    int b;                      // < 0: slot empty
};

// A tile that has left the registers for the workgroup's LDS: every lane keeps
// its own 16 values at its own addresses, so no barrier is needed.
struct StagedTile {
    int32_t tile;
    int idx;
    int b;                      // < 0: slot empty
    int slot;                   // which third of the stage buffer holds its p
};

__device__ __forceinline__ void stage_store(float *stage, int slot, const float4 (&p)[SUBROWS])
{
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) *reinterpret_cast<float4 *>(stage + slot * TILE + local_base(k)) = p[k];
}
__device__ __forceinline__ void stage_load(const float *stage, int slot, float4 (&p)[SUBROWS])
{
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) p[k] = *reinterpret_cast<const float4 *>(stage + slot * TILE + local_base(k));
}

constexpr int STAGE_DEPTH = 3;      // tiles a workgroup keeps in LDS behind the PIPE_DEPTH it keeps in registers

template <class Producer>
__device__ __forceinline__ void persistent_uniform(const Layout &L, const Scratch &X, Producer &prod, int n_part,
                                                   SyncShared &S, float *stage)
{
    const unsigned per_part = (unsigned)L.n_uniform;
    const unsigned total = per_part * (unsigned)n_part;

    HeldTile held[PIPE_DEPTH];
#pragma unroll
    for (int q = 0; q < PIPE_DEPTH; ++q) held[q].b = -1;
    StagedTile staged[STAGE_DEPTH];
#pragma unroll
    for (int q = 0; q < STAGE_DEPTH; ++q) {
        staged[q].b = -1;
        staged[q].slot = q;
        staged[q].tile = 0;
        staged[q].idx = 0;
    }
    Posted posted;
    clear_posted(posted);
    int posted_idx = 0;

    unsigned tk_next = 0;       // thread 0: the ticket taken ahead of need
    if (threadIdx.x == 0) tk_next = atomicAdd(X.ticket, 1u);

    for (;;) {
        // ---- next tile
        if (threadIdx.x == 0) S.ticket = tk_next;
        __syncthreads();
        const unsigned t = (unsigned)__builtin_amdgcn_readfirstlane((int)S.ticket);
        __syncthreads();
        if (t >= total) break;
        if (threadIdx.x == 0) tk_next = atomicAdd(X.ticket, 1u);   // the answer is read at the next tile
        const int idx = (int)(t / per_part);
        const int32_t tile = L.uniform_tiles[t % per_part];
        const int set = X.set_base + idx;

        // ---- this tile's loads go out first
        prod.issue(L, idx, tile);

        // ---- while they fly: follow up on the previous tile's post, write out the oldest tile held
        const int old_b = staged[0].b;
        const int old_idx = staged[0].idx;
        const int32_t old_tile = staged[0].tile;
        const unsigned long long peeked = peek_ready(old_b, L, X, X.set_base + (old_b >= 0 ? old_idx : 0));
        resolve_posted(posted, L, X, X.set_base + posted_idx, prod.scales(L, posted_idx), S);
        if (old_b >= 0) {
            // The block of the oldest tile cannot complete while this workgroup sits on a tile of
            // the same block that is not posted yet (the new one): then do not wait, park p and
            // leave the tile to the second pass.
            const bool may_wait = !(old_idx == idx && L.tile_fb[tile] == old_b);
            float4 pv_old[SUBROWS];
            stage_load(stage, staged[0].slot, pv_old);
            finish_uniform(pv_old, old_tile, TILE, old_b, peeked, prod.err_tile(old_idx, old_tile), L, X,
                           X.set_base + old_idx, S, may_wait);
        }
        {
            // the oldest register tile takes the LDS slot that has just become free
            const int free_slot = staged[0].slot;
#pragma unroll
            for (int q = 0; q + 1 < STAGE_DEPTH; ++q) staged[q] = staged[q + 1];
            StagedTile &in = staged[STAGE_DEPTH - 1];
            in.slot = free_slot;
            in.b = held[0].b;
            in.tile = held[0].tile;
            in.idx = held[0].idx;
            if (held[0].b >= 0) stage_store(stage, free_slot, held[0].p);
        }
#pragma unroll
        for (int q = 0; q + 1 < PIPE_DEPTH; ++q) held[q] = held[q + 1];

        // ---- the new tile
        float4 pv[SUBROWS];
        prod.produce(L, idx, tile, pv);
        HeldTile &slot = held[PIPE_DEPTH - 1];
        const int kind = compress_uniform(pv, L, tile, TILE, prod.signs(L, idx), prod.scales(L, idx),
                                          prod.err_tile(idx, tile), X, set, S, posted);
        posted_idx = idx;
        slot.b = -1;
        if (kind == UNI_PENDING) {
#pragma unroll
            for (int k = 0; k < SUBROWS; ++k) slot.p[k] = pv[k];
            slot.tile = tile;
            slot.idx = idx;
            slot.b = L.tile_fb[tile];
        }
    }

    // ---- drain, oldest first
    resolve_posted(posted, L, X, X.set_base + posted_idx, prod.scales(L, posted_idx), S);
#pragma unroll
    for (int q = 0; q < STAGE_DEPTH; ++q) {
        if (staged[q].b >= 0) {
            float4 pv_old[SUBROWS];
            stage_load(stage, staged[q].slot, pv_old);
            finish_uniform(pv_old, staged[q].tile, TILE, staged[q].b, 0ull, prod.err_tile(staged[q].idx, staged[q].tile),
                           L, X, X.set_base + staged[q].idx, S);
        }
    }
#pragma unroll
    for (int q = 0; q < PIPE_DEPTH; ++q) {
        if (held[q].b >= 0)
            finish_uniform(held[q].p, held[q].tile, TILE, held[q].b, 0ull, prod.err_tile(held[q].idx, held[q].tile), L,
                           X, X.set_base + held[q].idx, S);
    }
}

template <bool MOM>
struct WorkerProducer {
    WorkerArgs A;
    const Scratch *X;
    float4 gv[SUBROWS], mv[SUBROWS], ev[SUBROWS];
    LoadedCorrection corr;

    __device__ __forceinline__ uint64_t *signs(const Layout &L, int idx) const { return A.signs + (int64_t)idx * A.signs_stride; }
    __device__ __forceinline__ float *scales(const Layout &L, int idx) const { return A.scales + (int64_t)idx * A.scales_stride; }
    __device__ __forceinline__ float *err_tile(int idx, int32_t tile) const
    {
        return A.err + (int64_t)idx * A.state_stride + (int64_t)tile * TILE;
    }
    __device__ __forceinline__ void issue(const Layout &L, int idx, int32_t tile)
    {
        const int64_t tile_start = (int64_t)tile * TILE;
        corr = loaded_correction(L, tile, *X, X->set_base + idx);
        load_tile(A.grad + (int64_t)idx * A.grad_stride + tile_start, gv, TILE);
        if (MOM) load_tile(A.mom + (int64_t)idx * A.state_stride + tile_start, mv, TILE);
        load_tile(A.err + (int64_t)idx * A.state_stride + tile_start, ev, TILE);
    }
    __device__ __forceinline__ void produce(const Layout &L, int idx, int32_t tile, float4 (&p)[SUBROWS])
    {
        correct_loaded_residual(ev, corr);
        worker_values<MOM>(gv, mv, ev, A.mu, A.r);
        if (MOM) store_tile(A.mom + (int64_t)idx * A.state_stride + (int64_t)tile * TILE, mv, TILE);
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) p[k] = ev[k];
    }
};

template <bool MOM>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(3, 3)))
void k_worker_uniform(Layout L, ScratchRef R, WorkerArgs A, int n_workers)
{
    const Scratch X = open_call(R);
    __shared__ SyncShared S;
    __shared__ float stage[STAGE_DEPTH * TILE];     // 48 KiB: three workgroups per CU, as the registers allow
    WorkerProducer<MOM> prod;
    prod.A = A;
    prod.X = &X;
    persistent_uniform(L, X, prod, n_workers, S, stage);
}

// All tiles of all workers in one launch, one workgroup per (tile, worker): the mixed tiles first
// (the first n_mixed workgroups of every worker's row of the grid), then the whole tiles in
// ascending order.  A whole tile goes through the steps of the persistent kernel without the
// pipeline: the workgroup waits in place for its block's scale; the momentum tile is written at
// once, the residual tile when the scale is there, so the tiles of a block write their residuals
// in step.  The mixed tiles run the mixed-tile code and never wait for a whole tile (MIXED =
// false: the layout has no such tile, and the code for them is left out).  Relies on workgroups
// being dispatched in grid order (the mixed tiles' partial sums are posted before a block's last
// whole tile looks for them; fuse_limit keeps a block's tiles well inside what is resident at
// once) and on spin_limit where that fails.
// Eight workgroups per CU (64 VGPRs, a few spilled): the one-pass limit is half of what is
// resident, and 2048 resident workgroups let blocks of up to 1024 tiles (4 Mi elements) finish
// in one pass (measured: 27.1 -> 24.4 ms on the transformer-like layout, no change elsewhere).
template <bool MOM, bool QUAL>
__device__ __forceinline__ void worker_mixed_tile(const Layout &L, const Scratch &X, const WorkerArgs &A,
                                                  const QualityArgs &Q, int32_t tile, int worker, int n_valid,
                                                  TileShared &S)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const float *g = A.grad + (int64_t)worker * A.grad_stride + tile_start;
    float *m = MOM ? A.mom + (int64_t)worker * A.state_stride + tile_start : nullptr;
    float *e = A.err + (int64_t)worker * A.state_stride + tile_start;
    float4 gv[SUBROWS], mv[SUBROWS], pv[SUBROWS];
    load_tile(g, gv, n_valid);
    if (MOM) load_tile(m, mv, n_valid);
    load_tile(e, pv, n_valid);
    worker_values<MOM>(gv, mv, pv, A.mu, A.r);
    if (MOM) store_tile(m, mv, n_valid);
    if constexpr (QUAL) {
        float4 a[SUBROWS];
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) a[k] = pv[k];
        quality_of_tile(a, L, Q, tile, worker, n_valid, S);
    }
    compress_mixed(pv, L, tile, n_valid, A.signs + (int64_t)worker * A.signs_stride,
                   A.scales + (int64_t)worker * A.scales_stride, e, X, worker, S);
}

template <bool MIXED>
struct TilesShared {
    typedef SyncShared type;
};
template <>
struct TilesShared<true> {
    typedef TileShared type;
};

// QUAL = true: the compressor-quality sums of p (Section 3.2: Proposition 1's phi, Eq. (1)'s delta)
// are taken on the way, from the values the kernel holds anyway (see ef_quality.h).
template <bool MOM, bool MIXED, bool QUAL>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(8, 8)))
void k_worker_tiles(Layout L, ScratchRef R, WorkerArgs A, QualityArgs Q)
{
    const Scratch X = open_call(R);
    __shared__ typename TilesShared<MIXED || QUAL>::type S;
    const bool whole = !MIXED || (int)blockIdx.x >= L.n_mixed;
    // without mixed tiles the list of whole tiles is 0, 1, 2, ...: one dependent load less
    const int32_t tile = !MIXED ? (int32_t)blockIdx.x : whole ? L.uniform_tiles[blockIdx.x - L.n_mixed] : L.mixed_tiles[blockIdx.x];
    const int worker = blockIdx.y;
    const int n_valid = whole ? TILE : tile_valid(L, tile);
    const int64_t tile_start = (int64_t)tile * TILE;
    const float *g = A.grad + (int64_t)worker * A.grad_stride + tile_start;
    float *m = MOM ? A.mom + (int64_t)worker * A.state_stride + tile_start : nullptr;
    float *e = A.err + (int64_t)worker * A.state_stride + tile_start;
    float *scales_out = A.scales + (int64_t)worker * A.scales_stride;
    uint64_t *signs = A.signs + (int64_t)worker * A.signs_stride;
    float4 gv[SUBROWS], mv[SUBROWS], pv[SUBROWS];
    if (whole) {
        Posted P;
        const LoadedCorrection corr = loaded_correction(L, tile, X, worker);
        load_tile(g, gv, TILE);
        if (MOM) load_tile(m, mv, TILE);
        load_tile(e, pv, TILE);
        correct_loaded_residual(pv, corr);
        worker_values<MOM>(gv, mv, pv, A.mu, A.r);
        if (MOM) store_tile(m, mv, TILE);
        if constexpr (QUAL) {
            float4 a[SUBROWS];
#pragma unroll
            for (int k = 0; k < SUBROWS; ++k) a[k] = pv[k];
            quality_of_tile(a, L, Q, tile, worker, TILE, S);
        }
        const int kind = compress_uniform(pv, L, tile, TILE, signs, scales_out, e, X, worker, S, P, true);
        resolve_posted(P, L, X, worker, scales_out, S);
        if (kind == UNI_PENDING) {
            finish_uniform(pv, tile, TILE, L.tile_fb[tile], 0ull, e, L, X, worker, S);
        } else if (kind == UNI_HELD) {
            sync_group_wait(tile, L, X, worker, S);
            store_tile(e, pv, TILE);
        }
    } else if constexpr (MIXED) {
        worker_mixed_tile<MOM, QUAL>(L, X, A, Q, tile, worker, n_valid, S);
    }
}

}  // namespace ef
