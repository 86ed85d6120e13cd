// Bandwidth probe: the worker kernel's memory traffic with nothing else in it.
//
// Per 4096-element tile it reads g, m and e and writes m and e (20 bytes per element, Algorithm
// 4's worker state without the sign words), with the worker kernel's loads and stores, tile shape
// and hand-out of tiles by a ticket counter, but no compression, no cross-tile reduction and no
// waiting.  What it reaches is the practical ceiling of this access pattern on the machine at
// hand, to set beside the worker kernel's own rate.  The arithmetic only keeps the compiler from
// dropping the loads; the buffers' contents afterwards are of no use.
#pragma once
#include "ef_tile.h"

namespace ef {

__global__ void k_probe_reset(unsigned int *ticket)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *ticket = 0u;
}

__global__ __launch_bounds__(THREADS) void k_probe_stream(const float *g, float *m, float *e, unsigned n_tiles,
                                                          unsigned int *ticket)
{
    __shared__ unsigned s_ticket;
    for (;;) {
        if (threadIdx.x == 0) s_ticket = atomicAdd(ticket, 1u);
        __syncthreads();
        const unsigned t = s_ticket;
        __syncthreads();
        if (t >= n_tiles) break;
        const int64_t start = (int64_t)t * TILE;
        float4 gv[SUBROWS], mv[SUBROWS], ev[SUBROWS];
        load_tile(g + start, gv, TILE);
        load_tile(m + start, mv, TILE);
        load_tile(e + start, ev, TILE);
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) {
            mv[k].x = 0.5f * mv[k].x + gv[k].x;
            mv[k].y = 0.5f * mv[k].y + gv[k].y;
            mv[k].z = 0.5f * mv[k].z + gv[k].z;
            mv[k].w = 0.5f * mv[k].w + gv[k].w;
            ev[k].x = 0.5f * ev[k].x + mv[k].x;
            ev[k].y = 0.5f * ev[k].y + mv[k].y;
            ev[k].z = 0.5f * ev[k].z + mv[k].z;
            ev[k].w = 0.5f * ev[k].w + mv[k].w;
        }
        store_tile(m + start, mv, TILE);
        store_tile(e + start, ev, TILE);
    }
}

// The same traffic with one workgroup per tile, the residual-like array e written in step: the
// workgroups of `group` consecutive tiles write m at once, then wait (bounded) until all of them
// have loaded their tile, then write e.  `arrive` holds one word per tile, `line` one 128-byte line
// per tile (the group's last tile posts there); both carry the pass number, so nothing has to be
// cleared between passes.  This is the access pattern of the worker kernel's one-pass blocks and
// of its sync groups, without the compression.
__global__ __launch_bounds__(THREADS) void k_probe_grouped(const float *g, float *m, float *e, unsigned n_tiles,
                                                           int group, unsigned pass, unsigned int *arrive,
                                                           unsigned long long *line, int spin_limit)
{
    const unsigned t = blockIdx.x;
    if (t >= n_tiles) return;
    const int64_t start = (int64_t)t * TILE;
    float4 gv[SUBROWS], mv[SUBROWS], ev[SUBROWS];
    load_tile(g + start, gv, TILE);
    load_tile(m + start, mv, TILE);
    load_tile(e + start, ev, TILE);
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        mv[k].x = 0.5f * mv[k].x + gv[k].x;
        mv[k].y = 0.5f * mv[k].y + gv[k].y;
        mv[k].z = 0.5f * mv[k].z + gv[k].z;
        mv[k].w = 0.5f * mv[k].w + gv[k].w;
        ev[k].x = 0.5f * ev[k].x + mv[k].x;
        ev[k].y = 0.5f * ev[k].y + mv[k].y;
        ev[k].z = 0.5f * ev[k].z + mv[k].z;
        ev[k].w = 0.5f * ev[k].w + mv[k].w;
    }
    store_tile(m + start, mv, TILE);
    if (group > 1) {
        const unsigned g0 = t / (unsigned)group * (unsigned)group;
        const unsigned g1 = min(g0 + (unsigned)group - 1u, n_tiles - 1u);
        __syncthreads();                // every lane's loads have arrived
        if (threadIdx.x == 0) __hip_atomic_store(arrive + t, pass, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (t == g1) {
            const int others = (int)(g1 - g0);
            for (int it = 0; it < spin_limit; ++it) {
                int all = 1;
                if ((int)threadIdx.x < others)
                    all = __hip_atomic_load(arrive + g0 + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == pass;
                if (__syncthreads_and(all)) break;
                __builtin_amdgcn_s_sleep(8);
            }
            if (threadIdx.x == 0)
                __hip_atomic_store(line + (int64_t)g1 * READY_STRIDE, (unsigned long long)pass, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        } else {
            if (threadIdx.x == 0) {
                for (int it = 0; it < spin_limit; ++it) {
                    if (__hip_atomic_load(line + (int64_t)g1 * READY_STRIDE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                        (unsigned long long)pass)
                        break;
                    __builtin_amdgcn_s_sleep(8);
                }
            }
            __syncthreads();
        }
    }
    store_tile(e + start, ev, TILE);
}

}  // namespace ef
