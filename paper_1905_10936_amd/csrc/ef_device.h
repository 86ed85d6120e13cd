// Device side of libef: tile-based kernels for the worker, server and apply
// steps of Algorithm 4 (dist-EF-blockSGDM, arxiv 1905.10936), written for
// gfx950 (64-lane wavefronts, 256 CUs in 8 XCDs, HBM-bound streaming passes).
//
// Work decomposition
// ------------------
// The flat d-vector is cut into tiles of TILE = 4096 consecutive elements, one
// 256-thread workgroup per (tile, worker).  Tiles, not blocks, are the unit of
// work, so a block of 8M elements and a block of 1 element cost the same per
// element.  A tile is a whole number of 64-element sign words and starts on a
// 16 KiB boundary, so every fp32 access is a coalesced 128-bit access whatever
// the block boundaries are.  Inside a tile, wavefront w owns the 1024
// consecutive elements [1024w, 1024w+1024) as 4 sub-rows of 256; lane l of
// sub-row k holds the 4 consecutive elements 1024w + 256k + 4l .. +3.
//
// The blocks of the partition (Section 3.2) cut a tile into segments.  A
// segment whose block lies entirely inside the tile is "closed": its L1 norm,
// scale and residual are finished by the tile alone.  At most two segments of
// a tile are "open" (the block continues into a neighbouring tile).  Their fp64
// partial sums go to a per-(tile, slot) scratch word.  Whoever needs the
// block's scale adds the block's partials in one fixed order (thread t takes
// tiles t, t+256, ... in ascending order, then a fixed tree), so the scale has
// the same bits wherever and whenever it is computed.
//
// One pass over the state
// -----------------------
// e <- p - Delta needs the block's scale, i.e. every tile of the block.  For a
// block of at most `fuse_limit` tiles the workgroups keep p in registers, post
// their partial and poll (bounded) the partial words of the block's other tiles
// until all carry this call's tag, then write the finished residual, so every
// fp32 tensor is read once and written once.  A partial is never negative, so
// its sign bit is free to carry the tag, which flips on every call that uses
// the scratch set: a word is "of this call" exactly when its tag matches, and
// one relaxed agent-scope 64-bit store publishes value and tag together -- no
// counters, no fences (an agent-scope release fence would write back the whole
// L2 of streaming stores on every tile).  The wait cannot starve: all partials
// of a tile are posted before its first wait, workgroups are dispatched in grid
// order, and fuse_limit keeps a block's tiles well inside what is resident at
// once.  Should a wait still run out of its spin budget, or for blocks larger
// than fuse_limit, the workgroup parks p in the residual buffer instead; a small
// kernel then computes the scales still missing and another subtracts the
// decoded value where p was parked.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ef {

constexpr int TILE = 4096;      // elements per workgroup
constexpr int THREADS = 256;    // 4 wavefronts
constexpr int NWAVES = THREADS / 64;
constexpr int SUBROWS = 4;      // float4 per thread
constexpr int SMALL_SEG = 64;   // segments up to this length are summed by one thread
constexpr int MAX_LONG = TILE / SMALL_SEG;
constexpr int DEFER_WGS = 64;   // workgroups of the kernel that finishes deferred segments

struct Layout {
    int64_t d;                  // elements
    int64_t B;                  // blocks
    int64_t W;                  // sign words
    int32_t ntiles;
    int32_t fuse_limit;         // blocks of up to this many tiles finish in one pass
    const int64_t *offs;        // [B+1] device copy of block_offsets
    const int32_t *tile_fb;     // [ntiles] block holding the tile's first element
    const int32_t *tile_lb;     // [ntiles] block holding the tile's last valid element
};

// Scratch of one call.  A "set" is one worker, or the server.
struct Scratch {
    unsigned long long *part;   // [nsets][2*ntiles] tagged fp64 partial sums of open segments
    unsigned int *cnt;          // [nsets][B] arrivals per one-pass block, 0 between calls
    unsigned long long *ready;  // [nsets][B] (tag << 32) | scale bits, posted by the last arriver
    unsigned int *defer_cnt;    // entries in defer_list for this call
    unsigned long long *defer_list;  // parked segments: (set << 33) | (tile << 1) | slot
    unsigned int *fin_cnt;      // entries in fin_list for this call
    unsigned long long *fin_list;    // blocks whose scale is still to be written: (set << 32) | block
    unsigned long long tags;    // bit i = this call's tag of set (set_base + i)
    int set_base;               // first set this call uses (0 for workers, max_workers for the server)
    int spin_limit;             // polls before a waiting workgroup gives up and parks p
};

struct WorkerArgs {
    const float *grad; int64_t grad_stride;
    float *mom; float *err; int64_t state_stride;
    float mu, r;
    uint64_t *signs; float *scales;
};

struct ServerArgs {
    int M;
    const uint64_t *signs_in;   // [M][W]
    const float *scales_in;     // [M][B]
    float *err;                 // server residual
    float r, Mf;
    uint64_t *signs; float *scales;
};

// ---------------------------------------------------------------- helpers ---

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }
// first local element of this thread's float4 in sub-row k
__device__ __forceinline__ int local_base(int k) { return wave_id() * 1024 + k * 256 + lane_id() * 4; }

// The fp32 state is streamed: each element is read once and written once per
// call, so loads and stores carry the non-temporal hint and do not displace
// the little that is reused (offsets, scales, partial sums) from the caches.
typedef float vf4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4 stream_load4(const float *p)
{
    const vf4 v = __builtin_nontemporal_load(reinterpret_cast<const vf4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void stream_store4(float *p, float4 a)
{
    const vf4 v = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(v, reinterpret_cast<vf4 *>(p));
}

template <bool FULL>
__device__ __forceinline__ float4 load4(const float *base, int local, int n_valid)
{
    if (FULL || local + 4 <= n_valid) return stream_load4(base + local);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (local + 0 < n_valid) v.x = base[local + 0];
    if (local + 1 < n_valid) v.y = base[local + 1];
    if (local + 2 < n_valid) v.z = base[local + 2];
    return v;                   // local + 3 < n_valid would have taken the vector path
}

template <bool FULL>
__device__ __forceinline__ void store4(float *base, int local, int n_valid, float4 v)
{
    if (FULL || local + 4 <= n_valid) { stream_store4(base + local, v); return; }
    if (local + 0 < n_valid) base[local + 0] = v.x;
    if (local + 1 < n_valid) base[local + 1] = v.y;
    if (local + 2 < n_valid) base[local + 2] = v.z;
}

// Butterfly sum over the 64 lanes: every lane ends with the same bits.
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// Workgroup sum in a fixed order; every thread gets the same bits.
__device__ __forceinline__ double block_sum(double v, double *red)
{
    v = wave_sum(v);
    if (lane_id() == 0) red[wave_id()] = v;
    __syncthreads();
    double t = ((red[0] + red[1]) + red[2]) + red[3];
    __syncthreads();
    return t;
}

// value the payload stands for: +s if bit else -s (negation is exact)
__device__ __forceinline__ float signed_scale(float s, bool plus) { return plus ? s : -s; }
// e' = p - Delta for one element whose block has scale s
__device__ __forceinline__ float residual(float p, float s) { return p - signed_scale(s, p >= 0.f); }

// Pack the signs of this thread's 16 values into the wavefront's 16 sign words
// and store them.  nib[k] holds the 4 sign bits of sub-row k (bit c = element c).
// Within a sub-row, 16 consecutive lanes make one 64-bit word.
__device__ __forceinline__ void pack_and_store_signs(const unsigned nib[SUBROWS], uint64_t *signs,
                                                     int64_t tile_start, int64_t W)
{
    const int lane = lane_id();
    const int l16 = lane & 15;
    const unsigned sh = (unsigned)(l16 & 7) * 4u;
    unsigned mylo = 0, myhi = 0;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        unsigned lo = (l16 < 8) ? (nib[k] << sh) : 0u;
        unsigned hi = (l16 >= 8) ? (nib[k] << sh) : 0u;
#pragma unroll
        for (int off = 1; off <= 8; off <<= 1) {
            lo |= (unsigned)__shfl_xor((int)lo, off);
            hi |= (unsigned)__shfl_xor((int)hi, off);
        }
        if (l16 == k) { mylo = lo; myhi = hi; }
    }
    if (l16 < SUBROWS) {
        // lane 16q + k holds word 4k + q of the wavefront's 16 words
        const int64_t w = (tile_start + wave_id() * 1024) / 64 + 4 * l16 + (lane >> 4);
        if (w < W) signs[w] = ((uint64_t)myhi << 32) | (uint64_t)mylo;
    }
}

struct TileShared {
    float val[TILE];            // |p| per element, then the element's scale (closed segments)
    double red[NWAVES];
    double open_sum[2];
    int long_list[MAX_LONG];
    int n_long;
    int last[2];                // this workgroup arrived last at its first / last segment's block
    int flag[2];
};

// Per-call view of one set's scratch and outputs.
struct SetCtx {
    unsigned long long *part;   // [2*ntiles]
    unsigned int *cnt;          // [B]
    unsigned long long *ready;  // [B]
    unsigned int *defer_cnt;
    unsigned long long *defer_list;
    unsigned int *fin_cnt;
    unsigned long long *fin_list;
    unsigned long long tag;     // 0 or 1
    int spin_limit;
    int set;
    float *scales_out;          // [B]
};

__device__ __forceinline__ SetCtx make_ctx(const Scratch &X, const Layout &L, int set, float *scales_out)
{
    SetCtx c;
    c.part = X.part + (int64_t)set * 2 * L.ntiles;
    c.cnt = X.cnt + (int64_t)set * L.B;
    c.ready = X.ready + (int64_t)set * L.B;
    c.defer_cnt = X.defer_cnt;
    c.defer_list = X.defer_list;
    c.fin_cnt = X.fin_cnt;
    c.fin_list = X.fin_list;
    c.tag = (X.tags >> (set - X.set_base)) & 1ull;
    c.spin_limit = X.spin_limit;
    c.set = set;
    c.scales_out = scales_out;
    return c;
}

// ------------------------------------------ cross-tile block reductions ---

constexpr unsigned long long TAG_BIT = 1ull << 63;
constexpr int MAX_PER_THREAD = 4;                       // partial words a thread polls
constexpr int FUSE_LIMIT_MAX = MAX_PER_THREAD * THREADS; // tiles of the largest one-pass block

__device__ __forceinline__ int block_tiles(const Layout &L, int64_t b)
{
    return (int)((L.offs[b + 1] - 1) / TILE - L.offs[b] / TILE + 1);
}

// Scratch word of block b's segment in tile t (t0 = b's first tile): slot 1 of
// tile t0 if b starts inside that tile (it is then the tile's last segment),
// slot 0 everywhere else (first or only segment).
__device__ __forceinline__ int64_t part_index(int64_t t, int64_t t0, int64_t bs)
{
    return 2 * t + ((t == t0 && (bs % TILE) != 0) ? 1 : 0);
}

// Post the partial sum of an open segment of block b and, for a one-pass
// block, count the arrival.  which: 0 = the tile's first (or only) segment,
// 1 = its last segment.  Never waits; S.last[which] is valid after the next
// __syncthreads().
__device__ __forceinline__ void post_partial(double partial, int which, int32_t tile, int64_t b, const Layout &L,
                                             const SetCtx &C, TileShared &S)
{
    if (threadIdx.x == 0) {
        const unsigned long long w = (unsigned long long)__double_as_longlong(partial) | (C.tag ? TAG_BIT : 0ull);
        __hip_atomic_store(C.part + 2 * (int64_t)tile + which, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int last = 0;
        const int n = block_tiles(L, b);
        if (n <= L.fuse_limit) {
            // The store above need not have landed when the count does: whoever
            // reads the partials checks their tags.
            const unsigned prev = __hip_atomic_fetch_add(C.cnt + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            last = (prev + 1u == (unsigned)n) ? 1 : 0;
        }
        S.last[which] = last;
    }
}

// Sum of block b's partials once the kernel that posted them has finished.
// Same order as gather_scale.  Called by every thread of the workgroup.
__device__ __forceinline__ double sum_block_partials(const Layout &L, int64_t b, const unsigned long long *part,
                                                     double *red)
{
    const int64_t bs = L.offs[b], be = L.offs[b + 1];
    const int64_t t0 = bs / TILE, t1 = (be - 1) / TILE;
    double acc = 0.0;
    for (int64_t t = t0 + threadIdx.x; t <= t1; t += THREADS)
        acc += __longlong_as_double((long long)(part[part_index(t, t0, bs)] & ~TAG_BIT));
    return block_sum(acc, red);
}

// Wait (bounded) until every tile of block b has posted this call's partial,
// then form the block's scale.  Called by every thread of the workgroup with
// the same arguments; returns the same answer to all of them.
__device__ __forceinline__ bool gather_scale(int64_t b, const Layout &L, const SetCtx &C, TileShared &S, float *s)
{
    const int64_t bs = L.offs[b], be = L.offs[b + 1];
    const int64_t t0 = bs / TILE, t1 = (be - 1) / TILE;
    const int n = (int)(t1 - t0 + 1);                   // <= fuse_limit <= FUSE_LIMIT_MAX
    double v[MAX_PER_THREAD];
    unsigned have = 0;
#pragma unroll
    for (int q = 0; q < MAX_PER_THREAD; ++q) v[q] = 0.0;
    bool ok = false;
    for (int it = 0; it < C.spin_limit; ++it) {
        int all = 1;
#pragma unroll
        for (int q = 0; q < MAX_PER_THREAD; ++q) {
            const int i = (int)threadIdx.x + q * THREADS;
            if (i < n && !((have >> q) & 1u)) {
                const unsigned long long w = __hip_atomic_load(C.part + part_index(t0 + i, t0, bs), __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT);
                if ((w >> 63) == C.tag) {
                    v[q] = __longlong_as_double((long long)(w & ~TAG_BIT));
                    have |= 1u << q;
                } else {
                    all = 0;
                }
            }
        }
        if (__syncthreads_and(all)) {
            ok = true;
            break;
        }
        __builtin_amdgcn_s_sleep(8);
    }
    if (!ok) return false;
    double acc = 0.0;
#pragma unroll
    for (int q = 0; q < MAX_PER_THREAD; ++q) acc += v[q];   // absent words were left at +0
    const double total = block_sum(acc, S.red);
    *s = (float)(total / (double)(be - bs));
    return true;
}

// The workgroup that arrived last at one-pass block b forms the scale from the
// partials (waiting, bounded, for those still in flight), writes it out and
// posts it for the block's other tiles.  Called by every thread of that
// workgroup.  Does not depend on the progress of any other workgroup.
__device__ __forceinline__ bool finish_block(int64_t b, const Layout &L, const SetCtx &C, TileShared &S, float *s)
{
    const bool ok = gather_scale(b, L, C, S, s);
    if (threadIdx.x == 0) {
        __hip_atomic_store(C.cnt + b, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (ok) {
            C.scales_out[b] = *s;
            __hip_atomic_store(C.ready + b, (C.tag << 32) | (unsigned long long)__float_as_uint(*s), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        } else {
            const unsigned k = atomicAdd(C.fin_cnt, 1u);
            C.fin_list[k] = ((unsigned long long)C.set << 32) | (unsigned long long)b;
        }
    }
    return ok;
}

// Wait (bounded) until the last arriver has posted block b's scale of this call.
// Called by every thread of the workgroup; same answer to all of them.
__device__ __forceinline__ bool wait_ready(int64_t b, const SetCtx &C, TileShared &S, float *s)
{
    if (threadIdx.x == 0) {
        int found = 0;
        unsigned bits = 0;
        for (int it = 0; it < C.spin_limit; ++it) {
            const unsigned long long w = __hip_atomic_load(C.ready + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((w >> 32) == C.tag) {
                found = 1;
                bits = (unsigned)w;
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        S.flag[0] = found;
        S.flag[1] = (int)bits;
    }
    __syncthreads();
    const bool ok = S.flag[0] != 0;
    *s = __uint_as_float((unsigned)S.flag[1]);
    __syncthreads();
    return ok;
}

// Leave an open segment whose p gets parked in the residual buffer to the
// kernels that run after this one.
__device__ __forceinline__ void defer_segment(int32_t tile, int which, const SetCtx &C)
{
    if (threadIdx.x == 0) {
        const unsigned i = atomicAdd(C.defer_cnt, 1u);
        C.defer_list[i] = ((unsigned long long)C.set << 33) | ((unsigned long long)tile << 1) | (unsigned)which;
    }
}

// Compress the tile whose corrected values are in p[][] (Section 3.2): sign
// words, block sums, scales, and the residual e' = p - Delta (Algorithm 4).
template <bool FULL>
__device__ __forceinline__ void compress_tile(float4 (&p)[SUBROWS], const Layout &L, int32_t tile, int n_valid,
                                              uint64_t *signs, float *err_tile, const SetCtx &C, TileShared &S)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];

    // --- signs
    unsigned nib[SUBROWS];
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        const int lb0 = local_base(k);
        unsigned n = (p[k].x >= 0.f ? 1u : 0u) | (p[k].y >= 0.f ? 2u : 0u) | (p[k].z >= 0.f ? 4u : 0u) |
                     (p[k].w >= 0.f ? 8u : 0u);
        if (!FULL) {
            unsigned vm = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) vm |= (lb0 + c < n_valid) ? (1u << c) : 0u;
            n &= vm;
        }
        nib[k] = n;
    }
    pack_and_store_signs(nib, signs, tile_start, L.W);

    if (fb == lb) {
        // --- one block covers the whole tile
        double acc = 0.0;
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) {
            const int lb0 = local_base(k);
            const float a[4] = {fabsf(p[k].x), fabsf(p[k].y), fabsf(p[k].z), fabsf(p[k].w)};
#pragma unroll
            for (int c = 0; c < 4; ++c) acc += (FULL || lb0 + c < n_valid) ? (double)a[c] : 0.0;
        }
        const double total = block_sum(acc, S.red);
        const int64_t bs = L.offs[fb], be = L.offs[fb + 1];
        const bool closed = (bs >= tile_start) && (be <= tile_start + TILE);
        float s = 0.f;
        bool have_scale = closed;
        if (closed) {
            s = (float)(total / (double)(be - bs));
            if (threadIdx.x == 0) C.scales_out[fb] = s;
        } else {
            post_partial(total, 0, tile, fb, L, C, S);
            if (block_tiles(L, fb) <= L.fuse_limit) {
                __syncthreads();
                have_scale = S.last[0] ? finish_block(fb, L, C, S, &s) : wait_ready(fb, C, S, &s);
                if (!have_scale) defer_segment(tile, 0, C);
            }
        }
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) {
            float4 e = p[k];
            if (have_scale) {
                e.x = residual(p[k].x, s);
                e.y = residual(p[k].y, s);
                e.z = residual(p[k].z, s);
                e.w = residual(p[k].w, s);
            }
            store4<FULL>(err_tile, local_base(k), n_valid, e);
        }
        return;
    }

    // --- several blocks meet in this tile: segmented sums through LDS
    const int nseg = lb - fb + 1;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        float4 a = make_float4(fabsf(p[k].x), fabsf(p[k].y), fabsf(p[k].z), fabsf(p[k].w));
        *reinterpret_cast<float4 *>(&S.val[local_base(k)]) = a;
    }
    if (threadIdx.x == 0) S.n_long = 0;
    __syncthreads();
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
        double acc = 0.0;
        for (int j = lo; j < hi; ++j) acc += (double)S.val[j];
        const bool open = (sg == 0 && head_open) || (sg == nseg - 1 && tail_open);
        if (open) {
            S.open_sum[sg == 0 ? 0 : 1] = acc;
        } else {
            const float sc = (float)(acc / (double)(be - bs));
            C.scales_out[b] = sc;
            for (int j = lo; j < hi; ++j) S.val[j] = sc;
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
        double acc = 0.0;
        for (int j = lo + lane_id(); j < hi; j += 64) acc += (double)S.val[j];
        acc = wave_sum(acc);
        const bool open = (sg == 0 && head_open) || (sg == nseg - 1 && tail_open);
        if (open) {
            if (lane_id() == 0) S.open_sum[sg == 0 ? 0 : 1] = acc;
        } else {
            const float sc = (float)(acc / (double)(be - bs));
            if (lane_id() == 0) C.scales_out[b] = sc;
            for (int j = lo + lane_id(); j < hi; j += 64) S.val[j] = sc;
        }
    }
    __syncthreads();
    const int head_end = head_open ? (int)min(L.offs[fb + 1] - tile_start, (int64_t)n_valid) : 0;
    const int tail_begin = tail_open ? (int)(L.offs[lb] - tile_start) : TILE;
    // post everything this tile owes to others before waiting for anything
    if (threadIdx.x == 0) S.last[0] = S.last[1] = 0;
    if (head_open) post_partial(S.open_sum[0], 0, tile, fb, L, C, S);
    if (tail_open) post_partial(S.open_sum[1], 1, tile, lb, L, C, S);
    __syncthreads();
    const bool head_fused = head_open && block_tiles(L, fb) <= L.fuse_limit;
    const bool tail_fused = tail_open && block_tiles(L, lb) <= L.fuse_limit;
    const bool head_last = head_fused && S.last[0], tail_last = tail_fused && S.last[1];
    float s_head = 0.f, s_tail = 0.f;
    bool have_head = false, have_tail = false;
    // first what others wait for from this workgroup, then what it waits for itself
    if (head_last) have_head = finish_block(fb, L, C, S, &s_head);
    if (tail_last) have_tail = finish_block(lb, L, C, S, &s_tail);
    if (head_fused && !head_last) have_head = wait_ready(fb, C, S, &s_head);
    if (tail_fused && !tail_last) have_tail = wait_ready(lb, C, S, &s_tail);
    if (head_fused && !have_head) defer_segment(tile, 0, C);
    if (tail_fused && !have_tail) defer_segment(tile, 1, C);
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        const int lb0 = local_base(k);
        const float4 sc = *reinterpret_cast<const float4 *>(&S.val[lb0]);
        const float pv[4] = {p[k].x, p[k].y, p[k].z, p[k].w};
        const float sv[4] = {sc.x, sc.y, sc.z, sc.w};
        float ev[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = lb0 + c;
            if (j < head_end) ev[c] = have_head ? residual(pv[c], s_head) : pv[c];
            else if (j >= tail_begin) ev[c] = have_tail ? residual(pv[c], s_tail) : pv[c];
            else ev[c] = residual(pv[c], sv[c]);
        }
        store4<FULL>(err_tile, lb0, n_valid, make_float4(ev[0], ev[1], ev[2], ev[3]));
    }
}

// Fill S.val (read as int) with the segment index of every element of a tile
// that several blocks share, so that element j can look up scale[fb + seg].
__device__ __forceinline__ void build_segment_index(const Layout &L, int32_t tile, int n_valid, int32_t fb,
                                                    int nseg, TileShared &S)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    int *seg = reinterpret_cast<int *>(S.val);
    if (threadIdx.x == 0) S.n_long = 0;
    __syncthreads();
    for (int sg = threadIdx.x; sg < nseg; sg += THREADS) {
        const int lo = (int)max(L.offs[fb + sg] - tile_start, (int64_t)0);
        const int hi = (int)min(L.offs[fb + sg + 1] - tile_start, (int64_t)n_valid);
        if (hi - lo > SMALL_SEG) {
            S.long_list[atomicAdd(&S.n_long, 1)] = sg;
            continue;
        }
        for (int j = lo; j < hi; ++j) seg[j] = sg;
    }
    __syncthreads();
    const int n_long = S.n_long;
    for (int q = wave_id(); q < n_long; q += NWAVES) {
        const int sg = S.long_list[q];
        const int lo = (int)max(L.offs[fb + sg] - tile_start, (int64_t)0);
        const int hi = (int)min(L.offs[fb + sg + 1] - tile_start, (int64_t)n_valid);
        for (int j = lo + lane_id(); j < hi; j += 64) seg[j] = sg;
    }
    __syncthreads();
}

// ------------------------------------------------------------- kernels ---

// Worker (Algorithm 4, "on each worker i"): momentum, corrected value p, sign
// words, block scales, residual.
template <bool FULL>
__device__ __forceinline__ void worker_tile(const Layout &L, const Scratch &X, const WorkerArgs &A, int32_t tile,
                                            int worker, int n_valid, TileShared &S)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const float *g = A.grad + (int64_t)worker * A.grad_stride + tile_start;
    float *m = A.mom + (int64_t)worker * A.state_stride + tile_start;
    float *e = A.err + (int64_t)worker * A.state_stride + tile_start;
    float4 p[SUBROWS];
    float4 gv[SUBROWS], mv[SUBROWS], ev[SUBROWS];
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        gv[k] = load4<FULL>(g, local_base(k), n_valid);
        mv[k] = load4<FULL>(m, local_base(k), n_valid);
        ev[k] = load4<FULL>(e, local_base(k), n_valid);
    }
    const float mu = A.mu, r = A.r;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        float4 mn;
        mn.x = mu * mv[k].x + gv[k].x;
        mn.y = mu * mv[k].y + gv[k].y;
        mn.z = mu * mv[k].z + gv[k].z;
        mn.w = mu * mv[k].w + gv[k].w;
        store4<FULL>(m, local_base(k), n_valid, mn);
        p[k].x = (mu * mn.x + gv[k].x) + r * ev[k].x;
        p[k].y = (mu * mn.y + gv[k].y) + r * ev[k].y;
        p[k].z = (mu * mn.z + gv[k].z) + r * ev[k].z;
        p[k].w = (mu * mn.w + gv[k].w) + r * ev[k].w;
    }
    const SetCtx C = make_ctx(X, L, worker, A.scales + (int64_t)worker * L.B);
    compress_tile<FULL>(p, L, tile, n_valid, A.signs + (int64_t)worker * L.W, e, C, S);
}

__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_worker(Layout L, Scratch X, WorkerArgs A)
{
    __shared__ TileShared S;
    const int32_t tile = blockIdx.x;
    const int worker = blockIdx.y;
    const int64_t left = L.d - (int64_t)tile * TILE;
    if (left >= TILE) worker_tile<true>(L, X, A, tile, worker, TILE, S);
    else worker_tile<false>(L, X, A, tile, worker, (int)left, S);
}

// Server (Algorithm 4, "on server"): decode and add the M payloads in worker
// order, divide by M, add the rescaled server residual, compress.
template <bool FULL>
__device__ __forceinline__ void server_tile(const Layout &L, const Scratch &X, const ServerArgs &A, int32_t tile,
                                            int set, int n_valid, TileShared &S)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    float *te = A.err + tile_start;
    float4 tv[SUBROWS];
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) tv[k] = load4<FULL>(te, local_base(k), n_valid);

    float acc[SUBROWS][4];
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[k][c] = 0.0f;

    // this lane's 4 sign bits of sub-row k live in the 32-bit half-word below
    const uint32_t *s32 = reinterpret_cast<const uint32_t *>(A.signs_in);
    int64_t hw[SUBROWS];
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) hw[k] = (tile_start + local_base(k)) >> 5;
    const unsigned sh = (unsigned)(lane_id() & 7) * 4u;
    const int64_t n_hw = 2 * L.W;

    int segi[SUBROWS][4];
    if (fb != lb) {
        build_segment_index(L, tile, n_valid, fb, lb - fb + 1, S);
        const int *seg = reinterpret_cast<const int *>(S.val);
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int j = local_base(k) + c;
                segi[k][c] = (j < n_valid) ? seg[j] : 0;
            }
        __syncthreads();        // S.val is reused by compress_tile
    }
    for (int i = 0; i < A.M; ++i) {
        const float *sc_i = A.scales_in + (int64_t)i * L.B + fb;
        const float s_uniform = sc_i[0];
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) {
            const uint32_t word = (hw[k] < n_hw) ? s32[(int64_t)i * n_hw + hw[k]] : 0u;
            const unsigned nibble = (word >> sh) & 0xFu;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float s = (fb == lb) ? s_uniform : sc_i[segi[k][c]];
                acc[k][c] = acc[k][c] + signed_scale(s, (nibble >> c) & 1u);
            }
        }
    }
    float4 p[SUBROWS];
    const float r = A.r, Mf = A.Mf;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        p[k].x = acc[k][0] / Mf + r * tv[k].x;
        p[k].y = acc[k][1] / Mf + r * tv[k].y;
        p[k].z = acc[k][2] / Mf + r * tv[k].z;
        p[k].w = acc[k][3] / Mf + r * tv[k].w;
    }
    const SetCtx C = make_ctx(X, L, set, A.scales);
    compress_tile<FULL>(p, L, tile, n_valid, A.signs, te, C, S);
}

__global__ __launch_bounds__(THREADS) void k_server(Layout L, Scratch X, ServerArgs A, int set)
{
    __shared__ TileShared S;
    const int32_t tile = blockIdx.x;
    const int64_t left = L.d - (int64_t)tile * TILE;
    if (left >= TILE) server_tile<true>(L, X, A, tile, set, TILE, S);
    else server_tile<false>(L, X, A, tile, set, (int)left, S);
}

// e <- p - Delta on one open segment of a tile whose p was parked in the
// residual buffer (e_{t+1} = p_t - Delta_t of Algorithm 4), now that every scale
// exists.  The sign is taken from p itself.  which: 0 = first (or only)
// segment of the tile, 1 = last segment.
__device__ __forceinline__ void residual_segment(const Layout &L, int32_t tile, int which, float *err_set,
                                                 const float *scales)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const int64_t left = L.d - tile_start;
    const int n_valid = left >= TILE ? TILE : (int)left;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    float *err_tile = err_set + tile_start;
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
            v.x = residual(v.x, s);
            v.y = residual(v.y, s);
            v.z = residual(v.z, s);
            v.w = residual(v.w, s);
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

// Scales the first kernel of a call did not write: those of blocks larger than
// fuse_limit (list fixed per layout: workgroups 0 .. n_big*nsets-1) and those
// whose first tile gave up waiting (list filled by the first kernel: the last
// DEFER_WGS workgroups).
__global__ __launch_bounds__(THREADS) void k_finalize_scales(Layout L, Scratch X, const int32_t *big_blocks,
                                                             int n_big, int nsets, float *scales)
{
    __shared__ double red[NWAVES];
    const int n_static = n_big * nsets;
    if ((int)blockIdx.x < n_static) {
        const int64_t b = big_blocks[blockIdx.x % n_big];
        const int w = blockIdx.x / n_big;
        const double total =
            sum_block_partials(L, b, X.part + (int64_t)(X.set_base + w) * 2 * L.ntiles, red);
        if (threadIdx.x == 0) scales[(int64_t)w * L.B + b] = (float)(total / (double)(L.offs[b + 1] - L.offs[b]));
        return;
    }
    const unsigned n = *X.fin_cnt;
    for (unsigned i = blockIdx.x - n_static; i < n; i += DEFER_WGS) {
        const unsigned long long it = X.fin_list[i];
        const int set = (int)(it >> 32);
        const int64_t b = (int64_t)(it & 0xffffffffull);
        const double total = sum_block_partials(L, b, X.part + (int64_t)set * 2 * L.ntiles, red);
        if (threadIdx.x == 0)
            scales[(int64_t)(set - X.set_base) * L.B + b] = (float)(total / (double)(L.offs[b + 1] - L.offs[b]));
    }
}

// e <- p - Delta wherever the first kernel parked p: the open segments of blocks
// larger than fuse_limit (list fixed per layout: workgroups 0 .. n_items*nsets-1)
// and the segments whose wait ran out (list filled by the first kernel: the last
// DEFER_WGS workgroups).  Also clears the list counters the next call will use.
__global__ __launch_bounds__(THREADS) void k_residual_parked(Layout L, Scratch X, const uint32_t *items,
                                                             int n_items, int nsets, unsigned int *next_defer_cnt,
                                                             unsigned int *next_fin_cnt, float *err,
                                                             int64_t err_stride, const float *scales)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *next_defer_cnt = 0u;
        *next_fin_cnt = 0u;
    }
    const int n_static = n_items * nsets;
    if ((int)blockIdx.x < n_static) {
        const uint32_t it = items[blockIdx.x % n_items];
        const int w = blockIdx.x / n_items;
        residual_segment(L, (int32_t)(it >> 1), (int)(it & 1u), err + (int64_t)w * err_stride,
                         scales + (int64_t)w * L.B);
        return;
    }
    const unsigned n = *X.defer_cnt;
    for (unsigned i = blockIdx.x - n_static; i < n; i += DEFER_WGS) {
        const unsigned long long it = X.defer_list[i];
        const int w = (int)(it >> 33) - X.set_base;
        const int32_t tile = (int32_t)((it >> 1) & 0xffffffffull);
        residual_segment(L, tile, (int)(it & 1ull), err + (int64_t)w * err_stride, scales + (int64_t)w * L.B);
    }
}

// Parameter update x <- x - eta * Delta~ (Algorithm 4).
template <bool FULL>
__device__ __forceinline__ void apply_tile(const Layout &L, int32_t tile, int n_valid, float *x,
                                           const uint64_t *signs, const float *scales, float eta, TileShared &S)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    float *xt = x + tile_start;
    const uint32_t *s32 = reinterpret_cast<const uint32_t *>(signs);
    const unsigned sh = (unsigned)(lane_id() & 7) * 4u;
    const int64_t n_hw = 2 * L.W;
    const int *seg = reinterpret_cast<const int *>(S.val);
    if (fb != lb) build_segment_index(L, tile, n_valid, fb, lb - fb + 1, S);
    const float s_uniform = scales[fb];
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        const int lb0 = local_base(k);
        if (!FULL && lb0 >= n_valid) continue;
        const float4 v = load4<FULL>(xt, lb0, n_valid);
        const int64_t hw = (tile_start + lb0) >> 5;
        const uint32_t word = (hw < n_hw) ? s32[hw] : 0u;
        const unsigned nibble = (word >> sh) & 0xFu;
        float xv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = lb0 + c;
            float s = s_uniform;
            if (fb != lb) s = scales[fb + ((FULL || j < n_valid) ? seg[j] : 0)];
            const float u = eta * signed_scale(s, (nibble >> c) & 1u);
            xv[c] = xv[c] - u;
        }
        store4<FULL>(xt, lb0, n_valid, make_float4(xv[0], xv[1], xv[2], xv[3]));
    }
}

__global__ __launch_bounds__(THREADS) void k_apply(Layout L, float *x, const uint64_t *signs,
                                                   const float *scales, float eta)
{
    __shared__ TileShared S;
    const int32_t tile = blockIdx.x;
    const int64_t left = L.d - (int64_t)tile * TILE;
    if (left >= TILE) apply_tile<true>(L, tile, TILE, x, signs, scales, eta, S);
    else apply_tile<false>(L, tile, (int)left, x, signs, scales, eta, S);
}

}  // namespace ef
