// Device side of libef: tile-based kernels for the worker, server and apply
// steps of Algorithm 4 (dist-EF-blockSGDM, arxiv 1905.10936), written for
// gfx950 (64-lane wavefronts, 256 CUs, HBM-bound streaming passes).
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
// a tile are "open" (the block continues into a neighbouring tile): their fp64
// partial sums go to a per-(tile, slot) scratch word, an arrival counter per
// block is bumped, and the workgroup that arrives last adds the partials in a
// fixed order (so the scale does not depend on which workgroup that was) and
// writes the block's scale.  Elements of open segments have their corrected
// value p parked in the residual buffer; a second pass subtracts the decoded
// value once the scale exists.
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

struct Layout {
    int64_t d;                  // elements
    int64_t B;                  // blocks
    int64_t W;                  // sign words
    int32_t ntiles;
    const int64_t *offs;        // [B+1] device copy of block_offsets
    const int32_t *tile_fb;     // [ntiles] block holding the tile's first element
    const int32_t *tile_lb;     // [ntiles] block holding the tile's last valid element
};

struct Scratch {                // one set per worker (+1 for the server)
    unsigned long long *part;   // [nsets][2*ntiles] fp64 partial sums of open segments (bit patterns)
    unsigned int *cnt;          // [nsets][B] arrivals per block, 0 between calls
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

template <bool FULL>
__device__ __forceinline__ float4 load4(const float *base, int local, int n_valid)
{
    if (FULL || local + 4 <= n_valid) return *reinterpret_cast<const float4 *>(base + local);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (local + 0 < n_valid) v.x = base[local + 0];
    if (local + 1 < n_valid) v.y = base[local + 1];
    if (local + 2 < n_valid) v.z = base[local + 2];
    return v;                   // local + 3 < n_valid would have taken the vector path
}

template <bool FULL>
__device__ __forceinline__ void store4(float *base, int local, int n_valid, float4 v)
{
    if (FULL || local + 4 <= n_valid) { *reinterpret_cast<float4 *>(base + local) = v; return; }
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

// ------------------------------------------ cross-tile block reductions ---

// Called by every thread of the workgroup with the same arguments.  Publishes
// the partial sum of an open segment of block b and, in the workgroup that
// arrives last, adds all partials of b in ascending tile order and writes the
// scale.  slot: 0 = the tile's first (or only) segment, 1 = its last segment.
__device__ __forceinline__ void publish_open_segment(double partial, int which, int32_t tile, int64_t b,
                                                     const Layout &L, unsigned long long *part,
                                                     unsigned int *cnt, float *scales_out,
                                                     double *red, int *flag)
{
    const int64_t bs = L.offs[b], be = L.offs[b + 1];
    const int64_t t0 = bs / TILE, t1 = (be - 1) / TILE;
    if (threadIdx.x == 0) {
        // All traffic of this hand-off is relaxed agent-scope atomics, which the
        // hardware performs at the point where the 8 XCDs' L2 caches meet.  The
        // exchange returns only once the partial is there, and the counter bump
        // is made to depend on its return value, so a workgroup that sees the
        // final count also sees every partial.  (An agent-scope release fence
        // would order them too, but it writes back the whole L2 of streaming
        // stores on every tile.)
        unsigned long long old =
            __hip_atomic_exchange(part + 2 * (int64_t)tile + which, (unsigned long long)__double_as_longlong(partial),
                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned inc = 1u;
        asm volatile("" : "+v"(inc) : "v"((unsigned)old), "v"((unsigned)(old >> 32)) : "memory");
        unsigned prev = __hip_atomic_fetch_add(cnt + b, inc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = (prev + 1u == (unsigned)(t1 - t0 + 1)) ? 1 : 0;
    }
    __syncthreads();
    const int last = *flag;
    __syncthreads();
    if (!last) return;
    const int first_slot = (bs % TILE != 0) ? 1 : 0;   // b is the last segment of tile t0 unless it starts there
    double acc = 0.0;
    for (int64_t t = t0 + threadIdx.x; t <= t1; t += THREADS) {
        const int sl = (t == t0) ? first_slot : 0;
        unsigned long long bits = __hip_atomic_load(part + 2 * t + sl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        acc += __longlong_as_double((long long)bits);
    }
    const double total = block_sum(acc, red);
    if (threadIdx.x == 0) {
        scales_out[b] = (float)(total / (double)(be - bs));
        __hip_atomic_store(cnt + b, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

struct TileShared {
    float val[TILE];            // |p| per element, then the element's scale (closed segments)
    double red[NWAVES];
    double open_sum[2];
    int long_list[MAX_LONG];
    int n_long;
    int flag;
};

// Compress the tile whose corrected values are in p[][] (Section 3.2): sign
// words, block sums, scales of closed blocks, residual e' = p - Delta for closed
// segments, p itself for open ones (finished by k_residual_pass2).
template <bool FULL>
__device__ __forceinline__ void compress_tile(float4 (&p)[SUBROWS], const Layout &L, int32_t tile, int n_valid,
                                              uint64_t *signs, float *scales_out, float *err_tile,
                                              unsigned long long *part, unsigned int *cnt, TileShared &S)
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
        if (closed) {
            const float s = (float)(total / (double)(be - bs));
            if (threadIdx.x == 0) scales_out[fb] = s;
#pragma unroll
            for (int k = 0; k < SUBROWS; ++k) {
                float4 e;
                e.x = p[k].x - signed_scale(s, p[k].x >= 0.f);
                e.y = p[k].y - signed_scale(s, p[k].y >= 0.f);
                e.z = p[k].z - signed_scale(s, p[k].z >= 0.f);
                e.w = p[k].w - signed_scale(s, p[k].w >= 0.f);
                store4<FULL>(err_tile, local_base(k), n_valid, e);
            }
        } else {
#pragma unroll
            for (int k = 0; k < SUBROWS; ++k) store4<FULL>(err_tile, local_base(k), n_valid, p[k]);
            publish_open_segment(total, 0, tile, fb, L, part, cnt, scales_out, S.red, &S.flag);
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
    for (int s = threadIdx.x; s < nseg; s += THREADS) {
        const int64_t b = fb + s;
        const int64_t bs = L.offs[b], be = L.offs[b + 1];
        const int lo = (int)max(bs - tile_start, (int64_t)0);
        const int hi = (int)min(be - tile_start, (int64_t)n_valid);
        if (hi - lo > SMALL_SEG) {
            S.long_list[atomicAdd(&S.n_long, 1)] = s;
            continue;
        }
        double acc = 0.0;
        for (int j = lo; j < hi; ++j) acc += (double)S.val[j];
        const bool open = (s == 0 && head_open) || (s == nseg - 1 && tail_open);
        if (open) {
            S.open_sum[s == 0 ? 0 : 1] = acc;
        } else {
            const float sc = (float)(acc / (double)(be - bs));
            scales_out[b] = sc;
            for (int j = lo; j < hi; ++j) S.val[j] = sc;
        }
    }
    __syncthreads();
    const int n_long = S.n_long;
    for (int q = wave_id(); q < n_long; q += NWAVES) {
        const int s = S.long_list[q];
        const int64_t b = fb + s;
        const int64_t bs = L.offs[b], be = L.offs[b + 1];
        const int lo = (int)max(bs - tile_start, (int64_t)0);
        const int hi = (int)min(be - tile_start, (int64_t)n_valid);
        double acc = 0.0;
        for (int j = lo + lane_id(); j < hi; j += 64) acc += (double)S.val[j];
        acc = wave_sum(acc);
        const bool open = (s == 0 && head_open) || (s == nseg - 1 && tail_open);
        if (open) {
            if (lane_id() == 0) S.open_sum[s == 0 ? 0 : 1] = acc;
        } else {
            const float sc = (float)(acc / (double)(be - bs));
            if (lane_id() == 0) scales_out[b] = sc;
            for (int j = lo + lane_id(); j < hi; j += 64) S.val[j] = sc;
        }
    }
    __syncthreads();
    const int head_end = head_open ? (int)min(L.offs[fb + 1] - tile_start, (int64_t)n_valid) : 0;
    const int tail_begin = tail_open ? (int)(L.offs[lb] - tile_start) : TILE;
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
            const bool is_open = (j < head_end) || (j >= tail_begin);
            ev[c] = is_open ? pv[c] : pv[c] - signed_scale(sv[c], pv[c] >= 0.f);
        }
        store4<FULL>(err_tile, lb0, n_valid, make_float4(ev[0], ev[1], ev[2], ev[3]));
    }
    if (head_open) publish_open_segment(S.open_sum[0], 0, tile, fb, L, part, cnt, scales_out, S.red, &S.flag);
    if (tail_open) publish_open_segment(S.open_sum[1], 1, tile, lb, L, part, cnt, scales_out, S.red, &S.flag);
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
    for (int s = threadIdx.x; s < nseg; s += THREADS) {
        const int lo = (int)max(L.offs[fb + s] - tile_start, (int64_t)0);
        const int hi = (int)min(L.offs[fb + s + 1] - tile_start, (int64_t)n_valid);
        if (hi - lo > SMALL_SEG) {
            S.long_list[atomicAdd(&S.n_long, 1)] = s;
            continue;
        }
        for (int j = lo; j < hi; ++j) seg[j] = s;
    }
    __syncthreads();
    const int n_long = S.n_long;
    for (int q = wave_id(); q < n_long; q += NWAVES) {
        const int s = S.long_list[q];
        const int lo = (int)max(L.offs[fb + s] - tile_start, (int64_t)0);
        const int hi = (int)min(L.offs[fb + s + 1] - tile_start, (int64_t)n_valid);
        for (int j = lo + lane_id(); j < hi; j += 64) seg[j] = s;
    }
    __syncthreads();
}

// ------------------------------------------------------------- kernels ---

// Worker, first pass (Algorithm 4, "on each worker i"): momentum, corrected
// value p, sign words, block sums; see compress_tile for what is left open.
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
    compress_tile<FULL>(p, L, tile, n_valid, A.signs + (int64_t)worker * L.W, A.scales + (int64_t)worker * L.B, e,
                        X.part + (int64_t)worker * 2 * L.ntiles, X.cnt + (int64_t)worker * L.B, S);
}

__global__ __launch_bounds__(THREADS) void k_worker_pass1(Layout L, Scratch X, WorkerArgs A)
{
    __shared__ TileShared S;
    const int32_t tile = blockIdx.x;
    const int worker = blockIdx.y;
    const int64_t left = L.d - (int64_t)tile * TILE;
    if (left >= TILE) worker_tile<true>(L, X, A, tile, worker, TILE, S);
    else worker_tile<false>(L, X, A, tile, worker, (int)left, S);
}

// Server, first pass (Algorithm 4, "on server"): decode and add the M payloads
// in worker order, divide by M, add the rescaled server residual, compress.
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
    compress_tile<FULL>(p, L, tile, n_valid, A.signs, A.scales, te, X.part + (int64_t)set * 2 * L.ntiles,
                        X.cnt + (int64_t)set * L.B, S);
}

__global__ __launch_bounds__(THREADS) void k_server_pass1(Layout L, Scratch X, ServerArgs A, int set)
{
    __shared__ TileShared S;
    const int32_t tile = blockIdx.x;
    const int64_t left = L.d - (int64_t)tile * TILE;
    if (left >= TILE) server_tile<true>(L, X, A, tile, set, TILE, S);
    else server_tile<false>(L, X, A, tile, set, (int)left, S);
}

// Second pass of worker and server: e <- p - Delta on the open segments of each
// tile (e_{t+1} = p_t - Delta_t of Algorithm 4), now that every scale exists.
// err holds p there; the sign is taken from p itself.
template <bool FULL>
__device__ __forceinline__ void residual_tile(const Layout &L, int32_t tile, int n_valid, float *err_tile,
                                              const float *scales)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    int head_end = 0, tail_begin = TILE;
    float sh = 0.f, st = 0.f;
    if (fb == lb) {
        const bool open = (L.offs[fb] < tile_start) || (L.offs[fb + 1] > tile_start + TILE);
        if (open) { head_end = n_valid; sh = scales[fb]; }
    } else {
        if (L.offs[fb] < tile_start) {
            head_end = (int)min(L.offs[fb + 1] - tile_start, (int64_t)n_valid);
            sh = scales[fb];
        }
        if (L.offs[lb + 1] > tile_start + TILE) {
            tail_begin = (int)(L.offs[lb] - tile_start);
            st = scales[lb];
        }
    }
    if (head_end == 0 && tail_begin == TILE) return;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        const int lb0 = local_base(k);
        if (lb0 >= n_valid) continue;
        if (lb0 >= head_end && lb0 + 3 < tail_begin) continue;
        const float4 v = load4<FULL>(err_tile, lb0, n_valid);
        float pv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = lb0 + c;
            if (j < head_end) pv[c] = pv[c] - signed_scale(sh, pv[c] >= 0.f);
            else if (j >= tail_begin) pv[c] = pv[c] - signed_scale(st, pv[c] >= 0.f);
        }
        store4<FULL>(err_tile, lb0, n_valid, make_float4(pv[0], pv[1], pv[2], pv[3]));
    }
}

__global__ __launch_bounds__(THREADS) void k_residual_pass2(Layout L, float *err, int64_t err_stride,
                                                            const float *scales)
{
    const int32_t tile = blockIdx.x;
    const int w = blockIdx.y;
    const int64_t tile_start = (int64_t)tile * TILE;
    const int64_t left = L.d - tile_start;
    float *e = err + (int64_t)w * err_stride + tile_start;
    const float *sc = scales + (int64_t)w * L.B;
    if (left >= TILE) residual_tile<true>(L, tile, TILE, e, sc);
    else residual_tile<false>(L, tile, (int)left, e, sc);
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
