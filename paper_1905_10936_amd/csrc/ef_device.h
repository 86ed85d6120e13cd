// Device side of libef: tile-based kernels for the worker, server and apply
// steps of Algorithm 4 (dist-EF-blockSGDM, arxiv 1905.10936), written for
// gfx950 (64-lane wavefronts, 256 CUs in 8 XCDs, HBM-bound streaming passes).
//
// Work decomposition
// ------------------
// The flat d-vector is cut into tiles of TILE = 4096 consecutive elements, the
// unit of work of a 256-thread workgroup.  Tiles, not blocks, are the unit, so
// a block of 8M elements and a block of 1 element cost the same per element.
// A tile is a whole number of 64-element sign words and starts on a 16 KiB
// boundary, so every fp32 access is a coalesced 128-bit access whatever the
// block boundaries are.  Inside a tile, wavefront w owns the 1024 consecutive
// elements [1024w, 1024w+1024) as 4 sub-rows of 256; lane l of sub-row k holds
// the 4 consecutive elements 1024w + 256k + 4l .. +3.
//
// The blocks of the partition (Section 3.2) cut a tile into segments.  A full
// tile that lies inside one block is "uniform"; a tile where several blocks
// meet, and the ragged last tile of the vector, is "mixed".  A segment whose block lies entirely inside the tile is "closed":
// its L1 norm, scale and residual are finished by the tile alone (in fp64, in
// ascending order for short segments).  The other segments are "open": their
// fp64 partial sums go to a per-(tile, slot) scratch word, and whoever needs
// the block's scale adds the block's partials in one fixed order (thread t
// takes tiles t, t+256, ... ascending, then a fixed tree), so the scale has the
// same bits wherever and whenever it is computed.
//
// One pass over the state
// -----------------------
// e <- p - Delta needs the block's scale, i.e. every tile of the block.  For a
// block of at most `fuse_limit` tiles the workgroups of its uniform tiles keep
// p in registers until the scale exists and then write the finished residual,
// so every fp32 tensor is read once and written once.  The hand-off between
// workgroups uses relaxed agent-scope atomics only (an agent-scope release
// fence would write back the whole L2 of streaming stores on every tile):
//   * a partial is never negative, so its sign bit carries a tag that flips on
//     every call that uses the scratch set; one 64-bit store publishes value
//     and tag together;
//   * the workgroup that takes the block's last whole tile gathers the
//     partials (re-reading those whose tag is still old: tiles are handed out
//     in ascending order, so the others are at most a tile-time behind),
//     writes the scale and posts (call number, scale) in the block's "ready"
//     word -- no counter, hence no read-modify-write on a shared address;
//   * the others look at the ready word when they come to write the tile.
// Mixed tiles never wait: their open segments, like all tiles of blocks larger
// than fuse_limit and any tile whose (bounded) wait ran out, get p parked in
// the residual buffer; a small kernel then computes the scales still missing
// and another subtracts the decoded value where p was parked.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ef {

constexpr int TILE = 4096;      // elements per workgroup and step
constexpr int THREADS = 256;    // 4 wavefronts
constexpr int NWAVES = THREADS / 64;
constexpr int SUBROWS = 4;      // float4 per thread
constexpr int SMALL_SEG = 64;   // segments up to this length are summed by one thread
constexpr int MAX_LONG = TILE / SMALL_SEG;
constexpr int DEFER_WGS = 64;   // workgroups that serve the run-time lists of the second-pass kernels
#ifndef EF_PIPE_DEPTH
#define EF_PIPE_DEPTH 3
#endif
constexpr int PIPE_DEPTH = EF_PIPE_DEPTH;     // tiles a persistent workgroup keeps in registers while their scales form
constexpr unsigned long long TAG_BIT = 1ull << 63;
constexpr int MAX_PER_THREAD = 6;                        // partial words a thread gathers
constexpr int FUSE_LIMIT_MAX = MAX_PER_THREAD * THREADS; // tiles of the largest one-pass block

struct Layout {
    int64_t d;                  // elements
    int64_t B;                  // blocks
    int64_t W;                  // sign words
    int32_t ntiles;
    int32_t fuse_limit;         // blocks of up to this many tiles finish in one pass
    int32_t n_mixed, n_uniform;
    const int64_t *offs;        // [B+1] device copy of block_offsets
    const int32_t *tile_fb;     // [ntiles] block holding the tile's first element
    const int32_t *tile_lb;     // [ntiles] block holding the tile's last valid element
    const int32_t *mixed_tiles;   // [n_mixed] ascending
    const int32_t *uniform_tiles; // [n_uniform] ascending
};

// What changes from call to call lives in device memory, so that the kernel
// arguments of a call are the same every time (a captured HIP graph of the
// calls can be replayed): the number of calls made on the plan and the tag each
// scratch set's partial words carry since the last call that used the set.
// The last kernel of a call (k_advance) moves it on.
struct CallState {
    unsigned int calls;
    unsigned int server_tag;            // bit 0
    unsigned long long worker_tags;     // bit i: worker i
};

// Kernel argument: the plan's scratch.  A "set" is one worker, or the server.
struct ScratchRef {
    unsigned long long *part;
    unsigned long long *ready;
    unsigned long long *defer_list;
    unsigned long long *fin_list;
    unsigned int *list_cnt;             // [6]: defer_cnt[2], fin_cnt[2], ticket[2]; a call uses those of its parity
    const CallState *state;
    int set_base;                       // first set this call uses (0 for workers, max_workers for the server)
    int spin_limit;
};

// Scratch of one call, formed by every kernel from ScratchRef and CallState (open_call).
struct Scratch {
    unsigned long long *part;   // [nsets][2*ntiles] tagged fp64 partial sums of open segments
    unsigned long long *ready;  // [nsets][B] (epoch << 32) | scale bits, posted by the block's gatherer
    unsigned int *defer_cnt;    // entries in defer_list for this call
    unsigned long long *defer_list;  // parked segments: (set << 33) | (tile << 1) | slot
    unsigned int *fin_cnt;      // entries in fin_list for this call
    unsigned long long *fin_list;    // blocks whose scale is still to be written: (set << 32) | block
    unsigned int *ticket;       // next chunk of tiles to hand out (persistent kernels), 0 at call start
    unsigned long long tags;    // bit i = this call's tag of set (set_base + i), carried by its partial words
    unsigned int epoch;         // this call's number on the plan (never 0), carried by the ready words
    int set_base;               // first set this call uses (0 for workers, max_workers for the server)
    int spin_limit;             // polls before a waiting workgroup gives up and parks p
    unsigned int *next_cnt;     // the three list counters of the next call (zeroed by this call's last kernel)
};

__device__ __forceinline__ unsigned uniform_u32(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }

__device__ __forceinline__ Scratch open_call(const ScratchRef &R)
{
    Scratch X;
    const unsigned calls = uniform_u32(R.state->calls);
    const unsigned cur = calls & 1u;
    X.part = R.part;
    X.ready = R.ready;
    X.defer_list = R.defer_list;
    X.fin_list = R.fin_list;
    X.defer_cnt = R.list_cnt + cur;
    X.fin_cnt = R.list_cnt + 2 + cur;
    X.ticket = R.list_cnt + 4 + cur;
    X.next_cnt = R.list_cnt + (cur ^ 1u);
    // this call's tags are the stored ones flipped
    if (R.set_base == 0) {
        const unsigned long long t = R.state->worker_tags;
        X.tags = ~(((unsigned long long)uniform_u32((unsigned)(t >> 32)) << 32) | uniform_u32((unsigned)t));
    } else {
        X.tags = (unsigned long long)(uniform_u32(R.state->server_tag) ^ 1u);
    }
    X.epoch = calls % 0xffffffffu + 1u;     // never 0: 0 marks "no scale posted"
    X.set_base = R.set_base;
    X.spin_limit = R.spin_limit;
    return X;
}

struct WorkerArgs {
    const float *grad; int64_t grad_stride;
    float *mom; float *err; int64_t state_stride;
    float mu, r;
    uint64_t *signs; float *scales;
    int64_t signs_stride;       // 64-bit words between the payloads of two workers
    int64_t scales_stride;      // floats between the scale arrays of two workers
};

struct ServerArgs {
    int M;
    const uint64_t *signs_in;   // worker i at signs_in + i*in_signs_stride (64-bit words)
    const float *scales_in;     // worker i at scales_in + i*in_scales_stride (floats)
    int64_t in_signs_stride, in_scales_stride;
    float *err;                 // server residual
    float r, Mf;
    float Minv;                 // 1/M if M is a power of two (exact), else 0
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

__device__ __forceinline__ float4 guarded_load4(const float *base, int local, int n_valid)
{
    if (local + 4 <= n_valid) return stream_load4(base + local);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (local + 0 < n_valid) v.x = base[local + 0];
    if (local + 1 < n_valid) v.y = base[local + 1];
    if (local + 2 < n_valid) v.z = base[local + 2];
    return v;                   // local + 3 < n_valid would have taken the vector path
}

__device__ __forceinline__ void guarded_store4(float *base, int local, int n_valid, float4 v)
{
    if (local + 4 <= n_valid) { stream_store4(base + local, v); return; }
    if (local + 0 < n_valid) base[local + 0] = v.x;
    if (local + 1 < n_valid) base[local + 1] = v.y;
    if (local + 2 < n_valid) base[local + 2] = v.z;
}

// A thread's four float4 of one tile.  Only the last tile of a vector can be
// ragged; the test is uniform over the workgroup, so full tiles run straight
// through 128-bit accesses with no per-access branch.
__device__ __forceinline__ void load_tile(const float *base, float4 (&v)[SUBROWS], int n_valid)
{
    if (n_valid == TILE) {
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) v[k] = stream_load4(base + local_base(k));
    } else {
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) v[k] = guarded_load4(base, local_base(k), n_valid);
    }
}

__device__ __forceinline__ void store_tile(float *base, const float4 (&v)[SUBROWS], int n_valid)
{
    if (n_valid == TILE) {
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) stream_store4(base + local_base(k), v[k]);
    } else {
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) guarded_store4(base, local_base(k), n_valid, v[k]);
    }
}

__device__ __forceinline__ int tile_valid(const Layout &L, int32_t tile)
{
    const int64_t left = L.d - (int64_t)tile * TILE;
    return left >= TILE ? TILE : (int)left;
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

__device__ __forceinline__ void residual4(float4 &v, float s)
{
    v.x = residual(v.x, s);
    v.y = residual(v.y, s);
    v.z = residual(v.z, s);
    v.w = residual(v.w, s);
}

// Sign words of the tile whose values are in p (bit = p >= 0, Appendix A with
// sign(0) read as +1; elements past n_valid give 0 bits).  Within a sub-row, 16
// consecutive lanes make one 64-bit word; each wavefront stores its 16 words.
__device__ __forceinline__ void store_signs(const float4 (&p)[SUBROWS], int n_valid, uint64_t *signs,
                                            int64_t tile_start, int64_t W)
{
    const int lane = lane_id();
    const int l16 = lane & 15;
    const unsigned sh = (unsigned)(l16 & 7) * 4u;
    unsigned mylo = 0, myhi = 0;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        const int lb0 = local_base(k);
        unsigned nib = (p[k].x >= 0.f ? 1u : 0u) | (p[k].y >= 0.f ? 2u : 0u) | (p[k].z >= 0.f ? 4u : 0u) |
                       (p[k].w >= 0.f ? 8u : 0u);
        if (n_valid != TILE) {
            unsigned vm = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) vm |= (lb0 + c < n_valid) ? (1u << c) : 0u;
            nib &= vm;
        }
        unsigned lo = (l16 < 8) ? (nib << sh) : 0u;
        unsigned hi = (l16 >= 8) ? (nib << sh) : 0u;
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

// fp64 sum of |p| over the thread's valid elements
__device__ __forceinline__ double abs_sum(const float4 (&p)[SUBROWS], int n_valid)
{
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        const int lb0 = local_base(k);
        const float a[4] = {fabsf(p[k].x), fabsf(p[k].y), fabsf(p[k].z), fabsf(p[k].w)};
#pragma unroll
        for (int c = 0; c < 4; ++c) acc += (n_valid == TILE || lb0 + c < n_valid) ? (double)a[c] : 0.0;
    }
    return acc;
}

struct TileShared {
    float val[TILE];            // |p| per element, then the element's scale (closed segments)
    double red[NWAVES];
    double open_sum[2];
    int long_list[MAX_LONG];
    int n_long;
    int flag[2];
    unsigned ticket;
};

// ------------------------------------------------- per-set scratch views ---

__device__ __forceinline__ unsigned long long *set_part(const Scratch &X, const Layout &L, int set)
{
    return X.part + (int64_t)set * 2 * L.ntiles;
}
__device__ __forceinline__ unsigned long long *set_ready(const Scratch &X, const Layout &L, int set)
{
    return X.ready + (int64_t)set * L.B;
}
__device__ __forceinline__ unsigned long long set_tag(const Scratch &X, int set)
{
    return (X.tags >> (set - X.set_base)) & 1ull;
}

// ------------------------------------------ cross-tile block reductions ---

struct BlockSpan {
    int64_t bs, be;             // element range
    int64_t t0;                 // first tile
    int n;                      // tiles
};

__device__ __forceinline__ BlockSpan block_span(const Layout &L, int64_t b)
{
    BlockSpan s;
    s.bs = L.offs[b];
    s.be = L.offs[b + 1];
    s.t0 = s.bs / TILE;
    s.n = (int)((s.be - 1) / TILE - s.t0 + 1);
    return s;
}

// Does the block own a whole tile?  Its first tile is shared (or ragged) if it
// starts inside it, its last tile if it ends inside it; the tiles between are
// its own.
__device__ __forceinline__ bool has_uniform_tile(const BlockSpan &s)
{
    return s.n - ((s.bs % TILE) != 0 ? 1 : 0) - ((s.be % TILE) != 0 ? 1 : 0) >= 1;
}

// One-pass blocks: their scale is formed and posted inside the first kernels.
__device__ __forceinline__ bool is_counted(const Layout &L, const BlockSpan &s)
{
    return s.n >= 2 && s.n <= L.fuse_limit && has_uniform_tile(s);
}

// Scratch word of block b's segment in tile t: slot 1 of the block's first tile
// if b starts inside that tile (it is then the tile's last segment), slot 0
// everywhere else (first or only segment).
__device__ __forceinline__ int64_t part_index(int64_t t, const BlockSpan &s)
{
    return 2 * t + ((t == s.t0 && (s.bs % TILE) != 0) ? 1 : 0);
}

// The block's last whole tile: the workgroup that takes it forms the scale.
__device__ __forceinline__ int64_t gatherer_tile(const BlockSpan &s)
{
    return s.t0 + s.n - 1 - ((s.be % TILE) != 0 ? 1 : 0);
}

// What a uniform tile has to follow up on after posting its partial: the block
// whose scale it must form (it is that block's last whole tile), or -1.
struct Posted {
    int gather;
};

__device__ __forceinline__ void clear_posted(Posted &P) { P.gather = -1; }

// Post the partial sum of an open segment.  which: 0 = the tile's first (or
// only) segment, 1 = its last segment.  Never waits.
__device__ __forceinline__ void store_partial(double partial, int which, int32_t tile, const Layout &L,
                                              const Scratch &X, int set)
{
    if (threadIdx.x == 0) {
        const unsigned long long w =
            (unsigned long long)__double_as_longlong(partial) | (set_tag(X, set) ? TAG_BIT : 0ull);
        __hip_atomic_store(set_part(X, L, set) + 2 * (int64_t)tile + which, w, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Sum of block b's partials once the kernel that posted them has finished.
// Same order as gather_scale.  Called by every thread of the workgroup.
__device__ __forceinline__ double sum_block_partials(const Layout &L, int64_t b, const unsigned long long *part,
                                                     double *red)
{
    const BlockSpan sp = block_span(L, b);
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < sp.n; i += THREADS)
        acc += __longlong_as_double((long long)(part[part_index(sp.t0 + i, sp)] & ~TAG_BIT));
    return block_sum(acc, red);
}

// Wait (bounded) until every tile of block b has posted this call's partial,
// then form the block's scale.  Called by every thread of the workgroup with
// the same arguments; returns the same answer to all of them.
__device__ __forceinline__ bool gather_scale(int64_t b, const Layout &L, const Scratch &X, int set, TileShared &S,
                                             float *s)
{
    const BlockSpan sp = block_span(L, b);          // sp.n <= fuse_limit <= FUSE_LIMIT_MAX
    const unsigned long long *part = set_part(X, L, set);
    const unsigned long long tag = set_tag(X, set);
    double v[MAX_PER_THREAD];
    unsigned have = 0;
#pragma unroll
    for (int q = 0; q < MAX_PER_THREAD; ++q) v[q] = 0.0;
    bool ok = false;
    for (int it = 0; it < X.spin_limit; ++it) {
        int all = 1;
#pragma unroll
        for (int q = 0; q < MAX_PER_THREAD; ++q) {
            const int i = (int)threadIdx.x + q * THREADS;
            if (i < sp.n && !((have >> q) & 1u)) {
                const unsigned long long w =
                    __hip_atomic_load(part + part_index(sp.t0 + i, sp), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((w >> 63) == tag) {
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
    *s = (float)(total / (double)(sp.be - sp.bs));
    return true;
}

// The workgroup that holds the last whole tile of counted block b forms the
// scale from the partials (waiting, bounded, for those still in flight: every
// other tile of the block was handed out earlier), writes it out and posts it
// for the block's other tiles.  Called by every thread of that workgroup.
__device__ __forceinline__ void finish_block(int64_t b, const Layout &L, const Scratch &X, int set,
                                             float *scales_out, TileShared &S)
{
    float s;
    const bool ok = gather_scale(b, L, X, set, S, &s);
    if (threadIdx.x == 0) {
        if (ok) {
            scales_out[b] = s;
            __hip_atomic_store(set_ready(X, L, set) + b,
                               ((unsigned long long)X.epoch << 32) | (unsigned long long)__float_as_uint(s),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            const unsigned k = atomicAdd(X.fin_cnt, 1u);
            X.fin_list[k] = ((unsigned long long)set << 32) | (unsigned long long)b;
        }
    }
}

// Follow up on what a uniform tile posted: if it is its block's last whole
// tile, finish that block.  Called by every thread of the workgroup.
__device__ __forceinline__ void resolve_posted(const Posted &P, const Layout &L, const Scratch &X, int set,
                                               float *scales_out, TileShared &S)
{
    if (P.gather >= 0) finish_block(P.gather, L, X, set, scales_out, S);
}

// Thread 0's early look at the ready word of block b (b < 0: none).
__device__ __forceinline__ unsigned long long peek_ready(int b, const Layout &L, const Scratch &X, int set)
{
    unsigned long long w = 0ull;           // epoch 0 is never used
    if (threadIdx.x == 0 && b >= 0)
        w = __hip_atomic_load(set_ready(X, L, set) + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return w;
}

// Wait (bounded) until the block's gatherer has posted block b's scale of this call.
// `peeked` is thread 0's earlier look at the word (see peek_ready).  Called by
// every thread of the workgroup; same answer to all of them.
__device__ __forceinline__ bool wait_ready(int64_t b, unsigned long long peeked, const Layout &L, const Scratch &X,
                                           int set, TileShared &S, float *s)
{
    if (threadIdx.x == 0) {
        const unsigned long long *word = set_ready(X, L, set) + b;
        unsigned long long w = peeked;
        int found = ((unsigned)(w >> 32) == X.epoch) ? 1 : 0;
        for (int it = 0; !found && it < X.spin_limit; ++it) {
            w = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            found = ((unsigned)(w >> 32) == X.epoch) ? 1 : 0;
            if (!found) __builtin_amdgcn_s_sleep(8);
        }
        if (X.spin_limit <= 0) found = 0;   // a zero budget means: never take the one-pass route
        S.flag[0] = found;
        S.flag[1] = (int)(unsigned)w;
    }
    __syncthreads();
    const bool ok = S.flag[0] != 0;
    *s = __uint_as_float((unsigned)S.flag[1]);
    __syncthreads();
    return ok;
}

// Leave a segment whose p gets parked in the residual buffer to the kernels
// that run after this one.
__device__ __forceinline__ void defer_segment(int32_t tile, int which, const Scratch &X, int set)
{
    if (threadIdx.x == 0) {
        const unsigned i = atomicAdd(X.defer_cnt, 1u);
        X.defer_list[i] = ((unsigned long long)set << 33) | ((unsigned long long)tile << 1) | (unsigned)which;
    }
}

// ------------------------------------------------------- tile compression ---

// Mixed tile (several blocks meet): sign words; segmented fp64 sums through LDS;
// scales and residuals e' = p - Delta of the closed segments; partial sums of
// the (at most two) open segments posted, their elements stored as p for the
// second-pass kernels.  Never waits for another workgroup.  (Section 3.2 and
// e_{t+1} = p_t - Delta_t of Algorithm 4.)
__device__ __forceinline__ void compress_mixed(float4 (&p)[SUBROWS], const Layout &L, int32_t tile, int n_valid,
                                               uint64_t *signs, float *scales_out, float *err_tile,
                                               const Scratch &X, int set, TileShared &S)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    store_signs(p, n_valid, signs, tile_start, L.W);

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
            scales_out[b] = sc;
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
            if (lane_id() == 0) scales_out[b] = sc;
            for (int j = lo + lane_id(); j < hi; j += 64) S.val[j] = sc;
        }
    }
    __syncthreads();
    const int head_end = head_open ? (int)min(L.offs[fb + 1] - tile_start, (int64_t)n_valid) : 0;
    const int tail_begin = tail_open ? (int)(L.offs[lb] - tile_start) : TILE;
    if (head_open) store_partial(S.open_sum[0], 0, tile, L, X, set);
    if (tail_open) store_partial(S.open_sum[1], 1, tile, L, X, set);
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
            ev[c] = (j < head_end || j >= tail_begin) ? pv[c] : residual(pv[c], sv[c]);
        }
        p[k] = make_float4(ev[0], ev[1], ev[2], ev[3]);
    }
    store_tile(err_tile, p, n_valid);
    __syncthreads();            // S.val is free again
}

// Uniform tile (inside one block b): sign words and the tile's fp64 sum.
// Returns what is left to do with it:
//   UNI_DONE    the block is this tile alone: scale and residual written;
//   UNI_PARKED  block larger than fuse_limit: partial posted, p parked for the
//               second-pass kernels;
//   UNI_PENDING partial posted: p stays with the caller until the block's
//               scale is posted; P says whether this tile must form it.
enum { UNI_DONE = 0, UNI_PARKED = 1, UNI_PENDING = 2 };

__device__ __forceinline__ int compress_uniform(float4 (&p)[SUBROWS], const Layout &L, int32_t tile, int n_valid,
                                                uint64_t *signs, float *scales_out, float *err_tile,
                                                const Scratch &X, int set, TileShared &S, Posted &P)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t b = L.tile_fb[tile];
    clear_posted(P);
    store_signs(p, n_valid, signs, tile_start, L.W);
    const double total = block_sum(abs_sum(p, n_valid), S.red);
    const BlockSpan sp = block_span(L, b);
    if (sp.bs >= tile_start && sp.be <= tile_start + TILE) {
        const float s = (float)(total / (double)(sp.be - sp.bs));
        if (threadIdx.x == 0) scales_out[b] = s;
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) residual4(p[k], s);
        store_tile(err_tile, p, n_valid);
        return UNI_DONE;
    }
    store_partial(total, 0, tile, L, X, set);
    if (!is_counted(L, sp)) {
        store_tile(err_tile, p, n_valid);
        return UNI_PARKED;
    }
    if ((int64_t)tile == gatherer_tile(sp)) P.gather = b;
    return UNI_PENDING;
}

// Write the residual of a uniform tile of counted block b whose p was kept
// (e_{t+1} = p_t - Delta_t, Algorithm 4), waiting (bounded) for the scale; if
// the wait runs out, p is parked and the segment deferred.
__device__ __forceinline__ void finish_uniform(float4 (&p)[SUBROWS], int32_t tile, int n_valid, int b,
                                               unsigned long long peeked, float *err_tile, const Layout &L,
                                               const Scratch &X, int set, TileShared &S, bool may_wait = true)
{
    float s = 0.f;
    const bool ok = may_wait && wait_ready(b, peeked, L, X, set, S, &s);
    if (ok) {
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) residual4(p[k], s);
    } else {
        defer_segment(tile, 0, X, set);
    }
    store_tile(err_tile, p, n_valid);
}

// Fill S.val (read as int) with the segment index of every element of a mixed
// tile, so that element j can look up scale[fb + seg].
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
// are in flight write out the oldest of the PIPE_DEPTH tiles it holds in
// registers (their blocks' scales have had PIPE_DEPTH tile-times to form, so
// the wait is normally over before it starts); then compute the new tile, post
// its partial sum and keep it in turn.  Tiles are handed out one by one through
// a ticket counter, so at any moment the resident workgroups
// work on one compact, advancing window of the fp32 streams (best DRAM page
// locality, no dependence on dispatch order).  A workgroup never waits for a
// block of which it still holds an unposted tile, so a wait only ever depends
// on workgroups that wait for strictly older blocks; it could starve only if
// one block had more than (resident workgroups x PIPE_DEPTH) uniform tiles,
// which fuse_limit rules out, and it is bounded by spin_limit in any case.
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

template <class Producer>
__device__ __forceinline__ void persistent_uniform(const Layout &L, const Scratch &X, Producer &prod, int n_part,
                                                   TileShared &S)
{
    const unsigned per_part = (unsigned)L.n_uniform;
    const unsigned total = per_part * (unsigned)n_part;

    HeldTile held[PIPE_DEPTH];
#pragma unroll
    for (int q = 0; q < PIPE_DEPTH; ++q) held[q].b = -1;
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
        HeldTile &old = held[0];
        const unsigned long long peeked = peek_ready(old.b, L, X, X.set_base + (old.b >= 0 ? old.idx : 0));
        resolve_posted(posted, L, X, X.set_base + posted_idx, prod.scales(L, posted_idx), S);
        if (old.b >= 0) {
            // The block of the oldest tile cannot complete while this workgroup sits on a tile of
            // the same block that is not posted yet (the new one): then do not wait, park p and
            // leave the tile to the second pass.
            const bool may_wait = !(old.idx == idx && L.tile_fb[tile] == old.b);
            finish_uniform(old.p, old.tile, TILE, old.b, peeked, prod.err_tile(old.idx, old.tile), L, X,
                           X.set_base + old.idx, S, may_wait);
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

    // ---- drain
    resolve_posted(posted, L, X, X.set_base + posted_idx, prod.scales(L, posted_idx), S);
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
    float4 gv[SUBROWS], mv[SUBROWS], ev[SUBROWS];

    __device__ __forceinline__ uint64_t *signs(const Layout &L, int idx) const { return A.signs + (int64_t)idx * A.signs_stride; }
    __device__ __forceinline__ float *scales(const Layout &L, int idx) const { return A.scales + (int64_t)idx * A.scales_stride; }
    __device__ __forceinline__ float *err_tile(int idx, int32_t tile) const
    {
        return A.err + (int64_t)idx * A.state_stride + (int64_t)tile * TILE;
    }
    __device__ __forceinline__ void issue(const Layout &, int idx, int32_t tile)
    {
        const int64_t tile_start = (int64_t)tile * TILE;
        load_tile(A.grad + (int64_t)idx * A.grad_stride + tile_start, gv, TILE);
        if (MOM) load_tile(A.mom + (int64_t)idx * A.state_stride + tile_start, mv, TILE);
        load_tile(A.err + (int64_t)idx * A.state_stride + tile_start, ev, TILE);
    }
    __device__ __forceinline__ void produce(const Layout &, int idx, int32_t tile, float4 (&p)[SUBROWS])
    {
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
    __shared__ TileShared S;
    WorkerProducer<MOM> prod;
    prod.A = A;
    persistent_uniform(L, X, prod, n_workers, S);
}

// Uniform tiles of all workers, one workgroup per (tile, worker): the same
// steps without the pipeline; the workgroup waits in place for its block's
// scale.  Relies on workgroups being dispatched in grid order (fuse_limit keeps
// a block's tiles well inside what is resident at once) and on spin_limit.
// Eight workgroups per CU (64 VGPRs, a few spilled): the one-pass limit is half
// of what is resident, and 2048 resident workgroups let blocks of up to 1024
// tiles (4 Mi elements) finish in one pass (measured: 27.1 -> 24.4 ms on the
// transformer-like layout, no change elsewhere).
template <bool MOM>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(8, 8)))
void k_worker_uniform_direct(Layout L, ScratchRef R, WorkerArgs A)
{
    const Scratch X = open_call(R);
    __shared__ TileShared S;
    const int32_t tile = L.uniform_tiles[blockIdx.x];
    const int worker = blockIdx.y;
    constexpr int n_valid = TILE;
    const int64_t tile_start = (int64_t)tile * TILE;
    const float *g = A.grad + (int64_t)worker * A.grad_stride + tile_start;
    float *m = MOM ? A.mom + (int64_t)worker * A.state_stride + tile_start : nullptr;
    float *e = A.err + (int64_t)worker * A.state_stride + tile_start;
    Posted P;
    float4 gv[SUBROWS], mv[SUBROWS], pv[SUBROWS];
    load_tile(g, gv, n_valid);
    if (MOM) load_tile(m, mv, n_valid);
    load_tile(e, pv, n_valid);
    worker_values<MOM>(gv, mv, pv, A.mu, A.r);
    if (MOM) store_tile(m, mv, n_valid);
    float *scales_out = A.scales + (int64_t)worker * A.scales_stride;
    const int kind = compress_uniform(pv, L, tile, n_valid, A.signs + (int64_t)worker * A.signs_stride, scales_out, e, X, worker,
                                      S, P);
    resolve_posted(P, L, X, worker, scales_out, S);
    if (kind == UNI_PENDING) finish_uniform(pv, tile, n_valid, L.tile_fb[tile], 0ull, e, L, X, worker, S);
}

// -------------------------------------------------------- server kernels ---

// (1/M) * acc as Algorithm 4 writes it: one correctly rounded fp32 division, or,
// when M is a power of two, the product with the exact reciprocal, which is the
// same real number and therefore rounds to the same bits.
__device__ __forceinline__ float mean_of(float acc, float Mf, float Minv)
{
    return Minv != 0.0f ? acc * Minv : acc / Mf;
}

// acc[c] += (+s if bit sh+c of `word` is set, else -s), c = 0..3: what one
// worker's payload stands for in this lane's four elements.  The sign bit of
// the addend is sign(s) XOR NOT(bit), built without a compare: `flip` is ~0 for
// s >= 0 and 0 for s < 0, so word ^ flip has a 1 exactly where the addend is
// negative; that bit is extracted, shifted to the top and or-ed onto `mag`, the
// magnitude bits of s (one bit-field extract, one shift-or, one add per
// element).  Negation by sign bit is exact for every s.
__device__ __forceinline__ void add_decoded4(float (&acc)[4], uint32_t word, unsigned sh, uint32_t flip, uint32_t mag)
{
    const uint32_t x = word ^ flip;
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = acc[c] + __uint_as_float((((x >> (sh + c)) & 1u) << 31) | mag);
}

constexpr int SERVER_CHUNK = 8;     // workers whose sign words are in flight together

// Server part of Algorithm 4 on the tiles that lie inside one block:
// decode and add the M payloads in worker order, divide by M, add the rescaled
// server residual, compress.  One workgroup per tile; it waits in the kernel
// for its block's scale.  The sign words of SERVER_CHUNK workers are loaded
// together (one 32-bit word per worker and sub-row holds this lane's 4 bits),
// the block's M scales come through scalar loads.
// Six workgroups per CU (80 VGPRs): measured 0.58 ms against 0.63 ms at five and 0.73 ms at eight
// (where a third of the tile spills) on 2^28 elements and 8 workers.
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(6, 8)))
void k_server_uniform(Layout L, ScratchRef R, ServerArgs A, int set)
{
    const Scratch X = open_call(R);
    __shared__ TileShared S;
    const int32_t tile = L.uniform_tiles[blockIdx.x];
    constexpr int n_valid = TILE;
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t b = L.tile_fb[tile];
    float *te = A.err + tile_start;
    Posted P;
    float4 tv[SUBROWS];
    load_tile(te, tv, n_valid);

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
#pragma unroll
        for (int u = 0; u < SERVER_CHUNK; ++u) {
            if (i0 + u < A.M) {
                const uint32_t sb = __float_as_uint(sc[u]);
                const uint32_t flip = ~(uint32_t)((int32_t)sb >> 31), mag = sb & 0x7fffffffu;
#pragma unroll
                for (int k = 0; k < SUBROWS; ++k) add_decoded4(acc[k], word[u][k], sh, flip, mag);
            }
        }
    }
    float4 p[SUBROWS];
    const float r = A.r, Mf = A.Mf, Minv = A.Minv;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        p[k].x = mean_of(acc[k][0], Mf, Minv) + r * tv[k].x;
        p[k].y = mean_of(acc[k][1], Mf, Minv) + r * tv[k].y;
        p[k].z = mean_of(acc[k][2], Mf, Minv) + r * tv[k].z;
        p[k].w = mean_of(acc[k][3], Mf, Minv) + r * tv[k].w;
    }
    const int kind = compress_uniform(p, L, tile, n_valid, A.signs, A.scales, te, X, set, S, P);
    resolve_posted(P, L, X, set, A.scales, S);
    if (kind == UNI_PENDING) finish_uniform(p, tile, n_valid, b, 0ull, te, L, X, set, S);
}

// Server on the mixed tiles (several blocks meet, or the ragged last tile): a
// per-element segment index in LDS selects each worker's scale.  Never waits.
__global__ __launch_bounds__(THREADS) void k_server_mixed(Layout L, ScratchRef R, ServerArgs A, int set)
{
    const Scratch X = open_call(R);
    __shared__ TileShared S;
    const int32_t tile = L.mixed_tiles[blockIdx.x];
    const int n_valid = tile_valid(L, tile);
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    float *te = A.err + tile_start;
    float4 tv[SUBROWS];
    load_tile(te, tv, n_valid);

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
    const int64_t in_hw = 2 * A.in_signs_stride;

    int segi[SUBROWS][4];
    build_segment_index(L, tile, n_valid, fb, lb - fb + 1, S);
    {
        const int *seg = reinterpret_cast<const int *>(S.val);
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int j = local_base(k) + c;
                segi[k][c] = (j < n_valid) ? seg[j] : 0;
            }
    }
    __syncthreads();            // S.val is reused by compress_mixed
    for (int i = 0; i < A.M; ++i) {
        const float *sc_i = A.scales_in + (int64_t)i * A.in_scales_stride + fb;
#pragma unroll
        for (int k = 0; k < SUBROWS; ++k) {
            const uint32_t word = (hw[k] < n_hw) ? s32[(int64_t)i * in_hw + hw[k]] : 0u;
            const unsigned nibble = (word >> sh) & 0xFu;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                acc[k][c] = acc[k][c] + signed_scale(sc_i[segi[k][c]], (nibble >> c) & 1u);
        }
    }
    float4 p[SUBROWS];
    const float r = A.r, Mf = A.Mf, Minv = A.Minv;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) {
        p[k].x = mean_of(acc[k][0], Mf, Minv) + r * tv[k].x;
        p[k].y = mean_of(acc[k][1], Mf, Minv) + r * tv[k].y;
        p[k].z = mean_of(acc[k][2], Mf, Minv) + r * tv[k].z;
        p[k].w = mean_of(acc[k][3], Mf, Minv) + r * tv[k].w;
    }
    compress_mixed(p, L, tile, n_valid, A.signs, A.scales, te, X, set, S);
}

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
        if (threadIdx.x == 0) scales[(int64_t)w * scales_stride + b] = (float)(total / (double)(L.offs[b + 1] - L.offs[b]));
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
__global__ void k_advance(CallState *state, int set_base, int nsets)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state->calls = state->calls + 1u;
        if (set_base == 0)
            state->worker_tags ^= nsets >= 64 ? ~0ull : ((1ull << nsets) - 1ull);
        else
            state->server_tag ^= 1u;
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

// ------------------------------------------------- compressor quality ---
//
// phi(v) = min_b ||v_Gb||_1^2 / (d_b ||v_Gb||_2^2) (Proposition 1) and
// delta(v) = ||v||_1^2 / (d ||v||_2^2) (non-block compressor, Eq. (1)), in
// fp64.  Three small kernels: out[2i] = 1 (the ratio of an all-zero block,
// which the compressor reproduces exactly); per tile the sums of |v| and v^2
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

__global__ __launch_bounds__(THREADS) void k_quality_tiles(Layout L, QualityArgs Q)
{
    __shared__ TileShared S;
    __shared__ double seg_sum[2][2];            // [head, tail][l1, l2] of the open segments
    const int32_t tile = blockIdx.x;
    const int vec = blockIdx.y;
    const int n_valid = tile_valid(L, tile);
    const int64_t tile_start = (int64_t)tile * TILE;
    const int32_t fb = L.tile_fb[tile], lb = L.tile_lb[tile];
    unsigned long long *phi_bits = reinterpret_cast<unsigned long long *>(Q.out + 2 * (int64_t)vec);
    float4 a[SUBROWS];
    load_tile(Q.v + (int64_t)vec * Q.stride + tile_start, a, n_valid);     // elements past d read as 0
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
    __shared__ unsigned long long tile_min;
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
