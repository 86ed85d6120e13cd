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
// Mixed tiles are handed out before the whole tiles (first in the grid of the
// kernel that runs one workgroup per tile; in a kernel of their own before the
// persistent worker kernel), so their partial sums are there when a block's
// last whole tile comes to form the scale.  They never wait for a whole tile:
// a block without whole tiles is finished among the mixed tiles themselves
// (its last tile forms its scale, the others wait for it), while the segments
// that a block with whole tiles has in mixed tiles get p parked in the
// residual buffer.  Parked p (those segments, all tiles of blocks larger than
// fuse_limit, any tile whose bounded wait ran out) is finished by one kernel
// after the main one, which also computes the scales still missing and steps
// the plan to its next call.
//
// Deferred correction (optional)
// ------------------------------
// With Layout::lazy set, the whole tiles of blocks larger than fuse_limit are
// left out of that last kernel: the buffer keeps p, the block's scale is kept
// in Scratch::lazy_scales, a bit per set in CallState says so, and the next
// call subtracts the decoded value as it loads the tile (loaded_correction).
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
constexpr int DEFER_WGS = 16;   // workgroups that serve the run-time lists in the kernel that ends a call
constexpr int FIN_WGS_MAX = 512;    // most workgroups that kernel gives to the scales of blocks larger than fuse_limit ...
constexpr int RES_WGS_MAX = 2048;   // ... and to the segments whose p was parked
constexpr int RES_IN_TAIL_MAX = 4 * RES_WGS_MAX;    // longer lists of parked segments get a kernel of their own
#ifndef EF_PIPE_DEPTH
#define EF_PIPE_DEPTH 3
#endif
constexpr int PIPE_DEPTH = EF_PIPE_DEPTH;     // tiles a persistent workgroup keeps in registers while their scales form
constexpr unsigned long long TAG_BIT = 1ull << 63;
constexpr int FUSE_LIMIT_MAX = 4096;                     // most tiles a one-pass block may be given through ef_plan_tune

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
    // Deferred correction (see Scratch::lazy_scales): on or off, and for every block its position
    // among the blocks larger than fuse_limit (-1 for the others).
    int32_t lazy;
    const int32_t *late_index;    // [B]
    // Whole tiles of blocks larger than fuse_limit are written out in groups of this many
    // consecutive tiles (see sync_group_wait); 0 or 1: every tile on its own.
    int32_t sync_group;
};

// What changes from call to call lives in device memory, so that the kernel
// arguments of a call are the same every time (a captured HIP graph of the
// calls can be replayed): the number of calls made on the plan and the tag each
// scratch set's partial words carry since the last call that used the set.
// The last workgroup of the kernel that ends a call (k_tail) moves it on.
struct CallState {
    unsigned int calls;
    unsigned int server_tag;            // bit 0
    unsigned long long worker_tags;     // bit i: worker i
    unsigned long long worker_pending;  // bit i: worker i's residual buffer holds uncorrected p in its large blocks
    unsigned int server_pending;        // bit 0: the same for the server residual
};

// Kernel argument: the plan's scratch.  A "set" is one worker, or the server.
struct ScratchRef {
    unsigned long long *part;
    unsigned long long *ready;
    unsigned long long *defer_list;
    unsigned long long *fin_list;
    unsigned int *list_cnt;             // [8]: defer_cnt[2], fin_cnt[2], ticket[2] (a call uses those of its parity), done, unused
    float *lazy_scales;                 // [nsets][lazy_stride] last scale of every block larger than fuse_limit
    int lazy_stride;
    const CallState *state;
    int set_base;                       // first set this call uses (0 for workers, max_workers for the server)
    int spin_limit;
};

// Scratch of one call, formed by every kernel from ScratchRef and CallState (open_call).
struct Scratch {
    unsigned long long *part;   // [nsets][2*ntiles] tagged fp64 partial sums of open segments
    unsigned long long *ready;  // [nsets][ntiles][READY_STRIDE]: (epoch << 32) | scale bits in the line of the block's gatherer tile
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
    unsigned int *done;         // workgroups of the call's last kernel that have finished (0 between calls)
    // Deferred correction.  A block larger than fuse_limit cannot have its residual finished in
    // the first kernel; instead of a second pass over it (p written, read back, e written: 8 more
    // bytes per element), the residual buffer keeps p, the block's scale is remembered here, and
    // the next call that loads the buffer subtracts the decoded value on the fly: the same fp32
    // operation on the same operands, one call later.  `pending` says for which sets that is due.
    float *lazy_scales;
    int lazy_stride;
    unsigned long long pending;  // bit i: set (set_base + i)
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
    X.done = R.list_cnt + 6;
    // this call's tags are the stored ones flipped
    if (R.set_base == 0) {
        const unsigned long long t = R.state->worker_tags;
        X.tags = ~(((unsigned long long)uniform_u32((unsigned)(t >> 32)) << 32) | uniform_u32((unsigned)t));
    } else {
        X.tags = (unsigned long long)(uniform_u32(R.state->server_tag) ^ 1u);
    }
    X.lazy_scales = R.lazy_scales;
    X.lazy_stride = R.lazy_stride;
    if (R.set_base == 0) {
        const unsigned long long t = R.state->worker_pending;
        X.pending = ((unsigned long long)uniform_u32((unsigned)(t >> 32)) << 32) | uniform_u32((unsigned)t);
    } else {
        X.pending = (unsigned long long)(uniform_u32(R.state->server_pending) & 1u);
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

// Data-parallel-primitive moves inside a row of 16 lanes: the value of the lane
// whose index differs in bit 0 / bit 1, and of the mirror lane within 8 / 16
// lanes.  Applied in this order to an associative, commutative operation they
// leave its result over the whole row in every lane of the row (after the
// first two steps a group of four lanes agrees, and the mirrors pair up whole
// groups), with no LDS traffic.
#define EF_DPP_XOR1 0xB1            // quad_perm [1,0,3,2]
#define EF_DPP_XOR2 0x4E            // quad_perm [2,3,0,1]
#define EF_DPP_HALF_MIRROR 0x141    // lane i <- lane 7-i of its group of 8
#define EF_DPP_MIRROR 0x140         // lane i <- lane 15-i of its row
template <int CTRL>
__device__ __forceinline__ unsigned row_move(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ double row_move(double v)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const unsigned lo = row_move<CTRL>((unsigned)b), hi = row_move<CTRL>((unsigned)(b >> 32));
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// Sum over the 64 lanes in a fixed order: every lane ends with the same bits.
__device__ __forceinline__ double wave_sum(double v)
{
    v += row_move<EF_DPP_XOR1>(v);
    v += row_move<EF_DPP_XOR2>(v);
    v += row_move<EF_DPP_HALF_MIRROR>(v);
    v += row_move<EF_DPP_MIRROR>(v);
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
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
        // OR over the 16 lanes of the word
        lo |= row_move<EF_DPP_XOR1>(lo);
        hi |= row_move<EF_DPP_XOR1>(hi);
        lo |= row_move<EF_DPP_XOR2>(lo);
        hi |= row_move<EF_DPP_XOR2>(hi);
        lo |= row_move<EF_DPP_HALF_MIRROR>(lo);
        hi |= row_move<EF_DPP_HALF_MIRROR>(hi);
        lo |= row_move<EF_DPP_MIRROR>(lo);
        hi |= row_move<EF_DPP_MIRROR>(hi);
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

// LDS of a workgroup: what every kernel needs for reductions and broadcasts ...
struct SyncShared {
    double red[NWAVES];
    int flag[2];
    unsigned ticket;
};
// ... and what the kernels that cut a tile into segments need on top of it.
struct TileShared : SyncShared {
    float val[TILE];            // |p| per element, then the element's scale (closed segments)
    double open_sum[2];
    int long_list[MAX_LONG];
    int n_long;
};

// ------------------------------------------------- per-set scratch views ---

__device__ __forceinline__ unsigned long long *set_part(const Scratch &X, const Layout &L, int set)
{
    return X.part + (int64_t)set * 2 * L.ntiles;
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

// One-pass blocks: their scale is formed and posted inside the main kernel(s) of the call.
__device__ __forceinline__ bool is_counted(const Layout &L, const BlockSpan &s)
{
    return s.n >= 2 && s.n <= L.fuse_limit;
}

// A one-pass block without a whole tile: all its tiles are mixed ones, which form its scale (in
// the block's last tile) and finish its segments among themselves.
__device__ __forceinline__ bool finishes_with_mixed(const Layout &L, const BlockSpan &s)
{
    return is_counted(L, s) && !has_uniform_tile(s);
}

// Scratch word of block b's segment in tile t: slot 1 of the block's first tile
// if b starts inside that tile (it is then the tile's last segment), slot 0
// everywhere else (first or only segment).
__device__ __forceinline__ int64_t part_index(int64_t t, const BlockSpan &s)
{
    return 2 * t + ((t == s.t0 && (s.bs % TILE) != 0) ? 1 : 0);
}

// The block's last whole tile (meaningful if it has one).
__device__ __forceinline__ int64_t last_whole_tile(const BlockSpan &s)
{
    return s.t0 + s.n - 1 - ((s.be % TILE) != 0 ? 1 : 0);
}

// The tile whose workgroup forms the block's scale: the block's last whole tile, or its last tile
// if it has no whole one.
__device__ __forceinline__ int64_t gatherer_tile(const Layout &L, const BlockSpan &s)
{
    return has_uniform_tile(s) ? last_whole_tile(s) : s.t0 + s.n - 1;
}

// The ready word of a block that spans tiles: where its scale is posted with the call number and
// the workgroups of its other tiles look for it.  Every block has a 128-byte line of its own, found
// through its gatherer tile (different blocks have different gatherer tiles): with the words of
// neighbouring blocks in one line, the gatherers' stores and the other tiles' polls of up to 16
// blocks met in that line, which cost the kernels that wait in place up to a third of their
// time on blocks of 16 to 64 tiles (worker 9.0 -> 6.7 ms, server 0.81 -> 0.44 ms on 2^28 elements
// in blocks of 2^16) and a few percent on blocks of 256 tiles.
constexpr int READY_STRIDE = 16;    // 64-bit words
__device__ __forceinline__ unsigned long long *ready_word(const Scratch &X, const Layout &L, int set, int64_t b)
{
    return X.ready + ((int64_t)set * L.ntiles + gatherer_tile(L, block_span(L, b))) * READY_STRIDE;
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
constexpr int GATHER_KEEP = 4;      // partial words per thread whose values are kept while polling

__device__ __forceinline__ bool gather_scale(int64_t b, const Layout &L, const Scratch &X, int set, SyncShared &S,
                                             float *s)
{
    const BlockSpan sp = block_span(L, b);
    const unsigned long long *part = set_part(X, L, set);
    const unsigned long long tag = set_tag(X, set);
    // Thread t is in charge of tiles t, t + 256, ...  All of them are polled in every round, so
    // that the loads of a round overlap.  The values of the first GATHER_KEEP (blocks of up to
    // 1024 tiles: all) are kept as they arrive; words beyond that are only checked for this
    // call's tag and read once more when everything has arrived.
    double v[GATHER_KEEP];
    unsigned have = 0;
#pragma unroll
    for (int q = 0; q < GATHER_KEEP; ++q) v[q] = 0.0;
    bool complete = false;
    for (int it = 0; it < X.spin_limit; ++it) {
        int all = 1;
#pragma unroll
        for (int q = 0; q < GATHER_KEEP; ++q) {
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
        for (int i = (int)threadIdx.x + GATHER_KEEP * THREADS; i < sp.n; i += THREADS) {
            const unsigned long long w =
                __hip_atomic_load(part + part_index(sp.t0 + i, sp), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((w >> 63) != tag) all = 0;
        }
        if (__syncthreads_and(all)) {
            complete = true;
            break;
        }
        __builtin_amdgcn_s_sleep(8);
    }
    if (!complete) return false;
    double acc = 0.0;               // same order as sum_block_partials: thread t adds tiles t, t + 256, ... ascending
#pragma unroll
    for (int q = 0; q < GATHER_KEEP; ++q) acc += v[q];   // absent words were left at +0
    for (int i = (int)threadIdx.x + GATHER_KEEP * THREADS; i < sp.n; i += THREADS) {
        const unsigned long long w =
            __hip_atomic_load(part + part_index(sp.t0 + i, sp), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        acc += __longlong_as_double((long long)(w & ~TAG_BIT));
    }
    const double total = block_sum(acc, S.red);
    *s = (float)(total / (double)(sp.be - sp.bs));
    return true;
}

// The workgroup that holds the gatherer tile of one-pass block b forms the
// scale from the partials (waiting, bounded, for those still in flight: every
// other tile of the block was handed out earlier), writes it out and posts it
// for the block's other tiles.  Called by every thread of that workgroup;
// returns to all of them whether the scale could be formed, and the scale.
__device__ __forceinline__ bool finish_block(int64_t b, const Layout &L, const Scratch &X, int set,
                                             float *scales_out, SyncShared &S, float *scale)
{
    float s = 0.f;
    const bool ok = gather_scale(b, L, X, set, S, &s);
    if (threadIdx.x == 0) {
        if (ok) {
            scales_out[b] = s;
            __hip_atomic_store(ready_word(X, L, set, b),
                               ((unsigned long long)X.epoch << 32) | (unsigned long long)__float_as_uint(s),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            const unsigned k = atomicAdd(X.fin_cnt, 1u);
            X.fin_list[k] = ((unsigned long long)set << 32) | (unsigned long long)b;
        }
    }
    *scale = s;
    return ok;
}

// Follow up on what a uniform tile posted: if it is its block's last whole
// tile, finish that block.  Called by every thread of the workgroup.
__device__ __forceinline__ void resolve_posted(const Posted &P, const Layout &L, const Scratch &X, int set,
                                               float *scales_out, SyncShared &S)
{
    float s;
    if (P.gather >= 0) (void)finish_block(P.gather, L, X, set, scales_out, S, &s);
}

// Thread 0's early look at the ready word of block b (b < 0: none).
__device__ __forceinline__ unsigned long long peek_ready(int b, const Layout &L, const Scratch &X, int set)
{
    unsigned long long w = 0ull;           // epoch 0 is never used
    if (threadIdx.x == 0 && b >= 0)
        w = __hip_atomic_load(ready_word(X, L, set, b), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return w;
}

// Wait (bounded) until the block's gatherer has posted block b's scale of this call.
// `peeked` is thread 0's earlier look at the word (see peek_ready).  Called by
// every thread of the workgroup; same answer to all of them.
__device__ __forceinline__ bool wait_ready(int64_t b, unsigned long long peeked, const Layout &L, const Scratch &X,
                                           int set, SyncShared &S, float *s)
{
    if (threadIdx.x == 0) {
        const unsigned long long *word = ready_word(X, L, set, b);
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

// Mixed tile (several blocks meet, or the ragged end of the vector): sign words;
// segmented fp64 sums through LDS; scales and residuals e' = p - Delta of the
// closed segments; partial sums of the (at most two) open segments posted, and
// their residuals finished too where the block's scale forms inside this kernel
// (bounded waits), else their elements stored as p for the kernel that ends the
// call.  (Section 3.2 and e_{t+1} = p_t - Delta_t of Algorithm 4.)
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
    // An open segment whose block has no whole tile is finished in place: all tiles of such a
    // block are mixed ones, handed out before any whole tile and in ascending order.  The first
    // segment's block ends in this tile, which makes this workgroup the one that forms its scale;
    // the last segment's block goes on, and its scale comes from the next mixed tile.  The segments
    // of other blocks, and any whose wait runs out, keep p in the residual buffer for the kernel
    // that ends the call.
    float s_head = 0.f, s_tail = 0.f;
    bool fin_head = false, fin_tail = false;
    if (head_open && finishes_with_mixed(L, block_span(L, fb))) {
        fin_head = finish_block(fb, L, X, set, scales_out, S, &s_head);
        if (!fin_head) defer_segment(tile, 0, X, set);
    }
    if (tail_open && finishes_with_mixed(L, block_span(L, lb))) {
        fin_tail = wait_ready(lb, 0ull, L, X, set, S, &s_tail);
        if (!fin_tail) defer_segment(tile, 1, X, set);
    }
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
            if (j < head_end)
                ev[c] = fin_head ? residual(pv[c], s_head) : pv[c];
            else if (j >= tail_begin)
                ev[c] = fin_tail ? residual(pv[c], s_tail) : pv[c];
            else
                ev[c] = residual(pv[c], sv[c]);
        }
        p[k] = make_float4(ev[0], ev[1], ev[2], ev[3]);
    }
    store_tile(err_tile, p, n_valid);
    __syncthreads();            // S.val is free again
}

// Deferred correction of a uniform tile's residual as loaded (see Scratch::lazy_scales): if the
// tile's block is larger than fuse_limit and the set's last call left p in the buffer, what that
// call's payload stood for is subtracted.  The scale is looked up before the tile's loads are
// issued (two dependent scalar loads that then overlap with them) and applied once they are in.
// Called by every thread with the same tile and set.
struct LoadedCorrection {
    float s;
    bool on;
};
__device__ __forceinline__ LoadedCorrection loaded_correction(const Layout &L, int32_t tile, const Scratch &X, int set)
{
    LoadedCorrection c;
    c.s = 0.f;
    c.on = false;
    if (!L.lazy || !((X.pending >> (set - X.set_base)) & 1ull)) return c;
    const int32_t li = L.late_index[L.tile_fb[tile]];
    if (li < 0) return c;
    c.s = X.lazy_scales[(int64_t)set * X.lazy_stride + li];
    c.on = true;
    return c;
}
__device__ __forceinline__ void correct_loaded_residual(float4 (&e)[SUBROWS], const LoadedCorrection &c)
{
    if (!c.on) return;
#pragma unroll
    for (int k = 0; k < SUBROWS; ++k) residual4(e[k], c.s);
}

// Uniform tile (inside one block b): sign words and the tile's fp64 sum.
// Returns what is left to do with it:
//   UNI_DONE    the block is this tile alone: scale and residual written;
//   UNI_PARKED  block larger than fuse_limit: partial posted, p parked for the
//               kernel that ends the call;
//   UNI_PENDING partial posted: p stays with the caller until the block's
//               scale is posted; P says whether this tile must form it.
//   UNI_HELD    (only with hold = true) as UNI_PARKED, but p is still to be written by the caller,
//               after sync_group_wait.
enum { UNI_DONE = 0, UNI_PARKED = 1, UNI_PENDING = 2, UNI_HELD = 3 };

__device__ __forceinline__ int compress_uniform(float4 (&p)[SUBROWS], const Layout &L, int32_t tile, int n_valid,
                                                uint64_t *signs, float *scales_out, float *err_tile,
                                                const Scratch &X, int set, SyncShared &S, Posted &P,
                                                bool hold = false)
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
        if (hold && L.sync_group > 1) return UNI_HELD;
        store_tile(err_tile, p, n_valid);
        return UNI_PARKED;
    }
    if ((int64_t)tile == gatherer_tile(L, sp)) P.gather = b;
    return UNI_PENDING;
}

// Write the residual of a uniform tile of counted block b whose p was kept
// (e_{t+1} = p_t - Delta_t, Algorithm 4), waiting (bounded) for the scale; if
// the wait runs out, p is parked and the segment deferred.
__device__ __forceinline__ void finish_uniform(float4 (&p)[SUBROWS], int32_t tile, int n_valid, int b,
                                               unsigned long long peeked, float *err_tile, const Layout &L,
                                               const Scratch &X, int set, SyncShared &S, bool may_wait = true)
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

// Writing the residual out in step.  Measured on this machine: workgroups that take consecutive
// tiles and hold their residual tile back until all of them have posted their partial sums (as
// the tiles of a small one-pass block do, which wait for one scale) stream faster than workgroups
// that each write as soon as they are done (2^28 elements, 8 workers: 6.6 ms in blocks of 8 to
// 16 tiles against 7.7 ms without any wait; the momentum tile is written at once in both cases,
// holding it back as well was measured slower).  For a uniform tile of a block larger than
// fuse_limit nothing has to be waited for, so the kernel that runs one workgroup per tile makes
// it wait for its neighbours instead: the whole tiles of the block form groups of L.sync_group
// consecutive tiles; the last tile of a group looks for this call's tag on the partial words of
// the others (posted just before) and then posts the call number in its own ready line, where
// the others look for it.  Both waits are bounded, and nothing depends on their outcome:
// whoever runs out of patience just writes.
// Called by every thread of the workgroup, after compress_uniform returned UNI_HELD.
__device__ __forceinline__ void sync_group_wait(int32_t tile, const Layout &L, const Scratch &X, int set, SyncShared &S)
{
    const BlockSpan sp = block_span(L, L.tile_fb[tile]);
    const int64_t first_whole = sp.t0 + ((sp.bs % TILE) != 0 ? 1 : 0);
    const int64_t last_whole = last_whole_tile(sp);
    const int64_t g0 = first_whole + ((int64_t)tile - first_whole) / L.sync_group * L.sync_group;
    const int64_t g1 = min(g0 + L.sync_group - 1, last_whole);
    if (g1 == g0) return;
    // the second word of the tile's line: the first may be the block's ready word
    unsigned long long *line = X.ready + ((int64_t)set * L.ntiles + g1) * READY_STRIDE + 1;
    if ((int64_t)tile == g1) {
        const unsigned long long *part = set_part(X, L, set);
        const unsigned long long tag = set_tag(X, set);
        const int others = (int)(g1 - g0);
        for (int it = 0; it < X.spin_limit; ++it) {
            int all = 1;
            if ((int)threadIdx.x < others) {
                const unsigned long long w = __hip_atomic_load(part + 2 * (g0 + threadIdx.x), __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT);
                all = (w >> 63) == tag ? 1 : 0;
            }
            if (__syncthreads_and(all)) break;
            __builtin_amdgcn_s_sleep(8);
        }
        if (threadIdx.x == 0)
            __hip_atomic_store(line, (unsigned long long)X.epoch << 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        if (threadIdx.x == 0) {
            for (int it = 0; it < X.spin_limit; ++it) {
                const unsigned long long w = __hip_atomic_load(line, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((unsigned)(w >> 32) == X.epoch) break;
                __builtin_amdgcn_s_sleep(8);
            }
        }
        __syncthreads();
    }
}

// Fill S.val (read as int) with the segment index of every element of a mixed
// tile (0 past the end of the vector), so that element j can look up scale[fb + seg].
__device__ __forceinline__ void build_segment_index(const Layout &L, int32_t tile, int n_valid, int32_t fb,
                                                    int nseg, TileShared &S)
{
    const int64_t tile_start = (int64_t)tile * TILE;
    int *seg = reinterpret_cast<int *>(S.val);
    if (threadIdx.x == 0) S.n_long = 0;
    __syncthreads();
    for (int j = n_valid + (int)threadIdx.x; j < TILE; j += THREADS) seg[j] = 0;
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

}  // namespace ef
