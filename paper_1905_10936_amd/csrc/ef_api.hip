// Host side of libef: plan construction, argument checks and kernel launches
// behind the C ABI declared in include/ef.h.
#include "ef.h"
#include "ef_debug.h"
#include "ef_device.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

struct ef_plan {
    ef::Layout L;
    ef::ScratchRef X;
    int max_workers;
    int device;
    int spin_limit;
    ef::CallState *d_state;         // calls made so far and the tags of the scratch sets: advanced on the device
    std::vector<int64_t> offs_host;
    std::vector<int32_t> fb_host, lb_host;
    // What depends on the one-pass limit, which differs between the kernels (each is bounded by what
    // the kernel's own grid keeps resident): role 0 = the persistent worker kernel, 1 = the server,
    // 2 = the worker kernel that runs one workgroup per tile.
    struct Role {
        int32_t fuse_limit;
        uint32_t n_static;          // segments whose p the first kernels always park
        uint32_t n_late;            // blocks whose scale the first kernels never write
        uint32_t *d_static;         // [2*ntiles] capacity
        int32_t *d_late;            // [min(B, 2*ntiles)] capacity
        // deferred correction: position of every block in d_late if it is larger than fuse_limit, else -1;
        // the whole tiles of those blocks (left out of d_static while the mode is on)
        int32_t *d_late_index;      // [B]
        int32_t *d_lazy_tiles;      // [ntiles] capacity
        uint32_t n_lazy_tiles;
    } role[3];
    int sync_group;                 // tiles of a large block that are written out in step (ef_plan_set_sync_group)
    int lazy;                       // deferred correction on (ef_plan_set_lazy)
    ef_state *state;                // the library-held state that lives on this plan, if any
    // Host-side guard of the deferred mode: the residual buffers (workers, server) the last calls
    // left waiting for their correction, so that a call with other buffers is refused.  The
    // device-side CallState is what the kernels go by; this only catches misuse at the boundary.
    mutable const float *lazy_buf[2];
    mutable int64_t lazy_stride_seen;
    mutable int lazy_sets_seen;     // most workers any call since the last full flush has used
    float *d_lazy_scales;           // [nsets][lazy_stride]
    int lazy_stride;
    int32_t lim_persistent, lim_direct, lim_server;   // automatic limits
    int32_t user_fuse_limit;        // >= 0: set through ef_plan_tune, overrides the automatic limits
    // device allocations owned by the plan
    int64_t *d_offs;
    int32_t *d_tile_fb;
    int32_t *d_tile_lb;
    unsigned long long *d_part;
    unsigned long long *d_ready;
    unsigned int *d_list_cnt;       // [8]: defer_cnt[2], fin_cnt[2], ticket[2] (alternating between calls), done, unused
    int worker_grid;                // workgroups of the persistent worker kernel
    int persistent;                 // worker: 1 pipelined persistent kernel, 0 one workgroup per tile
    int persistent_auto;            // what plan creation chose for this layout
    int persistent_forced;          // 1 after ef_plan_set_persistent(plan, 1): also for the momentum-free worker
    unsigned long long *d_defer_list;
    unsigned long long *d_fin_list;
    int32_t *d_mixed, *d_uniform;   // tile lists
    // compressor-quality diagnostics
    int32_t *d_cross;               // blocks that span several tiles
    int32_t n_cross;
    double *d_qtile, *d_qpart;      // [max_workers][ntiles][2], [max_workers][2*ntiles][2]
};

// Scratch of ef_compressor_quality_static: device memory that exists from the moment the library
// is loaded on a GPU, so that the call allocates nothing.  In host code the array's name is only a
// stand-in for the symbol; the memory is reached through the per-device address that
// static_scratch() looks up once per device.
static __device__ __align__(256) double scratch[(size_t)EF_QUALITY_STATIC_MAX_TILE_VECTORS * 6];

// Optimizer state held by the library (ef_state_create): Algorithm 4's m_i and e_i of n_workers
// workers and the server's e~, in device memory the caller never addresses, which lets every call
// on it run in the deferred-correction mode.
struct ef_state {
    ef_plan *plan;
    int n_workers;
    int64_t stride;                 // elements between two workers' rows: d rounded up to a multiple of 4
    float *mom, *err;               // [n_workers][stride]
    float *server_err;              // [d]
};

namespace {

enum { ROLE_TICKET = 0, ROLE_SERVER = 1, ROLE_TILES = 2 };

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
double *g_scratch_ptr[MAX_DEVICES];     // [device] address of `scratch` on that device, once looked up

thread_local char g_errbuf[512];
thread_local hipError_t g_last_hip = hipSuccess;

int hip_fail(hipError_t e)
{
    g_last_hip = e;
    return EF_ERR_HIP;
}

#define EF_HIP(call)                                  \
    do {                                              \
        hipError_t e_ = (call);                       \
        if (e_ != hipSuccess) return hip_fail(e_);    \
    } while (0)

// A plan's tables, scratch and state live on the device it was created on: a call made with another
// device current would launch kernels there on memory they cannot reach.
int on_plan_device(const ef_plan *plan)
{
    int device = -1;
    EF_HIP(hipGetDevice(&device));
    return device == plan->device ? EF_OK : EF_ERR_ARG;
}

// Address of the static scratch on the current device (which must be `device`).  The first call
// per device asks the runtime for the symbol's address; no memory is allocated.
int static_scratch(int device, double **out)
{
    if (device < 0 || device >= MAX_DEVICES) return EF_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return hip_fail(e != hipSuccess ? e : hipErrorInvalidSymbol);
        g_scratch_ptr[device] = static_cast<double *>(ptr);
    }
    *out = g_scratch_ptr[device];
    return EF_OK;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Do the byte ranges [a, a + na) and [b, b + nb) share a byte?
bool overlap(const void *a, size_t na, const void *b, size_t nb)
{
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + nb && b0 < a0 + na;
}

// Bytes spanned by n rows of `row` items that lie `stride` items apart (item size `item`).
size_t span_bytes(int n, int64_t stride, int64_t row, size_t item)
{
    return ((size_t)(n - 1) * (size_t)stride + (size_t)row) * item;
}

int check_offsets(const int64_t *offs, int64_t B)
{
    if (!offs) return EF_ERR_NULL;
    if (B < 1 || B > (int64_t)0x7fffffff - 1) return EF_ERR_OFFSETS;
    if (offs[0] != 0) return EF_ERR_OFFSETS;
    for (int64_t b = 0; b < B; ++b)
        if (offs[b + 1] <= offs[b]) return EF_ERR_OFFSETS;
    // tiles are indexed with 32-bit integers
    if ((offs[B] + ef::TILE - 1) / ef::TILE > (int64_t)0x7fffffff) return EF_ERR_OFFSETS;
    return EF_OK;
}

bool good_eta(float eta_prev, float eta)
{
    return std::isfinite(eta) && std::isfinite(eta_prev) && eta > 0.0f && eta_prev >= 0.0f;
}

void destroy_device(ef_plan *p)
{
    if (p->d_offs) (void)hipFree(p->d_offs);
    if (p->d_tile_fb) (void)hipFree(p->d_tile_fb);
    if (p->d_tile_lb) (void)hipFree(p->d_tile_lb);
    if (p->d_part) (void)hipFree(p->d_part);
    if (p->d_ready) (void)hipFree(p->d_ready);
    if (p->d_list_cnt) (void)hipFree(p->d_list_cnt);
    if (p->d_state) (void)hipFree(p->d_state);
    if (p->d_lazy_scales) (void)hipFree(p->d_lazy_scales);
    if (p->d_defer_list) (void)hipFree(p->d_defer_list);
    if (p->d_fin_list) (void)hipFree(p->d_fin_list);
    for (auto &r : p->role) {
        if (r.d_static) (void)hipFree(r.d_static);
        if (r.d_late) (void)hipFree(r.d_late);
        if (r.d_late_index) (void)hipFree(r.d_late_index);
        if (r.d_lazy_tiles) (void)hipFree(r.d_lazy_tiles);
    }
    if (p->d_mixed) (void)hipFree(p->d_mixed);
    if (p->d_uniform) (void)hipFree(p->d_uniform);
    if (p->d_cross) (void)hipFree(p->d_cross);
    if (p->d_qtile) (void)hipFree(p->d_qtile);
    if (p->d_qpart) (void)hipFree(p->d_qpart);
}

int64_t tiles_of_block(const ef_plan *p, int64_t b)
{
    const int64_t *o = p->offs_host.data();
    return (o[b + 1] - 1) / ef::TILE - o[b] / ef::TILE + 1;
}

bool has_uniform_tile(const ef_plan *p, int64_t b)
{
    const int64_t *o = p->offs_host.data();
    return tiles_of_block(p, b) - (o[b] % ef::TILE != 0 ? 1 : 0) - (o[b + 1] % ef::TILE != 0 ? 1 : 0) >= 1;
}

// A one-pass block without a whole tile is finished among the mixed tiles.  (Host mirror of
// finishes_with_mixed in ef_tile.h.)
bool finishes_with_mixed(const ef_plan *p, const ef_plan::Role &r, int64_t b)
{
    const int64_t n = tiles_of_block(p, b);
    return n >= 2 && n <= r.fuse_limit && !has_uniform_tile(p, b);
}

// What the main kernels of a call always leave to the kernel that ends it: the scales of the
// blocks larger than fuse_limit, and the residual of every open segment that is not finished
// where it is computed (the segments of those large blocks, and the segments that blocks with
// whole tiles have in mixed tiles).
int upload_static_list(ef_plan *p, ef_plan::Role &r)
{
    std::vector<uint32_t> items;
    std::vector<int32_t> late, late_index((size_t)p->L.B, -1), lazy_tiles;
    const int64_t *o = p->offs_host.data();
    for (int64_t b = 0; b < p->L.B; ++b) {
        const int64_t n = tiles_of_block(p, b);
        if (n < 2 || n <= r.fuse_limit) continue;
        if (has_uniform_tile(p, b)) late_index[(size_t)b] = (int32_t)late.size();
        late.push_back((int32_t)b);
    }
    for (int32_t t = 0; t < p->L.ntiles; ++t) {
        const int64_t start = (int64_t)t * ef::TILE, end = start + ef::TILE;
        const int32_t fb = p->fb_host[t], lb = p->lb_host[t];
        const bool full = end <= p->L.d;
        if (fb == lb && full) {
            // a whole tile parks p only for blocks beyond fuse_limit
            const bool open = (o[fb] < start) || (o[fb + 1] > end);
            if (open && tiles_of_block(p, fb) > r.fuse_limit) {
                if (p->lazy)
                    lazy_tiles.push_back(t);        // deferred: corrected when the buffer is next loaded
                else
                    items.push_back(((uint32_t)t << 1) | 0u);
            }
        } else {
            // a tile the mixed-tile code handles (several blocks, or the ragged end of the vector)
            if (o[fb] < start && !finishes_with_mixed(p, r, fb)) items.push_back(((uint32_t)t << 1) | 0u);
            if (o[lb + 1] > end && !finishes_with_mixed(p, r, lb)) items.push_back(((uint32_t)t << 1) | 1u);
        }
    }
    r.n_late = (uint32_t)late.size();
    r.n_static = (uint32_t)items.size();
    r.n_lazy_tiles = (uint32_t)lazy_tiles.size();
    EF_HIP(hipMemcpy(r.d_late_index, late_index.data(), sizeof(int32_t) * late_index.size(), hipMemcpyHostToDevice));
    if (!lazy_tiles.empty())
        EF_HIP(hipMemcpy(r.d_lazy_tiles, lazy_tiles.data(), sizeof(int32_t) * lazy_tiles.size(), hipMemcpyHostToDevice));
    if (!late.empty()) EF_HIP(hipMemcpy(r.d_late, late.data(), sizeof(int32_t) * late.size(), hipMemcpyHostToDevice));
    if (!items.empty())
        EF_HIP(hipMemcpy(r.d_static, items.data(), sizeof(uint32_t) * items.size(), hipMemcpyHostToDevice));
    return EF_OK;
}

// Pick each role's one-pass limit and rebuild the lists that depend on it.
// Deferred mode, one workgroup per tile: blocks of up to this many tiles still wait for their
// scale in the kernel (measured: 6.6-6.75 ms on 2^28 elements and 8 workers for blocks of 2 to
// 64 tiles, as fast as anything else in that mode, and their residual is finished at once).
constexpr int32_t LAZY_WAIT_LIMIT = 64;

int refresh_limits_unguarded(ef_plan *p)
{
    auto clamp = [](int64_t v) { return (int32_t)(v < 0 ? 0 : (v > ef::FUSE_LIMIT_MAX ? ef::FUSE_LIMIT_MAX : v)); };
    ef_plan::Role &ticket = p->role[ROLE_TICKET], &server = p->role[ROLE_SERVER], &tiles = p->role[ROLE_TILES];
    if (p->user_fuse_limit >= 0) {
        ticket.fuse_limit = server.fuse_limit = tiles.fuse_limit = clamp(p->user_fuse_limit);
    } else if (p->lazy) {
        // With the correction deferred nothing has to wait for a block's scale.  The server and
        // the persistent worker kernel then run fastest without any wait; the worker kernel with
        // one workgroup per tile runs fastest when consecutive tiles are written out in step,
        // which small blocks get by waiting for their scale as usual and larger ones through
        // Layout::sync_group.  Both worker roles get the same limit: the buffers a call leaves
        // behind must fit the lists of whichever worker call comes next.
        ticket.fuse_limit = tiles.fuse_limit = p->persistent_forced ? 0 : LAZY_WAIT_LIMIT;
        server.fuse_limit = 0;
    } else {
        ticket.fuse_limit = clamp(p->lim_persistent);
        server.fuse_limit = clamp(p->lim_server);
        tiles.fuse_limit = clamp(p->lim_direct);
    }
    p->L.fuse_limit = p->role[0].fuse_limit;
    for (auto &r : p->role) {
        int rc = upload_static_list(p, r);
        if (rc) return rc;
    }
    return EF_OK;
}

// The lists are built in host vectors: a failed allocation there becomes an error code, not an
// exception crossing the C boundary.
int refresh_limits(ef_plan *p)
{
    try {
        return refresh_limits_unguarded(p);
    } catch (const std::bad_alloc &) {
        return EF_ERR_ARG;
    }
}

int build_device(ef_plan *p)
{
    const int64_t B = p->L.B, d = p->L.d;
    const int32_t ntiles = p->L.ntiles;
    const int nsets = p->max_workers + 1;    // workers 0..max_workers-1, then the server
    std::vector<int32_t> &fb = p->fb_host, &lb = p->lb_host;
    fb.resize(ntiles);
    lb.resize(ntiles);
    {
        // block of the first and of the last valid element of every tile
        int64_t b = 0;
        const int64_t *o = p->offs_host.data();
        for (int32_t t = 0; t < ntiles; ++t) {
            const int64_t first = (int64_t)t * ef::TILE;
            int64_t last = first + ef::TILE - 1;
            if (last > d - 1) last = d - 1;
            while (o[b + 1] <= first) ++b;
            fb[t] = (int32_t)b;
            int64_t c = b;
            while (o[c + 1] <= last) ++c;
            lb[t] = (int32_t)c;
        }
    }
    EF_HIP(hipGetDevice(&p->device));
    EF_HIP(hipMalloc(&p->d_offs, sizeof(int64_t) * (B + 1)));
    EF_HIP(hipMalloc(&p->d_tile_fb, sizeof(int32_t) * ntiles));
    EF_HIP(hipMalloc(&p->d_tile_lb, sizeof(int32_t) * ntiles));
    EF_HIP(hipMalloc(&p->d_part, sizeof(unsigned long long) * 2 * (size_t)ntiles * nsets));
    EF_HIP(hipMemcpy(p->d_offs, p->offs_host.data(), sizeof(int64_t) * (B + 1), hipMemcpyHostToDevice));
    EF_HIP(hipMemcpy(p->d_tile_fb, fb.data(), sizeof(int32_t) * ntiles, hipMemcpyHostToDevice));
    EF_HIP(hipMemcpy(p->d_tile_lb, lb.data(), sizeof(int32_t) * ntiles, hipMemcpyHostToDevice));
    EF_HIP(hipMemset(p->d_part, 0, sizeof(unsigned long long) * 2 * (size_t)ntiles * nsets));
    // a block that crosses a tile boundary owns at least one of the 2*ntiles open segments
    const size_t max_cross = (size_t)(2 * (int64_t)ntiles < B ? 2 * (int64_t)ntiles : B);
    // one 128-byte line per tile and set: a block's ready word sits in the line of its gatherer tile
    EF_HIP(hipMalloc(&p->d_ready, sizeof(unsigned long long) * ef::READY_STRIDE * (size_t)ntiles * nsets));
    EF_HIP(hipMemset(p->d_ready, 0, sizeof(unsigned long long) * ef::READY_STRIDE * (size_t)ntiles * nsets));
    EF_HIP(hipMalloc(&p->d_list_cnt, sizeof(unsigned int) * 8));
    EF_HIP(hipMalloc(&p->d_defer_list, sizeof(unsigned long long) * 2 * (size_t)ntiles * nsets));
    EF_HIP(hipMalloc(&p->d_fin_list, sizeof(unsigned long long) * max_cross * nsets));
    for (auto &r : p->role) {
        EF_HIP(hipMalloc(&r.d_static, sizeof(uint32_t) * 2 * (size_t)ntiles));
        EF_HIP(hipMalloc(&r.d_late, sizeof(int32_t) * max_cross));
        EF_HIP(hipMalloc(&r.d_late_index, sizeof(int32_t) * (size_t)B));
        EF_HIP(hipMalloc(&r.d_lazy_tiles, sizeof(int32_t) * (size_t)ntiles));
    }
    p->lazy_stride = (int)max_cross;
    EF_HIP(hipMalloc(&p->d_lazy_scales, sizeof(float) * max_cross * nsets));
    EF_HIP(hipMemset(p->d_lazy_scales, 0, sizeof(float) * max_cross * nsets));
    {
        std::vector<int32_t> mixed, uniform;
        for (int32_t t = 0; t < ntiles; ++t) {
            const bool full = ((int64_t)t + 1) * ef::TILE <= d;
            (fb[t] == lb[t] && full ? uniform : mixed).push_back(t);
        }
        p->L.n_mixed = (int32_t)mixed.size();
        p->L.n_uniform = (int32_t)uniform.size();
        EF_HIP(hipMalloc(&p->d_mixed, sizeof(int32_t) * (mixed.size() + 1)));
        EF_HIP(hipMalloc(&p->d_uniform, sizeof(int32_t) * (uniform.size() + 1)));
        if (!mixed.empty())
            EF_HIP(hipMemcpy(p->d_mixed, mixed.data(), sizeof(int32_t) * mixed.size(), hipMemcpyHostToDevice));
        if (!uniform.empty())
            EF_HIP(hipMemcpy(p->d_uniform, uniform.data(), sizeof(int32_t) * uniform.size(), hipMemcpyHostToDevice));
        p->L.mixed_tiles = p->d_mixed;
        p->L.uniform_tiles = p->d_uniform;
    }
    EF_HIP(hipMemset(p->d_list_cnt, 0, sizeof(unsigned int) * 8));
    EF_HIP(hipMalloc(&p->d_state, sizeof(ef::CallState)));
    EF_HIP(hipMemset(p->d_state, 0, sizeof(ef::CallState)));     // the zeroed partial words carry tag 0
    p->L.offs = p->d_offs;
    p->L.tile_fb = p->d_tile_fb;
    p->L.tile_lb = p->d_tile_lb;
    p->X.part = p->d_part;
    p->X.ready = p->d_ready;
    p->X.defer_list = p->d_defer_list;
    p->X.fin_list = p->d_fin_list;
    p->X.list_cnt = p->d_list_cnt;
    p->X.state = p->d_state;
    p->X.lazy_scales = p->d_lazy_scales;
    p->X.lazy_stride = p->lazy_stride;
    // A block finishes in one pass if its tiles fit twice over into the
    // workgroups resident at once (see ef_tile.h).
    {
        hipDeviceProp_t prop;
        EF_HIP(hipGetDeviceProperties(&prop, p->device));
        int occ_w = 0, occ_s = 0;
        EF_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ_w, ef::k_worker_uniform<true>, ef::THREADS, 0));
        EF_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ_s, ef::k_server_tiles<true>, ef::THREADS, 0));
        if (occ_w < 1) occ_w = 1;
        p->worker_grid = prop.multiProcessorCount * occ_w;
        // one-pass blocks must fit twice over into the tiles a kernel's workgroups hold at once:
        // grid x (PIPE_DEPTH + STAGE_DEPTH) for the persistent kernel, the resident workgroups for the kernels that
        // run one workgroup per tile (dispatched in grid order).  Larger limits were measured slower:
        // a block that fills most of the machine makes its first tiles wait for its last.
        int occ_d = 0;
        EF_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ_d, (ef::k_worker_tiles<true, true, false>), ef::THREADS, 0));
        p->lim_persistent = (int32_t)((int64_t)p->worker_grid * (ef::PIPE_DEPTH + ef::STAGE_DEPTH) / 2);
        p->lim_direct = (int32_t)((int64_t)prop.multiProcessorCount * occ_d / 2);
        p->lim_server = (int32_t)((int64_t)prop.multiProcessorCount * occ_s / 2);
    }
    p->user_fuse_limit = -1;
    // Which worker kernel for this layout.  The persistent kernel needs enough tiles per workgroup
    // to fill its pipeline; beyond that the choice follows the measured cost per tile of each
    // kernel by block size (2^28 elements, 8 workers, relative to the persistent kernel's 7.0 ms,
    // which does not depend on the block size up to its one-pass limit): the kernel with one
    // workgroup per tile is faster on blocks of up to 256 tiles, level up to 512, slower beyond,
    // and sends blocks above its own limit through the second pass.
    {
        const int64_t tiles_per_wg = (int64_t)p->L.n_uniform * p->max_workers / (p->worker_grid > 0 ? p->worker_grid : 1);
        const int64_t lim_hi = p->lim_persistent < ef::FUSE_LIMIT_MAX ? p->lim_persistent : ef::FUSE_LIMIT_MAX;
        const int64_t lim_lo = p->lim_direct < ef::FUSE_LIMIT_MAX ? p->lim_direct : ef::FUSE_LIMIT_MAX;
        double cost_direct = 0.0, cost_persistent = 0.0;
        for (int64_t b = 0; b < B; ++b) {
            const int64_t n = tiles_of_block(p, b);
            if (n < 2 || !has_uniform_tile(p, b)) continue;
            const double two_pass = 1.4;        // 28.125 instead of 20.125 bytes per element
            cost_persistent += (double)n * (n <= lim_hi ? 1.0 : two_pass);
            cost_direct += (double)n * (n > lim_lo ? two_pass - 0.03 : n <= 128 ? 0.94 : n <= 256 ? 0.98 : n <= 512 ? 1.0 : 1.05);
        }
        // a clear difference (blocks that only the persistent kernel finishes in one pass) decides from
        // 16 tiles per workgroup on, a small one only once the pipeline is well filled
        p->persistent_auto = ((tiles_per_wg >= 64 && cost_persistent < cost_direct) ||
                              (tiles_per_wg >= 16 && cost_persistent < 0.9 * cost_direct)) ? 1 : 0;
    }
    {
        // compressor-quality diagnostics: the blocks that span several tiles, and the per-tile sums
        std::vector<int32_t> cross;
        for (int64_t b = 0; b < B; ++b)
            if (tiles_of_block(p, b) >= 2) cross.push_back((int32_t)b);
        const size_t nt = (size_t)ntiles, nv = (size_t)p->max_workers;
        EF_HIP(hipMalloc(&p->d_cross, sizeof(int32_t) * (cross.size() + 1)));
        if (!cross.empty())
            EF_HIP(hipMemcpy(p->d_cross, cross.data(), sizeof(int32_t) * cross.size(), hipMemcpyHostToDevice));
        p->n_cross = (int32_t)cross.size();
        EF_HIP(hipMalloc(&p->d_qpart, sizeof(double) * 4 * nt * nv));
        EF_HIP(hipMalloc(&p->d_qtile, sizeof(double) * 2 * nt * nv));
    }
    {
        double *unused = nullptr;       // the static scratch of this device, looked up once, ahead of the first call that needs it
        int rc_scratch = static_scratch(p->device, &unused);
        if (rc_scratch) return rc_scratch;
    }
    // Measured on an otherwise idle GPU: every wait of every benchmark layout ends within 64 polls
    // (about 1.2 us each); 2048 polls leave a factor of 32 for a GPU that is shared, and a wait that
    // is lost (its gatherer not resident) costs about 2.5 ms before the tile takes the second pass.
    p->spin_limit = 1 << 11;
    p->persistent = p->persistent_auto;
    p->persistent_forced = 0;
    int rc = refresh_limits(p);
    if (rc) return rc;
    EF_HIP(hipDeviceSynchronize());
    return EF_OK;
}

// Which worker kernel a call runs.  The persistent kernel (ROLE_TICKET) where plan creation or
// the caller chose it, with two exceptions.  The momentum-free worker moves 48 KiB per tile
// instead of 80: one ticket per tile would make the ticket counter (about 84 tickets per
// microsecond) its bottleneck, so it runs one workgroup per tile unless the persistent kernel
// was asked for explicitly.  And in the deferred mode the kernel with one workgroup per tile is
// the faster one (see refresh_limits).
int worker_role(const ef_plan *plan, bool has_mom)
{
    const bool ticketed = plan->L.n_uniform && plan->persistent &&
                          (plan->lazy ? plan->persistent_forced != 0 : (has_mom || plan->persistent_forced));
    return ticketed ? ROLE_TICKET : ROLE_TILES;
}

// Scratch argument of one call over the sets [set_base, set_base + nsets).  Everything that
// differs between two calls of the same kind is read by the kernels from device memory.
struct CallScratch {
    ef::ScratchRef X;
};

CallScratch next_call(const ef_plan *plan, int set_base, int nsets)
{
    (void)nsets;
    CallScratch c;
    c.X = plan->X;
    c.X.set_base = set_base;
    c.X.spin_limit = plan->spin_limit;
    return c;
}

// The kernel after the main one(s): missing scales, parked residuals, and the step to the next call.
ef::Layout role_layout(const ef_plan *plan, int role)
{
    ef::Layout L = plan->L;
    L.fuse_limit = plan->role[role].fuse_limit;
    L.lazy = plan->lazy;
    L.late_index = plan->role[role].d_late_index;
    L.sync_group = plan->sync_group;
    return L;
}

int launch_tail(const ef_plan *plan, int role, const CallScratch &c, int nsets, float *err, int64_t err_stride,
                float *scales, int64_t scales_stride, hipStream_t s)
{
    const ef_plan::Role &r = plan->role[role];
    const ef::Layout L = role_layout(plan, role);
    ef::TailArgs T;
    T.late_blocks = r.d_late;
    T.n_late = (int)r.n_late;
    T.items = r.d_static;
    T.n_items = (int)r.n_static;
    T.nsets = nsets;
    T.err = err;
    T.err_stride = err_stride;
    T.scales = scales;
    T.scales_stride = scales_stride;
    const int64_t n_fin = (int64_t)r.n_late * nsets, n_res = (int64_t)r.n_static * nsets;
    // a long list of parked segments is streamed by a kernel of its own, after this one has formed the scales
    const bool res_apart = n_res > ef::RES_IN_TAIL_MAX;
    if (res_apart) T.n_items = 0;
    T.fin_wgs = (int)(n_fin < ef::FIN_WGS_MAX ? n_fin : ef::FIN_WGS_MAX);
    T.res_wgs = res_apart ? 0 : (int)(n_res < ef::RES_WGS_MAX ? n_res : ef::RES_WGS_MAX);
    T.state = plan->d_state;
    T.lazy = plan->lazy;
    hipLaunchKernelGGL(ef::k_tail, dim3((unsigned)(T.fin_wgs + T.res_wgs + ef::DEFER_WGS)), dim3(ef::THREADS), 0, s, L,
                       c.X, T);
    EF_HIP(hipGetLastError());
    if (res_apart) {
        hipLaunchKernelGGL(ef::k_residual_static, dim3(r.n_static, (unsigned)nsets), dim3(ef::THREADS), 0, s, L,
                           (const uint32_t *)r.d_static, (int)r.n_static, err, err_stride, (const float *)scales,
                           scales_stride);
        EF_HIP(hipGetLastError());
    }
    return EF_OK;
}

// Bytes of one fused message: W sign words, then B fp32 scales, padded to 16.
size_t payload_bytes(const ef_plan *plan)
{
    const size_t raw = (size_t)plan->L.W * 8u + (size_t)plan->L.B * 4u;
    return (raw + 15u) / 16u * 16u;
}

int worker_step_impl(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride, float *mom,
                     float *err, int64_t state_stride, float mu, float eta_prev, float eta, uint64_t *packed_signs,
                     int64_t signs_stride, float *scales, int64_t scales_stride, void *stream, double *quality = nullptr);
int server_step_impl(const ef_plan *plan, int M, const uint64_t *packed_signs, int64_t in_signs_stride,
                     const float *scales, int64_t in_scales_stride, float *server_err, float eta_prev, float eta,
                     uint64_t *out_signs, float *out_scales, void *stream);

}  // namespace

extern "C" {

size_t ef_sign_words(const ef_plan *plan) { return plan ? (size_t)plan->L.W : 0; }

int ef_plan_create(ef_plan **out, const int64_t *block_offsets_host, int64_t B, int max_workers, void *stream)
{
    (void)stream;
    if (!out) return EF_ERR_NULL;
    *out = nullptr;
    int rc = check_offsets(block_offsets_host, B);
    if (rc) return rc;
    if (max_workers < 1 || max_workers > EF_MAX_WORKERS) return EF_ERR_ARG;
    ef_plan *p = new (std::nothrow) ef_plan();
    if (!p) return EF_ERR_ARG;
    p->max_workers = max_workers;
    p->L.B = B;
    p->L.d = block_offsets_host[B];
    p->L.W = (p->L.d + 63) / 64;
    p->L.ntiles = (int32_t)((p->L.d + ef::TILE - 1) / ef::TILE);
    p->d_offs = nullptr;
    p->d_tile_fb = p->d_tile_lb = nullptr;
    p->d_part = nullptr;
    p->d_ready = nullptr;
    p->d_list_cnt = nullptr;
    p->d_state = nullptr;
    p->d_lazy_scales = nullptr;
    p->lazy = 0;
    p->state = nullptr;
    p->sync_group = 16;
    p->lazy_buf[0] = p->lazy_buf[1] = nullptr;
    p->lazy_stride_seen = 0;
    p->lazy_sets_seen = 0;
    p->d_defer_list = nullptr;
    p->d_fin_list = nullptr;
    for (auto &r : p->role) {
        r.d_static = nullptr;
        r.d_late = nullptr;
        r.d_late_index = r.d_lazy_tiles = nullptr;
        r.n_static = r.n_late = r.n_lazy_tiles = 0;
        r.fuse_limit = 0;
    }
    p->d_mixed = p->d_uniform = nullptr;
    p->d_cross = nullptr;
    p->n_cross = 0;
    p->d_qtile = p->d_qpart = nullptr;

    try {
        p->offs_host.assign(block_offsets_host, block_offsets_host + B + 1);
        rc = build_device(p);
    } catch (const std::bad_alloc &) {      // host memory for the layout tables
        rc = EF_ERR_ARG;
    }
    if (rc) {
        destroy_device(p);
        delete p;
        return rc;
    }
    *out = p;
    return EF_OK;
}

int ef_plan_destroy(ef_plan *plan)
{
    if (!plan) return EF_ERR_NULL;
    if (plan->state) return EF_ERR_ARG;     // ef_state_destroy first
    (void)hipDeviceSynchronize();
    destroy_device(plan);
    delete plan;
    return EF_OK;
}

// Residual buffers whose large blocks still hold uncorrected p (deferred correction): the lists
// that say which blocks those are must not change under them.
static int residuals_pending(ef_plan *plan, bool *pending)
{
    ef::CallState st;
    EF_HIP(hipDeviceSynchronize());
    EF_HIP(hipMemcpy(&st, plan->d_state, sizeof st, hipMemcpyDeviceToHost));
    *pending = st.worker_pending != 0ull || st.server_pending != 0u;
    return EF_OK;
}

static int set_lazy(ef_plan *plan, int on);

int ef_plan_set_lazy(ef_plan *plan, int on)
{
    if (!plan) return EF_ERR_NULL;
    if (plan->state) return EF_ERR_ARG;     // a library-held state keeps the mode on
    return set_lazy(plan, on);
}

static int set_lazy(ef_plan *plan, int on)
{
    bool pending = false;
    int rc = residuals_pending(plan, &pending);
    if (rc) return rc;
    if (pending) return EF_ERR_ARG;
    plan->lazy = on ? 1 : 0;
    plan->lazy_buf[0] = plan->lazy_buf[1] = nullptr;
    plan->lazy_sets_seen = 0;
    return refresh_limits(plan);
}

int ef_plan_is_lazy(const ef_plan *plan) { return plan ? plan->lazy : 0; }

int ef_plan_set_sync_group(ef_plan *plan, int tiles)
{
    if (!plan) return EF_ERR_NULL;
    if (tiles < 0 || tiles > 256) return EF_ERR_ARG;
    EF_HIP(hipDeviceSynchronize());
    plan->sync_group = tiles;
    return EF_OK;
}

int ef_flush(const ef_plan *plan, int n_workers, float *err, int64_t state_stride, float *server_err, void *stream)
{
    if (!plan) return EF_ERR_NULL;
    { const int rc_dev = on_plan_device(plan); if (rc_dev) return rc_dev; }
    if (err && (n_workers < 1 || n_workers > plan->max_workers ||
                (n_workers > 1 && (state_stride < plan->L.d || state_stride % 4))))
        return EF_ERR_ARG;
    if ((err && !aligned(err, 16)) || (server_err && !aligned(server_err, 16))) return EF_ERR_ALIGN;
    // other buffers than the ones that wait for their correction: refuse rather than corrupt them
    if (err && plan->lazy_buf[0] && (plan->lazy_buf[0] != err || plan->lazy_stride_seen != state_stride)) return EF_ERR_ARG;
    if (server_err && plan->lazy_buf[1] && plan->lazy_buf[1] != server_err) return EF_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int role = 0; role < 2; ++role) {
        float *buf = role == 0 ? err : server_err;
        if (!buf) continue;
        if (role == 1) {
            plan->lazy_buf[1] = nullptr;
        } else if (n_workers >= plan->lazy_sets_seen) {
            plan->lazy_buf[0] = nullptr;
            plan->lazy_sets_seen = 0;
        }
        const ef_plan::Role &r = plan->role[role == 0 ? ROLE_TILES : ROLE_SERVER];
        const int nsets = role == 0 ? n_workers : 1;
        const CallScratch c = next_call(plan, role == 0 ? 0 : plan->max_workers, nsets);
        if (r.n_lazy_tiles) {
            hipLaunchKernelGGL(ef::k_flush, dim3(r.n_lazy_tiles, (unsigned)nsets), dim3(ef::THREADS), 0, s,
                               role_layout(plan, role == 0 ? ROLE_TILES : ROLE_SERVER), c.X, (const int32_t *)r.d_lazy_tiles, (int)r.n_lazy_tiles, buf,
                               role == 0 ? state_stride : (int64_t)0);
            EF_HIP(hipGetLastError());
        }
        hipLaunchKernelGGL(ef::k_flush_done, dim3(1), dim3(64), 0, s, plan->d_state, c.X.set_base, nsets);
        EF_HIP(hipGetLastError());
    }
    return EF_OK;
}

int ef_plan_tune(ef_plan *plan, int fuse_limit, int spin_limit)
{
    if (!plan) return EF_ERR_NULL;
    if (spin_limit >= 0) plan->spin_limit = spin_limit;
    if (fuse_limit >= 0) {
        bool pending = false;
        int rc = residuals_pending(plan, &pending);
        if (rc) return rc;
        if (pending) return EF_ERR_ARG;
        plan->user_fuse_limit = fuse_limit;
        return refresh_limits(plan);
    }
    return EF_OK;
}

int ef_plan_fuse_limit(const ef_plan *plan)
{
    if (!plan) return 0;
    return plan->role[worker_role(plan, true)].fuse_limit;
}
int ef_plan_is_persistent(const ef_plan *plan)
{
    if (!plan) return 0;
    return plan->lazy ? (plan->persistent && plan->persistent_forced) : plan->persistent;
}

int ef_plan_last_fallbacks(ef_plan *plan, unsigned int *parked_tiles, unsigned int *late_blocks)
{
    if (!plan) return EF_ERR_NULL;
    EF_HIP(hipDeviceSynchronize());
    unsigned int a = 0, b = 0;
    ef::CallState st;
    EF_HIP(hipMemcpy(&st, plan->d_state, sizeof st, hipMemcpyDeviceToHost));
    if (st.calls > 0) {         // the most recent call used the counters of parity (calls - 1) & 1
        const unsigned last = (st.calls - 1u) & 1u;
        EF_HIP(hipMemcpy(&a, plan->d_list_cnt + last, sizeof a, hipMemcpyDeviceToHost));
        EF_HIP(hipMemcpy(&b, plan->d_list_cnt + 2 + last, sizeof b, hipMemcpyDeviceToHost));
    }
    if (parked_tiles) *parked_tiles = a;
    if (late_blocks) *late_blocks = b;
    return EF_OK;
}

int ef_plan_set_persistent(ef_plan *plan, int on)
{
    if (!plan) return EF_ERR_NULL;
    bool pending = false;
    int rc = residuals_pending(plan, &pending);
    if (rc) return rc;
    if (pending) return EF_ERR_ARG;
    plan->persistent = on < 0 ? plan->persistent_auto : (on ? 1 : 0);
    plan->persistent_forced = on > 0 ? 1 : 0;
    return refresh_limits(plan);
}

int64_t ef_plan_d(const ef_plan *plan) { return plan ? plan->L.d : 0; }
int64_t ef_plan_blocks(const ef_plan *plan) { return plan ? plan->L.B : 0; }

int ef_worker_step(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride, float *mom,
                   float *err, int64_t state_stride, float mu, float eta_prev, float eta,
                   uint64_t *packed_signs, float *scales, void *stream)
{
    if (!plan || !mom) return EF_ERR_NULL;
    return worker_step_impl(plan, n_workers, grad, grad_stride, mom, err, state_stride, mu, eta_prev, eta,
                            packed_signs, plan->L.W, scales, plan->L.B, stream);
}

int ef_worker_step_quality(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride, float *mom,
                           float *err, int64_t state_stride, float mu, float eta_prev, float eta,
                           uint64_t *packed_signs, float *scales, double *quality, void *stream)
{
    if (!plan || !mom || !quality) return EF_ERR_NULL;
    return worker_step_impl(plan, n_workers, grad, grad_stride, mom, err, state_stride, mu, eta_prev, eta,
                            packed_signs, plan->L.W, scales, plan->L.B, stream, quality);
}

int ef_worker_step_sgd(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride, float *err,
                       int64_t state_stride, float eta_prev, float eta, uint64_t *packed_signs, float *scales,
                       void *stream)
{
    if (!plan) return EF_ERR_NULL;
    return worker_step_impl(plan, n_workers, grad, grad_stride, nullptr, err, state_stride, 0.0f, eta_prev, eta,
                            packed_signs, plan->L.W, scales, plan->L.B, stream);
}

size_t ef_payload_bytes(const ef_plan *plan) { return plan ? payload_bytes(plan) : 0; }
size_t ef_payload_scales_offset(const ef_plan *plan) { return plan ? (size_t)plan->L.W * 8u : 0; }

int ef_worker_step_fused(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride, float *mom,
                         float *err, int64_t state_stride, float mu, float eta_prev, float eta, void *payloads,
                         void *stream)
{
    if (!plan || !payloads || !mom) return EF_ERR_NULL;
    if (!aligned(payloads, 16)) return EF_ERR_ALIGN;
    const size_t pb = payload_bytes(plan);
    char *base = static_cast<char *>(payloads);
    return worker_step_impl(plan, n_workers, grad, grad_stride, mom, err, state_stride, mu, eta_prev, eta,
                            reinterpret_cast<uint64_t *>(base), (int64_t)(pb / 8u),
                            reinterpret_cast<float *>(base + (size_t)plan->L.W * 8u), (int64_t)(pb / 4u), stream);
}

int ef_server_step_fused(const ef_plan *plan, int M, const void *payloads, float *server_err, float eta_prev,
                         float eta, void *out_payload, void *stream)
{
    if (!plan || !payloads || !out_payload) return EF_ERR_NULL;
    if (!aligned(payloads, 16) || !aligned(out_payload, 16)) return EF_ERR_ALIGN;
    const size_t pb = payload_bytes(plan), so = (size_t)plan->L.W * 8u;
    if (M >= 1) {  // the output message may not overlap any input message
        const char *in0 = static_cast<const char *>(payloads), *o = static_cast<const char *>(out_payload);
        if (o < in0 + pb * (size_t)M && in0 < o + pb) return EF_ERR_ARG;
    }
    const char *in = static_cast<const char *>(payloads);
    char *out = static_cast<char *>(out_payload);
    return server_step_impl(plan, M, reinterpret_cast<const uint64_t *>(in), (int64_t)(pb / 8u),
                            reinterpret_cast<const float *>(in + so), (int64_t)(pb / 4u), server_err, eta_prev, eta,
                            reinterpret_cast<uint64_t *>(out), reinterpret_cast<float *>(out + so), stream);
}

int ef_apply_fused(const ef_plan *plan, float *params, const void *payload, float eta, void *stream)
{
    if (!plan || !payload) return EF_ERR_NULL;
    if (!aligned(payload, 16)) return EF_ERR_ALIGN;
    const char *in = static_cast<const char *>(payload);
    return ef_apply(plan, params, reinterpret_cast<const uint64_t *>(in),
                    reinterpret_cast<const float *>(in + (size_t)plan->L.W * 8u), eta, stream);
}

}  // extern "C"

namespace {

int worker_step_impl(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride, float *mom,
                     float *err, int64_t state_stride, float mu, float eta_prev, float eta, uint64_t *packed_signs,
                     int64_t signs_stride, float *scales, int64_t scales_stride, void *stream, double *quality)
{
    // mom == nullptr selects Algorithm 3 (callers of the momentum entry points have checked theirs)
    const bool has_mom = mom != nullptr;
    if (!plan || !grad || !err || !packed_signs || !scales) return EF_ERR_NULL;
    { const int rc_dev = on_plan_device(plan); if (rc_dev) return rc_dev; }
    if (n_workers < 1 || n_workers > plan->max_workers) return EF_ERR_ARG;
    if (!(mu >= 0.0f && mu < 1.0f) || !good_eta(eta_prev, eta)) return EF_ERR_ARG;
    // with one worker the strides are never used
    if (n_workers > 1 && (grad_stride < plan->L.d || state_stride < plan->L.d || grad_stride % 4 || state_stride % 4))
        return EF_ERR_ARG;
    {
        // in-place aliasing is the contract for mom and err only: nothing else may overlap
        const int64_t d = plan->L.d;
        const size_t g_bytes = span_bytes(n_workers, grad_stride, d, 4), s_bytes = span_bytes(n_workers, state_stride, d, 4);
        const size_t w_bytes = span_bytes(n_workers, signs_stride, plan->L.W, 8);
        const size_t c_bytes = span_bytes(n_workers, scales_stride, plan->L.B, 4);
        if (overlap(grad, g_bytes, err, s_bytes) || (has_mom && (overlap(grad, g_bytes, mom, s_bytes) ||
                                                                 overlap(mom, s_bytes, err, s_bytes))))
            return EF_ERR_ARG;
        const void *in[3] = {grad, err, mom};
        const size_t in_bytes[3] = {g_bytes, s_bytes, s_bytes};
        for (int k = 0; k < (has_mom ? 3 : 2); ++k)
            if (overlap(packed_signs, w_bytes, in[k], in_bytes[k]) || overlap(scales, c_bytes, in[k], in_bytes[k]))
                return EF_ERR_ARG;
    }
    if (!aligned(grad, 16) || (has_mom && !aligned(mom, 16)) || !aligned(err, 16) || !aligned(scales, 4) ||
        !aligned(packed_signs, 8))
        return EF_ERR_ALIGN;
    ef::WorkerArgs A;
    A.grad = grad;
    A.grad_stride = grad_stride;
    A.mom = mom;
    A.err = err;
    A.state_stride = state_stride;
    A.mu = mu;
    A.r = eta_prev / eta;
    A.signs = packed_signs;
    A.scales = scales;
    A.signs_stride = signs_stride;
    A.scales_stride = scales_stride;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->lazy) {
        if (plan->lazy_buf[0] && (plan->lazy_buf[0] != err || plan->lazy_stride_seen != state_stride)) return EF_ERR_ARG;
        plan->lazy_buf[0] = err;
        plan->lazy_stride_seen = state_stride;
        if (n_workers > plan->lazy_sets_seen) plan->lazy_sets_seen = n_workers;
    }
    const CallScratch c = next_call(plan, 0, n_workers);
    const int role = quality ? (int)ROLE_TILES : worker_role(plan, has_mom);
    const ef::Layout L = role_layout(plan, role);
    if (quality) {
        if (!aligned(quality, 8)) return EF_ERR_ALIGN;
        hipLaunchKernelGGL(ef::k_quality_init, dim3(1), dim3(ef::THREADS), 0, s, quality, n_workers);
        EF_HIP(hipGetLastError());
    }
    if (role == ROLE_TICKET) {
        // the mixed tiles first, in a kernel of their own, then the persistent kernel
        if (plan->L.n_mixed) {
            const dim3 grid((unsigned)plan->L.n_mixed, (unsigned)n_workers);
            if (has_mom)
                hipLaunchKernelGGL(ef::k_worker_mixed<true>, grid, dim3(ef::THREADS), 0, s, L, c.X, A);
            else
                hipLaunchKernelGGL(ef::k_worker_mixed<false>, grid, dim3(ef::THREADS), 0, s, L, c.X, A);
            EF_HIP(hipGetLastError());
        }
        int64_t wgs = (int64_t)plan->L.n_uniform * n_workers;
        if (wgs > plan->worker_grid) wgs = plan->worker_grid;
        const dim3 grid((unsigned)wgs), block(ef::THREADS);
        if (has_mom)
            hipLaunchKernelGGL(ef::k_worker_uniform<true>, grid, block, 0, s, L, c.X, A, n_workers);
        else
            hipLaunchKernelGGL(ef::k_worker_uniform<false>, grid, block, 0, s, L, c.X, A, n_workers);
        EF_HIP(hipGetLastError());
    } else {
        // every tile in one launch, the mixed tiles first
        const dim3 grid((unsigned)plan->L.ntiles, (unsigned)n_workers), block(ef::THREADS);
        const bool mixed = plan->L.n_mixed != 0;
        ef::QualityArgs Q;
        Q.v = nullptr;
        Q.stride = 0;
        Q.tile_sums = plan->d_qtile;
        Q.part_sums = plan->d_qpart;
        Q.out = quality;
        if (quality && has_mom)
            hipLaunchKernelGGL((ef::k_worker_tiles<true, true, true>), grid, block, 0, s, L, c.X, A, Q);
        else if (quality)
            hipLaunchKernelGGL((ef::k_worker_tiles<false, true, true>), grid, block, 0, s, L, c.X, A, Q);
        else if (has_mom && mixed)
            hipLaunchKernelGGL((ef::k_worker_tiles<true, true, false>), grid, block, 0, s, L, c.X, A, Q);
        else if (has_mom)
            hipLaunchKernelGGL((ef::k_worker_tiles<true, false, false>), grid, block, 0, s, L, c.X, A, Q);
        else if (mixed)
            hipLaunchKernelGGL((ef::k_worker_tiles<false, true, false>), grid, block, 0, s, L, c.X, A, Q);
        else
            hipLaunchKernelGGL((ef::k_worker_tiles<false, false, false>), grid, block, 0, s, L, c.X, A, Q);
        EF_HIP(hipGetLastError());
    }
    int rc = launch_tail(plan, role, c, n_workers, err, state_stride, scales, scales_stride, s);
    if (rc || !quality) return rc;
    // the quality sums of the tiles are there: combine them per block and per vector
    ef::QualityArgs Q;
    Q.v = nullptr;
    Q.stride = 0;
    Q.tile_sums = plan->d_qtile;
    Q.part_sums = plan->d_qpart;
    Q.out = quality;
    hipLaunchKernelGGL(ef::k_quality_blocks, dim3((unsigned)plan->n_cross + 1u, (unsigned)n_workers), dim3(ef::THREADS), 0,
                       s, plan->L, Q, (const int32_t *)plan->d_cross, (int)plan->n_cross);
    EF_HIP(hipGetLastError());
    return EF_OK;
}

int server_step_impl(const ef_plan *plan, int M, const uint64_t *packed_signs, int64_t in_signs_stride,
                     const float *scales, int64_t in_scales_stride, float *server_err, float eta_prev, float eta,
                     uint64_t *out_signs, float *out_scales, void *stream)
{
    if (!plan || !packed_signs || !scales || !server_err || !out_signs || !out_scales) return EF_ERR_NULL;
    { const int rc_dev = on_plan_device(plan); if (rc_dev) return rc_dev; }
    if (M < 1 || M > plan->max_workers) return EF_ERR_ARG;
    if (!good_eta(eta_prev, eta)) return EF_ERR_ARG;
    {
        // the server residual is updated in place; the payloads may overlap neither it nor each other
        const size_t in_w = span_bytes(M, in_signs_stride, plan->L.W, 8), in_c = span_bytes(M, in_scales_stride, plan->L.B, 4);
        const size_t out_w = (size_t)plan->L.W * 8u, out_c = (size_t)plan->L.B * 4u, e_bytes = (size_t)plan->L.d * 4u;
        if (overlap(out_signs, out_w, packed_signs, in_w) || overlap(out_signs, out_w, scales, in_c) ||
            overlap(out_scales, out_c, packed_signs, in_w) || overlap(out_scales, out_c, scales, in_c) ||
            overlap(out_signs, out_w, out_scales, out_c))
            return EF_ERR_ARG;
        if (overlap(server_err, e_bytes, packed_signs, in_w) || overlap(server_err, e_bytes, scales, in_c) ||
            overlap(server_err, e_bytes, out_signs, out_w) || overlap(server_err, e_bytes, out_scales, out_c))
            return EF_ERR_ARG;
    }
    if (!aligned(server_err, 16) || !aligned(packed_signs, 8) || !aligned(out_signs, 8) ||
        !aligned(scales, 4) || !aligned(out_scales, 4))
        return EF_ERR_ALIGN;
    ef::ServerArgs A;
    A.M = M;
    A.signs_in = packed_signs;
    A.scales_in = scales;
    A.in_signs_stride = in_signs_stride;
    A.in_scales_stride = in_scales_stride;
    A.err = server_err;
    A.r = eta_prev / eta;
    A.Mf = (float)M;
    A.Minv = (M & (M - 1)) == 0 ? 1.0f / (float)M : 0.0f;
    A.signs = out_signs;
    A.scales = out_scales;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->lazy) {
        if (plan->lazy_buf[1] && plan->lazy_buf[1] != server_err) return EF_ERR_ARG;
        plan->lazy_buf[1] = server_err;
    }
    const CallScratch c = next_call(plan, plan->max_workers, 1);
    const ef::Layout L = role_layout(plan, ROLE_SERVER);
    if (L.n_mixed)
        hipLaunchKernelGGL(ef::k_server_tiles<true>, dim3((unsigned)L.ntiles), dim3(ef::THREADS), 0, s, L, c.X, A,
                           plan->max_workers);
    else
        hipLaunchKernelGGL(ef::k_server_tiles<false>, dim3((unsigned)L.ntiles), dim3(ef::THREADS), 0, s, L, c.X, A,
                           plan->max_workers);
    EF_HIP(hipGetLastError());
    return launch_tail(plan, ROLE_SERVER, c, 1, server_err, (int64_t)0, out_scales, (int64_t)0, s);
}

}  // namespace

extern "C" {

int ef_server_step(const ef_plan *plan, int M, const uint64_t *packed_signs, const float *scales,
                   float *server_err, float eta_prev, float eta, uint64_t *out_signs, float *out_scales,
                   void *stream)
{
    if (!plan) return EF_ERR_NULL;
    return server_step_impl(plan, M, packed_signs, plan->L.W, scales, plan->L.B, server_err, eta_prev, eta,
                            out_signs, out_scales, stream);
}

int ef_apply(const ef_plan *plan, float *params, const uint64_t *packed_signs, const float *scales, float eta,
             void *stream)
{
    if (!plan || !params || !packed_signs || !scales) return EF_ERR_NULL;
    { const int rc_dev = on_plan_device(plan); if (rc_dev) return rc_dev; }
    if (!(std::isfinite(eta) && eta > 0.0f)) return EF_ERR_ARG;
    if (!aligned(params, 16) || !aligned(packed_signs, 8) || !aligned(scales, 4)) return EF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    dim3 grid((unsigned)plan->L.ntiles, 1u);
    hipLaunchKernelGGL(ef::k_apply, grid, dim3(ef::THREADS), 0, s, plan->L, params, packed_signs, scales, eta);
    EF_HIP(hipGetLastError());
    return EF_OK;
}

int ef_apply_wd(const ef_plan *plan, float *params, float *decay_mom, const uint64_t *packed_signs,
                const float *scales, float eta, float mu, float lambda, void *stream)
{
    if (!plan || !params || !decay_mom || !packed_signs || !scales) return EF_ERR_NULL;
    { const int rc_dev = on_plan_device(plan); if (rc_dev) return rc_dev; }
    if (!(std::isfinite(eta) && eta > 0.0f)) return EF_ERR_ARG;
    if (!(mu >= 0.0f && mu < 1.0f)) return EF_ERR_ARG;
    if (!(std::isfinite(lambda) && lambda >= 0.0f)) return EF_ERR_ARG;
    if (!aligned(params, 16) || !aligned(decay_mom, 16) || !aligned(packed_signs, 8) || !aligned(scales, 4))
        return EF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    dim3 grid((unsigned)plan->L.ntiles, 1u);
    hipLaunchKernelGGL(ef::k_apply_wd, grid, dim3(ef::THREADS), 0, s, plan->L, params, decay_mom, packed_signs,
                       scales, eta, mu, lambda);
    EF_HIP(hipGetLastError());
    return EF_OK;
}

static int quality_launch(const ef_plan *plan, int n_vectors, const float *v, int64_t stride, double *out,
                          double *tile_sums, double *part_sums, hipStream_t s)
{
    ef::QualityArgs Q;
    Q.v = v;
    Q.stride = stride;
    Q.tile_sums = tile_sums;
    Q.part_sums = part_sums;
    Q.out = out;
    hipLaunchKernelGGL(ef::k_quality_init, dim3(1), dim3(ef::THREADS), 0, s, out, n_vectors);
    EF_HIP(hipGetLastError());
    hipLaunchKernelGGL(ef::k_quality_tiles, dim3((unsigned)plan->L.ntiles, (unsigned)n_vectors), dim3(ef::THREADS), 0,
                       s, plan->L, Q);
    EF_HIP(hipGetLastError());
    hipLaunchKernelGGL(ef::k_quality_blocks, dim3((unsigned)plan->n_cross + 1u, (unsigned)n_vectors),
                       dim3(ef::THREADS), 0, s, plan->L, Q, (const int32_t *)plan->d_cross, (int)plan->n_cross);
    EF_HIP(hipGetLastError());
    return EF_OK;
}

static int quality_args(const ef_plan *plan, int n_vectors, const float *v, int64_t stride, const double *out)
{
    if (!plan || !v || !out) return EF_ERR_NULL;
    { const int rc_dev = on_plan_device(plan); if (rc_dev) return rc_dev; }
    if (n_vectors < 1 || n_vectors > plan->max_workers) return EF_ERR_ARG;
    if (n_vectors > 1 && (stride < plan->L.d || stride % 4)) return EF_ERR_ARG;
    if (!aligned(v, 16) || !aligned(out, 8)) return EF_ERR_ALIGN;
    return EF_OK;
}

int ef_compressor_quality(ef_plan *plan, int n_vectors, const float *v, int64_t stride, double *out, void *stream)
{
    const int rc = quality_args(plan, n_vectors, v, stride, out);
    if (rc) return rc;
    return quality_launch(plan, n_vectors, v, stride, out, plan->d_qtile, plan->d_qpart, static_cast<hipStream_t>(stream));
}

int ef_compressor_quality_static(const ef_plan *plan, int n_vectors, const float *v, int64_t stride, double *out,
                                 void *stream)
{
    int rc = quality_args(plan, n_vectors, v, stride, out);
    if (rc) return rc;
    const int64_t tile_vectors = (int64_t)plan->L.ntiles * n_vectors;
    if (tile_vectors > (int64_t)EF_QUALITY_STATIC_MAX_TILE_VECTORS) return EF_ERR_SIZE;
    double *base = nullptr;
    rc = static_scratch(plan->device, &base);      // quality_args has checked that the plan's device is current
    if (rc) return rc;
    // [n][ntiles][2] tile sums, then [n][2*ntiles][2] sums of open segments; every word the kernels read
    // is written earlier in the same call, so nothing has to be cleared
    return quality_launch(plan, n_vectors, v, stride, out, base, base + 2 * tile_vectors, static_cast<hipStream_t>(stream));
}

int ef_state_create(ef_plan *plan, int n_workers, ef_state **out, void *stream)
{
    if (!plan || !out) return EF_ERR_NULL;
    *out = nullptr;
    if (n_workers < 1 || n_workers > plan->max_workers || plan->state) return EF_ERR_ARG;
    { const int rc_dev = on_plan_device(plan); if (rc_dev) return rc_dev; }
    int rc = set_lazy(plan, 1);             // refused (EF_ERR_ARG) while caller-owned buffers wait for a correction
    if (rc) return rc;
    ef_state *st = new (std::nothrow) ef_state();
    if (!st) return EF_ERR_ARG;
    st->plan = plan;
    st->n_workers = n_workers;
    st->stride = (plan->L.d + 3) / 4 * 4;
    st->mom = st->err = st->server_err = nullptr;
    const size_t rows = sizeof(float) * (size_t)st->stride * (size_t)n_workers, one = sizeof(float) * (size_t)plan->L.d;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipMalloc(&st->mom, rows);
    if (e == hipSuccess) e = hipMalloc(&st->err, rows);
    if (e == hipSuccess) e = hipMalloc(&st->server_err, one);
    // m_0 = e_0 = e~_0 = 0 (Algorithm 4, input line)
    if (e == hipSuccess) e = hipMemsetAsync(st->mom, 0, rows, s);
    if (e == hipSuccess) e = hipMemsetAsync(st->err, 0, rows, s);
    if (e == hipSuccess) e = hipMemsetAsync(st->server_err, 0, one, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        if (st->mom) (void)hipFree(st->mom);
        if (st->err) (void)hipFree(st->err);
        if (st->server_err) (void)hipFree(st->server_err);
        delete st;
        (void)set_lazy(plan, 0);
        return hip_fail(e);
    }
    plan->state = st;
    *out = st;
    return EF_OK;
}

int ef_state_destroy(ef_state *state)
{
    if (!state) return EF_ERR_NULL;
    ef_plan *plan = state->plan;
    (void)hipDeviceSynchronize();
    (void)hipFree(state->mom);
    (void)hipFree(state->err);
    (void)hipFree(state->server_err);
    plan->state = nullptr;
    delete state;
    // the buffers that waited for a correction are gone: clear the marks, leave the mode
    hipLaunchKernelGGL(ef::k_flush_done, dim3(1), dim3(64), 0, nullptr, plan->d_state, 0, plan->max_workers);
    hipLaunchKernelGGL(ef::k_flush_done, dim3(1), dim3(64), 0, nullptr, plan->d_state, plan->max_workers, 1);
    EF_HIP(hipGetLastError());
    plan->lazy_buf[0] = plan->lazy_buf[1] = nullptr;
    plan->lazy_sets_seen = 0;
    return set_lazy(plan, 0);
}

int ef_worker_step_state(const ef_plan *plan, ef_state *state, const float *grad, int64_t grad_stride, float mu,
                         float eta_prev, float eta, uint64_t *packed_signs, float *scales, void *stream)
{
    if (!plan || !state) return EF_ERR_NULL;
    if (state->plan != plan) return EF_ERR_ARG;
    return worker_step_impl(plan, state->n_workers, grad, grad_stride, state->mom, state->err, state->stride, mu,
                            eta_prev, eta, packed_signs, plan->L.W, scales, plan->L.B, stream);
}

int ef_server_step_state(const ef_plan *plan, ef_state *state, int M, const uint64_t *packed_signs, const float *scales,
                         float eta_prev, float eta, uint64_t *out_signs, float *out_scales, void *stream)
{
    if (!plan || !state) return EF_ERR_NULL;
    if (state->plan != plan) return EF_ERR_ARG;
    return server_step_impl(plan, M, packed_signs, plan->L.W, scales, plan->L.B, state->server_err, eta_prev, eta,
                            out_signs, out_scales, stream);
}

// Copies between the library-held state and caller buffers, row by row (the strides may differ).
static int copy_state(const ef_plan *plan, ef_state *state, float *mom, float *err, int64_t state_stride,
                      float *server_err, bool to_caller, hipStream_t s)
{
    const size_t row = sizeof(float) * (size_t)plan->L.d;
    const size_t mine = sizeof(float) * (size_t)state->stride, theirs = sizeof(float) * (size_t)state_stride;
    float *pairs[2][2] = {{state->mom, mom}, {state->err, err}};
    for (auto &pr : pairs) {
        if (!pr[1]) continue;
        if (to_caller)
            EF_HIP(hipMemcpy2DAsync(pr[1], theirs, pr[0], mine, row, (size_t)state->n_workers, hipMemcpyDeviceToDevice, s));
        else
            EF_HIP(hipMemcpy2DAsync(pr[0], mine, pr[1], theirs, row, (size_t)state->n_workers, hipMemcpyDeviceToDevice, s));
    }
    if (server_err) {
        if (to_caller)
            EF_HIP(hipMemcpyAsync(server_err, state->server_err, row, hipMemcpyDeviceToDevice, s));
        else
            EF_HIP(hipMemcpyAsync(state->server_err, server_err, row, hipMemcpyDeviceToDevice, s));
    }
    return EF_OK;
}

static int state_copy_args(const ef_plan *plan, const ef_state *state, const float *mom, const float *err,
                           int64_t state_stride, const float *server_err)
{
    if (!plan || !state) return EF_ERR_NULL;
    if (state->plan != plan) return EF_ERR_ARG;
    { const int rc_dev = on_plan_device(plan); if (rc_dev) return rc_dev; }
    if ((mom || err) && state->n_workers > 1 && state_stride < plan->L.d) return EF_ERR_ARG;
    if ((mom && !aligned(mom, 4)) || (err && !aligned(err, 4)) || (server_err && !aligned(server_err, 4))) return EF_ERR_ALIGN;
    return EF_OK;
}

int ef_state_export(const ef_plan *plan, ef_state *state, float *mom, float *err, int64_t state_stride,
                    float *server_err, void *stream)
{
    int rc = state_copy_args(plan, state, mom, err, state_stride, server_err);
    if (rc) return rc;
    // write the corrections that are still waiting, then the buffers hold m, e and e~ of Algorithm 4
    rc = ef_flush(plan, state->n_workers, state->err, state->stride, state->server_err, stream);
    if (rc) return rc;
    return copy_state(plan, state, mom, err, state_stride, server_err, true, static_cast<hipStream_t>(stream));
}

int ef_state_import(const ef_plan *plan, ef_state *state, const float *mom, const float *err, int64_t state_stride,
                    const float *server_err, void *stream)
{
    int rc = state_copy_args(plan, state, mom, err, state_stride, server_err);
    if (rc) return rc;
    // what is brought in is finished state: no correction may be left waiting for the buffers it replaces
    rc = ef_flush(plan, state->n_workers, err ? state->err : nullptr, state->stride, server_err ? state->server_err : nullptr,
                  stream);
    if (rc) return rc;
    return copy_state(plan, state, const_cast<float *>(mom), const_cast<float *>(err), state_stride,
                      const_cast<float *>(server_err), false, static_cast<hipStream_t>(stream));
}

const char *ef_strerror(int code)
{
    const char *t;
    switch (code) {
    case EF_OK: t = "ok"; break;
    case EF_ERR_NULL: t = "a required pointer is NULL"; break;
    case EF_ERR_OFFSETS: t = "block_offsets is not a partition (0 = o[0] < o[1] < ... < o[B] = d)"; break;
    case EF_ERR_ARG: t = "argument out of range"; break;
    case EF_ERR_ALIGN: t = "pointer not aligned (fp32 arrays 16 bytes, sign words 8 bytes)"; break;
    case EF_ERR_SIZE:
        t = "input too large for the static scratch of ef_compressor_quality_static (tiles x vectors above "
            "EF_QUALITY_STATIC_MAX_TILE_VECTORS): use ef_compressor_quality";
        break;
    case EF_ERR_HIP:
        snprintf(g_errbuf, sizeof g_errbuf, "HIP runtime error: %s", hipGetErrorString(g_last_hip));
        return g_errbuf;
    default: t = "unknown error code"; break;
    }
    snprintf(g_errbuf, sizeof g_errbuf, "%s", t);
    return g_errbuf;
}

}  // extern "C"
