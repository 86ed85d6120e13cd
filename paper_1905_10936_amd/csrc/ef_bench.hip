// libef_bench: the bandwidth probes declared in include/ef_bench.h.  A library of its own, so that
// libef itself holds nothing that allocates, times or synchronises after plan creation.
#include "ef.h"
#include "ef_bench.h"
#include "ef_probe.h"

namespace {
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
}  // namespace

extern "C" {

int ef_stream_probe(const float *g, float *m, float *e, int64_t n_elements, int repeats, float *ms_per_pass, void *stream)
{
    if (!g || !m || !e || !ms_per_pass) return EF_ERR_NULL;
    if (n_elements < ef::TILE || n_elements / ef::TILE > 0x7fffffffll || repeats < 1 || repeats > 1000) return EF_ERR_ARG;
    if (!aligned(g, 16) || !aligned(m, 16) || !aligned(e, 16)) return EF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned n_tiles = (unsigned)(n_elements / ef::TILE);
    hipDeviceProp_t prop;
    int dev = 0, occ = 0;
    if (hipGetDevice(&dev) != hipSuccess) return EF_ERR_HIP;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return EF_ERR_HIP;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, ef::k_probe_stream, ef::THREADS, 0) != hipSuccess) return EF_ERR_HIP;
    if (occ < 1) occ = 1;
    unsigned grid = (unsigned)prop.multiProcessorCount * (unsigned)occ;
    if (grid > n_tiles) grid = n_tiles;
    unsigned int *ticket = nullptr;
    hipEvent_t t0 = nullptr, t1 = nullptr;
    int rc = EF_OK;
    float ms = 0.f;
    auto pass = [&]() {
        hipLaunchKernelGGL(ef::k_probe_reset, dim3(1), dim3(64), 0, s, ticket);
        hipLaunchKernelGGL(ef::k_probe_stream, dim3(grid), dim3(ef::THREADS), 0, s, g, m, e, n_tiles, ticket);
    };
    if (hipMalloc(&ticket, sizeof(unsigned int)) != hipSuccess || hipEventCreate(&t0) != hipSuccess ||
        hipEventCreate(&t1) != hipSuccess) {
        rc = EF_ERR_HIP;
    } else {
        pass();                                     // warm-up
        bool ok = hipEventRecord(t0, s) == hipSuccess;
        for (int r = 0; r < repeats; ++r) pass();
        ok = ok && hipEventRecord(t1, s) == hipSuccess && hipEventSynchronize(t1) == hipSuccess &&
             hipEventElapsedTime(&ms, t0, t1) == hipSuccess && hipGetLastError() == hipSuccess;
        if (ok)
            *ms_per_pass = ms / (float)repeats;
        else
            rc = EF_ERR_HIP;
    }
    if (t0) (void)hipEventDestroy(t0);
    if (t1) (void)hipEventDestroy(t1);
    if (ticket) (void)hipFree(ticket);
    return rc;
}

int ef_stream_probe_grouped(const float *g, float *m, float *e, int64_t n_elements, int group, int repeats,
                            float *ms_per_pass, void *stream)
{
    if (!g || !m || !e || !ms_per_pass) return EF_ERR_NULL;
    if (n_elements < ef::TILE || n_elements / ef::TILE > 0x7fffffffll || repeats < 1 || repeats > 1000 || group < 0 ||
        group > 256)
        return EF_ERR_ARG;
    if (!aligned(g, 16) || !aligned(m, 16) || !aligned(e, 16)) return EF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned n_tiles = (unsigned)(n_elements / ef::TILE);
    unsigned int *arrive = nullptr;
    unsigned long long *line = nullptr;
    hipEvent_t t0 = nullptr, t1 = nullptr;
    int rc = EF_OK;
    float ms = 0.f;
    unsigned pass = 0;
    auto run = [&]() {
        ++pass;         // never 0, the value of the cleared words
        hipLaunchKernelGGL(ef::k_probe_grouped, dim3(n_tiles), dim3(ef::THREADS), 0, s, g, m, e, n_tiles, group, pass,
                           arrive, line, 1 << 14);
    };
    const size_t line_bytes = sizeof(unsigned long long) * ef::READY_STRIDE * (size_t)n_tiles;
    if (hipMalloc(&arrive, sizeof(unsigned int) * (size_t)n_tiles) != hipSuccess ||
        hipMalloc(&line, line_bytes) != hipSuccess || hipEventCreate(&t0) != hipSuccess ||
        hipEventCreate(&t1) != hipSuccess ||
        hipMemsetAsync(arrive, 0, sizeof(unsigned int) * (size_t)n_tiles, s) != hipSuccess ||
        hipMemsetAsync(line, 0, line_bytes, s) != hipSuccess) {
        rc = EF_ERR_HIP;
    } else {
        run();                                      // warm-up
        bool ok = hipEventRecord(t0, s) == hipSuccess;
        for (int r = 0; r < repeats; ++r) run();
        ok = ok && hipEventRecord(t1, s) == hipSuccess && hipEventSynchronize(t1) == hipSuccess &&
             hipEventElapsedTime(&ms, t0, t1) == hipSuccess && hipGetLastError() == hipSuccess;
        if (ok)
            *ms_per_pass = ms / (float)repeats;
        else
            rc = EF_ERR_HIP;
    }
    if (t0) (void)hipEventDestroy(t0);
    if (t1) (void)hipEventDestroy(t1);
    if (arrive) (void)hipFree(arrive);
    if (line) (void)hipFree(line);
    return rc;
}

}  // extern "C"
