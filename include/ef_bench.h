/*
 * ef_bench.h -- C ABI of libef_bench: bandwidth probes that bench.py runs
 * beside the library.  Measurement aids, not part of Algorithm 4 and not part
 * of libef: they allocate, create events and synchronise, which no entry point
 * of libef does after plan creation.  Error codes are those of ef.h.
 */
#ifndef EF_BENCH_H
#define EF_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement aid, not part of Algorithm 4: streams the worker step's memory
 * traffic with nothing else in it.  For every whole 4096-element tile of
 * g, m, e (device, >= n_elements floats each, 16-byte aligned, distinct) it
 * reads all three and writes m and e, 20 bytes per element, with the worker
 * kernel's loads, stores, tile shape and ticket order, but no compression and
 * no waiting; m and e hold garbage afterwards.  Runs one warm-up pass and
 * `repeats` (1..1000) timed passes on `stream`, waits for them, and stores
 * the mean time of a pass in *ms_per_pass (host): 20 * (n_elements rounded
 * down to whole tiles) bytes / that time is the practical ceiling of this
 * access pattern on the machine, to set beside ef_worker_step's rate.
 * Allocates a counter and two events for the duration of the call.
 * EF_ERR_ARG for fewer than 4096 elements or repeats out of range.
 */
int ef_stream_probe(const float *g, float *m, float *e, int64_t n_elements, int repeats, float *ms_per_pass,
                    void *stream);

/*
 * The same traffic as ef_stream_probe with one workgroup per tile in grid
 * order and the third array written in step: the workgroups of `group`
 * consecutive tiles (0..256; 0 or 1: no waiting) write m at once, wait
 * (bounded) until all of them have loaded their tile, and then write e.  This
 * is how the worker kernel's one-pass blocks and its sync groups
 * (ef_plan_set_sync_group) access memory, without the compression: the
 * ceiling of that pattern.  Arguments, result and errors as for
 * ef_stream_probe; allocates 132 bytes per tile for the duration of the call.
 */
int ef_stream_probe_grouped(const float *g, float *m, float *e, int64_t n_elements, int group, int repeats,
                            float *ms_per_pass, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EF_BENCH_H */
