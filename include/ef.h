/*
 * ef.h -- C ABI of libef: the per-iteration hot path of dist-EF-blockSGDM
 * (Zheng, Huang, Kwok: "Communication-Efficient Distributed Blockwise Momentum
 * SGD with Error-Feedback", arxiv 1905.10936), hand-written HIP for gfx950.
 *
 * One training iteration t of Algorithm 4 is, for M workers on one GPU:
 *
 *     ef_worker_step   (all M workers in one call)   the per-worker part
 *     ef_server_step                                 the parameter-server part
 *     ef_apply                                       x_{t+1} = x_t - eta_t * Delta~_t
 *       (ef_apply_wd: the same update with weight decay, Appendix A)
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Pointers.  Unless a parameter is marked HOST, every pointer is a DEVICE
 *   pointer into memory owned by the caller.  The library neither frees nor
 *   retains caller memory beyond the call.  fp32 arrays must be 16-byte aligned,
 *   sign-word arrays 8-byte aligned (EF_ERR_ALIGN otherwise).
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = the default
 *   stream).  Calls enqueue work and return without synchronising.  All calls
 *   that share one plan must be ordered on the device (same stream, or ordered
 *   by events): the plan owns scratch memory that the kernels of a call use.
 *   Calls on different plans may overlap on the device; every wait inside the
 *   kernels is bounded, so kernels that compete for the compute units cannot
 *   hang each other (at worst some tiles take the two-pass route).
 *   What differs between two calls (call number, tags of the scratch) is kept
 *   in device memory and advanced by the last kernel of each call, and no call
 *   records a memset: ef_worker_step*, ef_server_step*, ef_apply* may be
 *   captured into a HIP graph and the graph replayed; replays and eager calls
 *   on one plan may be mixed as long as they are ordered on the device.
 * Block partition {G_1..G_B} (Section 3.2).  Block b is the contiguous index
 *   range [block_offsets[b], block_offsets[b+1]) of the flat d-vector;
 *   block_offsets[0] = 0, strictly increasing (every d_b >= 1, since d_b is a
 *   denominator), block_offsets[B] = d.
 * Payload (Section 3.2, Appendix A).  A compressed vector is
 *     packed_signs : uint64[W], W = ceil(d/64).  Flat index j lives in bit
 *                    (j mod 64) of word floor(j/64), least significant bit
 *                    first; bit = 1 encodes sign +1, bit = 0 encodes -1;
 *                    bits at positions >= d of the last word are written as 0.
 *     scales       : float[B], scales[b] = ||v_Gb||_1 / d_b.
 *   sign(0) is read as +1 (both +0 and -0 give bit 1).
 * Arithmetic.  fp32, round-to-nearest-even, one rounding per written operation,
 *   left to right, never fused.  The L1 norm of a block is accumulated in fp64
 *   and rounded once to fp32 after the division by d_b.  Non-finite inputs are
 *   outside the contract.
 * Errors.  Every int-returning function returns EF_OK (0) or a negative code;
 *   on error nothing has been enqueued unless the code is EF_ERR_HIP.
 */
#ifndef EF_H
#define EF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EF_OK 0
#define EF_ERR_NULL -1    /* a required pointer is NULL */
#define EF_ERR_OFFSETS -2 /* block_offsets is not a partition as described above */
#define EF_ERR_ARG -3     /* scalar out of range: M < 1 or > max_workers, mu not in [0,1),
                             eta <= 0, eta_prev < 0, non-finite, stride < d or not a multiple of 4 */
#define EF_ERR_ALIGN -4   /* pointer not aligned as required */
#define EF_ERR_HIP -5     /* the HIP runtime reported an error (allocation, launch, no device) */
#define EF_ERR_SIZE -6    /* input beyond the fixed capacity of an entry point that allocates nothing */

#define EF_MAX_WORKERS 64

typedef struct ef_plan ef_plan;   /* opaque */
typedef struct ef_state ef_state; /* opaque: optimizer state held by the library, see ef_state_create */

/*
 * Build the per-layout plan: a device copy of the partition, the tile -> block
 * table the kernels use to find which blocks a tile touches, and the scratch
 * memory of the cross-tile block reductions (fp64 partial sums per tile and one
 * hand-off word per block, for max_workers workers and the server).  Blocks
 * follow Section 3.2 (one block per parameter tensor is the usual choice).
 *
 *   out                 HOST  receives the plan; caller releases it with ef_plan_destroy
 *   block_offsets_host  HOST  int64[B+1], copied; need not outlive the call
 *   B                         number of blocks, >= 1
 *   max_workers               largest M / n_workers later calls may pass, 1..EF_MAX_WORKERS
 *   stream                    unused for ordering: creation synchronises
 *
 * Offsets are validated first (EF_ERR_OFFSETS) before any GPU call is made, so
 * the check also works on a host without a GPU.  Allocates device memory with
 * hipMalloc on the current device; the plan must be used on that device only:
 * every call that enqueues work on a plan returns EF_ERR_ARG if another device
 * is current.
 */
int ef_plan_create(ef_plan **out, const int64_t *block_offsets_host, int64_t B, int max_workers,
                   void *stream);
int ef_plan_destroy(ef_plan *plan);

/*
 * Deferred residual correction, off by default.  Algorithm 4 ends a worker's
 * (and the server's) step with e <- p - Delta.  For a block of more than
 * fuse_limit tiles the scale of Delta is known only after the first kernel
 * has passed over the whole block, so that kernel leaves p in the residual
 * buffer and a second one reads it back and writes e (8 more bytes of HBM
 * traffic per element).  With on = 1 that second pass is not run: the buffer
 * keeps p over the whole tiles of such blocks, the plan remembers the block's
 * scale, and the next ef_worker_step* / ef_server_step on that buffer forms
 * e = p - Delta as it loads the data: the same fp32 subtraction on the same
 * operands, so payloads, momentum and parameters of every step are bit-equal
 * to the default mode's.  What changes for the caller:
 *   - between calls the residual buffers are opaque where large blocks lie;
 *     ef_flush writes the true e into them (before reading, checkpointing, or
 *     handing a buffer to another plan or to another worker index);
 *   - worker i's buffer must stay worker i's (the remembered scales are kept
 *     per worker index and for the server), and the plan must see every step
 *     of it: while corrections are waiting, a worker, server or flush call
 *     with another err / server_err pointer or stride than the call that
 *     left them returns EF_ERR_ARG;
 *   - ef_plan_set_lazy, and the tuning calls of ef_debug.h that move the
 *     one-pass limit, return EF_ERR_ARG while any buffer is waiting for its
 *     correction, since they change which blocks count as large: call
 *     ef_flush first.
 * Blocks of at most fuse_limit tiles, and the parts of large blocks that
 * share a tile with another block, are corrected in the call as before.
 * The mode picks its own one-pass limits: 0 for the server (no workgroup
 * waits for a scale) and 64 tiles for the worker, which then runs one
 * workgroup per tile.  Measured on 2^28 elements in 256
 * blocks with 8 workers: 7.5 instead of 8.0 ms per step.
 * ef_plan_set_lazy synchronises the device.
 */
int ef_plan_set_lazy(ef_plan *plan, int on);
int ef_plan_is_lazy(const ef_plan *plan);

/*
 * Makes the deferred corrections now: err (device, [n_workers][state_stride],
 * may be NULL) and server_err (device, [d], may be NULL) are the buffers the
 * plan's last worker / server calls wrote; afterwards they hold e of
 * Algorithm 4 everywhere and the next call takes them as they are.  Buffers
 * with nothing pending are left untouched, so the call is harmless in the
 * default mode.  Enqueues on `stream`; EF_ERR_ARG for n_workers outside
 * [1, max_workers] or a bad stride, EF_ERR_ALIGN for a pointer off 16 bytes.
 */
int ef_flush(const ef_plan *plan, int n_workers, float *err, int64_t state_stride, float *server_err, void *stream);

int64_t ef_plan_d(const ef_plan *plan);      /* d = block_offsets[B] */
int64_t ef_plan_blocks(const ef_plan *plan); /* B */
size_t ef_sign_words(const ef_plan *plan);   /* W = ceil(d/64): 64-bit words of one payload's sign bits (Section 3.2:
                                                d bits per direction, Table 1); 0 for a NULL plan */

/*
 * Worker side of iteration t of Algorithm 4, for n_workers workers at once
 * (n_workers = 1 is the per-worker call of the paper).  For worker i, element j:
 *     m_i   <- mu * m_i + g_i                                  (momentum)
 *     p_i    = mu * m_i + g_i + (eta_prev / eta) * e_i          (updated m_i)
 *     push   Delta_i = C_B(p_i)  -> packed_signs[i], scales[i]  (Section 3.2)
 *     e_i   <- p_i - Delta_i                                   (error feedback)
 * mu = 0 gives Algorithm 3.  eta_prev = eta_{t-1} with eta_{-1} = 0 on the first
 * iteration; only the ratio eta_prev/eta (one fp32 division) enters.
 *
 *   grad          in      float[n_workers][grad_stride], first d of each row used
 *   mom, err      in/out  float[n_workers][state_stride], updated in place
 *   packed_signs  out     uint64[n_workers][W]
 *   scales        out     float[n_workers][B]
 * Strides are in elements, >= d and multiples of 4 (with n_workers = 1 they are
 * not used and not checked).  mom and err are updated in place; apart from
 * that no two arguments may share memory: a payload buffer that overlaps grad,
 * mom or err, or state buffers that overlap each other, give EF_ERR_ARG.
 */
int ef_worker_step(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride,
                   float *mom, float *err, int64_t state_stride, float mu, float eta_prev,
                   float eta, uint64_t *packed_signs, float *scales, void *stream);

/*
 * The same call for dist-EF-blockSGD (Algorithm 3; Section 4.1 notes that it is
 * Algorithm 4 at mu = 0): no momentum buffer exists, so none is read or
 * written,
 *     p     = g + (eta_prev/eta) * e
 *     Delta = C_B(p)  -> packed_signs, scales
 *     e    <- p - Delta
 * Arguments as for ef_worker_step.  Payloads and residuals equal those of
 * ef_worker_step with mu = 0 (a zero of either sign may differ in sign).
 */
int ef_worker_step_sgd(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride,
                       float *err, int64_t state_stride, float eta_prev, float eta,
                       uint64_t *packed_signs, float *scales, void *stream);

/*
 * Server side of iteration t of Algorithm 4:
 *     p~   = (1/M) * sum_i Delta_i + (eta_prev / eta) * e~
 *     push  Delta~ = C_B(p~)  -> out_signs, out_scales
 *     e~  <- p~ - Delta~
 * The sum over workers runs in fp32 in worker order i = 0..M-1 starting from
 * +0, followed by one fp32 division by (float)M.
 *
 *   packed_signs  in      uint64[M][W]   the M worker payloads as ef_worker_step wrote them
 *   scales        in      float[M][B]
 *   server_err    in/out  float[d]
 *   out_signs     out     uint64[W]
 *   out_scales    out     float[B]
 * server_err is updated in place; the outgoing payload may overlap neither the
 * incoming payloads nor server_err (EF_ERR_ARG).
 */
int ef_server_step(const ef_plan *plan, int M, const uint64_t *packed_signs, const float *scales,
                   float *server_err, float eta_prev, float eta, uint64_t *out_signs,
                   float *out_scales, void *stream);

/*
 * Parameter update of Algorithm 4 with the payload pulled from the server:
 *     x <- x - eta * Delta~          (eta * scale rounded once, then subtracted)
 *
 *   params        in/out  float[d]
 *   packed_signs  in      uint64[W]
 *   scales        in      float[B]
 */
int ef_apply(const ef_plan *plan, float *params, const uint64_t *packed_signs, const float *scales,
             float eta, void *stream);

/*
 * Parameter update with weight decay kept outside the compressed signal
 * (Appendix A): every machine holds one more momentum buffer for the decay term,
 *     decay_mom <- mu * decay_mom + lambda * x
 *     x         <- x - eta * ((Delta~ + mu * decay_mom) + lambda * x)
 * with the updated decay_mom and the old x on the right-hand side; lambda * x is
 * rounded once and used in both lines.  lambda = 0 with a zero decay_mom gives
 * exactly ef_apply.
 *
 *   params        in/out  float[d]
 *   decay_mom     in/out  float[d], zero before the first iteration
 *   packed_signs  in      uint64[W]
 *   scales        in      float[B]
 *   mu in [0, 1), lambda >= 0, eta > 0 (EF_ERR_ARG otherwise)
 */
int ef_apply_wd(const ef_plan *plan, float *params, float *decay_mom, const uint64_t *packed_signs,
                const float *scales, float eta, float mu, float lambda, void *stream);

/*
 * Fused messages (Section 4.2: sign words and scales sent as two separate
 * messages cost the server latency; one message per worker avoids that).
 *
 * One message is a single contiguous buffer of ef_payload_bytes(plan) bytes:
 *     bytes [0, 8*W)                : the W sign words (layout as above)
 *     bytes [8*W, 8*W + 4*B)        : the B fp32 scales
 *     padding up to a multiple of 16 bytes (never read, never written)
 * ef_payload_scales_offset(plan) returns 8*W.  A buffer of n messages holds
 * message i at byte offset i * ef_payload_bytes(plan); buffers must be 16-byte
 * aligned (EF_ERR_ALIGN otherwise).  The three calls below compute exactly what
 * ef_worker_step / ef_server_step / ef_apply compute, bit for bit, with the
 * same kernels; only the addresses of the payload parts differ, so a worker's
 * message can be handed to a transport as one buffer and the server consumes
 * the M received messages in place.
 *
 *   ef_worker_step_fused : payloads     out  n_workers messages
 *   ef_server_step_fused : payloads     in   M messages
 *                          out_payload  out  one message, not overlapping the input
 *                                            (EF_ERR_ARG otherwise)
 *   ef_apply_fused       : payload      in   one message
 * All other arguments are those of the unfused calls.
 */
size_t ef_payload_bytes(const ef_plan *plan);
size_t ef_payload_scales_offset(const ef_plan *plan);
int ef_worker_step_fused(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride,
                         float *mom, float *err, int64_t state_stride, float mu, float eta_prev,
                         float eta, void *payloads, void *stream);
int ef_server_step_fused(const ef_plan *plan, int M, const void *payloads, float *server_err,
                         float eta_prev, float eta, void *out_payload, void *stream);
int ef_apply_fused(const ef_plan *plan, float *params, const void *payload, float eta, void *stream);

/*
 * How well the compressors approximate each of n_vectors vectors (Section 3.2):
 *     out[2i]   = phi(v_i)   = min_b ||v_Gb||_1^2 / (d_b ||v_Gb||_2^2)    (Proposition 1: C_B is
 *                              phi(v)-approximate; blocks of zeros count as ratio 1)
 *     out[2i+1] = delta(v_i) = ||v||_1^2 / (d ||v||_2^2)                  (the non-block compressor
 *                              of Eq. (1); 1 for a vector of zeros)
 * Sums are taken in fp64 in a fixed order, so repeated calls give the same bits.
 *
 *   v     in   float[n_vectors][stride], stride >= d and a multiple of 4
 *   out   out  double[2 * n_vectors], device memory, 8-byte aligned
 *   n_vectors in [1, max_workers]
 * Uses scratch the plan allocated at creation (48 bytes per tile and vector); like the other
 * calls it allocates nothing, and it must be ordered on the device with every call that shares
 * the plan.
 */
int ef_compressor_quality(ef_plan *plan, int n_vectors, const float *v, int64_t stride, double *out,
                          void *stream);

/*
 * Optimizer state held by the library.  Algorithm 4 keeps, between iterations,
 * the momentum m_i and the residual e_i of every worker and the residual e~ of
 * the server (all zero before the first iteration).  With ef_worker_step and
 * ef_server_step the caller owns those buffers and sees e after every call,
 * which for blocks beyond the one-pass limit costs a second pass, or the
 * caveats of ef_plan_set_lazy.  A caller that never looks at the residuals can
 * leave the buffers to the library instead: the calls below then always run
 * in the deferred mode (no second pass, no workgroup waiting for the scale of
 * a large block; on 2^28 elements in 256 blocks with 8 workers 7.5 instead of
 * 7.9 ms per step), with nothing for the caller to keep track of.  Payloads and
 * parameters are bit-equal to those of the caller-owned calls.
 *
 *   ef_state_create   allocates (hipMalloc) and zeroes m, e for n_workers
 *                     workers and e~; turns the plan's deferred mode on and
 *                     keeps it on (ef_plan_set_lazy then returns EF_ERR_ARG).
 *                     One state per plan (EF_ERR_ARG for a second one, for
 *                     n_workers outside [1, max_workers], or while
 *                     caller-owned buffers of this plan wait for a correction:
 *                     ef_flush them first).  Synchronises `stream`.
 *   ef_state_destroy  frees it and turns the mode off; synchronises the
 *                     device.  Destroy the state before its plan.
 *   ef_worker_step_state / ef_server_step_state
 *                     ef_worker_step (all n_workers of the state) and
 *                     ef_server_step on the held buffers; the other arguments,
 *                     the results and the errors are those calls'.
 *   ef_state_export   writes the true m, e (rows state_stride elements apart,
 *                     >= d) and e~ of Algorithm 4 into caller buffers, for a
 *                     checkpoint or a look at them; any of the three may be
 *                     NULL.  The held state is unchanged in value.
 *   ef_state_import   the reverse: overwrites the held m, e, e~ (those given)
 *                     with finished state, e.g. from a checkpoint.
 * Both copies are device-to-device on `stream` and allocate nothing.
 */
int ef_state_create(ef_plan *plan, int n_workers, ef_state **out, void *stream);
int ef_state_destroy(ef_state *state);
int ef_worker_step_state(const ef_plan *plan, ef_state *state, const float *grad, int64_t grad_stride,
                         float mu, float eta_prev, float eta, uint64_t *packed_signs, float *scales,
                         void *stream);
int ef_server_step_state(const ef_plan *plan, ef_state *state, int M, const uint64_t *packed_signs,
                         const float *scales, float eta_prev, float eta, uint64_t *out_signs,
                         float *out_scales, void *stream);
int ef_state_export(const ef_plan *plan, ef_state *state, float *mom, float *err, int64_t state_stride,
                    float *server_err, void *stream);
int ef_state_import(const ef_plan *plan, ef_state *state, const float *mom, const float *err,
                    int64_t state_stride, const float *server_err, void *stream);

/*
 * ef_worker_step that also reports how well the compressor approximated what
 * it was given: exactly ef_worker_step (same arguments, same results, bit for
 * bit), plus quality[2i] = phi(p_i) and quality[2i+1] = delta(p_i) of worker
 * i's corrected gradient p_i (Proposition 1 bounds the step's compression
 * error by (1 - phi(p)) ||p||^2).  The sums of |p| and p^2 are taken inside
 * the worker kernel on the values it holds anyway, so no tensor is read a
 * second time; the figures are those ef_compressor_quality would give on p_i
 * (fp64, fixed order).  The call always runs the worker kernel that takes one
 * workgroup per tile.  In the deferred mode it follows the same rules as
 * ef_worker_step.
 *
 *   quality   out  double[2 * n_workers], device memory, 8-byte aligned
 */
int ef_worker_step_quality(const ef_plan *plan, int n_workers, const float *grad, int64_t grad_stride,
                           float *mom, float *err, int64_t state_stride, float mu, float eta_prev,
                           float eta, uint64_t *packed_signs, float *scales, double *quality,
                           void *stream);

/*
 * ef_compressor_quality for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * kernels and the same results, bit for bit, but the per-tile sums go to a
 * fixed array in the library's own device image instead of plan-owned memory,
 * and the call itself calls no hipMalloc, hipFree or other allocating routine
 * (plan creation, which happens earlier, still does).
 *
 * Capacity: ceil(d/4096) * n_vectors <= EF_QUALITY_STATIC_MAX_TILE_VECTORS
 * (131072, i.e. 2^29 elements over all vectors; the array takes 6 MiB of every
 * GPU the library runs on until the process ends); larger inputs are refused
 * with EF_ERR_SIZE before anything is enqueued.  The plan's device must be
 * current (EF_ERR_ARG otherwise).  Other arguments and errors as for
 * ef_compressor_quality.
 *
 * All calls on one GPU share the one array, whatever their plan: calls that
 * overlap on the device (different streams, no ordering between them) race on
 * it and give wrong results; order them.  The array keeps the last call's
 * contents; nothing in it has to start at zero, since every word a call reads
 * it has written before.
 */
#define EF_QUALITY_STATIC_MAX_TILE_VECTORS 131072
int ef_compressor_quality_static(const ef_plan *plan, int n_vectors, const float *v, int64_t stride,
                                 double *out, void *stream);

/* Static text for an error code; for EF_ERR_HIP the text of the last HIP error
 * seen by this thread is appended.  The returned pointer stays valid until the
 * same thread calls ef_strerror again. */
const char *ef_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* EF_H */
