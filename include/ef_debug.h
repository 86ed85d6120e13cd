/*
 * ef_debug.h -- tuning and diagnostic entry points of libef, kept apart from
 * the boundary of Algorithm 4 (ef.h).  Tests use them to force each route by
 * which a block's residual can be finished; a caller of the method needs none
 * of them: plan creation picks every setting from the layout.  Results never
 * depend on these settings, only the time taken does.
 */
#ifndef EF_DEBUG_H
#define EF_DEBUG_H

#include "ef.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Tuning knobs of the one-pass residual update (e <- p - Delta of Algorithm 4
 * needs the whole block's scale): workgroups of a block spanning at most
 * fuse_limit tiles of 4096 elements keep p in registers and wait for the scale,
 * polling at most spin_limit times before they fall back to the two-pass route
 * that larger blocks always take.  Results are identical on either route.
 * Negative values leave a setting unchanged; fuse_limit = 0 sends every block
 * through two passes, spin_limit = 0 makes every wait give up at once (used by
 * tests to exercise the fallback).  The default spin_limit is 2048 polls of
 * about 1.2 us: waits on an idle GPU were measured to end within 64, so a wait
 * that cannot succeed costs about 2.5 ms.  Synchronises the device.  By default each
 * kernel gets its own limit: half the tiles its workgroups can hold at once
 * (resident workgroups; times six for the persistent worker kernel, which
 * keeps three tiles in registers and three in LDS), at most 4096 tiles.  A
 * limit set here applies to worker and server alike.
 *
 * For the caller's choice of blocks this means: a block of up to about 9.4 M
 * elements (2304 tiles, the persistent worker kernel's default limit on a GPU
 * with 256 compute units) costs 20.125 bytes of HBM traffic per element and
 * worker; a larger block has its corrected gradient written out and read back
 * once more (28.125 bytes) unless the deferred mode is on (ef_plan_set_lazy).
 * Within one pass, blocks of 8 to 64 tiles (32 K to 256 K elements) stream
 * fastest (about 6 % faster than blocks of 256 tiles, 12 % faster than blocks
 * of 1024).  Proposition 1 favours finer blocks as well.
 */
int ef_plan_tune(ef_plan *plan, int fuse_limit, int spin_limit);
int ef_plan_fuse_limit(const ef_plan *plan);       /* the worker kernels' limit in force */

/*
 * Which kernel the worker calls run over the tiles that lie inside one block:
 * on = 1 a persistent kernel whose workgroups take tiles from a ticket counter
 * and keep several tiles in registers while their scales form; on = 0 one
 * workgroup per tile that waits in place for its block's scale; on < 0 the
 * choice plan creation made for this layout: the persistent kernel if every
 * workgroup gets at least 16 tiles and the layout's blocks are cheaper on it
 * by the measured cost per tile of either kernel (one workgroup per tile is
 * the faster on blocks of up to 256 tiles, the persistent kernel on larger
 * ones, and it finishes blocks of 1025 to 2304 tiles in one pass that the
 * other sends through the second pass).  ef_worker_step_sgd, and every worker
 * call in the deferred mode (ef_plan_set_lazy), use the persistent kernel only
 * after on = 1.  The server always runs one workgroup per tile.  Same results
 * either way.  Synchronises the device.
 */
int ef_plan_set_persistent(ef_plan *plan, int on);
int ef_plan_is_persistent(const ef_plan *plan);

/*
 * Writing the residual out in step.  In the worker kernel that runs one
 * workgroup per tile, the whole tiles of a block larger than fuse_limit have
 * nothing to wait for; they are made to wait (bounded by spin_limit, and with
 * nothing depending on the outcome) for their neighbours, in groups of `tiles`
 * consecutive tiles, before they write their residual tile: measured faster
 * than workgroups that each write when done (worker call on 2^28 elements,
 * 8 workers, deferred mode: 7.6 ms without, 6.75 ms in groups of 16, 6.9 ms
 * in groups of 24 or 32).  tiles = 0 or 1 turns it off; at most 256; default
 * 16.  Results do not depend on it.  Synchronises the device.
 */
int ef_plan_set_sync_group(ef_plan *plan, int tiles);

/*
 * How often the most recent ef_worker_step / ef_server_step on this plan left
 * the one-pass route at run time: tiles whose wait for the block scale was not
 * taken or ran out (p parked, finished by the second pass) and blocks whose
 * scale had to be formed by the second pass.  Results do not depend on these
 * counts; they are a performance diagnostic.  Synchronises the device.  Either
 * pointer may be NULL (HOST pointers).
 */
int ef_plan_last_fallbacks(ef_plan *plan, unsigned int *parked_tiles, unsigned int *late_blocks);

#ifdef __cplusplus
}
#endif
#endif /* EF_DEBUG_H */
