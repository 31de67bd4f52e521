/*
 * loqt_debug.h -- test, tuning and diagnostic hooks of libloqt.  NOT part of the production ABI of loqt.h.
 *
 * Everything here is process-wide state or host-side introspection: overrides of the implementation and tile
 * choices that the calls of loqt.h otherwise make from their sizes alone, and per-kernel timers for the
 * benchmark.  None of it is thread-safe; a production caller needs none of it.  The parity tests use the
 * overrides to run every implementation and every tile shape over small ragged inputs.
 */
#ifndef LOQT_DEBUG_H
#define LOQT_DEBUG_H

#include "loqt.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Implementation choice (process-wide override; not thread-safe; default LOQT_PATH_AUTO).
 * The three forms of the layer of sec. 2.2 / 2.4:
 *   LOQT_PATH_FUSED  : NF4 codes are expanded inside the GEMMs' operand staging (global memory
 *                      -> registers -> LDS), no extra pass over the weights.
 *   LOQT_PATH_PREPASS: NF4 operands are expanded to bf16 in the workspace by one streaming pass
 *                      per call (transposed where the product needs it), then every product is
 *                      a K-contiguous bf16 GEMM fed by direct global->LDS loads.
 *   LOQT_PATH_FOLDED : as PREPASS, but forward and backward first fold the rank-r term into the
 *                      bf16 copy of the weight, W_eff = deq(W_q) + s deq(P_q) B (a rank-r product of
 *                      2 out in r flop with fp32 accumulation), and then run single products
 *                      y = x W_eff^T and dx = dy W_eff.  The intermediate U is not formed; Z still is
 *                      (dB = Z^T x).  Cheaper than carrying the rank-r term through every token
 *                      (2 T r (in + out) flop per pass) from T = out in / (in + out) tokens up.
 *   LOQT_PATH_AUTO   : forward and backward always take the pre-pass family (measured ahead of the
 *                      fused form at every token count from 16 up), folded when T (in + out) >= out in --
 *                      except that the backward pass, which has Z = s dy deq(P_q) at hand anyway, keeps the
 *                      rank-r term as a second K segment of the dx product when out > 0.73 T (2 T r in flop at
 *                      the rate of the large products instead of 2 out in r at the rate of the fold);
 *                      the merge is fused below 1024 columns (`in`), pre-pass above.
 * All compute the same quantities; results differ only in rounding order, within the stated
 * tolerance.
 */
enum { LOQT_PATH_AUTO = 0, LOQT_PATH_FUSED = 1, LOQT_PATH_PREPASS = 2, LOQT_PATH_FOLDED = 3 };
loqt_status loqt_set_path(int path);
/* The implementation (FUSED, PREPASS or FOLDED) the current option selects for these sizes. */
int loqt_resolved_path(int op, int64_t T, int64_t out, int64_t in);

/*
 * Tile-shape option (process-wide, not thread-safe; for tests and tuning).  The products of the
 * pre-pass family (every product of the layer calls of sec. 2.2 / 2.4 and the merge of Alg. 1 line 5
 * when it takes that path) run on work-group tiles of 256x256, 256x128 or 128x128 outputs, chosen from
 * the sizes.  LOQT_TILE_AUTO keeps that choice; the other values force one shape for every such product
 * whatever its size (the compensation step of Alg. 2 and the dense merge always use 128x128).  All
 * shapes compute the same quantities; results differ only in summation order.  Returns
 * LOQT_INVALID_ARG for any other value.
 */
enum { LOQT_TILE_AUTO = 0, LOQT_TILE_256x256 = 1, LOQT_TILE_256x128 = 2, LOQT_TILE_128x128 = 3 };
loqt_status loqt_set_tile(int tile);
/*
 * Diagnostic (host only, no GPU work): how a bf16-output product of M rows and N columns (plus Nx extra
 * columns that share the left operand, 0 if none) that is large enough for 256x256 tiles is laid out
 * under LOQT_TILE_AUTO.  *n_large = 0: one launch of 256x256 tiles; otherwise the first *n_large columns
 * (a multiple of 256, < N) go out as 256x256 tiles in whole rounds of 256 and the remaining columns, with
 * the extra ones, as a second launch of 128x128 tiles.  *rounds = the estimated duration in rounds of
 * 256x256 tiles.  Either pointer may be NULL.  Returns LOQT_BAD_SHAPE for M, N <= 0 or Nx < 0.
 */
loqt_status loqt_plan_product(int64_t M, int64_t N, int64_t Nx, int64_t *n_large, double *rounds);

/*
 * Optional per-kernel timing (diagnostics for benchmarks; off by default).
 * While enabled, every kernel launch of the library is bracketed by HIP events recorded on
 * the launch stream (the event tables are host memory allocated at the first enable and kept; never enable
 * it around a stream capture).  loqt_timing_read synchronises with the recorded events and returns,
 * for kernel slot `slot` (0 <= slot < loqt_timing_slots()), its name, launch count and summed
 * device time in milliseconds since the last loqt_timing_enable(1).  Not thread-safe; at most
 * LOQT_TIMING_MAX_EVENTS launches are recorded per enable, later ones are not timed.
 */
#define LOQT_TIMING_MAX_EVENTS 65536
void loqt_timing_enable(int on);
int loqt_timing_slots(void);
loqt_status loqt_timing_read(int slot, const char **name, int64_t *launches, double *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* LOQT_DEBUG_H */
