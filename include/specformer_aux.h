/*
 * specformer_aux.h -- measurement and tuning aids of libspecformer (gfx950).  Not part of the decoding
 * path: bench and sweep programs use these to time kernel classes, to calibrate hardware byte counters and
 * to override the automatic kernel choices of ONE context.
 */
#ifndef SPECFORMER_AUX_H
#define SPECFORMER_AUX_H
#include "specformer.h"
#ifdef __cplusplus
extern "C" {
#endif

/* Force the linear kernels' tile configuration (1..sf_linear_num_tiles()) and split-K factor for every
 * later launch of this context; 0 = automatic choice.  A forced pair whose partial tiles do not fit the
 * workspace makes the launch fail with SF_EHIP. host. */
sf_status sf_tune_linear(sf_ctx *ctx, int32_t tile, int32_t split_k);
int32_t sf_linear_num_tiles(void);
/* The automatic choice for a bf16 linear layer of M rows whose weight [N][K] is also used with up to
 * plan_M >= M rows: *split_k is the same for every M <= plan_M (so a row's result does not depend on
 * the rows batched with it), *tile follows M; *tile_rows = rows per workgroup of that tile.  Pure
 * host arithmetic, no GPU needed.  host pointers. */
sf_status sf_linear_config(int32_t M, int32_t plan_M, int32_t N, int32_t K, size_t workspace_bytes,
                           int32_t *tile, int32_t *split_k, int32_t *tile_rows);
/* Force the attention's split-KV chunk size in 32-key tiles (>= 16) for this context; 0 = automatic. host. */
sf_status sf_tune_attention(sf_ctx *ctx, int32_t chunk_tiles);

/* Between sf_profile_begin and sf_profile_end every kernel launch of this context is bracketed by a pair
 * of HIP events on its stream.  sf_profile_end waits for the last one and returns, per kernel class, the
 * summed duration in ms and the number of launches (host arrays of n_class >= SF_N_KERNEL_CLASSES
 * entries).  Classes: 0 linear (GEMM), 1 attention, 2 attention split-KV combine, 3 RMSNorm, 4 rotary +
 * K/V append, 5 SwiGLU gate, 6 embedding / hook copies, 7 arg-max pass over stored logits, 8 arg-max
 * finish / accept-commit. */
#define SF_N_KERNEL_CLASSES 9
sf_status sf_profile_begin(sf_ctx *ctx);
sf_status sf_profile_end(sf_ctx *ctx, double *ms, int32_t *launches, int32_t n_class);
/* A plain device-to-device copy kernel (`calib_copy_kernel`) of `bytes` (multiple of 16, 16-byte aligned
 * pointers) that reads and writes every byte exactly once: the dispatch of known size against which
 * hardware byte counters (FETCH_SIZE, WRITE_SIZE) are scaled. */
sf_status sf_calib_copy(void *dst, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif
