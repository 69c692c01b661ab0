/*
 * polysci_ranker.h -- C ABI of the pairwise neural ranking of code variants (Section 4.2.2 of the paper).
 *
 * A code variant (here: a candidate tile of a convolution) is described by four numbers, the working-set sizes that
 * Algorithm 2 assigns to the three cache levels and to memory.  A small fully connected network looks at two
 * variants at a time and says which one it expects to be faster; every variant plays every other one and variants
 * are ranked by their number of wins.
 *
 * Conventions as in polysci_conv.h: data pointers marked "device" are device memory owned by the caller, `stream`
 * is a hipStream_t passed as void* (0 = default stream), device work is asynchronous on that stream, nothing is
 * allocated, freed or retained, and the return value is PS_OK or a negative ps_status.
 */
#ifndef POLYSCI_RANKER_H
#define POLYSCI_RANKER_H

#include <stdint.h>

#include "polysci_conv.h"

#ifdef __cplusplus
extern "C" {
#endif

#define PS_RANKER_STATS 4    /* statistics per variant: working-set size at level 1, 2, 3 and memory */
#define PS_RANKER_LEVELS 3
/* Parameters of the network of Section 4.2.2: layers of 64, 32, 16, 8 and 2 units on 2 * PS_RANKER_STATS inputs.
 * Flat float array, layer after layer: the weight matrix row-major as [inputs][units], then the bias [units].
 * 8*64+64 + 64*32+32 + 32*16+16 + 16*8+8 + 8*2+2 values. */
#define PS_RANKER_PARAMS 3338
#define PS_RANKER_MAX_VARIANTS 8192

/* HOST call.  The statistics of one candidate tile: the tile's launch is written as a loop nest at workgroup
 * granularity -- the two tile loops in launch order, the split of the reduction, the channel blocks of one split,
 * the filter taps -- whose array elements are the blocks a workgroup moves (its output tile, its input pixels for
 * one channel block, one filter tap of its channels), weighted by their size in bytes.  Algorithm 1 gives the
 * working-set sizes of the nest's dependences, Algorithm 2 assigns them to registers+LDS of one compute unit
 * (672 KiB), the L2 caches (32 MiB) and the Infinity Cache (256 MiB); level_ws receives the three sums, *mem_ws what
 * is left to memory (bytes).  PS_EUNSUPPORTED if the split does not divide the channel blocks (the nest would not be
 * rectangular) or the nest is too large to enumerate; PS_EINVAL for malformed arguments. */
int ps_tile_reuse_levels(const ps_conv_desc *desc, const ps_tile *tile, int64_t level_ws[PS_RANKER_LEVELS],
                         int64_t *mem_ws);

/* HOST call.  A second set of four statistics for the same network, in the units this hardware is limited by: the
 * parts the tile model (ps_tile_cost_ws_us) adds up, in microseconds -- matrix-core time including per-workgroup
 * overheads, traffic into the compute units, traffic beyond L2 (with the partial tiles of a split reduction),
 * launches and extra passes.  Same validity rules and return codes as ps_tile_cost_ws_us's tile: PS_EUNSUPPORTED
 * for a tile that is not valid for the descriptor. */
int ps_tile_level_times_ws(const ps_conv_desc *desc, const ps_tile *tile, double times_us[PS_RANKER_STATS]);

/* The tournament of Section 4.2.2 on the GPU.
 *   stats   device, float [n][PS_RANKER_STATS]: the statistics of the n variants (non-negative)
 *   params  device, float [PS_RANKER_PARAMS], layout above; activations relu, relu, softsign, relu, then softmax
 *   theta   an output above theta counts as fired (the paper uses 0.6); must lie in [0.5, 1) so that at most one
 *           output fires
 *   wins    device, int32 [n], overwritten: games won
 *   probs   device, float [n][n][2] or NULL: if given, probs[i][j] receives the two outputs of the game in which
 *           variant i is presented first and variant j second (the diagonal is set to zero)
 * Every ordered pair (i, j), i != j, is one game: the eight statistics of i and j are divided by their sum (all
 * zeros stay zeros) and fed to the network; the first output firing is a win for i, the second a win for j,
 * neither a draw.  All arithmetic is single precision; win counts are integer sums and do not depend on scheduling.
 * Two kernels are enqueued (wins is cleared by a fill kernel, not a memset, so the call can be captured in a graph).  n = 0 is allowed and does nothing; n above
 * PS_RANKER_MAX_VARIANTS is PS_EUNSUPPORTED. */
int ps_ranker_play(const float *stats, int n, const float *params, float theta, int32_t *wins, float *probs,
                   void *stream);

#define PS_RANKER_WORKING_SETS 0 /* statistics of ps_tile_reuse_levels (bytes) */
#define PS_RANKER_LEVEL_TIMES 1  /* statistics of ps_tile_level_times_ws (microseconds) */

/* Device bytes ps_tile_rank_dnn needs as scratch for this descriptor (statistics and win counts of every
 * candidate); 0 for an invalid descriptor. */
size_t ps_tile_rank_dnn_scratch_bytes(const ps_conv_desc *desc);

/* Ranks the candidate tiles of a descriptor with the network (the paper's "rank n variants, run the best k" with
 * the ranking of Section 4.2.2): every candidate that fits `workspace_bytes` of split-reduction workspace and has
 * statistics of kind `stats_kind` enters the tournament; the k candidates with the most wins are written to
 * tiles[0..) (HOST memory), most wins first, equal counts in enumeration order (ps_tile_get), with their win counts
 * in wins[0..) (HOST, may be NULL).  `params` is device memory as for ps_ranker_play; `scratch` is device memory of
 * at least ps_tile_rank_dnn_scratch_bytes(desc) bytes, 16-byte aligned, whose contents are overwritten.  Unlike
 * the other device calls this one WAITS for the stream: it returns after the win counts have come back.  Returns
 * the number of tiles written (<= k) or a negative ps_status (PS_EUNSUPPORTED if no candidate qualifies). */
int ps_tile_rank_dnn(const ps_conv_desc *desc, size_t workspace_bytes, int stats_kind, const float *params, float theta,
                     void *scratch, size_t scratch_bytes, int k, ps_tile *tiles, int32_t *wins, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* POLYSCI_RANKER_H */
