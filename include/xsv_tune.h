/* xsv_tune.h - tuning knobs and measurement aids of libxsv.
 *
 * Nothing here is part of the method: these calls change how the library launches its kernels (never what
 * they compute: results agree to rounding, and bit for bit where xsv.h promises it) or report how long
 * launches took.  Benchmarks, profiling runs and tests of the launch shapes use them; a model calls xsv.h only.
 * Conventions as in xsv.h: 0 or a negative error code, no exceptions, a context is not thread-safe.
 */
#ifndef XSV_TUNE_H
#define XSV_TUNE_H

#include "xsv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning: number of equal key ranges every (head, block of query rows) is cut into by the attention
 * kernel (partial results are merged by a second kernel), 1..16.  0 (default) = one workgroup per
 * slot of the chip, the key tiles of all (head, query block) pairs dealt out evenly among them. */
int xsv_set_attend_splits(xsv_ctx* ctx, int per_layer_calls, int batched_calls);
/* Tuning: compute units the attention launch of xsv_step / xsv_step_all_layers leaves free for the
 * overlapped score/select/re-quantize chain (0 .. half the chip).  Without spare units the chain only
 * starts when attention drains.  -1 (default) = a quarter of the chip, an eighth when the attention launch
 * is long (more than about 24 key tiles per workgroup).  Ignored when overlap is off or splits are fixed. */
int xsv_set_side_cus(xsv_ctx* ctx, int compute_units);
/* Tuning: in xsv_step / xsv_step_all_layers with overlap, cut every (head, query block) into one more key
 * range than the spare units allow, the extra one `percent` of a full range long (1..100; 0 = off; -1 = default: 35, or 50 in overlap mode 2): its
 * workgroups end early and hand their compute units to the chain for the rest of the attention launch. */
int xsv_set_short_range(xsv_ctx* ctx, int percent);
/* Tuning: what a key tile of the frame's own bf16 rows costs the attention kernel relative to a tile of the packed
 * cache, in percent (25..400, default 95: bf16 rows need no dequantization).  When every (head, query block) is cut into the same key ranges, the
 * ranges are chosen to cost the same by this measure, so that all workgroups of a launch end together. */
int xsv_set_frame_tile_cost(xsv_ctx* ctx, int percent);
/* Measurement aid.  While enabled, every attention launch of this context (xsv_dequant_attend, xsv_step,
 * xsv_step_all_layers) is bracketed by events on the context's stream: before the attention kernel,
 * between it and the kernel that merges key-range partials, after, and once more right behind.
 * xsv_attend_times waits for the stream, returns the number of launches recorded since the last call (or
 * since enabling), the average span of each of the two kernels in milliseconds and (event_ms, may be NULL)
 * the average span of the last two events, which have nothing between them: what an event pair itself adds
 * to a span.  It then starts a new series.  Enabling or disabling discards the series.  The events cost a
 * few microseconds per launch; leave this off in production. */
int xsv_set_attend_timing(xsv_ctx* ctx, int enabled);
int xsv_attend_times(xsv_ctx* ctx, int32_t* launches, float* attend_ms, float* merge_ms, float* event_ms);
/* With the same switch, xsv_step and xsv_step_all_layers also bracket their score + select launches and
 * their re-quantize launch with events on the stream those run on.  Returns the number of steps recorded,
 * the average span of the two stages in milliseconds (event cost included), and starts a new series.  In the
 * overlapped modes the spans include whatever the attention running beside them takes away. */
int xsv_chain_times(xsv_ctx* ctx, int32_t* steps, float* score_prune_ms, float* quantize_ms);
/* Grid (workgroups) of the most recent attention launch of this context, 0 before the first. */
int xsv_last_attend_workgroups(xsv_ctx* ctx, int32_t* workgroups);
/* Tuning: workgroup shape of the attention kernel (waves x query rows per wave).  3 = 8 x 64, 0 = 4 x 64,
 * 1 = 4 x 32, 2 = 8 x 32.  Default: 3, or 2 where blocks of 256 rows pad a frame's tokens less than blocks
 * of 512 (e.g. 1041 tokens).  Other values: XSV_ERR_ARG.  Results agree to rounding. */
int xsv_set_attend_variant(xsv_ctx* ctx, int variant);

/* Host only (no GPU call): where the attention launch of a step cuts a (head, query block)'s key tiles - `cache_tiles`
 * tiles of 64 cached tokens followed by `frame_tiles` tiles of the frame's own tokens - into `ranges` consecutive key
 * ranges of equal cost, a frame tile costing `frame_tile_cost` percent of a cache tile and the last range
 * `last_percent` percent of a full share.  begin[0] = 0 <= begin[1] < .. < begin[ranges] = all tiles; every range holds
 * at least one tile.  1 <= ranges <= min(16, tiles), 1 <= last_percent <= 100, 25 <= frame_tile_cost <= 400, else
 * XSV_ERR_ARG.  For tests and for sizing experiments; the library calls the same routine. */
int xsv_key_ranges(int cache_tiles, int frame_tiles, int ranges, int last_percent, int frame_tile_cost, int32_t* begin);

/* Host only: the other way an attention launch divides its work, used when the workgroup count is not a multiple of
 * the units - the `units * tiles` (unit, key tile) items in one line, cut into `workgroups` pieces that differ by at
 * most one item.  Piece `workgroup` is [*begin, *end); unit `unit` is touched by workgroups *first .. *last.  Any
 * pointer may be NULL.  units, tiles, workgroups >= 1, 0 <= workgroup < workgroups, 0 <= unit < units, else XSV_ERR_ARG. */
int xsv_line_partition(int64_t units, int tiles, int workgroups, int workgroup, int64_t* begin, int64_t* end, int64_t unit,
                       int32_t* first, int32_t* last);

/* Host only: what one step does to a cache of `cache_tokens` tokens that has seen `frames_seen` frames, under this
 * configuration (token counting of Sec. 3.2: nothing is pruned while the cache plus the frame fit the budget or on
 * the first frame; otherwise the middle of *middle tokens keeps its *keep best ones beside the first and the current
 * frame).  *new_len = cache length after the step.  Any pointer may be NULL.  The library's own step uses the same
 * routine.  cfg NULL or invalid counts: XSV_ERR_ARG. */
int xsv_step_plan(const xsv_config* cfg, int cache_tokens, int frames_seen, int32_t* middle, int32_t* keep, int32_t* new_len);

/* Measurement aid, synchronous.  The re-quantization leaves out blocks of 64 cached tokens that keep their place
 * (the first frame's, or all old blocks of a cache that is not pruned) once re-quantizing them has reproduced them
 * bit for bit: `settled` = (head, block) pairs of the layer in that state, `total` = (head, block) pairs it holds. */
int xsv_settled_blocks(xsv_ctx* ctx, int layer, int32_t* settled, int32_t* total);

/* Measurement aid, synchronous: two yardsticks of the current device - the rate of a loop of nothing but the bf16
 * MFMA instruction the attention kernel uses (TFLOP/s, all compute units busy) and of a plain streaming copy of
 * 512 MiB (GB/s, bytes read + bytes written).  Allocates and frees 1 GiB of temporaries; takes about 50 ms. */
int xsv_measure_peaks(void* hip_stream, float* mfma_bf16_tflops, float* copy_gbs);

#ifdef __cplusplus
}
#endif
#endif /* XSV_TUNE_H */
