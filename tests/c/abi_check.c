/* Plain C99 translation unit against include/xsv.h and include/xsv_tune.h: both headers must compile as C, and every
 * entry point must link.  Calls only what needs no GPU: the error strings and the argument checks of NULL contexts. */
#include <stdio.h>
#include <string.h>

#include "xsv.h"
#include "xsv_tune.h"

int main(void) {
  xsv_config cfg;
  xsv_tensor t;
  /* the addresses of all entry points: a missing symbol fails the link */
  typedef void (*fn)(void);
  const fn entry[] = {(fn)xsv_create, (fn)xsv_destroy, (fn)xsv_reset,
                         (fn)xsv_dequant_attend, (fn)xsv_frame_attend, (fn)xsv_score_prune,
                         (fn)xsv_quantize, (fn)xsv_step, (fn)xsv_step_all_layers,
                         (fn)xsv_cache_len, (fn)xsv_cache_export, (fn)xsv_cache_import,
                         (fn)xsv_last_selection, (fn)xsv_quantize_k, (fn)xsv_quantize_v,
                         (fn)xsv_score, (fn)xsv_score_noalloc, (fn)xsv_topk_keep, (fn)xsv_join,
                         (fn)xsv_set_overlap, (fn)xsv_strerror,
                         /* xsv_tune.h */
                         (fn)xsv_set_attend_splits, (fn)xsv_set_attend_variant, (fn)xsv_set_side_cus,
                         (fn)xsv_set_short_range, (fn)xsv_set_frame_tile_cost, (fn)xsv_last_attend_workgroups, (fn)xsv_settled_blocks, (fn)xsv_set_attend_timing,
                         (fn)xsv_attend_times, (fn)xsv_chain_times, (fn)xsv_measure_peaks, (fn)xsv_key_ranges, (fn)xsv_line_partition, (fn)xsv_step_plan};
  size_t i;
  memset(&cfg, 0, sizeof cfg);
  memset(&t, 0, sizeof t);
  for (i = 0; i < sizeof entry / sizeof entry[0]; ++i)
    if (!entry[i]) return 1;
  if (strcmp(xsv_strerror(XSV_OK), "ok") != 0) return 2;
  if (xsv_step(NULL, 0, t, t, t, NULL) != XSV_ERR_ARG) return 3;
  if (xsv_create(NULL, NULL, NULL) != XSV_ERR_ARG) return 4;
  if (xsv_destroy(NULL) != XSV_OK) return 5;
  if (xsv_set_attend_splits(NULL, 0, 0) != XSV_ERR_ARG) return 6;
  if (xsv_measure_peaks(NULL, NULL, NULL) != XSV_ERR_ARG) return 7;
  if (xsv_key_ranges(64, 22, 5, 50, 95, NULL) != XSV_ERR_ARG) return 8;
  printf("abi ok: %u entry points, config %u bytes, tensor %u bytes\n", (unsigned)(sizeof entry / sizeof entry[0]),
         (unsigned)sizeof cfg, (unsigned)sizeof t);
  return 0;
}
