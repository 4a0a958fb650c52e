// Host-side chunk-size selector for the mask-only logits path.
//
// Paper section 4.4: chunking of the logits operator along the sequence dimension is off by
// default and switched on only when memory is short; the search raises the chunk count of
// the operator that forms the peak by one, re-evaluates the footprint, and stops at the first
// configuration that fits, or fails when only non-chunkable memory is left.  On this path the one
// chunkable buffer is the array of partial (max, sum-exp, arg-max) triples, 12 bytes per row and
// vocabulary split (20 when the step samples with a temperature: two more values per partial), plus a fixed
// MOSAIC_SYNC_BYTES of round counters; its non-chunkable floor is one row tile with one split.
#include <stdint.h>

#include "mosaic_internal.h"

namespace mosaic {

// Workspace of one chunk: the partial results plus the round counters of the persistent grid.
int64_t partials_bytes(int64_t rows_padded, int32_t splits) {
  return 12 * rows_padded * (int64_t)splits + MOSAIC_SYNC_BYTES;
}
// sampling keeps two more planes per row and split (best perturbed score, the plain logit there)
int64_t sample_partials_bytes(int64_t rows_padded, int32_t splits) {
  return 20 * rows_padded * (int64_t)splits + MOSAIC_SYNC_BYTES;
}

// Number of vocabulary splits for `row_tiles` row tiles: the workgroups walk their units in rounds of
// `num_cus`; a round lasts as long as its longest unit.  Pick the S that minimises
// rounds * (tiles per unit + a fixed per-unit cost), the smallest S on ties.
int32_t choose_vocab_splits(int64_t row_tiles, int64_t vocab_tiles, int32_t num_cus) {
  if (row_tiles <= 0 || vocab_tiles <= 0) return 1;
  int64_t smax = vocab_tiles < MOSAIC_MAX_VOCAB_SPLITS ? vocab_tiles : MOSAIC_MAX_VOCAB_SPLITS;
  // At least four splits where the vocabulary allows: the 32 workgroups that share an L2 then work on 8 row tiles x
  // 4 splits.  With fewer splits they spread over more row tiles, whose hidden tiles no longer share the cache
  // (256 row tiles in one split each: 62 ms; in four: 47 ms).
  const int64_t smin = smax < 4 ? smax : 4;
  int32_t best = (int32_t)smin;
  int64_t best_cost = -1;
  for (int64_t s = smin; s <= smax; ++s) {
    const int64_t units = row_tiles * s;
    const int64_t rounds = (units + num_cus - 1) / num_cus;
    const int64_t longest = (vocab_tiles + s - 1) / s;
    const int64_t cost = rounds * (2 * longest + 1);  // half-tile units: pipeline fill, merge and partials of a unit ~ 1/2 tile
    if (best_cost < 0 || cost < best_cost) {
      best_cost = cost;
      best = (int32_t)s;
    }
  }
  return best;
}

// Which kernel(s) serve a call.  The hand-scheduled 4-wave kernel needs whole vocabulary tiles and addresses the 64
// rows a wave copies by 32-bit offsets from the lowest of them: always possible in a hidden tensor smaller than
// 4 GiB, and in a larger one unless such a group of rows lies 4 GiB or more apart, which only the device can tell
// (`wide`: both kernels are launched and a flag decides).  A vocabulary with a ragged last tile is covered by a pair
// of launches: the 4-wave kernel on the whole tiles with S - 1 splits and the general 8-wave kernel on the last
// tile as split S - 1.  Everything else (and plans that ask for it) goes to the general kernel alone.
KernelChoice choose_kernel(int64_t T, int64_t ld_h, int32_t d, int32_t V, const mosaic_plan& plan) {
  const int64_t vocab_tiles = ((int64_t)V + MOSAIC_VOCAB_TILE - 1) / MOSAIC_VOCAB_TILE;
  const bool fast_ok = (plan.flags & MOSAIC_PLAN_GENERAL_KERNEL) == 0 &&
                       (uint64_t)MOSAIC_VOCAB_TILE * (uint64_t)d * 2u < ((uint64_t)1 << 32);
  KernelChoice c;
  c.fast = fast_ok && V % MOSAIC_VOCAB_TILE == 0;
  c.paired = fast_ok && !c.fast && vocab_tiles >= 2 && plan.vocab_splits >= 2;
  c.wide = (c.fast || c.paired) && (uint64_t)T * (uint64_t)(ld_h * 2) >= ((uint64_t)1 << 32);
  return c;
}

const char* masked_logits_kernel_name(int64_t T, int64_t ld_h, int32_t d, int32_t V, const mosaic_plan& plan,
                                      bool sample) {
  const KernelChoice c = choose_kernel(T, ld_h, d, V, plan);
  if (c.wide)
    return sample ? "masked_logits_kernel_w4<true>, or masked_logits_kernel<3,2,true> where 64 consecutive rows of "
                    "the list lie 4 GiB apart (decided on the device)"
                  : "masked_logits_kernel_w4<false>, or masked_logits_kernel<3,2,false> where 64 consecutive rows of "
                    "the list lie 4 GiB apart (decided on the device)";
  if (c.fast) return sample ? "masked_logits_kernel_w4<true>" : "masked_logits_kernel_w4<false>";
  if (c.paired)
    return sample ? "masked_logits_kernel_w4<true> + masked_logits_kernel<3,2,true> (ragged last vocabulary tile)"
                  : "masked_logits_kernel_w4<false> + masked_logits_kernel<3,2,false> (ragged last vocabulary tile)";
  return sample ? "masked_logits_kernel<3,2,true>" : "masked_logits_kernel<3,2,false>";
}

}  // namespace mosaic

extern "C" int mosaic_plan_workspace(int64_t T, int64_t max_rows, int32_t d, int32_t V, int64_t budget_bytes,
                                     int32_t num_cus, int32_t sampling, mosaic_plan* out_plan) {
  using namespace mosaic;
  if (out_plan == nullptr || T < 0 || max_rows < 0 || max_rows > T || d <= 0 || V < 0 || (sampling != 0 && sampling != 1))
    return MOSAIC_ERR_INVALID_ARG;
  if (T >= (int64_t)1 << 31 || (int64_t)V >= ((int64_t)1 << 31) - MOSAIC_VOCAB_TILE || d % MOSAIC_K_TILE != 0)
    return MOSAIC_ERR_UNSUPPORTED_SHAPE;
  if (num_cus <= 0) num_cus = 256;
  const int64_t vocab_tiles = ((int64_t)V + MOSAIC_VOCAB_TILE - 1) / MOSAIC_VOCAB_TILE;
  const int64_t rows = max_rows > 0 ? max_rows : 1;

  for (int64_t K = 1;; ++K) {
    const int64_t per = (rows + K - 1) / K;
    const int64_t C = (per + MOSAIC_ROW_TILE - 1) / MOSAIC_ROW_TILE * MOSAIC_ROW_TILE;
    const int64_t row_tiles = C / MOSAIC_ROW_TILE;
    // A vocabulary with a ragged last tile is run as a pair of launches: the whole tiles in S - 1 splits chosen to
    // fill the chip, the last tile as one more split.
    const bool ragged = V % MOSAIC_VOCAB_TILE != 0 && vocab_tiles >= 2;
    int64_t S = ragged ? choose_vocab_splits(row_tiles, vocab_tiles - 1, num_cus) + 1
                       : choose_vocab_splits(row_tiles, vocab_tiles, num_cus);
    if (S > MOSAIC_MAX_VOCAB_SPLITS) S = MOSAIC_MAX_VOCAB_SPLITS;
    if (budget_bytes > 0) {
      // splits the budget allows (a sampling step keeps 20 bytes per row and split, a greedy one 12)
      const int64_t per_split = (sampling ? 20 : 12) * C;
      const int64_t fit = budget_bytes > MOSAIC_SYNC_BYTES ? (budget_bytes - MOSAIC_SYNC_BYTES) / per_split : 0;
      if (fit < S) S = fit;
    }
    if (S >= 1) {
      out_plan->workspace_bytes = sampling ? sample_partials_bytes(C, (int32_t)S) : partials_bytes(C, (int32_t)S);
      out_plan->num_chunks = (int32_t)((rows + C - 1) / C);  // chunks that actually hold rows
      out_plan->rows_per_chunk = (int32_t)C;
      out_plan->vocab_splits = (int32_t)S;
      out_plan->tile_panel = (int32_t)(row_tiles <= 8 ? row_tiles : 8);
      int64_t grid = row_tiles * S;
      if (grid > num_cus) grid = num_cus;
      out_plan->grid = (int32_t)grid;
      out_plan->flags = sampling ? MOSAIC_PLAN_SAMPLING : 0;
      return MOSAIC_OK;
    }
    if (C == MOSAIC_ROW_TILE) return MOSAIC_ERR_WORKSPACE_TOO_SMALL;  // nothing left to chunk
  }
}
