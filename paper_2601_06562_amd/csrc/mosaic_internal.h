// Internal declarations shared by the translation units of libmosaic (not part of the C ABI).
#ifndef MOSAIC_INTERNAL_H_
#define MOSAIC_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mosaic.h"

namespace mosaic {

// Enqueue a kernel and return THIS launch's status (0 / -1).  hipGetLastError() after a <<<>>> launch would also
// report an error left behind by earlier, unrelated HIP calls of the host program.
template <typename T>
struct launch_arg { using type = T; };
template <typename... P>
inline int launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t stream,
                         typename launch_arg<P>::type... args) {
  void* argv[] = {const_cast<void*>(static_cast<const void*>(&args))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv, 0, stream) == hipSuccess ? 0 : -1;
}

// ---- mask compaction (mosaic_compact.hip)
constexpr int kCompactBlockPositions = 4096;   // mask positions one block of the multi-block path counts and scatters
inline int64_t compact_num_blocks(int64_t T) { return (T + kCompactBlockPositions - 1) / kCompactBlockPositions; }
int launch_compact(const uint8_t* mask, int64_t T, int32_t* out_idx, int32_t* out_count, int32_t* block_counts,
                   hipStream_t stream);

// ---- fused gather-GEMM + vocabulary reduction (mosaic_logits.hip)
struct LogitsArgs {
  const void* hidden;   // bf16 [T, ld_h]
  int64_t T;            // rows of hidden
  int64_t ld_h;         // elements
  const void* w;        // bf16 [V, d]
  int32_t d;
  int32_t V;
  const int32_t* idx;   // hidden row to read per masked row (the masked positions themselves, or a shifted list)
  const int32_t* noise_idx = nullptr;  // sampling: position that keys each row's noise; nullptr = idx
  const int32_t* count; // device scalar M
  int64_t max_rows;
  int32_t* out_token;
  float* out_conf;
  float* out_lse;
  void* workspace;
  float temperature = 0.f;   // > 0: Gumbel-max sampling (needs the 20-byte-per-row-and-split workspace)
  uint64_t seed = 0;
};
int launch_masked_logits(const LogitsArgs& a, const mosaic_plan& plan, hipStream_t stream);
// Which kernel(s) serve a call (host-side decision, mosaic_plan.cpp).
struct KernelChoice {
  bool fast;     // 4-wave kernel alone
  bool paired;   // 4-wave kernel + general kernel on the ragged last vocabulary tile
  bool wide;     // hidden tensor of 4 GiB or more: the 4-wave launch(es) run only where every 64 consecutive rows of
                 // the list lie less than 4 GiB apart (checked on the device); else the general kernel does the work
};
KernelChoice choose_kernel(int64_t T, int64_t ld_h, int32_t d, int32_t V, const mosaic_plan& plan);
// Name(s) of the kernel(s) launch_masked_logits picks for these sizes and this plan (static storage).
const char* masked_logits_kernel_name(int64_t T, int64_t ld_h, int32_t d, int32_t V, const mosaic_plan& plan,
                                      bool sample);

// ---- sampling tail and shifted gather (mosaic_unmask.hip)
int launch_unmask_topn(const float* conf, const int32_t* token, const int32_t* idx, const int32_t* count,
                       int64_t max_rows, const int32_t* seq_starts, int32_t num_seqs, const int32_t* n_per_seq,
                       int32_t* tokens, uint8_t* mask, int64_t T, hipStream_t stream);
int launch_shift_indices(const int32_t* idx, const int32_t* count, int64_t max_rows, const int32_t* seq_starts,
                         int32_t num_seqs, int32_t* gather, hipStream_t stream);

// ---- measurement aid (mosaic_probe.hip)
int launch_mfma_probe(const void* operands, float* sink, int32_t iters, int32_t num_wgs, hipStream_t stream);

// ---- host-side selector (mosaic_plan.cpp)
int32_t choose_vocab_splits(int64_t row_tiles, int64_t vocab_tiles, int32_t num_cus);
int64_t partials_bytes(int64_t rows_padded, int32_t splits);
int64_t sample_partials_bytes(int64_t rows_padded, int32_t splits);

}  // namespace mosaic
#endif
