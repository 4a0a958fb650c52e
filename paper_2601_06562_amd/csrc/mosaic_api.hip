// C ABI entry points of libmosaic: argument validation, then enqueue.  See include/mosaic.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "mosaic_internal.h"

// Workspace of mosaic_masked_logits_reduce_static, the entry point for callers that cannot allocate: a fixed
// array in the library's own device image.  Each GPU the library runs on holds its own copy, at its own address,
// until the process ends.  The name is a host-side stand-in, not a device address: host code only ever uses the
// pointer that hipGetSymbolAddress returns for the current device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[MOSAIC_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // resolved once per device, on that device's first call

// Device address of `scratch` on the calling thread's current device.
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOSAIC_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return MOSAIC_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return MOSAIC_OK;
}
}  // namespace

extern "C" {

const char* mosaic_status_string(int status) {
  switch (status) {
    case MOSAIC_OK: return "MOSAIC_OK";
    case MOSAIC_ERR_INVALID_ARG: return "MOSAIC_ERR_INVALID_ARG";
    case MOSAIC_ERR_UNSUPPORTED_SHAPE: return "MOSAIC_ERR_UNSUPPORTED_SHAPE";
    case MOSAIC_ERR_WORKSPACE_TOO_SMALL: return "MOSAIC_ERR_WORKSPACE_TOO_SMALL";
    case MOSAIC_ERR_HIP: return "MOSAIC_ERR_HIP";
    default: return "MOSAIC_ERR_UNKNOWN";
  }
}

int mosaic_version(void) { return 1000; }

int64_t mosaic_compact_scratch_bytes(int64_t T) {
  if (T < 0) return 0;
  return 4 * (mosaic::compact_num_blocks(T) + 4);
}

int mosaic_mask_compact(const uint8_t* mask, int64_t T, int32_t* out_idx, int32_t* out_count, void* scratch,
                        int64_t scratch_bytes, void* stream) {
  if (T < 0 || out_idx == nullptr || out_count == nullptr || scratch == nullptr || (T > 0 && mask == nullptr))
    return MOSAIC_ERR_INVALID_ARG;
  if (T >= (int64_t)1 << 31) return MOSAIC_ERR_UNSUPPORTED_SHAPE;
  if (scratch_bytes < mosaic_compact_scratch_bytes(T) || (reinterpret_cast<uintptr_t>(scratch) & 3u) != 0)
    return MOSAIC_ERR_INVALID_ARG;
  const int rc = mosaic::launch_compact(mask, T, out_idx, out_count, static_cast<int32_t*>(scratch),
                                        static_cast<hipStream_t>(stream));
  return rc == 0 ? MOSAIC_OK : MOSAIC_ERR_HIP;
}

// Argument checks and launch shared by the greedy and the sampling entry points (temperature 0 = greedy).
static int reduce_checked(const void* hidden, int64_t T, int32_t d, int64_t ld_h, const void* w, int32_t V,
                          const int32_t* idx, const int32_t* noise_idx, const int32_t* count, int64_t max_rows,
                          int32_t* out_token,
                          float* out_conf, float* out_lse, const mosaic_plan* plan, void* workspace,
                          int64_t workspace_bytes, bool static_workspace, float temperature, uint64_t seed,
                          void* stream) {
  if (T < 0 || d <= 0 || V < 0 || max_rows < 0 || max_rows > T || plan == nullptr || count == nullptr)
    return MOSAIC_ERR_INVALID_ARG;
  if (T >= (int64_t)1 << 31 || (int64_t)V >= ((int64_t)1 << 31) - MOSAIC_VOCAB_TILE || d % MOSAIC_K_TILE != 0 ||
      ld_h < d || ld_h % 8 != 0)
    return MOSAIC_ERR_UNSUPPORTED_SHAPE;
  if (max_rows == 0 || V == 0) return MOSAIC_OK;
  if (hidden == nullptr || w == nullptr || idx == nullptr || out_token == nullptr || out_conf == nullptr ||
      out_lse == nullptr || (workspace == nullptr && !static_workspace))
    return MOSAIC_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(hidden) & 15u) || (reinterpret_cast<uintptr_t>(w) & 15u) ||
      (reinterpret_cast<uintptr_t>(workspace) & 15u))
    return MOSAIC_ERR_INVALID_ARG;
  // The plan must be one the selector could have produced for these sizes.
  const int64_t vocab_tiles = ((int64_t)V + MOSAIC_VOCAB_TILE - 1) / MOSAIC_VOCAB_TILE;
  if (plan->num_chunks < 1 || plan->rows_per_chunk < MOSAIC_ROW_TILE || plan->rows_per_chunk % MOSAIC_ROW_TILE != 0 ||
      plan->vocab_splits < 1 || plan->vocab_splits > MOSAIC_MAX_VOCAB_SPLITS || plan->vocab_splits > vocab_tiles ||
      plan->tile_panel < 1 || plan->grid < 1 || (int64_t)plan->num_chunks * plan->rows_per_chunk < max_rows)
    return MOSAIC_ERR_INVALID_ARG;
  // 12 bytes per row and split for a greedy pass, 20 for a sampling one -- whatever the plan was made for.
  const int64_t need = temperature > 0.f ? mosaic::sample_partials_bytes(plan->rows_per_chunk, plan->vocab_splits)
                                         : mosaic::partials_bytes(plan->rows_per_chunk, plan->vocab_splits);
  if (plan->workspace_bytes < mosaic::partials_bytes(plan->rows_per_chunk, plan->vocab_splits))
    return MOSAIC_ERR_WORKSPACE_TOO_SMALL;
  if (static_workspace) {   // the library's own fixed array: the plan must fit it, nothing is allocated
    if (need > MOSAIC_STATIC_WORKSPACE_BYTES) return MOSAIC_ERR_WORKSPACE_TOO_SMALL;
    const int rc = static_scratch(&workspace);
    if (rc != MOSAIC_OK) return rc;
    workspace_bytes = MOSAIC_STATIC_WORKSPACE_BYTES;
  }
  if (workspace_bytes < need) return MOSAIC_ERR_WORKSPACE_TOO_SMALL;

  mosaic::LogitsArgs a;
  a.hidden = hidden;
  a.T = T;
  a.ld_h = ld_h;
  a.w = w;
  a.d = d;
  a.V = V;
  a.idx = idx;
  a.noise_idx = noise_idx;
  a.count = count;
  a.max_rows = max_rows;
  a.out_token = out_token;
  a.out_conf = out_conf;
  a.out_lse = out_lse;
  a.workspace = workspace;
  a.temperature = temperature;
  a.seed = seed;
  const int rc = mosaic::launch_masked_logits(a, *plan, static_cast<hipStream_t>(stream));
  return rc == 0 ? MOSAIC_OK : MOSAIC_ERR_HIP;
}

int mosaic_masked_logits_reduce(const void* hidden, int64_t T, int32_t d, int64_t ld_h, const void* w, int32_t V,
                                const int32_t* idx, const int32_t* count, int64_t max_rows, int32_t* out_token,
                                float* out_conf, float* out_lse, const mosaic_plan* plan, void* workspace,
                                int64_t workspace_bytes, void* stream) {
  return reduce_checked(hidden, T, d, ld_h, w, V, idx, nullptr, count, max_rows, out_token, out_conf, out_lse, plan,
                        workspace, workspace_bytes, false, 0.f, 0, stream);
}

int mosaic_masked_logits_reduce_static(const void* hidden, int64_t T, int32_t d, int64_t ld_h, const void* w, int32_t V,
                                       const int32_t* idx, const int32_t* count, int64_t max_rows, int32_t* out_token,
                                       float* out_conf, float* out_lse, const mosaic_plan* plan, void* stream) {
  return reduce_checked(hidden, T, d, ld_h, w, V, idx, nullptr, count, max_rows, out_token, out_conf, out_lse, plan,
                        nullptr, 0, true, 0.f, 0, stream);
}

const char* mosaic_masked_logits_kernel_name(int64_t T, int32_t d, int64_t ld_h, int32_t V, const mosaic_plan* plan,
                                             int32_t sampling) {
  if (plan == nullptr || T < 0 || d <= 0 || V <= 0 || ld_h < d) return "";
  return mosaic::masked_logits_kernel_name(T, ld_h, d, V, *plan, sampling != 0);
}

int64_t mosaic_sample_workspace_bytes(const mosaic_plan* plan) {
  if (plan == nullptr || plan->rows_per_chunk < 1 || plan->vocab_splits < 1) return 0;
  return mosaic::sample_partials_bytes(plan->rows_per_chunk, plan->vocab_splits);
}

int mosaic_masked_logits_sample(const void* hidden, int64_t T, int32_t d, int64_t ld_h, const void* w, int32_t V,
                                const int32_t* idx, const int32_t* noise_idx, const int32_t* count, int64_t max_rows,
                                float temperature, uint64_t seed, int32_t* out_token, float* out_conf, float* out_lse,
                                const mosaic_plan* plan, void* workspace, int64_t workspace_bytes, void* stream) {
  if (!(temperature >= 0.f) || temperature > 1e30f) return MOSAIC_ERR_INVALID_ARG;   // also rejects NaN
  return reduce_checked(hidden, T, d, ld_h, w, V, idx, noise_idx, count, max_rows, out_token, out_conf, out_lse, plan,
                        workspace, workspace_bytes, false, temperature, seed, stream);
}

int64_t mosaic_mfma_probe_flops(int32_t iters, int32_t num_wgs) {
  if (iters < 0 || num_wgs < 0) return 0;
  return (int64_t)num_wgs * 4 * 64 * 16384 * (int64_t)iters;   // 4 waves, 64 instructions of 16*16*32*2 flop
}

int mosaic_mfma_probe(const void* operands, float* sink, int32_t iters, int32_t num_wgs, void* stream) {
  if (operands == nullptr || sink == nullptr || iters < 1 || iters > (1 << 20) || num_wgs < 1 || num_wgs > 65536 ||
      (reinterpret_cast<uintptr_t>(operands) & 15u))
    return MOSAIC_ERR_INVALID_ARG;
  const int rc = mosaic::launch_mfma_probe(operands, sink, iters, num_wgs, static_cast<hipStream_t>(stream));
  return rc == 0 ? MOSAIC_OK : MOSAIC_ERR_HIP;
}

int mosaic_unmask_topn(const float* conf, const int32_t* token, const int32_t* idx, const int32_t* count,
                       int64_t max_rows, const int32_t* seq_starts, int32_t num_seqs, const int32_t* n_per_seq,
                       int32_t* tokens, uint8_t* mask, int64_t T, void* stream) {
  if (T < 0 || max_rows < 0 || max_rows > T || num_seqs < 1 || count == nullptr || seq_starts == nullptr ||
      n_per_seq == nullptr)
    return MOSAIC_ERR_INVALID_ARG;
  if (T >= (int64_t)1 << 31) return MOSAIC_ERR_UNSUPPORTED_SHAPE;
  if (max_rows == 0) return MOSAIC_OK;
  if (conf == nullptr || token == nullptr || idx == nullptr || tokens == nullptr || mask == nullptr)
    return MOSAIC_ERR_INVALID_ARG;
  const int rc = mosaic::launch_unmask_topn(conf, token, idx, count, max_rows, seq_starts, num_seqs, n_per_seq, tokens,
                                            mask, T, static_cast<hipStream_t>(stream));
  return rc == 0 ? MOSAIC_OK : MOSAIC_ERR_HIP;
}

int mosaic_shift_indices(const int32_t* idx, const int32_t* count, int64_t max_rows, const int32_t* seq_starts,
                         int32_t num_seqs, int32_t* out_gather, void* stream) {
  if (max_rows < 0 || num_seqs < 1 || count == nullptr || seq_starts == nullptr) return MOSAIC_ERR_INVALID_ARG;
  if (max_rows >= (int64_t)1 << 31) return MOSAIC_ERR_UNSUPPORTED_SHAPE;
  if (max_rows == 0) return MOSAIC_OK;
  if (idx == nullptr || out_gather == nullptr) return MOSAIC_ERR_INVALID_ARG;
  const int rc = mosaic::launch_shift_indices(idx, count, max_rows, seq_starts, num_seqs, out_gather,
                                              static_cast<hipStream_t>(stream));
  return rc == 0 ? MOSAIC_OK : MOSAIC_ERR_HIP;
}

}  // extern "C"
