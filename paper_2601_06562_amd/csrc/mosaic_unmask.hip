// The tail of a denoising step, after mask-only logits: pick the positions to unmask and write their
// tokens (paper section 2.1: a step's drawn tokens replace a chosen subset of the still-masked positions;
// which subset is left open), and the index shift of Dream-style prediction (section 4.5, last paragraph).
// Integer / byte work: results are bit-exact by construction.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mosaic_internal.h"

namespace mosaic {

constexpr int kUnmaskThreads = 1024;

// First row j in [0, n) with idx[j] >= pos (idx ascending).
__device__ __forceinline__ int lower_bound_rows(const int32_t* __restrict__ idx, int n, int pos) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (idx[mid] < pos) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// Exclusive scan of one 0/1 flag per thread over the block, in thread order.  Returns the exclusive
// prefix; *total receives the block total.  wave_tot: LDS, one int per wave.
__device__ __forceinline__ int block_exclusive_scan_flag(int flag, int* wave_tot, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t ballot = __ballot(flag);
  const int excl = __popcll(ballot & ((1ull << lane) - 1ull));
  if (lane == 0) wave_tot[wave] = __popcll(ballot);
  __syncthreads();
  int before = 0, tot = 0;
  for (int w = 0; w < kUnmaskThreads / 64; ++w) {
    const int t = wave_tot[w];
    if (w < wave) before += t;
    tot += t;
  }
  __syncthreads();  // wave_tot is reused by the next call
  *total = tot;
  return before + excl;
}

// One block per sequence: exact top-n by confidence (ties: lower position) through a 4-pass radix
// select on the float bit patterns (confidences are non-negative, so the patterns order like the values).
__global__ __launch_bounds__(kUnmaskThreads) void unmask_topn_kernel(
    const float* __restrict__ conf, const int32_t* __restrict__ token, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ count, int32_t max_rows, const int32_t* __restrict__ seq_starts,
    const int32_t* __restrict__ n_per_seq, int32_t* __restrict__ tokens, uint8_t* __restrict__ mask, int32_t T) {
  __shared__ int hist[256];
  __shared__ int wave_tot[kUnmaskThreads / 64];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_need;
  const int b = blockIdx.x, tid = threadIdx.x;
  int total = *count;
  if (total > max_rows) total = max_rows;
  const int lo = lower_bound_rows(idx, total, seq_starts[b]);
  const int hi = lower_bound_rows(idx, total, seq_starts[b + 1]);
  const int m = hi - lo;
  int n = n_per_seq[b];
  if (n > m) n = m;
  if (n <= 0) return;
  const uint32_t* keys = reinterpret_cast<const uint32_t*>(conf);

  uint32_t prefix = 0;   // bytes of the threshold key decided so far
  int need = n;          // rows still to find among keys matching the prefix
  if (n < m) {
    for (int pass = 3; pass >= 0; --pass) {
      const int shift = 8 * pass;
      const uint32_t high_mask = (pass == 3) ? 0u : (0xffffffffu << (shift + 8));
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      for (int j = lo + tid; j < hi; j += kUnmaskThreads) {
        const uint32_t k = keys[j];
        if ((k & high_mask) == prefix) atomicAdd(&hist[(k >> shift) & 0xffu], 1);
      }
      __syncthreads();
      if (tid == 0) {
        int above = 0, byte = 255;
        for (; byte > 0; --byte) {          // largest byte value whose "at least" count reaches need
          if (above + hist[byte] >= need) break;
          above += hist[byte];
        }
        sh_prefix = prefix | ((uint32_t)byte << shift);
        sh_need = need - above;
      }
      __syncthreads();
      prefix = sh_prefix;
      need = sh_need;
      __syncthreads();
    }
  }
  // Rows above the threshold key are taken; of the rows equal to it, the first `need` in position order.
  int base = 0;
  for (int j0 = lo; j0 < hi; j0 += kUnmaskThreads) {
    const int j = j0 + tid;
    const bool valid = j < hi;
    const uint32_t k = valid ? keys[j] : 0u;
    const bool all = (n == m);
    const int eq = (valid && !all && k == prefix) ? 1 : 0;
    int eq_total;
    const int rank = base + block_exclusive_scan_flag(eq, wave_tot, &eq_total);
    base += eq_total;
    const bool take = valid && (all || k > prefix || (eq && rank < need));
    if (take) {
      const int t = idx[j];
      if (t >= 0 && t < T) {   // an entry outside [0, T) of a caller-built list is skipped, never written through
        tokens[t] = token[j];
        mask[t] = 0;
      }
    }
  }
}

// gather[j] = idx[j] - 1, except where idx[j] is the first position of its sequence.
__global__ __launch_bounds__(256) void shift_indices_kernel(const int32_t* __restrict__ idx,
                                                            const int32_t* __restrict__ count, int32_t max_rows,
                                                            const int32_t* __restrict__ seq_starts, int32_t num_seqs,
                                                            int32_t* __restrict__ gather) {
  int total = *count;
  if (total > max_rows) total = max_rows;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= total) return;
  const int pos = idx[j];
  int lo = 0, hi = num_seqs;            // largest b with seq_starts[b] <= pos
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (seq_starts[mid] <= pos) lo = mid; else hi = mid;
  }
  int g = (seq_starts[lo] == pos) ? pos : pos - 1;
  const int last = seq_starts[num_seqs] - 1;   // T - 1: an out-of-range entry is clamped, never passed on
  g = g > last ? last : g;
  gather[j] = g < 0 ? 0 : g;
}

int launch_unmask_topn(const float* conf, const int32_t* token, const int32_t* idx, const int32_t* count,
                       int64_t max_rows, const int32_t* seq_starts, int32_t num_seqs, const int32_t* n_per_seq,
                       int32_t* tokens, uint8_t* mask, int64_t T, hipStream_t stream) {
  return launch_kernel(unmask_topn_kernel, dim3((unsigned)num_seqs), dim3(kUnmaskThreads), stream, conf, token, idx,
                       count, (int32_t)max_rows, seq_starts, n_per_seq, tokens, mask, (int32_t)T);
}

int launch_shift_indices(const int32_t* idx, const int32_t* count, int64_t max_rows, const int32_t* seq_starts,
                         int32_t num_seqs, int32_t* gather, hipStream_t stream) {
  return launch_kernel(shift_indices_kernel, dim3((unsigned)((max_rows + 255) / 256)), dim3(256), stream, idx, count,
                       (int32_t)max_rows, seq_starts, num_seqs, gather);
}

}  // namespace mosaic
