// Stream compaction of the mask into ascending indices of masked positions.
//
// Paper section 4.2: the gather-GEMM kernel takes the list of masked positions as an input;
// the paper leaves its production to the framework.  Here it is an explicit
// exclusive prefix sum over (mask[t] != 0) followed by a scatter that never touches the host:
// one single-block launch for up to 65536 positions (a denoising step of one long sequence),
// otherwise three small launches (per-block counts, a scan of those counts, the scatter).
// Integer work only; the result is unique (stable order), so it is bit-exact by construction.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mosaic_internal.h"

namespace mosaic {

constexpr int kCompactThreads = 256;
constexpr int kBytesPerThread = 16;
constexpr int kCompactBlockElems = kCompactThreads * kBytesPerThread;  // 4096 positions per block
static_assert(kCompactBlockElems == kCompactBlockPositions, "the scratch size is computed from this constant");

// Loads the 16 mask bytes a thread owns as a bit set (bit j = mask[base + j] != 0).
__device__ __forceinline__ uint32_t load_flags(const uint8_t* __restrict__ mask, int64_t base, int64_t T,
                                               bool aligned16) {
  uint32_t bits = 0;
  if (base + kBytesPerThread <= T && aligned16) {
    const uint4 q = *reinterpret_cast<const uint4*>(mask + base);
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int b = 0; b < 4; ++b) bits |= (((w[i] >> (8 * b)) & 0xffu) != 0u ? 1u : 0u) << (4 * i + b);
    }
  } else {
#pragma unroll
    for (int j = 0; j < kBytesPerThread; ++j) {
      if (base + j < T) bits |= (mask[base + j] != 0 ? 1u : 0u) << j;
    }
  }
  return bits;
}

// Inclusive scan of one int per thread over a block of THREADS threads: wave shuffles, then the wave totals.
template <int THREADS = kCompactThreads>
__device__ __forceinline__ int block_inclusive_scan(int v, int* wave_totals /* LDS, THREADS/64 ints */,
                                                    int* block_total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(v, off, 64);
    if (lane >= off) v += up;
  }
  if (lane == 63) wave_totals[wave] = v;
  __syncthreads();
  int before = 0, total = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) {
    const int t = wave_totals[w];
    if (w < wave) before += t;
    total += t;
  }
  *block_total = total;
  return v + before;
}

__global__ __launch_bounds__(kCompactThreads) void compact_count_kernel(const uint8_t* __restrict__ mask, int64_t T,
                                                                        int32_t* __restrict__ block_counts) {
  __shared__ int wave_totals[kCompactThreads / 64];
  const bool aligned16 = (reinterpret_cast<uintptr_t>(mask) & 15u) == 0;
  const int64_t base = (int64_t)blockIdx.x * kCompactBlockElems + (int64_t)threadIdx.x * kBytesPerThread;
  const int c = __popc(load_flags(mask, base, T, aligned16));
  int total;
  (void)block_inclusive_scan(c, wave_totals, &total);
  if (threadIdx.x == 0) block_counts[blockIdx.x] = total;
}

// One block: block_counts[0..nb) -> exclusive offsets in place; the grand total goes to *out_count.
__global__ __launch_bounds__(1024) void compact_scan_kernel(int32_t* __restrict__ block_counts, int64_t nb,
                                                             int32_t* __restrict__ out_count) {
  __shared__ int part[1024];
  const int tid = threadIdx.x;
  const int64_t per = (nb + 1023) / 1024;
  const int64_t lo = (int64_t)tid * per, hi = (lo + per < nb) ? lo + per : nb;
  int sum = 0;
  for (int64_t i = lo; i < hi; ++i) sum += block_counts[i];
  part[tid] = sum;
  __syncthreads();
  // Hillis-Steele inclusive scan over the 1024 per-thread sums.
  for (int off = 1; off < 1024; off <<= 1) {
    int add = (tid >= off) ? part[tid - off] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  int run = part[tid] - sum;  // exclusive prefix of this thread's slice
  for (int64_t i = lo; i < hi; ++i) {
    const int c = block_counts[i];
    block_counts[i] = run;
    run += c;
  }
  if (tid == 1023) *out_count = part[1023];
}

__global__ __launch_bounds__(kCompactThreads) void compact_scatter_kernel(const uint8_t* __restrict__ mask, int64_t T,
                                                                          const int32_t* __restrict__ block_offsets,
                                                                          int32_t* __restrict__ out_idx) {
  __shared__ int wave_totals[kCompactThreads / 64];
  const bool aligned16 = (reinterpret_cast<uintptr_t>(mask) & 15u) == 0;
  const int64_t base = (int64_t)blockIdx.x * kCompactBlockElems + (int64_t)threadIdx.x * kBytesPerThread;
  uint32_t bits = load_flags(mask, base, T, aligned16);
  const int c = __popc(bits);
  int total;
  const int incl = block_inclusive_scan(c, wave_totals, &total);
  int64_t out = (int64_t)block_offsets[blockIdx.x] + (incl - c);
  while (bits) {
    const int j = __ffs(bits) - 1;
    bits &= bits - 1;
    out_idx[out++] = (int32_t)(base + j);
  }
}

// Everything in one block, for masks of up to kSingleMax positions: passes of 16384 positions, the running
// offset carried from pass to pass.  One launch instead of three where launches are all the cost.
constexpr int kSingleThreads = 1024;
constexpr int64_t kSingleMax = 65536;
__global__ __launch_bounds__(kSingleThreads) void compact_single_kernel(const uint8_t* __restrict__ mask, int64_t T,
                                                                        int32_t* __restrict__ out_idx,
                                                                        int32_t* __restrict__ out_count) {
  __shared__ int wave_totals[kSingleThreads / 64];
  const bool aligned16 = (reinterpret_cast<uintptr_t>(mask) & 15u) == 0;
  int running = 0;
  for (int64_t pass0 = 0; pass0 < T; pass0 += (int64_t)kSingleThreads * kBytesPerThread) {
    const int64_t base = pass0 + (int64_t)threadIdx.x * kBytesPerThread;
    uint32_t bits = load_flags(mask, base, T, aligned16);
    const int c = __popc(bits);
    int total;
    const int incl = block_inclusive_scan<kSingleThreads>(c, wave_totals, &total);
    int out = running + incl - c;
    while (bits) {
      const int j = __ffs(bits) - 1;
      bits &= bits - 1;
      out_idx[out++] = (int32_t)(base + j);
    }
    running += total;
    __syncthreads();   // the wave totals are rewritten by the next pass
  }
  if (threadIdx.x == 0) *out_count = running;
}

int launch_compact(const uint8_t* mask, int64_t T, int32_t* out_idx, int32_t* out_count, int32_t* block_counts,
                   hipStream_t stream) {
  if (T <= kSingleMax) {
    return launch_kernel(compact_single_kernel, dim3(1), dim3(kSingleThreads), stream, mask, T, out_idx, out_count);
  }
  const int64_t nb = compact_num_blocks(T);
  int rc = 0;
  if (nb > 0)
    rc |= launch_kernel(compact_count_kernel, dim3((unsigned)nb), dim3(kCompactThreads), stream, mask, T, block_counts);
  // nb == 0 still has to publish count = 0.
  rc |= launch_kernel(compact_scan_kernel, dim3(1), dim3(1024), stream, block_counts, nb, out_count);
  if (nb > 0)
    rc |= launch_kernel(compact_scatter_kernel, dim3((unsigned)nb), dim3(kCompactThreads), stream, mask, T, block_counts,
                        out_idx);
  return rc;
}

}  // namespace mosaic
