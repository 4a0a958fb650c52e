// Measurement aid: a register-only loop of the MFMA instruction the fused kernel is built on.  It reads 64 KiB
// of operands once, then issues nothing but matrix instructions, so its rate is what the matrix cores sustain
// at the clock the chip settles to under that load -- the practical ceiling the fused kernel is compared with,
// next to the datasheet peak.
#include "mosaic_internal.h"

namespace mosaic {
namespace {

using bf16x8 = __attribute__((ext_vector_type(8))) __bf16;
using f32x4 = __attribute__((ext_vector_type(4))) float;

// One wave per SIMD, an 8 x 8 grid of 16x16 accumulator blocks (the fused kernel's register tile): 64
// independent v_mfma_f32_16x16x32_bf16 per iteration and wave.
__global__ __launch_bounds__(256) void mfma_probe_kernel(const bf16x8* __restrict__ operands, float* __restrict__ sink,
                                                         int iters) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = operands[(threadIdx.x + 256 * i) & 4095];
    b[i] = operands[(threadIdx.x + 256 * (i + 8)) & 4095];
  }
  f32x4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) s += (acc[i][j][0] + acc[i][j][1]) + (acc[i][j][2] + acc[i][j][3]);
  sink[(blockIdx.x & 255) * 256 + threadIdx.x] = s;   // keeps the loop alive; the value is of no interest
}

}  // namespace

int launch_mfma_probe(const void* operands, float* sink, int32_t iters, int32_t num_wgs, hipStream_t stream) {
  return launch_kernel(mfma_probe_kernel, dim3((unsigned)num_wgs), dim3(256), stream,
                       static_cast<const bf16x8*>(operands), sink, (int)iters);
}

}  // namespace mosaic
