// Fused gather-GEMM + vocabulary reduction for mask-only logits on gfx950 (MI355X).
//
// Paper section 4.2 describes a gather-GEMM: the kernel gets the hidden states of all positions
// plus the indices of the masked ones, computes row addresses by pointer arithmetic, stages the
// scattered rows in on-chip memory, multiplies, accumulates, and discards each tile -- no gathered
// copy in global memory.  This kernel keeps that idea (the gather is folded into the global->LDS
// copy, one address per lane) and, unlike the paper's kernel, never writes logits either: every
// 256x256 tile of logits lives only in MFMA accumulators and is reduced on the spot to a running
// (max, sum-exp, arg-max) per token row.
//
// Shape of the computation.  The MFMA "A" operand is the LM-head tile (vocabulary ids along the
// instruction's rows), "B" is the gathered hidden tile (token rows along the instruction's columns).
// A lane then owns ONE token per accumulator block (column lane%16 with v_mfma_f32_16x16x32_bf16 in the
// 4-wave kernel, lane%32 with v_mfma_f32_32x32x16_bf16 in the general one) and several vocabulary ids,
// so the reduction over the vocabulary is almost entirely in-register; the cross-lane steps and the
// cross-wave step happen once per work unit, not per tile.
//
// Work decomposition.  A unit is (row tile of 256 masked tokens, vocabulary split); a workgroup (4 waves
// in the hand-scheduled kernel, 8 in the general one) walks the 256-wide vocabulary tiles of its split,
// carrying the running triple in registers, and writes one partial triple per row at the end.  A second
// tiny kernel merges the S partials per row in an order fixed by S (deterministic) and emits token,
// confidence and log-sum-exp.
//
// Sampling.  The SAMPLE instantiations of both kernels draw the token by the Gumbel-max form of categorical
// sampling at temperature tau (paper section 2.1 leaves the sampler open): arg-max of x + tau*g with g from a
// Philox4x32-10 stream keyed by (seed, position, vocabulary id), next to the unperturbed max / sum-exp.
//
// Data movement.  Global->LDS copies use the direct-to-LDS 16-byte loads of gfx950; both tiles are
// K-contiguous ([256 rows][64 k] bf16 = 128 B per row, i.e. whole 128-byte lines per request) and
// 16-byte chunks are XOR-swizzled by row so that the ds_read_b128 operand fetches of 32 consecutive
// rows spread over all LDS banks.  Each operand has its own ring of 32 KiB slots: three for the LM-head
// tiles (two K-tiles ahead), two for the hidden tiles (one ahead) -- 160 KiB, all of a CU's LDS; the
// merge scratch aliases slot 0 at the end of a unit.  One workgroup barrier per K-tile.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>
#include <stdlib.h>

#include "mosaic_internal.h"

namespace mosaic {

using bf16x8 = __attribute__((ext_vector_type(8))) __bf16;
using f32x16 = __attribute__((ext_vector_type(16))) float;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

constexpr int kTileRows = MOSAIC_ROW_TILE;     // masked tokens per tile (MFMA N side)
constexpr int kTileVocab = MOSAIC_VOCAB_TILE;  // vocabulary ids per tile (MFMA M side)
constexpr int kThreads = 512;                  // 8 waves: 2 (vocabulary halves) x 4 (token quarters)
constexpr float kNeg = -1.0e30f;                     // "minus infinity" that survives subtraction
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct KernelParams {
  const char* hidden;
  int64_t ldh_bytes;
  const char* w;
  int32_t d;
  int32_t V;
  const int32_t* idx;        // hidden row to read, per masked row
  const int32_t* noise_idx;  // sampling: the position that keys the row's noise (idx unless the gather is shifted)
  const int32_t* count;
  int32_t T;           // rows of hidden: gather entries are clamped to [0, T)
  int32_t row0;        // first compacted row of this chunk
  int32_t chunk_rows;  // capacity of the chunk (C)
  int32_t max_rows;
  int32_t splits;      // S
  int32_t panel;       // row tiles scheduled side by side
  int32_t vocab_tiles; // vocabulary tiles this launch covers (all ceil(V / 256) of them unless the launch is one of a pair)
  int32_t tile_first;  // first of those tiles
  int32_t split_first; // partial slot of this launch's split 0
  int32_t c_pad;       // row capacity of the partial arrays
  float* part_m;
  float* part_s;
  int32_t* part_i;
  int32_t* out_token;
  float* out_conf;
  float* out_lse;
  // sampling with temperature (tau > 0): two more partial planes and the generator key
  float tau;
  uint32_t seed_lo, seed_hi;
  float* part_ym;   // best perturbed score x + tau*g
  float* part_xa;   // the unperturbed logit at that arg-max
  int32_t* sync;    // round counters of the persistent grid (cleared before the launch), sync_slots of them
  int32_t sync_slots;
  // Hidden tensors of 4 GiB or more.  The 4-wave kernel addresses a wave's 64 rows by 32-bit offsets from the lowest of
  // them, which works unless those rows lie 4 GiB or more apart; a small kernel looks for such a group in the list
  // and raises *wide_flag, and of the two launches that follow (4-wave kernel, general kernel) the one whose
  // wide_run_if differs from the flag returns at once.  nullptr: no such check (the launch always runs).
  const int32_t* wide_flag;
  int32_t wide_run_if;
};

// (m, s, i) monoid: max, sum of exp relative to the max, lowest index attaining the max.
__device__ __forceinline__ void merge_triple(float& m, float& s, int& i, float m2, float s2, int i2) {
  const float mn = fmaxf(m, m2);
  const float a = __builtin_amdgcn_exp2f((m - mn) * kLog2e);
  const float b = __builtin_amdgcn_exp2f((m2 - mn) * kLog2e);
  const bool keep = (m > m2) || (m == m2 && i < i2);
  s = s * a + s2 * b;
  i = keep ? i : i2;
  m = mn;
}

// log-sum-exp pair alone (max, sum of exp relative to the max).
__device__ __forceinline__ void merge_ms(float& m, float& s, float m2, float s2) {
  const float mn = fmaxf(m, m2);
  s = s * __builtin_amdgcn_exp2f((m - mn) * kLog2e) + s2 * __builtin_amdgcn_exp2f((m2 - mn) * kLog2e);
  m = mn;
}

// Sampled candidate: best perturbed score, the plain logit there, its id (lowest id on equal scores).
__device__ __forceinline__ void merge_pick(float& ym, float& xa, int& i, float ym2, float xa2, int i2) {
  const bool keep = (ym > ym2) || (ym == ym2 && i < i2);
  ym = keep ? ym : ym2;
  xa = keep ? xa : xa2;
  i = keep ? i : i2;
}

// tau * Gumbel noise for the four vocabulary ids 4*v4 .. 4*v4+3 of one position.  Philox4x32-10 (Salmon et
// al., SC'11), key = seed, counter = (v4, position, 0, 0); word j -> u = ((word >> 9) + 1/2) * 2^-23 (exact in
// fp32, never 0 or 1); g = -ln(-ln u).  Near u = 1 the inner logarithm comes from the series of -ln(1 - e)
// (e = 1 - u is exact too), where the hardware log2 loses relative accuracy.
__device__ __forceinline__ void gumbel4(uint32_t k0, uint32_t k1, uint32_t pos, uint32_t v4, float tau, float (&n)[4]) {
  uint32_t c0 = v4, c1 = pos, c2 = 0u, c3 = 0u;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
  }
  const uint32_t w[4] = {c0, c1, c2, c3};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t k = w[j] >> 9;
    const float u = ((float)k + 0.5f) * 0x1p-23f;
    const float e = ((float)(8388607u - k) + 0.5f) * 0x1p-23f;   // 1 - u
    const float by_log = -__builtin_amdgcn_logf(u) * kLn2;
    const float by_series = e * (1.0f + e * (0.5f + e * (1.0f / 3.0f)));
    const float inner = (e < 0x1p-8f) ? by_series : by_log;       // -ln u  > 0
    n[j] = -__builtin_amdgcn_logf(inner) * kLn2 * tau;
  }
}

// Workgroups are dealt to the 8 XCDs round-robin by id, and the workgroups of one XCD share an L2.  This maps
// workgroup b of a grid of G to a position such that each XCD's workgroups hold one contiguous range of positions
// (XCD x owns ceil((G - x) / 8) of them), so that consecutive work units -- which share LM-head and hidden tiles --
// meet in one L2.  A bijection on [0, G) for any G.
__device__ __forceinline__ int xcd_contiguous_position(int b, int G) {
  const int x = b & 7;
  int first = 0;
  for (int y = 0; y < x; ++y) first += (G - y + 7) >> 3;
  return first + (b >> 3);
}

// Round alignment of the persistent grid.  A workgroup that takes more than one unit meets the others before each
// further one: the workgroups behind one L2 share LM-head and hidden tiles only while they walk their units in
// step, and once they have drifted apart (units end at slightly different times) every tile is fetched several
// times over; measured on 229 row tiles x 19 splits, 17 rounds: 43.6 ms without, 41.5 ms with the meeting.  It is a
// hint, not a synchronisation anything depends on: the wait is bounded (a workgroup that is not resident, or a
// counter that was never cleared, costs time, never a hang and never a wrong result), and rounds beyond the
// counters provided simply do not meet.
constexpr int kRoundSpins = 256;
__device__ __forceinline__ void meet_before_round(const KernelParams& p, int round, int n_units, int G, int tid) {
  if (p.sync != nullptr && round < p.sync_slots) {
    if (tid == 0) {
      const int left = n_units - G * round;
      const int expect = left > G ? G : left;            // workgroups that have a unit in this round
      int* ctr = p.sync + round;
      __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      for (int spin = 0; spin < kRoundSpins; ++spin) {
        if (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= expect) break;
        __builtin_amdgcn_s_sleep(2);
      }
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void clear_round_counters_kernel(int32_t* sync, int n) {
  if ((int)threadIdx.x < n) sync[threadIdx.x] = 0;
}

// For hidden tensors of 4 GiB or more: raises *flag when some group of 64 consecutive rows of the chunk's list (the
// rows one wave of the 4-wave kernel copies, the last group padded with the last row as that kernel does) spans
// rows whose byte offsets differ by 4 GiB or more.  One wave per group.
__global__ __launch_bounds__(256) void span_check_kernel(const int32_t* idx, const int32_t* count, int32_t row0,
                                                         int32_t chunk_rows, int32_t max_rows, int32_t T,
                                                         int64_t ldh_bytes, int32_t* flag) {
  int total = *count;
  if (total > max_rows) total = max_rows;
  int rows = total - row0;
  if (rows > chunk_rows) rows = chunk_rows;
  const int group = (int)blockIdx.x * 4 + ((int)threadIdx.x >> 6);
  if (rows <= 0 || group * 64 >= rows) return;
  int j = group * 64 + ((int)threadIdx.x & 63);
  if (j > rows - 1) j = rows - 1;
  int t = idx[row0 + j];
  t = t < 0 ? 0 : (t > T - 1 ? T - 1 : t);
  int lo = t, hi = t;
#pragma unroll
  for (int x = 32; x >= 1; x >>= 1) {
    const int a = __shfl_xor(lo, x, 64), b = __shfl_xor(hi, x, 64);
    lo = a < lo ? a : lo;
    hi = b > hi ? b : hi;
  }
  // the offset of a row from the group's lowest, plus the 16-byte chunk inside the row's K-tile, must fit 32 bits
  if (((int)threadIdx.x & 63) == 0 && (uint64_t)(hi - lo) * (uint64_t)ldh_bytes >= ((uint64_t)1 << 32) - 256)
    atomicOr(flag, 1);
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// exp(x - mn) as exp2.  Full tiles fold the subtraction into one fma against nml = -mn*log2(e).  Tail
// tiles hold the kNeg sentinel, whose magnitude would turn the rounding of nml into a huge exponent, so
// they subtract first (exact zero when x == mn).
template <bool TAIL>
__device__ __forceinline__ float exp_rel(float x, float mn, float nml) {
  if constexpr (TAIL) return __builtin_amdgcn_exp2f((x - mn) * kLog2e);
  else return __builtin_amdgcn_exp2f(__builtin_fmaf(x, kLog2e, nml));
}

// Reduce one finished 256x256 logits tile (this wave's 128 vocabulary ids x 64 tokens) into the
// lane's running triples.  vb = vocabulary id of this lane's element (block 0, register 0).
template <bool TAIL>
__device__ __forceinline__ void reduce_tile(f32x16 (&acc)[4][2], float (&m)[2], float (&s)[2], int (&ix)[2], int vb,
                                            int V) {
#pragma unroll
  for (int bj = 0; bj < 2; ++bj) {
    float mt = kNeg;
#pragma unroll
    for (int bi = 0; bi < 4; ++bi) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int code = bi * 32 + 8 * (r >> 2) + (r & 3);
        if (TAIL) {
          if (vb + code >= V) acc[bi][bj][r] = kNeg;
        }
        mt = fmaxf(mt, acc[bi][bj][r]);
      }
    }
    int sel = 0;
#pragma unroll
    for (int bi = 3; bi >= 0; --bi) {
#pragma unroll
      for (int r = 15; r >= 0; --r) {
        const int code = bi * 32 + 8 * (r >> 2) + (r & 3);
        sel = (acc[bi][bj][r] == mt) ? code : sel;  // descending scan: the lowest id wins
      }
    }
    const bool upd = mt > m[bj];  // strict: an equal maximum in a later tile has a higher id
    ix[bj] = upd ? vb + sel : ix[bj];
    const float mn = fmaxf(m[bj], mt);
    const float nml = -mn * kLog2e;
    float p0 = 0.f, p1 = 0.f, p2 = 0.f, p3 = 0.f;
#pragma unroll
    for (int bi = 0; bi < 4; ++bi) {
#pragma unroll
      for (int r = 0; r < 16; r += 4) {
        p0 += exp_rel<TAIL>(acc[bi][bj][r + 0], mn, nml);
        p1 += exp_rel<TAIL>(acc[bi][bj][r + 1], mn, nml);
        p2 += exp_rel<TAIL>(acc[bi][bj][r + 2], mn, nml);
        p3 += exp_rel<TAIL>(acc[bi][bj][r + 3], mn, nml);
      }
    }
    s[bj] = s[bj] * __builtin_amdgcn_exp2f((m[bj] - mn) * kLog2e) + ((p0 + p1) + (p2 + p3));
    m[bj] = mn;
  }
}

// Separate rings for the two operands: NW slots of W K-tiles, NH slots of H K-tiles (32 KiB each).
// The shallow ring runs one K-tile ahead, the deep one two; the shallow operand is issued first in
// every iteration so that the in-order vmcnt wait can leave the deep ring's newest tile in flight.
// Same tile under sampling: also tracks the arg-max of x + tau*g and the plain logit there.
template <bool TAIL>
__device__ __forceinline__ void reduce_tile_sample(f32x16 (&acc)[4][2], float (&m)[2], float (&s)[2], float (&ym)[2],
                                                   float (&xa)[2], int (&ix)[2], int vb, int V, const int (&pos)[2],
                                                   uint32_t k0, uint32_t k1, float tau) {
#pragma unroll
  for (int bj = 0; bj < 2; ++bj) {
    float mt = kNeg, yt = kNeg, xsel = 0.f;
    int sel = 0;
#pragma unroll
    for (int bi = 3; bi >= 0; --bi) {
#pragma unroll
      for (int r4 = 3; r4 >= 0; --r4) {
        const int code0 = bi * 32 + 8 * r4;
        float n[4];
        gumbel4(k0, k1, (uint32_t)pos[bj], (uint32_t)(vb + code0) >> 2, tau, n);
#pragma unroll
        for (int r = 3; r >= 0; --r) {
          // ids past the vocabulary: selects, not branches (a branch per element makes the compiler move whole
          // accumulator vectors through scratch)
          const bool past = TAIL && vb + code0 + r >= V;
          const float x = past ? kNeg : acc[bi][bj][4 * r4 + r];
          if (TAIL) acc[bi][bj][4 * r4 + r] = x;
          const float y = past ? kNeg : x + n[r];
          mt = fmaxf(mt, x);
          const bool better = y >= yt;   // descending scan: on equal scores the lower id replaces the higher
          sel = better ? code0 + r : sel;
          xsel = better ? x : xsel;
          yt = better ? y : yt;
        }
      }
    }
    const bool upd = yt > ym[bj];
    ix[bj] = upd ? vb + sel : ix[bj];
    xa[bj] = upd ? xsel : xa[bj];
    ym[bj] = upd ? yt : ym[bj];
    const float mn = fmaxf(m[bj], mt);
    const float nml = -mn * kLog2e;
    float p0 = 0.f, p1 = 0.f, p2 = 0.f, p3 = 0.f;
#pragma unroll
    for (int bi = 0; bi < 4; ++bi) {
#pragma unroll
      for (int r = 0; r < 16; r += 4) {
        p0 += exp_rel<TAIL>(acc[bi][bj][r + 0], mn, nml);
        p1 += exp_rel<TAIL>(acc[bi][bj][r + 1], mn, nml);
        p2 += exp_rel<TAIL>(acc[bi][bj][r + 2], mn, nml);
        p3 += exp_rel<TAIL>(acc[bi][bj][r + 3], mn, nml);
      }
    }
    s[bj] = s[bj] * __builtin_amdgcn_exp2f((m[bj] - mn) * kLog2e) + ((p0 + p1) + (p2 + p3));
    m[bj] = mn;
  }
}

template <int NW, int NH, bool SAMPLE>
__global__ __launch_bounds__(kThreads) void masked_logits_kernel(const KernelParams p) {
  static_assert((NW == 2 || NW == 3) && (NH == 2 || NH == 3) && NW + NH <= 5, "ring shape");
  constexpr int kTileK = 64;
  constexpr int kRowBytes = 128;
  constexpr int kOperandBytes = 256 * kRowBytes;        // 32 KiB
  constexpr int kSwzShift = 1;
  constexpr int kSubSteps = 4;
  constexpr int kDW = NW - 1, kDH = NH - 1;             // prefetch distance in K-tiles
  constexpr int kRing = (NW + NH) * kOperandBytes;
  constexpr int kLds = (NW + NH == 5) ? kRing : kRing + 5 * 256 * 4;
  constexpr int kRedOff = (NW + NH == 5) ? 0 : kRing;   // 5 slots fill the LDS: merge scratch aliases slot 0
  __shared__ __attribute__((aligned(1024))) char smem[kLds];
  float* red_m = reinterpret_cast<float*>(smem + kRedOff);
  float* red_s = red_m + 256;
  int* red_i = reinterpret_cast<int*>(red_s + 256);
  float* red_ym = reinterpret_cast<float*>(red_i + 256);   // sampling only
  float* red_xa = red_ym + 256;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wv = wave & 1;   // vocabulary half of the tile
  const int wt = wave >> 1;  // token quarter of the tile
  const int l32 = lane & 31, lhalf = lane >> 5;

  if (p.wide_flag != nullptr && *p.wide_flag != p.wide_run_if) return;   // the other kernel of the two serves this list
  int total = *p.count;
  if (total > p.max_rows) total = p.max_rows;
  int rows = total - p.row0;
  if (rows > p.chunk_rows) rows = p.chunk_rows;
  if (rows <= 0) return;
  const int n_tt = (rows + kTileRows - 1) / kTileRows;

  const int G = gridDim.x;
  const int pos = xcd_contiguous_position((int)blockIdx.x, G);
  const int S = p.splits;
  const int n_units = n_tt * S;
  const int A = p.panel < n_tt ? p.panel : n_tt;
  const int full_panel_units = A * S;
  const int n_panels = (n_tt + A - 1) / A;

  const int drow = wave * 32 + (lane >> 3);
  int src_chunk_bytes[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) src_chunk_bytes[i] = (((lane & 7) ^ (((drow + 8 * i) >> kSwzShift) & 7))) * 16;
  int rd_off[kSubSteps];
#pragma unroll
  for (int ks = 0; ks < kSubSteps; ++ks) rd_off[ks] = l32 * kRowBytes + (((2 * ks + lhalf) ^ ((l32 >> kSwzShift) & 7)) * 16);

  const int nk = p.d / kTileK;

  for (int u = pos, round = 0; u < n_units; u += G, ++round) {
    if (round > 0) meet_before_round(p, round, n_units, G, tid);
    int pnl = u / full_panel_units;
    if (pnl >= n_panels) pnl = n_panels - 1;
    const int ul = u - pnl * full_panel_units;
    const int hp = (n_tt - pnl * A) < A ? (n_tt - pnl * A) : A;
    const int sp = ul / hp;
    const int tt = pnl * A + ul % hp;
    const int vt0 = p.tile_first + (int)(((int64_t)sp * p.vocab_tiles) / S);
    const int vt1 = p.tile_first + (int)(((int64_t)(sp + 1) * p.vocab_tiles) / S);
    const int ntile = vt1 - vt0;
    const int total_steps = ntile * nk;

    const char* hptr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int j = tt * kTileRows + drow + 8 * i;
      if (j > rows - 1) j = rows - 1;
      int t = p.idx[p.row0 + j];
      t = t < 0 ? 0 : (t > p.T - 1 ? p.T - 1 : t);   // a bad entry of a caller-built list reads a valid row
      hptr[i] = p.hidden + (int64_t)t * p.ldh_bytes + src_chunk_bytes[i];
    }
    const char* wptr[4];

    // W loader: global step w_g = (vocab tile, k); slot w_g % NW.
    int w_g = 0, w_vt = vt0, w_k = 0, w_slot = 0;
    auto issue_w = [&]() {
      if (w_k == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          int v = w_vt * kTileVocab + drow + 8 * i;
          if (v > p.V - 1) v = p.V - 1;
          wptr[i] = p.w + (int64_t)v * ((int64_t)p.d * 2) + src_chunk_bytes[i];
        }
      }
      char* dst = smem + w_slot * kOperandBytes + (wave * 32) * kRowBytes;
      const int koff = w_k * kRowBytes;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(wptr[i] + koff), (lds_ptr_t)(dst + i * 1024), 16, 0, 0);
      w_k += 1;
      if (w_k == nk) { w_k = 0; w_vt += 1; }
      w_slot = (w_slot + 1 == NW) ? 0 : w_slot + 1;
      w_g += 1;
    };
    int h_g = 0, h_k = 0, h_slot = 0;
    auto issue_h = [&]() {
      char* dst = smem + (NW + h_slot) * kOperandBytes + (wave * 32) * kRowBytes;
      const int koff = h_k * kRowBytes;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(hptr[i] + koff), (lds_ptr_t)(dst + i * 1024), 16, 0, 0);
      h_k = (h_k + 1 == nk) ? 0 : h_k + 1;
      h_slot = (h_slot + 1 == NH) ? 0 : h_slot + 1;
      h_g += 1;
    };
    // One scheduling slot: at (virtual) iteration it, bring in W step it+kDW and H step it+kDH,
    // shallow ring first.
    auto issue_pair = [&](int it) {
      if constexpr (kDW <= kDH) {
        if (it + kDW >= 0 && it + kDW < total_steps) issue_w();
        if (it + kDH >= 0 && it + kDH < total_steps) issue_h();
      } else {
        if (it + kDH >= 0 && it + kDH < total_steps) issue_h();
        if (it + kDW >= 0 && it + kDW < total_steps) issue_w();
      }
    };
    constexpr int kDMax = kDW > kDH ? kDW : kDH;
    constexpr int kDMin = kDW < kDH ? kDW : kDH;

    float run_m[2] = {kNeg, kNeg};
    float run_s[2] = {0.f, 0.f};
    int run_i[2] = {INT_MAX, INT_MAX};
    float run_ym[2] = {kNeg, kNeg};   // sampling: best x + tau*g, the plain logit there
    float run_xa[2] = {0.f, 0.f};
    int pos[2] = {0, 0};              // sampling: the position whose row this lane's column holds
    if constexpr (SAMPLE) {
#pragma unroll
      for (int bj = 0; bj < 2; ++bj) {
        int j = tt * kTileRows + wt * 64 + bj * 32 + l32;
        if (j > rows - 1) j = rows - 1;
        pos[bj] = p.noise_idx[p.row0 + j];
      }
    }

    wait_vm<0>();
#pragma unroll
    for (int it = -kDMax; it < 0; ++it) issue_pair(it);

    int ws = 0, hs = 0, step = 0;
    for (int n = 0; n < ntile; ++n) {
      f32x16 acc[4][2];
#pragma unroll
      for (int bi = 0; bi < 4; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.f;

      for (int kt = 0; kt < nk; ++kt, ++step) {
        // Both operands of `step` must have landed.  The only loads issued after them are the deep
        // ring's tile step+kDMax... (one tile, 4 loads) when the rings differ in depth by one.
        if (kDMax > kDMin && step + kDMax - kDMin < total_steps && kDMin == 1) wait_vm<4>();
        else wait_vm<0>();
        __builtin_amdgcn_s_barrier();
        issue_pair(step);

        const char* wbase = smem + ws * kOperandBytes + (wv * 128) * kRowBytes;
        const char* hbase = smem + (NW + hs) * kOperandBytes + (wt * 64) * kRowBytes;
#pragma unroll
        for (int ks = 0; ks < kSubSteps; ++ks) {
          bf16x8 a[4], b[2];
#pragma unroll
          for (int bi = 0; bi < 4; ++bi) a[bi] = *reinterpret_cast<const bf16x8*>(wbase + bi * 32 * kRowBytes + rd_off[ks]);
#pragma unroll
          for (int bj = 0; bj < 2; ++bj) b[bj] = *reinterpret_cast<const bf16x8*>(hbase + bj * 32 * kRowBytes + rd_off[ks]);
#pragma unroll
          for (int bi = 0; bi < 4; ++bi)
#pragma unroll
            for (int bj = 0; bj < 2; ++bj)
              acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[bi], b[bj], acc[bi][bj], 0, 0, 0);
        }
        ws = (ws + 1 == NW) ? 0 : ws + 1;
        hs = (hs + 1 == NH) ? 0 : hs + 1;
      }

      const int v_tile0 = (vt0 + n) * kTileVocab;
      const int vb = v_tile0 + wv * 128 + 4 * lhalf;
      if constexpr (SAMPLE) {
        if (v_tile0 + kTileVocab > p.V)
          reduce_tile_sample<true>(acc, run_m, run_s, run_ym, run_xa, run_i, vb, p.V, pos, p.seed_lo, p.seed_hi, p.tau);
        else
          reduce_tile_sample<false>(acc, run_m, run_s, run_ym, run_xa, run_i, vb, p.V, pos, p.seed_lo, p.seed_hi, p.tau);
      } else {
        if (v_tile0 + kTileVocab > p.V) reduce_tile<true>(acc, run_m, run_s, run_i, vb, p.V);
        else reduce_tile<false>(acc, run_m, run_s, run_i, vb, p.V);
      }
    }

#pragma unroll
    for (int bj = 0; bj < 2; ++bj) {
      const float m2 = __shfl_xor(run_m[bj], 32, 64);
      const float s2 = __shfl_xor(run_s[bj], 32, 64);
      const int i2 = __shfl_xor(run_i[bj], 32, 64);
      if constexpr (SAMPLE) {
        merge_ms(run_m[bj], run_s[bj], m2, s2);
        merge_pick(run_ym[bj], run_xa[bj], run_i[bj], __shfl_xor(run_ym[bj], 32, 64), __shfl_xor(run_xa[bj], 32, 64), i2);
      } else {
        merge_triple(run_m[bj], run_s[bj], run_i[bj], m2, s2, i2);
      }
    }
    __syncthreads();  // every wave is done reading the ring (the merge scratch may alias it)
    if (wv == 1 && lhalf == 0) {
#pragma unroll
      for (int bj = 0; bj < 2; ++bj) {
        const int e = (wt * 2 + bj) * 32 + l32;
        red_m[e] = run_m[bj];
        red_s[e] = run_s[bj];
        red_i[e] = run_i[bj];
        if constexpr (SAMPLE) {
          red_ym[e] = run_ym[bj];
          red_xa[e] = run_xa[bj];
        }
      }
    }
    __syncthreads();
    if (wv == 0 && lhalf == 0) {
#pragma unroll
      for (int bj = 0; bj < 2; ++bj) {
        const int e = (wt * 2 + bj) * 32 + l32;
        const int64_t slot = (int64_t)(p.split_first + sp) * p.c_pad + tt * kTileRows + e;
        if constexpr (SAMPLE) {
          merge_ms(run_m[bj], run_s[bj], red_m[e], red_s[e]);
          merge_pick(run_ym[bj], run_xa[bj], run_i[bj], red_ym[e], red_xa[e], red_i[e]);
          p.part_ym[slot] = run_ym[bj];
          p.part_xa[slot] = run_xa[bj];
        } else {
          merge_triple(run_m[bj], run_s[bj], run_i[bj], red_m[e], red_s[e], red_i[e]);
        }
        p.part_m[slot] = run_m[bj];
        p.part_s[slot] = run_s[bj];
        p.part_i[slot] = run_i[bj];
      }
    }
    __syncthreads();  // the scratch is read before the next unit's copies may overwrite it
  }
}

// ---- 4-wave fast path: one wave per SIMD, 128 (vocab) x 128 (token) per wave as 8 x 8 blocks of
// v_mfma_f32_16x16x32_bf16 (the more power-efficient bf16 shape on this part), accumulators in AGPRs.
// A vocabulary tile is one hand-scheduled inline-asm statement (mosaic_w4_tile.inc greedy, mosaic_w4_tile_sample.inc
// sampling; both generated): the K-loop, then the tile's reduction into the running per-column state.  In the K-loop
// every MFMA is followed by at most one LDS read or one direct-to-LDS copy, fragments are double-
// buffered in fixed VGPRs, the LM-head ring runs two K-tiles ahead and the hidden ring one.
// Preconditions (checked by the launcher): V % 256 == 0, 256*d*2 < 4 GiB; and, in a hidden tensor of 4 GiB or more,
// no 64 consecutive rows of the list 4 GiB apart (checked on the device, see KernelParams::wide_flag).
template <bool SAMPLE>
__global__ __launch_bounds__(256) void masked_logits_kernel_w4(const KernelParams p) {
  constexpr int NW = 3, NH = 2;
  constexpr int kTileK = 64;
  constexpr int kRowBytes = 128;
  constexpr int kOperandBytes = 256 * kRowBytes;        // 32 KiB
  constexpr int kSwzShift = 1;
  __shared__ __attribute__((aligned(1024))) char smem[(NW + NH) * kOperandBytes];
  float* red_m = reinterpret_cast<float*>(smem);        // merge scratch aliases W slot 0 at unit end
  float* red_s = red_m + 256;
  int* red_i = reinterpret_cast<int*>(red_s + 256);
  float* red_ym = reinterpret_cast<float*>(red_i + 256);   // sampling only
  float* red_xa = red_ym + 256;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wv = wave & 1;   // vocabulary half of the tile
  const int wt = wave >> 1;  // token half of the tile
  const int l16 = lane & 15, q = lane >> 4;   // MFMA 16x16x32: row/column lane%16, k group lane/16

  if (p.wide_flag != nullptr && *p.wide_flag != p.wide_run_if) return;   // the other kernel of the two serves this list
  int total = *p.count;
  if (total > p.max_rows) total = p.max_rows;
  int rows = total - p.row0;
  if (rows > p.chunk_rows) rows = p.chunk_rows;
  if (rows <= 0) return;
  const int n_tt = (rows + kTileRows - 1) / kTileRows;

  const int G = gridDim.x;
  const int pos = xcd_contiguous_position((int)blockIdx.x, G);
  const int S = p.splits;
  const int n_units = n_tt * S;
  const int A = p.panel < n_tt ? p.panel : n_tt;
  const int full_panel_units = A * S;
  const int n_panels = (n_tt + A - 1) / A;

  // Direct-to-LDS copy: instruction i (0..7) of this wave fills rows wave*64 + 8*i + lane/8; the swizzle
  // of row drow + 8*i depends on i only through its parity.
  const int drow = wave * 64 + (lane >> 3);
  const uint32_t chunk_even = (uint32_t)(((lane & 7) ^ ((drow >> kSwzShift) & 7)) * 16);
  const uint32_t chunk_odd = (uint32_t)(((lane & 7) ^ (((drow + 8) >> kSwzShift) & 7)) * 16);
  const int nk = p.d / kTileK;
  const uint32_t w_row_bytes = (uint32_t)p.d * 2u;

  // LDS read offsets per half K-tile: row (lane%16) of this wave's first 16-row block, swizzled chunk.
  uint32_t rdw[2], rdh[2], woff[8];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const uint32_t o = (uint32_t)(l16 * kRowBytes + (((4 * ks + q) ^ ((l16 >> kSwzShift) & 7)) * 16));
    rdw[ks] = o + (uint32_t)(wv * 128 * kRowBytes);
    rdh[ks] = o + (uint32_t)(NW * kOperandBytes + wt * 128 * kRowBytes);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) woff[i] = (uint32_t)(drow + 8 * i) * w_row_bytes + ((i & 1) ? chunk_odd : chunk_even);

  // sampling: the generator's key (the statement derives the round keys from it), its multipliers, 1/tau and tau
  const uint32_t seed_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)p.seed_lo);
  const uint32_t seed_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)p.seed_hi);
  const uint32_t philox_m0 = 0xD2511F53u, philox_m1 = 0xCD9E8D57u;
  const float tau_s = p.tau;
  const float inv_tau_log2e = SAMPLE ? kLog2e / p.tau : 0.f;
  const uint32_t u_nk = (uint32_t)nk;
  const uint32_t u_wwrap = 256u * w_row_bytes - (uint32_t)(nk - 1) * 128u;
  const uint32_t u_hwrap = (uint32_t)(nk - 1) * 128u;
  const uint32_t wave_dst = (uint32_t)wave * 64u * kRowBytes;

  for (int u = pos, round = 0; u < n_units; u += G, ++round) {
    if (round > 0) meet_before_round(p, round, n_units, G, tid);
    int pnl = u / full_panel_units;
    if (pnl >= n_panels) pnl = n_panels - 1;
    const int ul = u - pnl * full_panel_units;
    const int hp = (n_tt - pnl * A) < A ? (n_tt - pnl * A) : A;
    const int sp = ul / hp;
    const int tt = pnl * A + ul % hp;
    const int vt0 = (int)(((int64_t)sp * p.vocab_tiles) / S);
    const int vt1 = (int)(((int64_t)(sp + 1) * p.vocab_tiles) / S);
    const int ntile = vt1 - vt0;
    const int total_steps = ntile * nk;
    const uint32_t u_total = (uint32_t)total_steps;

    // Gather: 32-bit byte offsets of the 8 hidden rows this lane copies, from the lowest of the 64 rows this wave
    // copies (rows past the end of the chunk re-read the last valid row; their results are never stored).  The
    // offsets fit 32 bits when the hidden tensor is smaller than 4 GiB, and otherwise because this launch only
    // runs when no wave's rows lie that far apart (span_check_kernel).
    int trow[8], tmin = INT_MAX;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int j = tt * kTileRows + drow + 8 * i;
      if (j > rows - 1) j = rows - 1;
      int t = p.idx[p.row0 + j];
      t = t < 0 ? 0 : (t > p.T - 1 ? p.T - 1 : t);   // a bad entry of a caller-built list reads a valid row
      trow[i] = t;
      tmin = t < tmin ? t : tmin;
    }
#pragma unroll
    for (int x = 32; x >= 1; x >>= 1) {
      const int other = __shfl_xor(tmin, x, 64);
      tmin = other < tmin ? other : tmin;
    }
    tmin = __builtin_amdgcn_readfirstlane(tmin);
    const char* hidden_wave = p.hidden + (int64_t)tmin * p.ldh_bytes;
    uint32_t hoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      hoff[i] = (uint32_t)(trow[i] - tmin) * (uint32_t)p.ldh_bytes + ((i & 1) ? chunk_odd : chunk_even);

    // Prologue copies, in this order: W0, H0, W1, W2, H1 (tile 0 is needed first, H1 at the first sync).
    auto copy_w = [&](int gw) {
      const char* src = p.w + ((int64_t)(vt0 + gw / nk) * kTileVocab) * (int64_t)w_row_bytes + (gw % nk) * kRowBytes;
      char* dst = smem + (gw % NW) * kOperandBytes + wave_dst;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(src + woff[i]), (lds_ptr_t)(dst + i * 1024), 16, 0, 0);
    };
    auto copy_h = [&](int gh) {
      const char* src = hidden_wave + (gh % nk) * kRowBytes;
      char* dst = smem + (NW + gh % NH) * kOperandBytes + wave_dst;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(src + hoff[i]), (lds_ptr_t)(dst + i * 1024), 16, 0, 0);
    };
    wait_vm<0>();
    copy_w(0);
    copy_h(0);
    int after0 = 0;
    if (1 < total_steps) { copy_w(1); after0 += 1; }
    if (2 < total_steps) { copy_w(2); after0 += 1; }
    if (1 < total_steps) { copy_h(1); after0 += 1; }
    if (after0 == 3) wait_vm<24>(); else if (after0 == 2) wait_vm<16>(); else if (after0 == 1) wait_vm<8>(); else wait_vm<0>();
    __builtin_amdgcn_s_barrier();

    // State of the asm loop: next tiles to copy are W(3) and H(2) (never issued if past the end).
    const int gw = 3, gh = 2;
    const uint64_t wsrc0 = (uint64_t)(p.w + ((int64_t)(vt0 + gw / nk) * kTileVocab) * (int64_t)w_row_bytes + (gw % nk) * kRowBytes);
    const uint64_t hsrc0 = (uint64_t)(hidden_wave + (gh % nk) * kRowBytes);
    uint32_t st_wsrc_lo = (uint32_t)wsrc0, st_wsrc_hi = (uint32_t)(wsrc0 >> 32);
    uint32_t st_hsrc_lo = (uint32_t)hsrc0, st_hsrc_hi = (uint32_t)(hsrc0 >> 32);
    uint32_t st_wrd = 0, st_hrd = 0;
    uint32_t st_wdst = (uint32_t)((gw % NW) * kOperandBytes) + wave_dst;
    uint32_t st_hdst = (uint32_t)((gh % NH) * kOperandBytes) + wave_dst;
    uint32_t st_wk = (uint32_t)(gw % nk), st_hk = (uint32_t)(gh % nk);
    uint32_t st_g = 0;

    float run_m[8], run_s[8], run_ym[8], run_xa[8];
    int run_i[8], pos[8];
#pragma unroll
    for (int tb = 0; tb < 8; ++tb) {
      run_m[tb] = kNeg; run_s[tb] = 0.f; run_i[tb] = INT_MAX; run_ym[tb] = kNeg; run_xa[tb] = 0.f; pos[tb] = 0;
      if constexpr (SAMPLE) {   // the position whose row this lane's column tb holds
        int j = tt * kTileRows + wt * 128 + tb * 16 + l16;
        if (j > rows - 1) j = rows - 1;
        pos[tb] = p.noise_idx[p.row0 + j];
      }
    }

    for (int n = 0; n < ntile; ++n) {
      st_wsrc_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_wsrc_lo);
      st_wsrc_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_wsrc_hi);
      st_hsrc_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_hsrc_lo);
      st_hsrc_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_hsrc_hi);
      st_wrd = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_wrd);
      st_hrd = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_hrd);
      st_wdst = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_wdst);
      st_hdst = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_hdst);
      st_wk = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_wk);
      st_hk = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_hk);
      st_g = (uint32_t)__builtin_amdgcn_readfirstlane((int)st_g);
      {
      const uint32_t st_total = (uint32_t)__builtin_amdgcn_readfirstlane((int)u_total);
      const uint32_t st_nk = (uint32_t)__builtin_amdgcn_readfirstlane((int)u_nk);
      const uint32_t st_wwrap = (uint32_t)__builtin_amdgcn_readfirstlane((int)u_wwrap);
      const uint32_t st_hwrap = (uint32_t)__builtin_amdgcn_readfirstlane((int)u_hwrap);
        uint32_t addr_tmp0, addr_tmp1;
        const int vb = (vt0 + n) * kTileVocab + wv * 128 + 4 * q;   // vocabulary id of this lane's element 0
        if constexpr (SAMPLE) {
          // sampling: the same, with the Gumbel-max draw in the reduction (fragments, accumulators, the
          // reduction's temporaries and the round keys all by number)
#include "mosaic_w4_tile_sample.inc"
        } else {
          // greedy: one statement clears the accumulators (the AGPR file, by number), runs the K-loop and folds
          // the tile into the running triples, so nothing of it is left to the compiler's scheduling
          bf16x8 frag_a[2][8], frag_b[2][8];   // written and consumed inside the statement only
          float red_x[32], red_t, red_mn, red_nml, red_y;
          int red_sel;
#include "mosaic_w4_tile.inc"
        }
      }
    }

    // Unit end: fold the four lanes that share a token (lane ^ 16, lane ^ 32), then the two waves that
    // share it (vocabulary halves) through LDS, and publish one partial triple per row.
#pragma unroll
    for (int tb = 0; tb < 8; ++tb) {
#pragma unroll
      for (int x = 16; x <= 32; x <<= 1) {
        const float m2 = __shfl_xor(run_m[tb], x, 64);
        const float s2 = __shfl_xor(run_s[tb], x, 64);
        const int i2 = __shfl_xor(run_i[tb], x, 64);
        if constexpr (SAMPLE) {
          merge_ms(run_m[tb], run_s[tb], m2, s2);
          merge_pick(run_ym[tb], run_xa[tb], run_i[tb], __shfl_xor(run_ym[tb], x, 64), __shfl_xor(run_xa[tb], x, 64), i2);
        } else {
          merge_triple(run_m[tb], run_s[tb], run_i[tb], m2, s2, i2);
        }
      }
    }
    __syncthreads();  // every wave is done with the ring (the merge scratch aliases it)
    if (wv == 1 && q == 0) {
#pragma unroll
      for (int tb = 0; tb < 8; ++tb) {
        const int e = wt * 128 + tb * 16 + l16;
        red_m[e] = run_m[tb];
        red_s[e] = run_s[tb];
        red_i[e] = run_i[tb];
        if constexpr (SAMPLE) {
          red_ym[e] = run_ym[tb];
          red_xa[e] = run_xa[tb];
        }
      }
    }
    __syncthreads();
    if (wv == 0 && q == 0) {
#pragma unroll
      for (int tb = 0; tb < 8; ++tb) {
        const int e = wt * 128 + tb * 16 + l16;
        const int64_t slot = (int64_t)sp * p.c_pad + tt * kTileRows + e;
        if constexpr (SAMPLE) {
          merge_ms(run_m[tb], run_s[tb], red_m[e], red_s[e]);
          merge_pick(run_ym[tb], run_xa[tb], run_i[tb], red_ym[e], red_xa[e], red_i[e]);
          p.part_ym[slot] = run_ym[tb];
          p.part_xa[slot] = run_xa[tb];
        } else {
          merge_triple(run_m[tb], run_s[tb], run_i[tb], red_m[e], red_s[e], red_i[e]);
        }
        p.part_m[slot] = run_m[tb];
        p.part_s[slot] = run_s[tb];
        p.part_i[slot] = run_i[tb];
      }
    }
    __syncthreads();
  }
}

// Merge the S partial results of every row and emit the outputs.  A block of 256 threads handles ROWS rows with
// G = 256 / ROWS thread groups: group g folds the splits g, g + G, g + 2G, ... in ascending order (their loads
// issued together), then the G group results are folded pairwise, group g with group g + stride for stride = G/2,
// G/4, ..., 1.  The order is a function of S alone (run-to-run and chunking-independent results) and a row's chain
// of dependent steps is S / G + log2 G long instead of S.  Few splits: 16 rows x 16 groups; many splits (one row
// tile spread over ~250 of them, where this kernel is a visible part of the step): 4 rows x 64 groups -- the
// sequential merge took 114 us there, 16 groups with a sequential second level 16 us.
template <int ROWS>
__global__ __launch_bounds__(256) void combine_kernel(const KernelParams p) {
  constexpr int G = 256 / ROWS;
  constexpr int kPerGroup = (MOSAIC_MAX_VOCAB_SPLITS + G - 1) / G;   // splits one group folds at most
  __shared__ float sh_m[G][ROWS], sh_s[G][ROWS], sh_ym[G][ROWS], sh_xa[G][ROWS];
  __shared__ int sh_i[G][ROWS];
  int total = *p.count;
  if (total > p.max_rows) total = p.max_rows;
  int rows = total - p.row0;
  if (rows > p.chunk_rows) rows = p.chunk_rows;
  const int lr = threadIdx.x % ROWS, g = threadIdx.x / ROWS;
  const int r = blockIdx.x * ROWS + lr;
  const bool valid = r < rows;
  const bool sample = p.tau > 0.f;   // sampling: the token is the arg-max of the perturbed scores
  float m = kNeg, s = 0.f, ym = kNeg, xa = 0.f;
  int i = INT_MAX;
  if (valid) {
    float lm[kPerGroup], ls[kPerGroup], lym[kPerGroup], lxa[kPerGroup];
    int li[kPerGroup];
#pragma unroll
    for (int k = 0; k < kPerGroup; ++k) {
      const int sp = g + k * G;
      const bool on = sp < p.splits;
      const int64_t slot = (int64_t)(on ? sp : 0) * p.c_pad + r;
      lm[k] = on ? p.part_m[slot] : kNeg;        // beyond S: the neutral element
      ls[k] = on ? p.part_s[slot] : 0.f;
      li[k] = on ? p.part_i[slot] : INT_MAX;
      lym[k] = (on && sample) ? p.part_ym[slot] : kNeg;
      lxa[k] = (on && sample) ? p.part_xa[slot] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < kPerGroup; ++k) {
      if (sample) {
        merge_ms(m, s, lm[k], ls[k]);
        merge_pick(ym, xa, i, lym[k], lxa[k], li[k]);
      } else {
        merge_triple(m, s, i, lm[k], ls[k], li[k]);
      }
    }
  }
  sh_m[g][lr] = m;
  sh_s[g][lr] = s;
  sh_i[g][lr] = i;
  sh_ym[g][lr] = ym;
  sh_xa[g][lr] = xa;
  __syncthreads();
#pragma unroll
  for (int stride = G / 2; stride >= 1; stride >>= 1) {
    if (g < stride) {
      if (sample) {
        merge_ms(m, s, sh_m[g + stride][lr], sh_s[g + stride][lr]);
        merge_pick(ym, xa, i, sh_ym[g + stride][lr], sh_xa[g + stride][lr], sh_i[g + stride][lr]);
      } else {
        merge_triple(m, s, i, sh_m[g + stride][lr], sh_s[g + stride][lr], sh_i[g + stride][lr]);
      }
      sh_m[g][lr] = m;
      sh_s[g][lr] = s;
      sh_i[g][lr] = i;
      sh_ym[g][lr] = ym;
      sh_xa[g][lr] = xa;
    }
    __syncthreads();
  }
  if (g != 0 || !valid) return;
  p.out_token[p.row0 + r] = i;
  p.out_lse[p.row0 + r] = m + __builtin_amdgcn_logf(s) * kLn2;
  p.out_conf[p.row0 + r] = sample ? __builtin_amdgcn_exp2f((xa - m) * kLog2e) / s : 1.0f / s;
}
constexpr int kWideMergeSplits = 64;   // from this many splits on, the 64-group merge

int launch_masked_logits(const LogitsArgs& a, const mosaic_plan& plan, hipStream_t stream) {
  KernelParams p;
  p.hidden = static_cast<const char*>(a.hidden);
  p.ldh_bytes = a.ld_h * 2;
  p.w = static_cast<const char*>(a.w);
  p.d = a.d;
  p.V = a.V;
  p.idx = a.idx;
  p.noise_idx = a.noise_idx != nullptr ? a.noise_idx : a.idx;
  p.count = a.count;
  p.T = (int32_t)a.T;
  p.chunk_rows = plan.rows_per_chunk;
  p.max_rows = (int32_t)a.max_rows;
  p.splits = plan.vocab_splits;
  p.panel = plan.tile_panel;
  p.vocab_tiles = (a.V + kTileVocab - 1) / kTileVocab;
  p.tile_first = 0;
  p.split_first = 0;
  p.c_pad = plan.rows_per_chunk;
  p.part_m = static_cast<float*>(a.workspace);
  p.part_s = p.part_m + (int64_t)plan.vocab_splits * plan.rows_per_chunk;
  p.part_i = reinterpret_cast<int32_t*>(p.part_s + (int64_t)plan.vocab_splits * plan.rows_per_chunk);
  p.out_token = a.out_token;
  p.out_conf = a.out_conf;
  p.out_lse = a.out_lse;
  const bool sample = a.temperature > 0.f;
  p.tau = sample ? a.temperature : 0.f;
  p.seed_lo = (uint32_t)a.seed;
  p.seed_hi = (uint32_t)(a.seed >> 32);
  p.part_ym = reinterpret_cast<float*>(p.part_i + (int64_t)plan.vocab_splits * plan.rows_per_chunk);
  p.part_xa = p.part_ym + (int64_t)plan.vocab_splits * plan.rows_per_chunk;
  // the round counters sit behind the partial planes (three for a greedy pass, five for a sampling one)
  constexpr int kSyncSlots = MOSAIC_SYNC_BYTES / 4 - 1;   // the last word is the flag of the span check
  p.sync = reinterpret_cast<int32_t*>(sample ? p.part_xa + (int64_t)plan.vocab_splits * plan.rows_per_chunk
                                             : p.part_ym);
  p.sync_slots = kSyncSlots;
  p.wide_flag = nullptr;
  p.wide_run_if = 0;

  const KernelChoice choice = choose_kernel(a.T, a.ld_h, a.d, a.V, plan);
  const bool fast = choice.fast, paired = choice.paired, wide = choice.wide;
  int32_t* const flag = p.sync + kSyncSlots;
  // The selector gives a ragged vocabulary one split more than fills the chip (for the pair's second launch);
  // the general kernel alone works best without it.
  if (!fast && !paired && a.V % kTileVocab != 0 && p.vocab_tiles >= 2 && p.splits >= 2) p.splits -= 1;
  KernelParams body = p, tail = p;   // the two launches of a pair
  if (paired) {
    body.vocab_tiles = p.vocab_tiles - 1;
    body.splits = plan.vocab_splits - 1;
    if (body.splits > body.vocab_tiles) body.splits = body.vocab_tiles;
    tail.vocab_tiles = 1;
    tail.tile_first = p.vocab_tiles - 1;
    tail.splits = 1;
    tail.split_first = body.splits;
    p.splits = body.splits + 1;        // what the merge reads
    body.sync_slots = tail.sync_slots = kSyncSlots / 2;   // each launch of the pair meets on its own counters
    tail.sync = p.sync + kSyncSlots / 2;
  }
  // A hidden tensor of 4 GiB or more: the 4-wave launch and a general-kernel launch of the same work both go out,
  // and the flag of the span check decides on the device which of the two does it.
  KernelParams fallback = paired ? body : p;
  if (wide) {
    p.wide_flag = body.wide_flag = fallback.wide_flag = flag;
    fallback.wide_run_if = 1;
  }
  int rc = 0;
  for (int c = 0; c < plan.num_chunks; ++c) {
    const int64_t row0 = (int64_t)c * plan.rows_per_chunk;
    if (row0 >= a.max_rows) break;
    p.row0 = body.row0 = tail.row0 = (int32_t)row0;
    int64_t cap = a.max_rows - row0;
    if (cap > plan.rows_per_chunk) cap = plan.rows_per_chunk;
    const int64_t tiles = (cap + kTileRows - 1) / kTileRows;
    const KernelParams& q = paired ? body : p;
    int64_t grid = tiles * q.splits;
    const bool several_rounds = grid > plan.grid || (paired && tiles > plan.grid);
    if (grid > plan.grid) grid = plan.grid;
    if (several_rounds || wide)
      rc |= launch_kernel(clear_round_counters_kernel, dim3(1), dim3(256), stream, p.sync, kSyncSlots + 1);
    if (wide)
      rc |= launch_kernel(span_check_kernel, dim3((unsigned)((cap + 255) / 256)), dim3(256), stream, a.idx, a.count,
                          (int32_t)row0, plan.rows_per_chunk, (int32_t)a.max_rows, (int32_t)a.T, p.ldh_bytes, flag);
    auto launch_general = [&](const KernelParams& kp, int64_t blocks) {
      return sample ? launch_kernel(masked_logits_kernel<3, 2, true>, dim3((unsigned)blocks), dim3(kThreads), stream, kp)
                    : launch_kernel(masked_logits_kernel<3, 2, false>, dim3((unsigned)blocks), dim3(kThreads), stream, kp);
    };
    if (fast || paired) {
      rc |= sample ? launch_kernel(masked_logits_kernel_w4<true>, dim3((unsigned)grid), dim3(256), stream, q)
                   : launch_kernel(masked_logits_kernel_w4<false>, dim3((unsigned)grid), dim3(256), stream, q);
      if (wide) {   // the same work on the general kernel, for lists the span check flags
        fallback.row0 = (int32_t)row0;
        rc |= launch_general(fallback, grid);
      }
    } else {
      rc |= launch_general(p, grid);
    }
    if (paired) rc |= launch_general(tail, tiles < plan.grid ? tiles : plan.grid);
    if (p.splits >= kWideMergeSplits)
      rc |= launch_kernel(combine_kernel<4>, dim3((unsigned)((cap + 3) / 4)), dim3(256), stream, p);
    else
      rc |= launch_kernel(combine_kernel<16>, dim3((unsigned)((cap + 15) / 16)), dim3(256), stream, p);
    if (rc != 0) break;
  }
  return rc;
}

}  // namespace mosaic
