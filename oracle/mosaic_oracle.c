/*
 * mosaic_oracle.c -- plain CPU oracle for the mask-only logits path of a dLLM
 * denoising step (Mosaic, arXiv 2601.06562).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is slow on purpose, shares
 * no code with the HIP library, and may be called only from tests, from the
 * smoke check and from the benchmark's cpu_baseline leg.
 *
 * What it computes (paper section 2.1 "Diffusion": a forward pass yields
 * logits, tokens are then picked from them for [MASK] positions; section 3
 * observation #2 and section 4.2: computing logits only for masked tokens is
 * pure redundancy elimination, i.e. it equals "logits for every position,
 * then keep the masked rows").  The paper does not say how a token is picked
 * from a row of logits; the reading taken here is the greedy one: per row the
 * arg-max vocabulary id (lowest id on ties), the soft-max probability of that
 * id ("confidence") and the log-sum-exp of the row.
 *
 * Definition, per position t (independent of the mask):
 *   x[t,v] = sum_k H[t,k] * W[v,k]      bf16 inputs widened exactly, the sum
 *                                       taken in fp64 and rounded once to fp32
 *   m[t]   = max_v x[t,v]       tok[t] = min{ v : x[t,v] == m[t] }
 *   s[t]   = sum_v exp(x[t,v]-m[t])     (fp64, on the fp32 logits)
 *   lse[t] = m[t] + ln s[t]     conf[t] = exp(m[t]-lse[t]) = 1/s[t]
 *   gap[t] = m[t] - max_{v != tok[t]} x[t,v]   (0 when the maximum is repeated)
 * Selection: idx = ascending positions t with mask[t] != 0; outputs are the
 * per-position values at idx[0..M-1].
 *
 * No blocking, no fusion, no reordering: one row of V logits at a time.
 * The only liberty is that the fp64 dot product may be summed in any order
 * (OpenMP simd reduction); its terms are exact products of bf16 values, so
 * the fp64 sum is exact or within 1 ulp(fp64) in every order, far below the
 * final rounding to fp32.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline float bf16_to_f32(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

/* Stable selection of the masked positions (paper section 4.2: the kernel takes the
 * list of masked positions as an input; ascending order is the reading taken here).
 * mask: T bytes, nonzero = still masked.  idx: room for T entries.
 * Returns M, the number of masked positions. */
int64_t oracle_mask_select(const uint8_t *mask, int64_t T, int32_t *idx) {
  int64_t M = 0;
  for (int64_t t = 0; t < T; ++t) {
    if (mask[t] != 0) {
      idx[M] = (int32_t)t;
      M += 1;
    }
  }
  return M;
}

/* One row of logits: x[v] = fp32( sum_k h[k] * W[v,k] ), fp64 accumulation.
 * h: d bf16 values; W: V rows of d bf16 values (row stride d). */
void oracle_row_logits(const uint16_t *h, const uint16_t *W, int32_t d,
                       int32_t V, float *x) {
  double *hd = (double *)malloc(sizeof(double) * (size_t)d);
  for (int32_t k = 0; k < d; ++k) hd[k] = (double)bf16_to_f32(h[k]);
  for (int32_t v = 0; v < V; ++v) {
    const uint16_t *w = W + (size_t)v * (size_t)d;
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int32_t k = 0; k < d; ++k) acc += hd[k] * (double)bf16_to_f32(w[k]);
    x[v] = (float)acc;
  }
  free(hd);
}

/* A second way to the same logits, for measuring how much the order of accumulation matters: plain fp32
 * accumulation in ascending k (each product of two bf16 values is exact in fp32, so rounding happens only in
 * the additions).  Not used for parity; the parity reference is oracle_row_logits. */
void oracle_row_logits_f32seq(const uint16_t *h, const uint16_t *W, int32_t d,
                              int32_t V, float *x) {
  for (int32_t v = 0; v < V; ++v) {
    const uint16_t *w = W + (size_t)v * (size_t)d;
    float acc = 0.0f;
    for (int32_t k = 0; k < d; ++k) acc += bf16_to_f32(h[k]) * bf16_to_f32(w[k]);
    x[v] = acc;
  }
}

/* Reduce one row of V fp32 logits to (tok, conf, lse, gap, rowmax). */
void oracle_row_reduce(const float *x, int32_t V, int32_t *tok, float *conf,
                       float *lse, float *gap, float *rowmax) {
  double m = (double)x[0];
  int32_t arg = 0;
  for (int32_t v = 1; v < V; ++v) {
    if ((double)x[v] > m) { /* strict: the lowest id wins a tie */
      m = (double)x[v];
      arg = v;
    }
  }
  double second = -INFINITY;
  for (int32_t v = 0; v < V; ++v) {
    if (v != arg && (double)x[v] > second) second = (double)x[v];
  }
  double s = 0.0;
  for (int32_t v = 0; v < V; ++v) s += exp((double)x[v] - m);
  double l = m + log(s);
  *tok = arg;
  *lse = (float)l;
  *conf = (float)exp(m - l);
  *gap = (V > 1) ? (float)(m - second) : INFINITY;
  *rowmax = (float)m;
}

/* The per-position results at an explicit list of positions.  Rows are
 * independent, so this is exactly the restriction of the full computation to
 * those positions; it is how the large workloads are checked on a sample.
 * H: [T, d] bf16 with row stride ld_h elements.  pos: n positions in [0,T).
 * Outputs have n entries.  logits_out (may be NULL): n*V fp32, the rows of
 * logits themselves.  Returns 0, or -1 on a position out of range. */
int oracle_positions(const uint16_t *H, int64_t T, int32_t d, int64_t ld_h,
                     const uint16_t *W, int32_t V, const int64_t *pos,
                     int64_t n, int32_t *tok, float *conf, float *lse,
                     float *gap, float *rowmax, float *logits_out) {
  for (int64_t j = 0; j < n; ++j)
    if (pos[j] < 0 || pos[j] >= T) return -1;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t j = 0; j < n; ++j) {
    float *x = logits_out ? logits_out + (size_t)j * (size_t)V
                          : (float *)malloc(sizeof(float) * (size_t)V);
    oracle_row_logits(H + (size_t)pos[j] * (size_t)ld_h, W, d, V, x);
    oracle_row_reduce(x, V, &tok[j], &conf[j], &lse[j], &gap[j], &rowmax[j]);
    if (!logits_out) free(x);
  }
  return 0;
}

/* The literal statement: results for EVERY position 0..T-1, then keep the
 * masked ones.  idx/tok/conf/lse/gap/rowmax: room for T entries each; the
 * first M are written.  Returns M. */
int64_t oracle_full_then_select(const uint16_t *H, int64_t T, int32_t d,
                                int64_t ld_h, const uint16_t *W, int32_t V,
                                const uint8_t *mask, int32_t *idx,
                                int32_t *tok, float *conf, float *lse,
                                float *gap, float *rowmax) {
  if (T <= 0) return 0;
  int32_t *tok_all = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
  float *conf_all = (float *)malloc(sizeof(float) * (size_t)T);
  float *lse_all = (float *)malloc(sizeof(float) * (size_t)T);
  float *gap_all = (float *)malloc(sizeof(float) * (size_t)T);
  float *max_all = (float *)malloc(sizeof(float) * (size_t)T);
  int64_t *all = (int64_t *)malloc(sizeof(int64_t) * (size_t)T);
  for (int64_t t = 0; t < T; ++t) all[t] = t;
  oracle_positions(H, T, d, ld_h, W, V, all, T, tok_all, conf_all, lse_all,
                   gap_all, max_all, NULL);
  int64_t M = oracle_mask_select(mask, T, idx);
  for (int64_t j = 0; j < M; ++j) {
    int32_t t = idx[j];
    tok[j] = tok_all[t];
    conf[j] = conf_all[t];
    lse[j] = lse_all[t];
    gap[j] = gap_all[t];
    rowmax[j] = max_all[t];
  }
  free(tok_all); free(conf_all); free(lse_all); free(gap_all); free(max_all);
  free(all);
  return M;
}

/* Number of threads oracle_positions runs on (for the benchmark's report). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif

/* ---- Sampling tail of a denoising step (paper section 2.1: the sampled tokens replace a selected
 * subset of the [MASK] positions).  The paper does not say which subset; the reading taken is the
 * one diffusion LLMs use for greedy decoding: per sequence, the n masked positions with the highest
 * confidence, ties going to the lower position.  Plain selection by repeated maximum, O(n*m).
 *
 * conf/tok/idx: the M per-row results in ascending position order.  seq_starts: B+1 ascending flat
 * positions delimiting the sequences.  n_per_seq: how many positions to unmask in each sequence
 * (all of them if it has fewer masked positions).  tokens (int32[T]) and mask (uint8[T]) are updated
 * in place.  Returns the number of positions unmasked. */
int64_t oracle_unmask_topn(const float *conf, const int32_t *tok, const int32_t *idx, int64_t M,
                           const int32_t *seq_starts, int32_t B, const int32_t *n_per_seq,
                           int32_t *tokens, uint8_t *mask) {
  int64_t done = 0;
  uint8_t *taken = (uint8_t *)calloc((size_t)(M > 0 ? M : 1), 1);
  for (int32_t b = 0; b < B; ++b) {
    for (int32_t k = 0; k < n_per_seq[b]; ++k) {
      int64_t best = -1;
      for (int64_t j = 0; j < M; ++j) {
        if (taken[j] || idx[j] < seq_starts[b] || idx[j] >= seq_starts[b + 1]) continue;
        if (best < 0 || conf[j] > conf[best]) best = j; /* strict: earlier (lower) position wins ties */
      }
      if (best < 0) break;
      taken[best] = 1;
      tokens[idx[best]] = tok[best];
      mask[idx[best]] = 0;
      done += 1;
    }
  }
  free(taken);
  return done;
}

/* Dream-style shifted gather (paper section 4.5, last paragraph: the logits shift and concatenation
 * of Dream replaced by a token-level alternative; no detail is given).  Reading: the prediction for
 * position p is made from the hidden state of position p-1, except at the first position of a
 * sequence, which keeps its own.  gather[j] = idx[j] - 1 unless idx[j] is a sequence start. */
void oracle_shift_indices(const int32_t *idx, int64_t M, const int32_t *seq_starts, int32_t B,
                          int32_t *gather) {
  for (int64_t j = 0; j < M; ++j) {
    int is_start = 0;
    for (int32_t b = 0; b < B; ++b)
      if (idx[j] == seq_starts[b]) is_start = 1;
    gather[j] = is_start ? idx[j] : idx[j] - 1;
  }
}

/* ---- Sampling with temperature (rest of the sampling tail; paper section 2.1 only says that tokens
 * are sampled from the logits).  Reading: the Gumbel-max rule diffusion LLMs use, noise scaled by the
 * temperature tau:   tok = argmax_v ( x[v] + tau * g[v] ),  g = -ln(-ln u),  u uniform in (0,1),
 * conf = softmax(x)[tok] = exp(x[tok] - lse)  (the probability of the token actually picked),
 * lse as before.  tau = 0 is the greedy rule.  The random numbers are a pure function of
 * (seed, position, vocabulary id), so the HIP path can draw the same ones: Philox4x32-10 (Salmon et al.,
 * "Parallel random numbers: as easy as 1, 2, 3", SC'11) with key = (seed low, seed high) and counter =
 * (v / 4, position, 0, 0); output word v % 4; u = ((word >> 9) + 1/2) * 2^-23, which is exact in fp32
 * as well (23 bits plus the half), never 0 and never 1. */
static inline uint32_t mulhi32(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32); }

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    uint32_t hi0 = mulhi32(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    uint32_t hi1 = mulhi32(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    uint32_t n0 = hi1 ^ c1 ^ k0, n1 = lo1, n2 = hi0 ^ c3 ^ k1, n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform in (0,1) for (seed, position, vocabulary id); 23 bits, never 0 or 1. */
double oracle_uniform(uint64_t seed, int32_t position, int32_t v) {
  uint32_t ctr[4] = {(uint32_t)v >> 2, (uint32_t)position, 0u, 0u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  oracle_philox4x32_10(ctr, key, out);
  return ((double)(out[v & 3] >> 9) + 0.5) * (1.0 / 8388608.0);
}

double oracle_gumbel(uint64_t seed, int32_t position, int32_t v) {
  return -log(-log(oracle_uniform(seed, position, v)));
}

/* One row: logits x[V] (fp32) -> sampled token, its probability, lse, and the top-2 gap of the
 * perturbed scores (for the acceptance rule). */
void oracle_row_sample(const float *x, int32_t V, double tau, uint64_t seed, int32_t position,
                       int32_t *tok, float *conf, float *lse, float *ygap) {
  double m = (double)x[0];
  for (int32_t v = 1; v < V; ++v) if ((double)x[v] > m) m = (double)x[v];
  double s = 0.0;
  for (int32_t v = 0; v < V; ++v) s += exp((double)x[v] - m);
  double l = m + log(s);
  double best = -INFINITY, second = -INFINITY;
  int32_t arg = 0;
  for (int32_t v = 0; v < V; ++v) {
    double y = (double)x[v] + (tau > 0.0 ? tau * oracle_gumbel(seed, position, v) : 0.0);
    if (y > best) { second = best; best = y; arg = v; }   /* strict: lowest id on ties */
    else if (y > second) second = y;
  }
  *tok = arg;
  *lse = (float)l;
  *conf = (float)exp((double)x[arg] - l);
  *ygap = (V > 1) ? (float)(best - second) : INFINITY;
}
