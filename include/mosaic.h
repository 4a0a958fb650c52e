/*
 * mosaic.h -- C ABI of libmosaic: the mask-only logits hot path of a diffusion-LLM
 * denoising step (Mosaic, arXiv 2601.06562), for AMD MI355X (gfx950).
 *
 * The path (paper section 2.1 "Diffusion", section 3 observation #2, section 4.2):
 * a denoising step needs logits only for the positions that are still [MASK]; the
 * kernel takes the hidden states of ALL positions plus the indices of the masked
 * ones, gathers rows by indirect addressing while it multiplies by the LM head, and
 * keeps no gathered copy in global memory.  This library goes one step further than
 * the paper's kernel: the vocabulary reduction that sampling needs (arg-max id, its
 * soft-max probability, the row's log-sum-exp) is fused into the GEMM epilogue, so
 * neither [T,V] nor [M,V] logits ever exist in memory.  Section 4.4's chunking of
 * the logits operator along the sequence dimension (chunk count K_logits: chunking stays
 * off unless memory is short, and K is then the smallest that fits) appears as mosaic_plan_workspace.
 *
 * Conventions for every call
 *   - "dev" pointers are device (HBM) pointers owned by the CALLER; "host" pointers
 *     are ordinary host memory.  The compute calls allocate and free no device memory
 *     and keep no state between calls.  The one exception is the mosaic_vmm_* object at
 *     the end of this header: it owns a virtual address range and the physical pages
 *     mapped behind it, and mosaic_vmm_resize / mosaic_vmm_destroy wait for the device.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work on it and return; they never synchronise the device
 *     (mosaic_vmm_* excepted, as above).
 *   - Return value: MOSAIC_OK (0) or a negative mosaic_status.  Argument and shape errors
 *     are found before anything is enqueued; MOSAIC_ERR_HIP reports a failed launch, and
 *     earlier launches of the same call may then already be in the stream (outputs are
 *     unspecified).  mosaic_status_string() names a status.
 *   - T = flat number of positions (a batch is the concatenation of its sequences,
 *     no padding -- paper section 5.1), M = number of masked positions, d = hidden
 *     size, V = vocabulary size.
 */
#ifndef MOSAIC_H_
#define MOSAIC_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOSAIC_OK = 0,
  MOSAIC_ERR_INVALID_ARG = -1,        /* null pointer, negative size, misaligned pointer     */
  MOSAIC_ERR_UNSUPPORTED_SHAPE = -2,  /* d, ld_h, T or V outside what the kernels handle      */
  MOSAIC_ERR_WORKSPACE_TOO_SMALL = -3,/* budget / workspace below the non-chunkable minimum   */
  MOSAIC_ERR_HIP = -4                 /* a HIP runtime call failed (launch, attribute query)  */
} mosaic_status;

/* Name of a status code; static storage, never NULL. */
const char *mosaic_status_string(int status);

/* Tile sizes of the fused kernel, exported so callers can size things:
 * rows of masked tokens per tile, vocabulary ids per tile, and the multiple d must have. */
#define MOSAIC_ROW_TILE 256
#define MOSAIC_VOCAB_TILE 256
#define MOSAIC_K_TILE 64
#define MOSAIC_MAX_VOCAB_SPLITS 256
/* Bytes at the end of every workspace for the round counters of the persistent grid (see mosaic_plan_workspace);
 * the last word is the flag of the device-side check described at MOSAIC_PLAN_GENERAL_KERNEL. */
#define MOSAIC_SYNC_BYTES 1024

/* Result of the chunk-size selector.  All fields are filled by mosaic_plan_workspace;
 * callers may read them and may set `flags`, nothing else. */
typedef struct {
  int64_t workspace_bytes; /* bytes mosaic_masked_logits_reduce needs in `workspace`    */
  int32_t num_chunks;      /* K_logits: number of sequential chunks over masked rows    */
  int32_t rows_per_chunk;  /* C: masked rows per chunk, a multiple of MOSAIC_ROW_TILE   */
  int32_t vocab_splits;    /* S: vocabulary ranges whose partial results are merged     */
  int32_t tile_panel;      /* row tiles scheduled side by side (cache-sharing group)    */
  int32_t grid;            /* persistent workgroups launched per chunk                  */
  int32_t flags;           /* MOSAIC_PLAN_* bits (see below)                              */
} mosaic_plan;

/* plan.flags bit: use the general 8-wave kernel even where the hand-scheduled 4-wave kernel applies
 * (it applies to the whole tiles of the vocabulary; in a hidden tensor of 4 GiB or more it needs every 64
 * consecutive rows of the gather list to lie less than 4 GiB apart, which a small kernel checks on the device
 * before the launch, handing lists with such a gap to the general kernel).  Both give the same results; the flag
 * exists for testing and tuning. */
#define MOSAIC_PLAN_GENERAL_KERNEL 1
/* plan.flags bit, set by the selector: the plan was sized for a sampling step (20 bytes per row and
 * vocabulary split in workspace_bytes instead of 12). */
#define MOSAIC_PLAN_SAMPLING 2

/*
 * Chunk-size selector (paper section 4.4: the lazy chunking strategy and its
 * bottleneck-driven search, restricted to the one chunkable operator on this path).
 * Host-only, pure function.  Starts from K = 1 (chunking off); while the workspace of
 * one chunk of C = roundup(ceil(max_rows / K), MOSAIC_ROW_TILE) rows exceeds
 * budget_bytes even with a single vocabulary split, K is raised by one; stops at the
 * first K that fits (the minimal one) and fails with MOSAIC_ERR_WORKSPACE_TOO_SMALL
 * when even one row tile with one split does not fit (the non-chunkable floor).
 * The workspace is 12 * S * C + MOSAIC_SYNC_BYTES bytes (one (max, sum-exp, arg-max) triple per
 * row and vocabulary split, and a fixed kilobyte of counters on which the workgroups of a launch
 * that each take several units meet between units) -- never O(C * V); 20 * S * C +
 * MOSAIC_SYNC_BYTES when the plan is for a sampling step (mosaic_masked_logits_sample with
 * temperature > 0 keeps two more values per partial), so that the budget bounds what that call
 * really needs.
 *   T          total positions, >= 0, < 2^31
 *   max_rows   host-side upper bound on M (the search in the paper is driven by the
 *              number of masks and the number of tokens; pass T if M is unknown), 0..T.  Results do
 *              not depend on it, speed does: the number of vocabulary splits is chosen so that
 *              max_rows rows fill the chip, so a bound far above the actual M leaves compute units idle
 *              (planning is a host-side function of a few microseconds: plan again as the masks shrink)
 *   d, V       hidden and vocabulary size; d must be a multiple of MOSAIC_K_TILE
 *   budget_bytes  <= 0 means unbounded
 *   num_cus    compute units to schedule for; <= 0 means 256 (one MI355X)
 *   sampling   0: plan for mosaic_masked_logits_reduce; 1: plan for mosaic_masked_logits_sample with
 *              temperature > 0 (sets MOSAIC_PLAN_SAMPLING); anything else is INVALID_ARG
 *   out_plan   host pointer, written on success
 */
int mosaic_plan_workspace(int64_t T, int64_t max_rows, int32_t d, int32_t V, int64_t budget_bytes,
                          int32_t num_cus, int32_t sampling, mosaic_plan *out_plan);

/*
 * Stream compaction of the mask (paper section 4.2: the gather-GEMM kernel takes the list of
 * masked positions as an input and does not say who builds it; this call builds it).  Exclusive prefix sum over
 * mask[t] != 0, then out_idx[scan[t]] = t: the masked positions in ascending order,
 * bit-exact.  Any nonzero byte counts as masked.
 *   mask       dev uint8[T]
 *   out_idx    dev int32[max(T,1)]; the first M entries are written, the rest untouched
 *   out_count  dev int32[1]; receives M
 *   scratch    dev, at least mosaic_compact_scratch_bytes(T) bytes, 4-byte aligned
 * T == 0 is valid (count = 0).  Errors: INVALID_ARG (null pointer, T < 0, scratch too
 * small), UNSUPPORTED_SHAPE (T >= 2^31), HIP.
 */
int64_t mosaic_compact_scratch_bytes(int64_t T);
int mosaic_mask_compact(const uint8_t *mask, int64_t T, int32_t *out_idx, int32_t *out_count, void *scratch,
                        int64_t scratch_bytes, void *stream);

/*
 * Mask-only logits with the vocabulary reduction fused in (paper section 4.2 for the
 * gather-GEMM; section 2.1 only says that a step draws tokens from the logits, and the
 * reduction here is this library's reading of that: greedy).  For every j < *count, with t = idx[j]:
 *   x[v]        = sum_k hidden[t,k] * w[v,k]      bf16 x bf16, fp32 accumulation, no bias
 *   out_token[j] = lowest v attaining max_v x[v]
 *   out_lse[j]   = log sum_v exp(x[v])
 *   out_conf[j]  = exp(max_v x[v] - out_lse[j])   (soft-max probability of out_token[j])
 * Rows are processed in plan->num_chunks sequential chunks of plan->rows_per_chunk.
 *   hidden     dev bf16[T, d], row-major, row stride ld_h elements (ld_h >= d,
 *              ld_h % 8 == 0), 16-byte aligned; only rows named by idx are read
 *   w          dev bf16[V, d], row-major, dense, 16-byte aligned
 *   idx        dev int32[>= *count], every entry in [0, T) (as mosaic_mask_compact makes).  An entry
 *              outside that range in a caller-built list is clamped to it on the device: the row's
 *              results are then those of row 0 or T - 1, and nothing outside `hidden` is read
 *   count      dev int32[1], read on the device: 0 <= *count <= max_rows.  If it exceeds
 *              max_rows only the first max_rows rows are produced.
 *   max_rows   the bound the plan was made for
 *   out_*      dev, max_rows entries each; entries >= *count are left untouched
 *   plan       host pointer, from mosaic_plan_workspace with the same T, max_rows, d, V
 *   workspace  dev, >= plan->workspace_bytes, 16-byte aligned; contents are scratch.  Calls that may run
 *              concurrently (different streams) need workspaces of their own
 * max_rows == 0 or V == 0 enqueue nothing.  Inputs must be finite; a NaN or Inf in a
 * row gives unspecified values for that row only.  The accuracy the tests hold the call to (2e-3 absolute
 * on out_lse and out_conf) is met for logits of magnitude up to a few thousand.  Errors: INVALID_ARG,
 * UNSUPPORTED_SHAPE (d % MOSAIC_K_TILE, ld_h, T >= 2^31, V >= 2^31 - 256),
 * WORKSPACE_TOO_SMALL, HIP.
 */
int mosaic_masked_logits_reduce(const void *hidden, int64_t T, int32_t d, int64_t ld_h, const void *w, int32_t V,
                                const int32_t *idx, const int32_t *count, int64_t max_rows, int32_t *out_token,
                                float *out_conf, float *out_lse, const mosaic_plan *plan, void *workspace,
                                int64_t workspace_bytes, void *stream);

/*
 * Name of the kernel (or pair of kernels) that mosaic_masked_logits_reduce (sampling = 0) or
 * mosaic_masked_logits_sample with temperature > 0 (sampling = 1) launches for these sizes and this plan, as it
 * appears in a profiler's kernel trace; for reports.  Host-only, static storage; "" for a NULL plan or sizes the
 * calls reject.
 */
const char *mosaic_masked_logits_kernel_name(int64_t T, int32_t d, int64_t ld_h, int32_t V, const mosaic_plan *plan,
                                             int32_t sampling);

/*
 * mosaic_masked_logits_reduce for callers that cannot allocate device memory or hand in a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors as mosaic_masked_logits_reduce, except that the partial results go to a fixed array of
 * MOSAIC_STATIC_WORKSPACE_BYTES inside the library's device image instead of a caller's `workspace`; the call
 * itself allocates and frees nothing.
 *   plan   must need at most MOSAIC_STATIC_WORKSPACE_BYTES (plan->workspace_bytes of a greedy plan), else
 *          MOSAIC_ERR_WORKSPACE_TOO_SMALL and nothing is enqueued: make the plan with
 *          budget_bytes = MOSAIC_STATIC_WORKSPACE_BYTES and the selector chunks the rows to fit
 * Every GPU the library runs on holds one copy of the array until the process ends, and every call on a GPU uses
 * that GPU's copy (the current device of the calling thread, which must be `stream`'s): calls that overlap on
 * one GPU -- different streams, or a captured graph replayed while another call runs -- race on it; calls in
 * one stream are ordered and safe.  Nothing in the array needs to start at zero (every partial that is read has
 * been written by the same call).  The first call on a device looks the array's address up (one
 * hipGetSymbolAddress, which may load the library's device image): make it before a capture begins.
 */
#define MOSAIC_STATIC_WORKSPACE_BYTES (4 << 20)
int mosaic_masked_logits_reduce_static(const void *hidden, int64_t T, int32_t d, int64_t ld_h, const void *w, int32_t V,
                                       const int32_t *idx, const int32_t *count, int64_t max_rows,
                                       int32_t *out_token, float *out_conf, float *out_lse, const mosaic_plan *plan,
                                       void *stream);

/*
 * The same fused pass with temperature sampling in place of the arg-max (paper section 2.1: tokens are
 * sampled from the logits; the paper fixes no sampler -- the reading here is the Gumbel-max form of
 * categorical sampling at temperature tau, which draws v with probability softmax(x / tau)[v] and needs
 * no second pass over the logits).  For every j < *count, with t = idx[j] and x as above:
 *   g[v]         = -ln(-ln u[v]),  u[v] = ((word >> 9) + 1/2) * 2^-23, where word is output word v % 4 of
 *                  Philox4x32-10 (Salmon et al., SC'11) with key = (low, high 32 bits of seed) and
 *                  counter = (v / 4, n, 0, 0), n = noise_idx[j] (idx[j] when noise_idx is NULL): the noise
 *                  depends on (seed, position, id) only, not on the chunking, the vocabulary split or the
 *                  launch shape
 *   out_token[j] = lowest v attaining max_v ( x[v] + temperature * g[v] )      (fp32)
 *   out_lse[j]   = log sum_v exp(x[v])                                          (of the unperturbed logits)
 *   out_conf[j]  = exp(x[out_token[j]] - out_lse[j])
 * temperature == 0 is exactly mosaic_masked_logits_reduce.  All other arguments are as there, except
 *   noise_idx  dev int32[>= *count] or NULL: the position whose prediction row j is.  It differs from
 *              idx[j] when the gather list is shifted (mosaic_shift_indices: position p reads hidden row
 *              p - 1, and a sequence start s and s + 1 both read row s); passing the unshifted positions
 *              here keeps the draws of different positions independent.  Any int32 value is valid
 *   workspace  dev, >= mosaic_sample_workspace_bytes(plan) when temperature > 0 (20 bytes per row of a
 *              chunk and vocabulary split instead of 12, plus MOSAIC_SYNC_BYTES; plan->workspace_bytes
 *              already says so when the plan was made with sampling = 1), 16-byte aligned
 *   seed       any value; callers advance it per denoising step
 * Additional errors: INVALID_ARG for a negative, NaN or infinite temperature.
 * mosaic_sample_workspace_bytes returns 0 for a NULL or unfilled plan.
 */
int64_t mosaic_sample_workspace_bytes(const mosaic_plan *plan);
int mosaic_masked_logits_sample(const void *hidden, int64_t T, int32_t d, int64_t ld_h, const void *w, int32_t V,
                                const int32_t *idx, const int32_t *noise_idx, const int32_t *count, int64_t max_rows,
                                float temperature, uint64_t seed, int32_t *out_token, float *out_conf, float *out_lse,
                                const mosaic_plan *plan, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * Sampling tail of a denoising step (paper section 2.1: the tokens sampled from the logits replace a
 * selected subset of the [MASK] positions; the paper does not say which subset -- the reading here is
 * greedy decoding's: per sequence the n masked positions with the highest confidence, ties going to the
 * lower position).  For every selected row j: tokens[idx[j]] = token[j] and mask[idx[j]] = 0; nothing
 * else is written, so the next step's mosaic_mask_compact sees the updated mask.
 *   conf, token, idx, count   dev, as produced by the two calls above (confidences are >= 0)
 *   max_rows                  bound on *count
 *   seq_starts                dev int32[num_seqs + 1], ascending flat positions delimiting the sequences
 *                             (seq_starts[0] = 0, seq_starts[num_seqs] = T)
 *   n_per_seq                 dev int32[num_seqs]; a sequence with fewer masked rows unmasks them all
 *   tokens                    dev int32[T], the token sequence(s); mask: dev uint8[T].  A row whose idx entry
 *                             lies outside [0, T) is skipped
 * One workgroup per sequence; selection is exact (radix select on the fp32 bit patterns).
 * Errors: INVALID_ARG (null pointer, negative size, num_seqs < 1), UNSUPPORTED_SHAPE (T or max_rows >= 2^31).
 */
int mosaic_unmask_topn(const float *conf, const int32_t *token, const int32_t *idx, const int32_t *count,
                       int64_t max_rows, const int32_t *seq_starts, int32_t num_seqs, const int32_t *n_per_seq,
                       int32_t *tokens, uint8_t *mask, int64_t T, void *stream);

/*
 * Dream-style shifted prediction without a shifted tensor (paper section 4.5, last paragraph: Dream's
 * logits shift and concatenation replaced by a token-level alternative; no detail is given).  Reading:
 * the prediction for position p comes from the hidden state of position p - 1, except at the first
 * position of a sequence, which keeps its own.  out_gather[j] = that hidden row for idx[j]; pass it as
 * `idx` to mosaic_masked_logits_reduce (outputs stay in the order of the masked positions).
 *   idx, count, max_rows, seq_starts, num_seqs   as above;  out_gather: dev int32[max_rows], every entry
 *                                                written is in [0, T) (T = seq_starts[num_seqs])
 */
int mosaic_shift_indices(const int32_t *idx, const int32_t *count, int64_t max_rows, const int32_t *seq_starts,
                         int32_t num_seqs, int32_t *out_gather, void *stream);

/*
 * Measurement aid, not part of the method: a register-only loop of the bf16 matrix instruction the fused
 * kernel is built on (v_mfma_f32_16x16x32_bf16, the kernel's own 8 x 8 accumulator grid, one wave per SIMD,
 * no memory traffic inside the loop).  Its rate is what the matrix cores sustain at the clock the chip
 * settles to under that load; bench.py reports the fused kernel against it as well as against the datasheet
 * peak.  Each of num_wgs workgroups (256 threads) issues iters x 4 x 64 instructions;
 * mosaic_mfma_probe_flops returns the flops of one launch (0 for negative arguments).
 *   operands   dev, 64 KiB of finite bf16 values, 16-byte aligned (read once)
 *   sink       dev float[65536]; overwritten with values of no interest
 * Errors: INVALID_ARG (null or misaligned pointer, iters outside [1, 2^20], num_wgs outside [1, 65536]), HIP.
 */
int64_t mosaic_mfma_probe_flops(int32_t iters, int32_t num_wgs);
int mosaic_mfma_probe(const void *operands, float *sink, int32_t iters, int32_t num_wgs, void *stream);

/*
 * Workspace on virtual memory (paper section 4.5, VMM-based allocator): reserve a large contiguous range of
 * virtual addresses once (no memory is taken), then map physical pages behind its start up to the planned
 * peak of each request; the pointer never changes, so it can be handed to the calls above as `workspace`
 * (or sliced by the offsets of a mosaic_graph plan).
 *   mosaic_vmm_create     reserves reserve_bytes (rounded up to the mapping granularity) on `device`, which
 *                         must be the current device of the calling thread for every later call on the object.
 *                         UNSUPPORTED_SHAPE if the device has no virtual memory management.
 *   mosaic_vmm_resize     makes exactly `bytes`, rounded up to the granularity, of the range usable.  A call
 *                         that does not change the rounded size does nothing.  Growth first tries to map further
 *                         pages behind the ones already there: no wait, the contents stay, and if the device has
 *                         no memory left the call returns HIP with the old pages still mapped.  If the driver
 *                         refuses that for another reason, and for a shrink or a first mapping, the call waits
 *                         for the device to be idle (hipDeviceSynchronize -- the only call of this library that
 *                         does), drops the old mapping and maps new pages at the same address: the contents do
 *                         NOT survive that; HIP if the driver refuses, e.g. out of memory (the range is then left
 *                         with nothing mapped: committed_bytes() == 0).  WORKSPACE_TOO_SMALL if bytes exceeds the
 *                         reservation (nothing changes).
 *   mosaic_vmm_kept_contents  nonzero if the last resize that changed the size kept what the range held (1: the
 *                         driver opened the whole mapped prefix in one call, 2: it refused that and opened the
 *                         new pages alone), else 0.
 *   mosaic_vmm_ptr        device pointer to the start of the range (granularity-aligned); only the first
 *                         mosaic_vmm_committed_bytes() bytes may be touched -- beyond them is unmapped
 *                         address space and an access faults.
 *   mosaic_vmm_destroy    waits for the device, unmaps, releases and frees the reservation; accepts NULL.
 * mosaic_vmm_resize and mosaic_vmm_destroy return INVALID_ARG when the calling thread's current device is not the
 * object's (the wait would act on the wrong device).
 * The object is owned by the caller and is not thread-safe.
 */
typedef struct mosaic_vmm mosaic_vmm;
int mosaic_vmm_create(int device, int64_t reserve_bytes, mosaic_vmm **out);
int mosaic_vmm_resize(mosaic_vmm *v, int64_t bytes);
void *mosaic_vmm_ptr(const mosaic_vmm *v);
int64_t mosaic_vmm_committed_bytes(const mosaic_vmm *v);
int64_t mosaic_vmm_reserved_bytes(const mosaic_vmm *v);
int64_t mosaic_vmm_granularity(const mosaic_vmm *v);
int mosaic_vmm_kept_contents(const mosaic_vmm *v);
/* Name of the driver call behind the most recent MOSAIC_ERR_HIP of mosaic_vmm_resize ("" if none) and, if
 * hip_error is not NULL, its hipError_t value.  Static storage. */
const char *mosaic_vmm_last_error(const mosaic_vmm *v, int *hip_error);
int mosaic_vmm_destroy(mosaic_vmm *v);

/* Library version, "major.minor" as major*1000 + minor. */
int mosaic_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MOSAIC_H_ */
