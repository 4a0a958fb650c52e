/*
 * mosaic_graph.h -- host-side memory planning for a dLLM denoising step: a registered graph template,
 * a single-request first-fit planner and the bottleneck-driven chunk search (C ABI, no GPU involved).
 *
 * Paper sections 4.3 (graph registrar: a parameterised graph template written down with primitives for
 * operators, address aliases and barriers, input-dependent dimensions left symbolic), 4.4 (lazy chunking:
 * chunk counts K per chunkable operator, found by a search that raises the K of the operator at the current
 * memory peak by one and re-plans, until the peak fits or no chunkable operator is at the peak) and 4.5
 * (single-request planner: lifetimes of all transient tensors over the whole graph, one offset per tensor
 * in one workspace, first-fit).  The paper gives no pseudo-code for any of them; the model below is this
 * library's reading, stated in full so that results can be checked by hand.
 *
 * Model.
 *   - A *dimension* is a runtime row count (number of tokens T, number of masked tokens M, ...).
 *   - A *chunk parameter* K belongs to one dimension; a tensor or operator tagged with it works on
 *     ceil(rows / K) rows at a time.
 *   - A *tensor* has bytes = bytes_per_row * rows, rounded up to 256; rows = the dimension's value, or
 *     ceil(value / K) if the tensor carries a chunk parameter, or 1 if it has no dimension.  Persistent
 *     tensors (weights, the step's input) live outside the workspace and are not planned.
 *   - *Operators* run in registration order.  A maximal run of consecutive operators carrying the same
 *     chunk parameter is a chunk loop: its body is repeated K times, and every tensor carrying that
 *     parameter gets a fresh instance per iteration.
 *   - Lifetime of a tensor instance = first to last step (operator execution) that names it.
 *     add_barrier(tensor, K) stretches it to the last step of K's loop(s); add_alias(a, b) makes b live
 *     at a's address: the two are planned as one block (size = the larger, lifetime = the union).
 *   - The planner places blocks in order of first step (ties: registration order, then iteration), each
 *     at the lowest offset where it overlaps no already placed block whose lifetime intersects its own.
 *     peak = max(offset + bytes).
 *   - The search starts from every K = 1.  While peak > budget: take the block that ends at the peak
 *     (ties: earliest first step), look at the operator running at that block's first step; if it
 *     carries a chunk parameter whose K is still below its dimension, raise that K by one and re-plan;
 *     otherwise report failure (the peak belongs to something that cannot be chunked).
 *
 * All functions are host-only and thread-compatible (no global state; one graph must not be mutated
 * concurrently).  Ids are dense non-negative integers in registration order; every function returns a
 * negative mosaic_status (see mosaic.h) on error.  Names are copied.
 */
#ifndef MOSAIC_GRAPH_H_
#define MOSAIC_GRAPH_H_

#include <stdint.h>

#include "mosaic.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mosaic_graph mosaic_graph;

#define MOSAIC_GRAPH_NONE (-1)
#define MOSAIC_GRAPH_ALIGN 256

/* Creates an empty template (NULL if out of memory); destroy accepts NULL. */
mosaic_graph *mosaic_graph_create(void);
void mosaic_graph_destroy(mosaic_graph *g);

/* Registers a symbolic dimension; returns its id. */
int mosaic_graph_add_dim(mosaic_graph *g, const char *name);
/* Registers a chunk parameter over dimension `dim`; returns its id. */
int mosaic_graph_add_chunk_param(mosaic_graph *g, const char *name, int dim);
/* Registers a tensor: dim = MOSAIC_GRAPH_NONE for a constant-size tensor (bytes_per_row bytes), chunk =
 * MOSAIC_GRAPH_NONE for a full-size one; a chunk parameter must belong to `dim`.  Returns the tensor id. */
int mosaic_graph_add_tensor(mosaic_graph *g, const char *name, int64_t bytes_per_row, int dim, int chunk,
                            int persistent);
/* Registers the next operator in execution order (section 4.3, add_op).  chunk = MOSAIC_GRAPH_NONE: runs
 * once.  Inputs and outputs are tensor ids (host arrays, copied).  Returns the operator id. */
int mosaic_graph_add_op(mosaic_graph *g, const char *name, const int32_t *inputs, int n_inputs,
                        const int32_t *outputs, int n_outputs, int chunk);
/* b lives at a's address (section 4.3, add_alias).  Both must be transient and carry the same chunk
 * parameter; chains are allowed (alias classes are merged). */
int mosaic_graph_add_alias(mosaic_graph *g, int tensor_a, int tensor_b);
/* The tensor stays live until the last step of the chunk loop(s) of `chunk` (section 4.3, add_barrier). */
int mosaic_graph_add_barrier(mosaic_graph *g, int tensor, int chunk);

/* One planned block of the workspace. */
typedef struct {
  int32_t tensor;     /* representative (lowest id) of the alias class                 */
  int32_t iteration;  /* chunk-loop iteration of the instance, 0 for full-size tensors */
  int32_t first_step; /* lifetime, in operator executions of the instantiated graph    */
  int32_t last_step;
  int64_t offset;     /* bytes from the start of the workspace, multiple of 256         */
  int64_t bytes;
} mosaic_placement;

/* Result summary of one planning pass. */
typedef struct {
  int64_t peak_bytes;      /* size of the single workspace request                               */
  int64_t num_blocks;      /* placements produced (may exceed the capacity passed in)            */
  int32_t num_steps;       /* operator executions of the instantiated graph                      */
  int32_t peak_block;      /* index into the placement list of the block that ends at the peak   */
  int32_t peak_op;         /* operator running at that block's first step                        */
  int32_t peak_chunk;      /* that operator's chunk parameter, or MOSAIC_GRAPH_NONE              */
} mosaic_plan_summary;

/*
 * Instantiates the template with dims[n_dims] and chunks[n_chunks] (every K >= 1; a K above its
 * dimension's value is clamped to max(value, 1)) and plans it (section 4.5, first-fit).
 *   out / capacity   host array for the placements, in placement order; may be NULL / 0 to get only
 *                    the summary.  At most `capacity` entries are written.
 * Errors: INVALID_ARG (null graph or summary, wrong counts, negative dimension, K < 1).
 */
int mosaic_graph_plan(const mosaic_graph *g, const int64_t *dims, int n_dims, const int32_t *chunks, int n_chunks,
                      mosaic_placement *out, int64_t capacity, mosaic_plan_summary *summary);

/*
 * Bottleneck-driven search (section 4.4): the minimal chunk counts, found by raising the K at the current
 * peak one at a time, whose planned peak fits `budget_bytes`.
 *   chunks_out[n_chunks]   receives the K of every chunk parameter (all 1 when no chunking is needed)
 *   summary                of the final plan (also filled on failure, for the last plan tried)
 *   evaluations            number of planning passes made (may be NULL)
 * Returns MOSAIC_OK, or MOSAIC_ERR_WORKSPACE_TOO_SMALL when the peak cannot be reduced further (the
 * operator at the peak carries no chunk parameter, or its K has reached its dimension).
 */
int mosaic_graph_search(const mosaic_graph *g, const int64_t *dims, int n_dims, int64_t budget_bytes,
                        int32_t *chunks_out, int n_chunks, mosaic_plan_summary *summary, int32_t *evaluations);

#ifdef __cplusplus
}
#endif
#endif /* MOSAIC_GRAPH_H_ */
