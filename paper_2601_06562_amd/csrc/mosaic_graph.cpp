// Host-side memory planning: graph registrar, chunk-loop instantiation, single-request first-fit planner and
// the bottleneck-driven chunk search (paper sections 4.3, 4.4, 4.5).  The model is stated in mosaic_graph.h.
//
// Everything here is plain host C++ on small data (a step's graph has tens of operators, an instantiated plan
// at most a few thousand blocks), so the planner keeps the placed blocks in one vector sorted by offset and
// scans it per block: O(n^2) in the worst case, microseconds in practice -- the search re-plans once per
// increment of a chunk count, and that has to stay negligible next to a denoising step (section 4.4).
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "mosaic_graph.h"

namespace {

struct Chunk {
  std::string name;
  int dim;
};
struct Tensor {
  std::string name;
  int64_t bytes_per_row;
  int dim, chunk;
  bool persistent;
};
struct Op {
  std::string name;
  std::vector<int32_t> inputs, outputs;
  int chunk;
};
struct Step {
  int32_t op, iteration, run;
};
struct Run {
  int32_t chunk, first, last;
};
struct Block {
  int32_t tensor, iteration, first, last;
  int64_t bytes, offset;
};

int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

}  // namespace

struct mosaic_graph {
  std::vector<std::string> dims;
  std::vector<Chunk> chunks;
  std::vector<Tensor> tensors;
  std::vector<Op> ops;
  std::vector<int32_t> alias_parent;                  // union-find over tensors, root = lowest id of the class
  std::vector<std::pair<int32_t, int32_t>> barriers;  // (tensor, chunk)

  int32_t find(int32_t t) const {
    while (alias_parent[t] != t) t = alias_parent[t];
    return t;
  }
};

namespace {

struct Instance {
  std::vector<int64_t> k;       // effective chunk counts
  std::vector<Step> steps;
  std::vector<Run> runs;
  std::vector<Block> blocks;    // in placement order, offsets filled
  mosaic_plan_summary summary;
};

bool has_barrier(const mosaic_graph& g, int32_t tensor, int32_t chunk) {
  for (const auto& b : g.barriers)
    if (b.first == tensor && b.second == chunk) return true;
  return false;
}

// Instantiate + plan.  dims / chunks are already validated.
void plan_instance(const mosaic_graph& g, const int64_t* dims, const int32_t* chunks, Instance& out) {
  const int n_chunks = (int)g.chunks.size();
  out.k.assign(n_chunks, 1);
  for (int c = 0; c < n_chunks; ++c) {
    const int64_t cap = std::max<int64_t>(dims[g.chunks[c].dim], 1);
    out.k[c] = std::max<int64_t>(1, std::min<int64_t>(chunks[c], cap));
  }
  // 1. chunk loops: maximal runs of consecutive operators with the same chunk parameter, body repeated K times
  out.steps.clear();
  out.runs.clear();
  const int n_ops = (int)g.ops.size();
  for (int i = 0; i < n_ops;) {
    const int c = g.ops[i].chunk;
    if (c < 0) {
      out.steps.push_back({i, 0, -1});
      ++i;
      continue;
    }
    int j = i;
    while (j < n_ops && g.ops[j].chunk == c) ++j;
    const int32_t first = (int32_t)out.steps.size();
    const int32_t run = (int32_t)out.runs.size();
    for (int64_t it = 0; it < out.k[c]; ++it)
      for (int o = i; o < j; ++o) out.steps.push_back({o, (int32_t)it, run});
    out.runs.push_back({c, first, (int32_t)out.steps.size() - 1});
    i = j;
  }
  // 2. lifetimes of the instances, merged over alias classes.  index: (class root, iteration) -> block
  const int n_t = (int)g.tensors.size();
  std::vector<int64_t> bytes(n_t);
  for (int t = 0; t < n_t; ++t) {
    const Tensor& x = g.tensors[t];
    int64_t rows = x.dim < 0 ? 1 : dims[x.dim];
    if (x.chunk >= 0) rows = (rows + out.k[x.chunk] - 1) / out.k[x.chunk];
    bytes[t] = round_up(x.bytes_per_row * rows, MOSAIC_GRAPH_ALIGN);
  }
  std::vector<std::vector<int32_t>> slot(n_t);   // slot[root][iteration] = block index or -1
  std::vector<Block> blocks;
  for (int32_t s = 0; s < (int32_t)out.steps.size(); ++s) {
    const Step st = out.steps[s];
    const Op& op = g.ops[st.op];
    for (int side = 0; side < 2; ++side) {
      const std::vector<int32_t>& list = side == 0 ? op.inputs : op.outputs;
      for (int32_t t : list) {
        const Tensor& x = g.tensors[t];
        if (x.persistent) continue;
        const int32_t inst = (x.chunk >= 0 && x.chunk == op.chunk) ? st.iteration : 0;
        const int32_t root = g.find(t);
        int32_t last = s;
        if (st.run >= 0 && has_barrier(g, t, out.runs[st.run].chunk)) last = out.runs[st.run].last;
        std::vector<int32_t>& sl = slot[root];
        if ((int32_t)sl.size() <= inst) sl.resize(inst + 1, -1);
        if (sl[inst] < 0) {
          sl[inst] = (int32_t)blocks.size();
          blocks.push_back({root, inst, s, last, bytes[t], 0});
        } else {
          Block& b = blocks[sl[inst]];
          b.first = std::min(b.first, s);
          b.last = std::max(b.last, last);
          b.bytes = std::max(b.bytes, bytes[t]);
        }
      }
    }
  }
  // 3. placement order: first step, then tensor id, then iteration
  std::sort(blocks.begin(), blocks.end(), [](const Block& a, const Block& b) {
    if (a.first != b.first) return a.first < b.first;
    if (a.tensor != b.tensor) return a.tensor < b.tensor;
    return a.iteration < b.iteration;
  });
  // 4. first-fit: lowest offset clear of every placed block whose lifetime intersects
  std::vector<int32_t> by_offset;   // indices of placed blocks, ascending offset
  for (int32_t i = 0; i < (int32_t)blocks.size(); ++i) {
    Block& b = blocks[i];
    int64_t cand = 0;
    for (int32_t j : by_offset) {
      const Block& p = blocks[j];
      if (p.last < b.first || b.last < p.first) continue;   // never live together
      if (cand + b.bytes <= p.offset) break;                // the gap before p is large enough
      cand = std::max(cand, p.offset + p.bytes);
    }
    b.offset = cand;
    auto pos = std::upper_bound(by_offset.begin(), by_offset.end(), i, [&](int32_t a, int32_t c) {
      return blocks[a].offset < blocks[c].offset;
    });
    by_offset.insert(pos, i);
  }
  // 5. summary: the block that ends at the peak (ties: earliest first step, then placement order)
  mosaic_plan_summary s{};
  s.peak_bytes = 0;
  s.peak_block = -1;
  s.peak_op = MOSAIC_GRAPH_NONE;
  s.peak_chunk = MOSAIC_GRAPH_NONE;
  for (int32_t i = 0; i < (int32_t)blocks.size(); ++i) {
    const int64_t end = blocks[i].offset + blocks[i].bytes;
    if (end > s.peak_bytes || (end == s.peak_bytes && s.peak_block >= 0 && blocks[i].first < blocks[s.peak_block].first)) {
      s.peak_bytes = end;
      s.peak_block = i;
    }
  }
  s.num_blocks = (int64_t)blocks.size();
  s.num_steps = (int32_t)out.steps.size();
  if (s.peak_block >= 0) {
    s.peak_op = out.steps[blocks[s.peak_block].first].op;
    s.peak_chunk = g.ops[s.peak_op].chunk;
  }
  out.blocks.swap(blocks);
  out.summary = s;
}

bool valid_inputs(const mosaic_graph* g, const int64_t* dims, int n_dims, int n_chunks) {
  if (g == nullptr || n_dims != (int)g->dims.size() || n_chunks != (int)g->chunks.size()) return false;
  if (n_dims > 0 && dims == nullptr) return false;
  for (int i = 0; i < n_dims; ++i)
    if (dims[i] < 0) return false;
  return true;
}

}  // namespace

extern "C" {

mosaic_graph* mosaic_graph_create(void) { return new (std::nothrow) mosaic_graph(); }

void mosaic_graph_destroy(mosaic_graph* g) { delete g; }

int mosaic_graph_add_dim(mosaic_graph* g, const char* name) {
  if (g == nullptr || name == nullptr) return MOSAIC_ERR_INVALID_ARG;
  g->dims.emplace_back(name);
  return (int)g->dims.size() - 1;
}

int mosaic_graph_add_chunk_param(mosaic_graph* g, const char* name, int dim) {
  if (g == nullptr || name == nullptr || dim < 0 || dim >= (int)g->dims.size()) return MOSAIC_ERR_INVALID_ARG;
  g->chunks.push_back({name, dim});
  return (int)g->chunks.size() - 1;
}

int mosaic_graph_add_tensor(mosaic_graph* g, const char* name, int64_t bytes_per_row, int dim, int chunk,
                            int persistent) {
  if (g == nullptr || name == nullptr || bytes_per_row < 0) return MOSAIC_ERR_INVALID_ARG;
  if (dim < MOSAIC_GRAPH_NONE || dim >= (int)g->dims.size()) return MOSAIC_ERR_INVALID_ARG;
  if (chunk < MOSAIC_GRAPH_NONE || chunk >= (int)g->chunks.size()) return MOSAIC_ERR_INVALID_ARG;
  if (chunk >= 0 && g->chunks[chunk].dim != dim) return MOSAIC_ERR_INVALID_ARG;   // K must chunk the tensor's own rows
  if (chunk >= 0 && persistent) return MOSAIC_ERR_INVALID_ARG;
  g->tensors.push_back({name, bytes_per_row, dim, chunk, persistent != 0});
  g->alias_parent.push_back((int32_t)g->tensors.size() - 1);
  return (int)g->tensors.size() - 1;
}

int mosaic_graph_add_op(mosaic_graph* g, const char* name, const int32_t* inputs, int n_inputs,
                        const int32_t* outputs, int n_outputs, int chunk) {
  if (g == nullptr || name == nullptr || n_inputs < 0 || n_outputs < 0) return MOSAIC_ERR_INVALID_ARG;
  if ((n_inputs > 0 && inputs == nullptr) || (n_outputs > 0 && outputs == nullptr)) return MOSAIC_ERR_INVALID_ARG;
  if (chunk < MOSAIC_GRAPH_NONE || chunk >= (int)g->chunks.size()) return MOSAIC_ERR_INVALID_ARG;
  Op op{name, {}, {}, chunk};
  for (int side = 0; side < 2; ++side) {
    const int32_t* list = side == 0 ? inputs : outputs;
    const int n = side == 0 ? n_inputs : n_outputs;
    for (int i = 0; i < n; ++i) {
      const int32_t t = list[i];
      if (t < 0 || t >= (int32_t)g->tensors.size()) return MOSAIC_ERR_INVALID_ARG;
      // a chunk of a tensor exists only inside the loop of its own chunk parameter
      if (g->tensors[t].chunk >= 0 && g->tensors[t].chunk != chunk) return MOSAIC_ERR_INVALID_ARG;
      (side == 0 ? op.inputs : op.outputs).push_back(t);
    }
  }
  // a chunked tensor may be named in one loop only: a later, separate run of the same parameter is refused
  if (chunk >= 0 && !g->ops.empty() && g->ops.back().chunk != chunk) {
    for (int side = 0; side < 2; ++side)
      for (int32_t t : (side == 0 ? op.inputs : op.outputs)) {
        if (g->tensors[t].chunk < 0) continue;
        for (const Op& prev : g->ops)
          for (int ps = 0; ps < 2; ++ps)
            for (int32_t u : (ps == 0 ? prev.inputs : prev.outputs))
              if (u == t) return MOSAIC_ERR_INVALID_ARG;
      }
  }
  g->ops.push_back(std::move(op));
  return (int)g->ops.size() - 1;
}

int mosaic_graph_add_alias(mosaic_graph* g, int a, int b) {
  if (g == nullptr || a < 0 || b < 0 || a >= (int)g->tensors.size() || b >= (int)g->tensors.size())
    return MOSAIC_ERR_INVALID_ARG;
  const Tensor& x = g->tensors[a];
  const Tensor& y = g->tensors[b];
  if (x.persistent || y.persistent || x.chunk != y.chunk) return MOSAIC_ERR_INVALID_ARG;
  const int32_t ra = g->find(a), rb = g->find(b);
  if (ra != rb) g->alias_parent[std::max(ra, rb)] = std::min(ra, rb);
  return MOSAIC_OK;
}

int mosaic_graph_add_barrier(mosaic_graph* g, int tensor, int chunk) {
  if (g == nullptr || tensor < 0 || tensor >= (int)g->tensors.size() || chunk < 0 || chunk >= (int)g->chunks.size())
    return MOSAIC_ERR_INVALID_ARG;
  if (g->tensors[tensor].persistent) return MOSAIC_ERR_INVALID_ARG;
  if (!has_barrier(*g, tensor, chunk)) g->barriers.emplace_back(tensor, chunk);
  return MOSAIC_OK;
}

int mosaic_graph_plan(const mosaic_graph* g, const int64_t* dims, int n_dims, const int32_t* chunks, int n_chunks,
                      mosaic_placement* out, int64_t capacity, mosaic_plan_summary* summary) {
  if (!valid_inputs(g, dims, n_dims, n_chunks) || summary == nullptr || capacity < 0 ||
      (capacity > 0 && out == nullptr) || (n_chunks > 0 && chunks == nullptr))
    return MOSAIC_ERR_INVALID_ARG;
  for (int c = 0; c < n_chunks; ++c)
    if (chunks[c] < 1) return MOSAIC_ERR_INVALID_ARG;
  Instance inst;
  plan_instance(*g, dims, chunks, inst);
  *summary = inst.summary;
  const int64_t n = std::min<int64_t>(capacity, (int64_t)inst.blocks.size());
  for (int64_t i = 0; i < n; ++i) {
    const Block& b = inst.blocks[i];
    out[i] = {b.tensor, b.iteration, b.first, b.last, b.offset, b.bytes};
  }
  return MOSAIC_OK;
}

int mosaic_graph_search(const mosaic_graph* g, const int64_t* dims, int n_dims, int64_t budget_bytes,
                        int32_t* chunks_out, int n_chunks, mosaic_plan_summary* summary, int32_t* evaluations) {
  if (!valid_inputs(g, dims, n_dims, n_chunks) || summary == nullptr || budget_bytes < 0 ||
      (n_chunks > 0 && chunks_out == nullptr))
    return MOSAIC_ERR_INVALID_ARG;
  std::vector<int32_t> k(n_chunks, 1);
  int32_t evals = 0;
  Instance inst;
  int rc;
  for (;;) {
    plan_instance(*g, dims, k.data(), inst);
    ++evals;
    if (inst.summary.peak_bytes <= budget_bytes) {
      rc = MOSAIC_OK;
      break;
    }
    const int32_t c = inst.summary.peak_chunk;   // the operator at the peak decides which K moves
    if (c < 0 || k[c] >= std::max<int64_t>(dims[g->chunks[c].dim], 1)) {
      rc = MOSAIC_ERR_WORKSPACE_TOO_SMALL;       // the peak is not chunkable (any further)
      break;
    }
    k[c] += 1;
  }
  for (int c = 0; c < n_chunks; ++c) chunks_out[c] = k[c];
  *summary = inst.summary;
  if (evaluations != nullptr) *evaluations = evals;
  return rc;
}

}  // extern "C"
