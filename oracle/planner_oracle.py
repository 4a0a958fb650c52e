"""CPU oracle for the host-side memory planning (TEST INFRASTRUCTURE ONLY: nothing in the product imports it).

Plain, slow Python written from the paper's description of the graph registrar (section 4.3), the lazy
chunking search (section 4.4) and the single-request first-fit planner (section 4.5).  The paper gives
no pseudo-code; the model is the one stated in the product's header, restated here step by step:

  * operators run in registration order; a maximal run of consecutive operators with the same chunk
    parameter is a loop whose body repeats K times (K clamped to the dimension's value, at least 1);
  * a tensor's bytes = bytes_per_row * rows rounded up to 256, rows = dim value, ceil(value / K) for a
    chunked tensor, 1 without a dimension; chunked tensors get a fresh instance per iteration;
  * lifetime = first..last step naming the instance; a barrier keeps every instance named inside a loop
    of its chunk parameter alive to that loop's last step; aliased tensors form one block;
  * first-fit: blocks in order of first step (ties: lowest tensor id, then iteration), each at the
    lowest offset at which it overlaps no placed block with an intersecting lifetime;
  * search: all K = 1; while the peak exceeds the budget, raise by one the K of the operator that runs
    at the first step of the block ending at the peak (ties: earliest first step, then placement order);
    fail when that operator has no chunk parameter or its K has reached its dimension.

Shares no code with the C++ implementation; pure Python, for small cases.
"""
from dataclasses import dataclass, field
from itertools import product

ALIGN = 256
NONE = -1


@dataclass
class Template:
    dims: list = field(default_factory=list)          # names
    chunks: list = field(default_factory=list)        # (name, dim)
    tensors: list = field(default_factory=list)       # (name, bytes_per_row, dim, chunk, persistent)
    ops: list = field(default_factory=list)           # (name, inputs, outputs, chunk)
    aliases: list = field(default_factory=list)       # (a, b)
    barriers: list = field(default_factory=list)      # (tensor, chunk)

    def add_dim(self, name):
        self.dims.append(name)
        return len(self.dims) - 1

    def add_chunk_param(self, name, dim):
        self.chunks.append((name, dim))
        return len(self.chunks) - 1

    def add_tensor(self, name, bytes_per_row, dim=NONE, chunk=NONE, persistent=False):
        self.tensors.append((name, bytes_per_row, dim, chunk, persistent))
        return len(self.tensors) - 1

    def add_op(self, name, inputs, outputs, chunk=NONE):
        self.ops.append((name, list(inputs), list(outputs), chunk))
        return len(self.ops) - 1

    def add_alias(self, a, b):
        self.aliases.append((a, b))

    def add_barrier(self, tensor, chunk):
        self.barriers.append((tensor, chunk))


def _round_up(x, a):
    return -(-x // a) * a


def effective_chunks(tpl, dims, ks):
    return [max(1, min(k, max(dims[tpl.chunks[c][1]], 1))) for c, k in enumerate(ks)]


def expand(tpl, dims, ks):
    """The instantiated graph: list of steps (op id, iteration, run index of its loop or -1)."""
    ks = effective_chunks(tpl, dims, ks)
    steps, runs = [], []          # runs: (chunk, first step, last step)
    i = 0
    while i < len(tpl.ops):
        c = tpl.ops[i][3]
        if c == NONE:
            steps.append((i, 0, -1))
            i += 1
            continue
        j = i
        while j < len(tpl.ops) and tpl.ops[j][3] == c:
            j += 1
        first = len(steps)
        for it in range(ks[c]):
            for o in range(i, j):
                steps.append((o, it, len(runs)))
        runs.append((c, first, len(steps) - 1))
        i = j
    return steps, runs


def tensor_bytes(tpl, dims, ks, t):
    _, bpr, dim, chunk, _ = tpl.tensors[t]
    ks = effective_chunks(tpl, dims, ks)
    rows = 1 if dim == NONE else dims[dim]
    if chunk != NONE:
        rows = -(-rows // ks[chunk])
    return _round_up(bpr * rows, ALIGN)


def blocks(tpl, dims, ks):
    """Blocks to place: dict key (class representative, iteration) -> [first, last, bytes]."""
    steps, runs = expand(tpl, dims, ks)
    rep = list(range(len(tpl.tensors)))            # alias classes by repeated relabelling (tiny inputs)
    for a, b in tpl.aliases:
        ra, rb = rep[a], rep[b]
        lo, hi = min(ra, rb), max(ra, rb)
        rep = [lo if r == hi else r for r in rep]
    barrier = set(tpl.barriers)
    out = {}
    for s, (o, it, run) in enumerate(steps):
        _, ins, outs, oc = tpl.ops[o]
        for t in ins + outs:
            _, _, _, tc, persistent = tpl.tensors[t]
            if persistent:
                continue
            inst = it if (tc != NONE and tc == oc) else 0
            key = (rep[t], inst)
            size = tensor_bytes(tpl, dims, ks, t)
            last = s
            if run >= 0 and (t, runs[run][0]) in barrier:
                last = runs[run][2]
            if key not in out:
                out[key] = [s, last, size]
            else:
                out[key][0] = min(out[key][0], s)
                out[key][1] = max(out[key][1], last)
                out[key][2] = max(out[key][2], size)
    return out, steps


def first_fit(block_list):
    """block_list: [(key, first, last, bytes)] in placement order.  Returns offsets in the same order."""
    placed = []      # (offset, bytes, first, last)
    offsets = []
    for _, first, last, size in block_list:
        conflicts = [(o, b) for (o, b, f, l) in placed if not (l < first or last < f)]
        candidates = sorted({0} | {o + b for (o, b) in conflicts})
        for cand in candidates:                      # the lowest feasible offset is 0 or the end of a conflicting block
            if all(cand + size <= o or o + b <= cand for (o, b) in conflicts):
                offsets.append(cand)
                placed.append((cand, size, first, last))
                break
    return offsets


def first_fit_literal(block_list):
    """The definition without the candidate-set shortcut: try every multiple of 256 upwards."""
    placed, offsets = [], []
    for _, first, last, size in block_list:
        cand = 0
        while any(not (l < first or last < f) and cand < o + b and o < cand + size for (o, b, f, l) in placed):
            cand += ALIGN
        offsets.append(cand)
        placed.append((cand, size, first, last))
    return offsets


def plan(tpl, dims, ks):
    """Returns (placements, summary); placements = list of dicts in placement order."""
    blk, steps = blocks(tpl, dims, ks)
    order = sorted(blk.items(), key=lambda kv: (kv[1][0], kv[0][0], kv[0][1]))
    block_list = [(k, v[0], v[1], v[2]) for k, v in order]
    offsets = first_fit(block_list)
    placements = [dict(tensor=k[0], iteration=k[1], first_step=f, last_step=l, offset=off, bytes=b)
                  for (k, f, l, b), off in zip(block_list, offsets)]
    peak, peak_block = 0, -1
    for i, p in enumerate(placements):
        end = p["offset"] + p["bytes"]
        if end > peak or (end == peak and peak_block >= 0 and p["first_step"] < placements[peak_block]["first_step"]):
            peak, peak_block = end, i
    peak_op = steps[placements[peak_block]["first_step"]][0] if peak_block >= 0 else NONE
    peak_chunk = tpl.ops[peak_op][3] if peak_op != NONE else NONE
    return placements, dict(peak_bytes=peak, num_blocks=len(placements), num_steps=len(steps), peak_block=peak_block,
                            peak_op=peak_op, peak_chunk=peak_chunk)


def check_plan(placements):
    """A plan is valid when no two blocks overlap in both time and address and offsets are aligned."""
    for i, p in enumerate(placements):
        assert p["offset"] % ALIGN == 0 and p["bytes"] % ALIGN == 0 and p["bytes"] >= 0
        for q in placements[:i]:
            in_time = not (p["last_step"] < q["first_step"] or q["last_step"] < p["first_step"])
            in_addr = p["offset"] < q["offset"] + q["bytes"] and q["offset"] < p["offset"] + p["bytes"]
            assert not (in_time and in_addr), (p, q)


def max_live_bytes(placements):
    """Lower bound on any plan's peak: the largest sum of bytes live at one step."""
    if not placements:
        return 0
    n = max(p["last_step"] for p in placements) + 1
    return max(sum(p["bytes"] for p in placements if p["first_step"] <= s <= p["last_step"]) for s in range(n))


def search(tpl, dims, budget):
    """Returns (ok, ks, summary, evaluations)."""
    ks = [1] * len(tpl.chunks)
    evaluations = 0
    while True:
        _, summary = plan(tpl, dims, ks)
        evaluations += 1
        if summary["peak_bytes"] <= budget:
            return True, ks, summary, evaluations
        c = summary["peak_chunk"]
        if c == NONE or ks[c] >= max(dims[tpl.chunks[c][1]], 1):
            return False, ks, summary, evaluations
        ks[c] += 1


def brute_force(tpl, dims, budget, kmax):
    """Every chunk setting in [1, kmax]^n whose planned peak fits the budget (the enumeration the paper
    compares its search against)."""
    feasible = []
    for ks in product(range(1, kmax + 1), repeat=len(tpl.chunks)):
        _, summary = plan(tpl, dims, list(ks))
        if summary["peak_bytes"] <= budget:
            feasible.append(ks)
    return feasible
