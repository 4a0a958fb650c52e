"""A pin of the planning oracle's lifetimes (oracle/planner_oracle.py: expand + blocks) that shares no structure
with it or with the library: a small run-time simulator.

The oracle derives a block's lifetime by folding min / max over the steps that name it.  The simulator below does
what an executing runtime with reference counts would do (paper section 4.3: operators run in order, an alias
binds an output to an existing address, a barrier keeps an input of a chunk loop until the loop is over;
section 4.5: a tensor occupies the workspace from its first to its last use): it interprets the template with a
program counter, re-enters chunk loops, allocates a buffer the first time an instruction touches it, counts the
touches that are still to come, frees a buffer after its last touch or -- if a barrier holds it -- when the
loop that holds it exits, and records the table of live buffers after every instruction.  The live tables, the
buffer sizes and the instruction trace must equal what the oracle's blocks imply, on hand-worked cases, on the
dLLM step template and on random templates.
"""
import random

import pytest

from oracle import planner_oracle as po
from paper_2601_06562_amd import graph_templates


class DisjointSets:
    def __init__(self, n):
        self.parent = list(range(n))

    def find(self, a):
        while self.parent[a] != a:
            self.parent[a] = self.parent[self.parent[a]]
            a = self.parent[a]
        return a

    def union(self, a, b):
        ra, rb = self.find(a), self.find(b)
        if ra != rb:
            self.parent[max(ra, rb)] = min(ra, rb)      # the lowest tensor id names the shared storage


def program(tpl, dims, ks):
    """The instruction trace of one instantiation: [(op, iteration, loop ordinal or None)], by interpretation."""
    trace, loops = [], 0
    pc = 0
    while pc < len(tpl.ops):
        c = tpl.ops[pc][3]
        if c == po.NONE:
            trace.append((pc, 0, None))
            pc += 1
            continue
        end = pc
        while end < len(tpl.ops) and tpl.ops[end][3] == c:
            end += 1
        size_of_dim = dims[tpl.chunks[c][1]]
        trips = min(max(ks[c], 1), max(size_of_dim, 1))
        for trip in range(trips):
            body_pc = pc
            while body_pc < end:
                trace.append((body_pc, trip, loops))
                body_pc += 1
        loops += 1
        pc = end
    return trace


def rows_of(tpl, dims, ks, t):
    _, _, dim, chunk, _ = tpl.tensors[t]
    if dim == po.NONE:
        return 1
    if chunk == po.NONE:
        return dims[dim]
    trips = min(max(ks[chunk], 1), max(dims[dim], 1))
    return (dims[dim] + trips - 1) // trips


def simulate(tpl, dims, ks):
    """Runs the trace with a table of live buffers.  Returns (trace, live tables per instruction, sizes):
    a live table is the set of buffer names (storage id, loop trip) that hold memory WHILE the instruction runs."""
    trace = program(tpl, dims, ks)
    sets = DisjointSets(len(tpl.tensors))
    for a, b in tpl.aliases:
        sets.union(a, b)

    def touched(instr):
        op, trip, _ = instr
        _, ins, outs, oc = tpl.ops[op]
        names = []
        for t in ins + outs:
            _, _, _, tc, persistent = tpl.tensors[t]
            if persistent:
                continue
            names.append((t, (sets.find(t), trip if (tc != po.NONE and tc == oc) else 0)))
        return names

    # pass 1: how often will each buffer still be touched
    remaining = {}
    for instr in trace:
        for _, name in touched(instr):
            remaining[name] = remaining.get(name, 0) + 1
    loop_end = {}
    for pos, (_, _, loop) in enumerate(trace):
        if loop is not None:
            loop_end[loop] = pos
    # pass 2: execute
    live, sizes, tables = set(), {}, []
    held = {}                                            # loop ordinal -> buffers a barrier keeps until it exits
    for pos, instr in enumerate(trace):
        op, trip, loop = instr
        chunk_of_loop = tpl.ops[op][3]
        done_here = []
        for t, name in touched(instr):
            live.add(name)                               # first touch allocates
            nbytes = -(-(tpl.tensors[t][1] * rows_of(tpl, dims, ks, t)) // po.ALIGN) * po.ALIGN
            sizes[name] = max(sizes.get(name, 0), nbytes)
            remaining[name] -= 1
            if loop is not None and (t, chunk_of_loop) in set(tpl.barriers):
                held.setdefault(loop, set()).add(name)
            if remaining[name] == 0:
                done_here.append(name)
        tables.append(frozenset(live))
        for name in done_here:
            if not any(name in h for h in held.values()):
                live.discard(name)
        if loop is not None and loop_end[loop] == pos:    # the loop exits: release what its barriers held
            for name in held.pop(loop, set()):
                if remaining[name] == 0 and not any(name in h for h in held.values()):
                    live.discard(name)
    assert not live, live                                # everything was freed by the end
    return trace, tables, sizes


def assert_oracle_agrees(tpl, dims, ks):
    trace, tables, sizes = simulate(tpl, dims, ks)
    blk, steps = po.blocks(tpl, dims, ks)
    assert [(o, it) for o, it, _ in steps] == [(o, it) for o, it, _ in trace]
    for s in range(len(trace)):
        from_oracle = frozenset(k for k, (first, last, _) in blk.items() if first <= s <= last)
        assert from_oracle == tables[s], (s, sorted(from_oracle ^ tables[s]))
    assert {k: v[2] for k, v in blk.items()} == sizes
    return trace, tables, blk


def test_two_loops_with_an_alias_across_the_boundary_by_hand():
    """x[T] -> loop A (K_a = 2): p = f(x), q += g(p) -> loop B (K_b = 3): r = h(q), y += s(r) -> z = u(y)
    with q written over x's storage (an alias that spans loop A's exit) and a barrier that keeps every r until loop
    B is over.  Instructions: 0 make_x | 1 f0 2 g0 3 f1 4 g1 | 5 h0 6 s0 7 h1 8 s1 9 h2 10 s2 | 11 u."""
    t = po.Template()
    T = t.add_dim("T")
    Ka = t.add_chunk_param("Ka", T)
    Kb = t.add_chunk_param("Kb", T)
    w = t.add_tensor("w", 64, po.NONE, po.NONE, True)
    x = t.add_tensor("x", 100, T)
    p = t.add_tensor("p", 40, T, Ka)
    q = t.add_tensor("q", 60, T)
    r = t.add_tensor("r", 30, T, Kb)
    y = t.add_tensor("y", 10, T)
    z = t.add_tensor("z", 8)
    t.add_op("make_x", [w], [x])
    t.add_op("f", [x], [p], Ka)
    t.add_op("g", [p], [q], Ka)
    t.add_op("h", [q], [r], Kb)
    t.add_op("s", [r], [y], Kb)
    t.add_op("u", [y], [z])
    t.add_alias(x, q)
    t.add_barrier(r, Kb)
    trace, tables, blk = assert_oracle_agrees(t, [90], [2, 3])
    assert [o for o, _, _ in trace] == [0, 1, 2, 1, 2, 3, 4, 3, 4, 3, 4, 5]
    X, P0, P1, R0, R1, R2, Y, Z = (x, 0), (p, 0), (p, 1), (r, 0), (r, 1), (r, 2), (y, 0), (z, 0)
    by_hand = [
        {X},                    # 0 make_x
        {X, P0},                # 1 f, trip 0
        {X, P0},                # 2 g, trip 0: q is x's storage, no new buffer
        {X, P1},                # 3 f, trip 1
        {X, P1},                # 4 g, trip 1
        {X, R0},                # 5 h, trip 0: x's storage is still live because q lives there
        {X, R0, Y},             # 6 s, trip 0
        {X, R0, R1, Y},         # 7 h, trip 1: r of trip 0 is held by the barrier
        {X, R0, R1, Y},         # 8
        {X, R0, R1, R2, Y},     # 9 h, trip 2: the last read of q
        {R0, R1, R2, Y},        # 10 s, trip 2: x/q is gone, every r is released when the loop exits
        {Y, Z},                 # 11 u
    ]
    assert [set(tb) for tb in tables] == by_hand
    up = lambda n: -(-n // 256) * 256
    assert blk[X] == [0, 9, up(100 * 90)]                # union of x (0-3) and q (2-9); the larger of the two sizes
    assert blk[P1] == [3, 4, up(40 * 45)]
    assert blk[R0] == [5, 10, up(30 * 30)] and blk[R2] == [9, 10, up(30 * 30)]
    assert (q, 0) not in blk
    # the plan built on these lifetimes: r's three instances may not share an address, p's two may
    placements, summary = po.plan(t, [90], [2, 3])
    po.check_plan(placements)
    off = {(b["tensor"], b["iteration"]): b["offset"] for b in placements}
    assert off[P0] == off[P1] and len({off[R0], off[R1], off[R2]}) == 3


def test_barrier_holds_only_inside_its_own_loop_by_hand():
    """A tensor read in two separate loops of the same chunk parameter, with a barrier: each loop holds it to its
    own end, and in between it lives only because the second loop still needs it."""
    t = po.Template()
    T = t.add_dim("T")
    K = t.add_chunk_param("K", T)
    a = t.add_tensor("a", 16, T)
    c = t.add_tensor("c", 16, T, K)
    m = t.add_tensor("m", 16, T)
    e = t.add_tensor("e", 16, T, K)
    t.add_op("mk", [], [a])
    t.add_op("l1", [a], [c], K)
    t.add_op("mid", [a], [m])
    t.add_op("l2", [m], [e], K)
    t.add_barrier(c, K)
    t.add_barrier(m, K)
    trace, tables, blk = assert_oracle_agrees(t, [64], [2])
    # 0 mk | 1 l1.0 2 l1.1 | 3 mid | 4 l2.0 5 l2.1
    assert blk[(c, 0)][:2] == [1, 2] and blk[(c, 1)][:2] == [2, 2]
    assert blk[(a, 0)][:2] == [0, 3] and blk[(m, 0)][:2] == [3, 5] and blk[(e, 0)][:2] == [4, 4]
    assert [len(tb) for tb in tables] == [1, 2, 3, 2, 2, 2]


@pytest.mark.parametrize("logits", ["materialised", "fused"])
@pytest.mark.parametrize("inplace", [True, False])
def test_dllm_step_lifetimes_equal_the_simulated_live_tables(logits, inplace):
    t = po.Template()
    graph_templates.dllm_step(t, layers=3, d=64, d_ff=256, vocab=2048, logits=logits, inplace_residual=inplace)
    for dims in ([512, 512], [4096, 300], [1000, 1], [7, 7], [1, 0], [0, 0]):
        for ks in ([1, 1], [2, 1], [1, 3], [4, 5], [16, 2], [100, 100]):
            assert_oracle_agrees(t, dims, ks)


class _OracleOnly(po.Template):
    """The random-template generator of the library tests talks to a builder with an `ora` attribute."""

    @property
    def ora(self):
        return self


@pytest.mark.parametrize("seed", range(40))
def test_random_template_lifetimes_equal_the_simulated_live_tables(seed):
    from test_graph_planner import random_template
    rng = random.Random(1000 + seed)
    t = _OracleOnly()
    n_dims, n_chunks = random_template(rng, t)
    for _ in range(5):
        dims = [rng.choice([0, 1, 5, 100, 1000]) for _ in range(n_dims)]
        ks = [rng.choice([1, 2, 3, 7]) for _ in range(n_chunks)]
        assert_oracle_agrees(t, dims, ks)


def test_the_simulator_catches_planted_mistakes():
    """The pin has teeth: an oracle whose barrier rule, alias rule or instance rule is broken disagrees with it."""
    t = po.Template()
    graph_templates.dllm_step(t, layers=2, d=64, d_ff=256, vocab=1024)
    K = t.chunks.index(("K_ffn", 0))
    act0 = [i for i, x in enumerate(t.tensors) if x[0] == "act0"][0]
    t.add_barrier(act0, K)                               # every chunk of act0 stays until the FFN loop is over
    good, _ = po.blocks(t, [512, 512], [3, 2])
    _, tables, _ = simulate(t, [512, 512], [3, 2])

    def tables_of(blk):
        return [frozenset(k for k, (f, l, _) in blk.items() if f <= s <= l) for s in range(len(tables))]
    assert tables_of(good) == tables
    # a dropped barrier: a chunk of act0 would end at its last read instead of at the loop's end
    no_barrier = po.Template(**{k: list(v) for k, v in vars(t).items()})
    no_barrier.barriers = []
    assert tables_of(po.blocks(no_barrier, [512, 512], [3, 2])[0]) != tables
    # a dropped alias: the residual sum would get a buffer of its own
    no_alias = po.Template(**{k: list(v) for k, v in vars(t).items()})
    no_alias.aliases = []
    assert tables_of(po.blocks(no_alias, [512, 512], [3, 2])[0]) != tables
    # chunk instances collapsed into one block per tensor
    merged = {}
    for (rep, _), (f, l, b) in good.items():
        cur = merged.setdefault((rep, 0), [f, l, b])
        cur[0], cur[1] = min(cur[0], f), max(cur[1], l)
    assert tables_of(merged) != tables
