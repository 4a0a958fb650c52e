"""Pins of the planning oracle (oracle/planner_oracle.py) against facts that do not come from it: hand-worked
placements, the literal definition of first-fit, the optimality of first-fit on equal-size intervals (an
interval-graph colouring fact), validity and the live-bytes lower bound, the hand-computed sizes and lifetimes
of a small chunk loop, and the search against exhaustive enumeration."""
import random

import pytest

from oracle import planner_oracle as po
from paper_2601_06562_amd import graph_templates


def blocks_of(spec):
    """spec: list of (first, last, bytes) -> block list in placement order (sorted by first, then index)."""
    order = sorted(range(len(spec)), key=lambda i: (spec[i][0], i))
    return [((i, 0), spec[i][0], spec[i][1], spec[i][2]) for i in order], order


def test_first_fit_hand_worked_case():
    # A lives 0-2 (512 B), B 1-3 (256), C 3-4 (768), D 2-5 (256), E 4-6 (512)
    #   A -> 0;  B overlaps A -> 512;  D (first 2) overlaps A, B -> 768;  C (first 3) overlaps B@512, D@768:
    #   hole [0,512) is too small for 768 -> 1024;  E (first 4) overlaps C@1024 and D@768 -> [0,512) is free -> 0
    spec = [(0, 2, 512), (1, 3, 256), (3, 4, 768), (2, 5, 256), (4, 6, 512)]
    bl, order = blocks_of(spec)
    off = dict(zip(order, po.first_fit(bl)))
    assert off == {0: 0, 1: 512, 3: 768, 2: 1024, 4: 0}


def test_first_fit_fills_a_hole_that_is_large_enough():
    # X 0-9 at 0 (256); Y 0-1 at 256 (512); Z 0-9 at 768 (256); W 2-9 (512) fits exactly in Y's hole; U 2-9 (768) does not
    spec = [(0, 9, 256), (0, 1, 512), (0, 9, 256), (2, 9, 512), (2, 9, 768)]
    bl, order = blocks_of(spec)
    off = dict(zip(order, po.first_fit(bl)))
    assert off == {0: 0, 1: 256, 2: 768, 3: 256, 4: 1024}


@pytest.mark.parametrize("seed", range(20))
def test_first_fit_equals_its_literal_definition_and_is_valid(seed):
    rng = random.Random(seed)
    spec = []
    for _ in range(rng.randint(1, 14)):
        f = rng.randint(0, 12)
        spec.append((f, f + rng.randint(0, 6), 256 * rng.randint(1, 5)))
    bl, _ = blocks_of(spec)
    a, b = po.first_fit(bl), po.first_fit_literal(bl)
    assert a == b
    placements = [dict(offset=o, bytes=s, first_step=f, last_step=l) for (_, f, l, s), o in zip(bl, a)]
    po.check_plan(placements)
    peak = max(p["offset"] + p["bytes"] for p in placements)
    assert po.max_live_bytes(placements) <= peak <= sum(p["bytes"] for p in placements)


@pytest.mark.parametrize("seed", range(10))
def test_equal_size_intervals_are_packed_optimally(seed):
    """First-fit in order of start time colours an interval graph with as many colours as its largest clique,
    so with equal sizes the peak equals the live-bytes lower bound exactly."""
    rng = random.Random(100 + seed)
    spec = []
    for _ in range(rng.randint(2, 25)):
        f = rng.randint(0, 20)
        spec.append((f, f + rng.randint(0, 8), 1024))
    bl, _ = blocks_of(spec)
    off = po.first_fit(bl)
    placements = [dict(offset=o, bytes=s, first_step=f, last_step=l) for (_, f, l, s), o in zip(bl, off)]
    assert max(p["offset"] + p["bytes"] for p in placements) == po.max_live_bytes(placements)


def small_loop():
    """x[T] -> loop K over T: a = f(x) chunked, b = g(a) chunked, y[T] += h(b)  -> z = r(y)."""
    t = po.Template()
    T = t.add_dim("T")
    K = t.add_chunk_param("K", T)
    x = t.add_tensor("x", 100, T)
    a = t.add_tensor("a", 300, T, K)
    b = t.add_tensor("b", 200, T, K)
    y = t.add_tensor("y", 100, T)
    z = t.add_tensor("z", 8)
    w = t.add_tensor("w", 1 << 20, po.NONE, po.NONE, True)
    t.add_op("make_x", [w], [x])
    t.add_op("f", [x, w], [a], K)
    t.add_op("g", [a], [b], K)
    t.add_op("h", [b], [y], K)
    t.add_op("r", [y], [z])
    return t, dict(x=x, a=a, b=b, y=y, z=z, K=K)


def test_chunk_loop_expansion_sizes_and_lifetimes_by_hand():
    t, ids = small_loop()
    steps, runs = po.expand(t, [1000], [3])
    # make_x, then (f g h) x 3, then r
    assert [s[0] for s in steps] == [0, 1, 2, 3, 1, 2, 3, 1, 2, 3, 4]
    assert [s[1] for s in steps] == [0, 0, 0, 0, 1, 1, 1, 2, 2, 2, 0]
    assert runs == [(ids["K"], 1, 9)]
    blk, _ = po.blocks(t, [1000], [3])
    rows = 334                                           # ceil(1000 / 3)
    up = lambda n: -(-n // 256) * 256
    assert blk[(ids["x"], 0)] == [0, 7, up(100 * 1000)]   # read by f in every iteration: live through the loop
    assert blk[(ids["a"], 0)] == [1, 2, up(300 * rows)]
    assert blk[(ids["a"], 2)] == [7, 8, up(300 * rows)]
    assert blk[(ids["b"], 1)] == [5, 6, up(200 * rows)]
    assert blk[(ids["y"], 0)] == [3, 10, up(100 * 1000)]  # first written by h in iteration 0, read by r
    assert blk[(ids["z"], 0)] == [10, 10, 256]
    assert (5, 0) not in blk                              # the persistent tensor is not planned
    # K above the dimension is clamped
    assert po.effective_chunks(t, [2], [5]) == [2] and po.effective_chunks(t, [0], [5]) == [1]


def test_barrier_and_alias_semantics_by_hand():
    t, ids = small_loop()
    t.add_barrier(ids["b"], ids["K"])                    # every chunk of b stays until the loop ends
    blk, _ = po.blocks(t, [1000], [3])
    assert [blk[(ids["b"], i)][:2] for i in range(3)] == [[2, 9], [5, 9], [8, 9]]
    assert blk[(ids["a"], 0)][:2] == [1, 2]              # unaffected
    t2, ids2 = small_loop()
    t2.add_alias(ids2["x"], ids2["y"])                   # y is accumulated over x's storage
    blk2, _ = po.blocks(t2, [1000], [3])
    assert (ids2["y"], 0) not in blk2
    assert blk2[(ids2["x"], 0)][:2] == [0, 10]           # union of both lifetimes
    p2, s2 = po.plan(t2, [1000], [3])
    p1, s1 = po.plan(small_loop()[0], [1000], [3])
    po.check_plan(p1)
    po.check_plan(p2)
    assert s2["peak_bytes"] == s1["peak_bytes"] - (-(-100 * 1000 // 256) * 256)   # one full-size buffer saved


def test_plan_of_the_small_loop_by_hand():
    t, ids = small_loop()
    p, s = po.plan(t, [1000], [1])
    # K = 1, steps make_x f g h r = 0..4.  Lifetimes: x 0-1, a 1-2, b 2-3, y 3-4, z 4.
    # x@0; a meets x -> X; b meets a only, the hole [0, X) is too small for it -> X + A; y meets b only -> 0;
    # z meets y only -> X (the end of y, which has x's size).
    by = {(q["tensor"], q["iteration"]): q for q in p}
    X, A, B = 100096, 300032, 200192
    assert by[(ids["x"], 0)]["offset"] == 0 and by[(ids["x"], 0)]["bytes"] == X
    assert by[(ids["a"], 0)]["offset"] == X
    assert by[(ids["b"], 0)]["offset"] == X + A
    assert by[(ids["y"], 0)]["offset"] == 0
    assert by[(ids["z"], 0)]["offset"] == X
    assert s["peak_bytes"] == X + A + B and s["num_steps"] == 5
    assert s["peak_op"] == 2 and s["peak_chunk"] == ids["K"]    # the block ending at the peak is b, first made by g
    po.check_plan(p)
    assert po.max_live_bytes(p) <= s["peak_bytes"]


@pytest.mark.parametrize("logits", ["materialised", "fused"])
@pytest.mark.parametrize("T,M", [(512, 512), (2048, 1024), (4096, 200), (4096, 4096), (300, 7)])
def test_search_against_exhaustive_enumeration(logits, T, M):
    """The search's answer is feasible, no feasible setting is component-wise smaller, and it fails only when
    the enumeration finds nothing (section 4.4: the search is compared with brute force over all combinations)."""
    t = po.Template()
    graph_templates.dllm_step(t, layers=2, d=64, d_ff=256, vocab=1024, logits=logits)
    _, unchunked = po.plan(t, [T, M], [1, 1])
    kmax = 10
    for frac in (1.0, 0.8, 0.6, 0.45, 0.3, 0.2, 0.1, 0.02):
        budget = int(unchunked["peak_bytes"] * frac)
        ok, ks, summary, evals = po.search(t, [T, M], budget)
        feasible = po.brute_force(t, [T, M], budget, kmax)
        if ok and max(ks) <= kmax:
            assert tuple(ks) in feasible
            assert not [f for f in feasible if all(a <= b for a, b in zip(f, ks)) and tuple(f) != tuple(ks)]
            assert evals == sum(ks) - len(ks) + 1            # one plan per increment, nothing else
            assert evals <= len(feasible) + kmax * kmax      # never more work than the enumeration
        elif not ok:
            assert feasible == [] or max(ks) >= max(1, min(T, M))
        if frac == 1.0:
            assert ok and ks == [1, 1] and evals == 1        # lazy: no chunking when everything fits


def test_bottleneck_moves_with_the_mask_ratio():
    """Section 3 / 4.4: with materialised logits the peak sits at the logits operator when most tokens are masked
    and at the feed-forward network when few are; with the fused reduction it is never at the logits."""
    t = po.Template()
    ids = graph_templates.dllm_step(t, layers=2, d=64, d_ff=256, vocab=4096, logits="materialised")
    _, high = po.plan(t, [4096, 4096], [1, 1])
    _, low = po.plan(t, [4096, 64], [1, 1])
    assert high["peak_chunk"] == ids["k_logits"] and low["peak_chunk"] == ids["k_ffn"]
    f = po.Template()
    idf = graph_templates.dllm_step(f, layers=2, d=64, d_ff=256, vocab=4096, logits="fused")
    for M in (4096, 1024, 64):
        _, s = po.plan(f, [4096, M], [1, 1])
        assert s["peak_chunk"] == idf["k_ffn"]
    _, fused_high = po.plan(f, [4096, 4096], [1, 1])
    assert fused_high["peak_bytes"] < high["peak_bytes"] / 4
