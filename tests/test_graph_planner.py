"""The host-side planner behind the C ABI (mosaic_graph_*) against the plain-Python oracle: identical
placements block by block, identical search trajectories, and argument validation.  No GPU involved."""
import ctypes
import random

import pytest

from oracle import planner_oracle as po
from paper_2601_06562_amd import binding, graph_templates
from paper_2601_06562_amd.binding import GraphTemplate


class Both:
    """Feeds every registrar call to the library and to the oracle; ids must agree."""

    def __init__(self):
        self.lib, self.ora = GraphTemplate(), po.Template()

    def _same(self, a, b):
        assert a == b
        return a

    def add_dim(self, name):
        return self._same(self.lib.add_dim(name), self.ora.add_dim(name))

    def add_chunk_param(self, name, dim):
        return self._same(self.lib.add_chunk_param(name, dim), self.ora.add_chunk_param(name, dim))

    def add_tensor(self, name, bytes_per_row, dim=-1, chunk=-1, persistent=False):
        return self._same(self.lib.add_tensor(name, bytes_per_row, dim, chunk, persistent),
                          self.ora.add_tensor(name, bytes_per_row, dim, chunk, persistent))

    def add_op(self, name, inputs, outputs, chunk=-1):
        return self._same(self.lib.add_op(name, inputs, outputs, chunk), self.ora.add_op(name, inputs, outputs, chunk))

    def add_alias(self, a, b):
        self.lib.add_alias(a, b)
        self.ora.add_alias(a, b)

    def add_barrier(self, t, c):
        self.lib.add_barrier(t, c)
        self.ora.add_barrier(t, c)

    def check(self, dims, ks):
        got, gs = self.lib.plan(dims, ks)
        want, ws = po.plan(self.ora, dims, ks)
        assert got == want
        assert gs == ws
        po.check_plan(got)
        return got, gs


@pytest.mark.parametrize("logits", ["materialised", "fused"])
@pytest.mark.parametrize("layers", [1, 3])
def test_dllm_step_plans_match_the_oracle(logits, layers):
    b = Both()
    graph_templates.dllm_step(b, layers=layers, d=64, d_ff=256, vocab=2048, logits=logits)
    for dims in ([512, 512], [4096, 300], [1000, 1], [7, 7], [1, 0], [0, 0]):
        for ks in ([1, 1], [2, 1], [1, 3], [4, 5], [16, 2], [100, 100]):
            b.check(dims, ks)


def random_template(rng, b):
    n_dims = rng.randint(1, 3)
    dims = [b.add_dim(f"D{i}") for i in range(n_dims)]
    chunks = [b.add_chunk_param(f"K{i}", rng.choice(dims)) for i in range(rng.randint(0, 3))]
    chunk_dim = {}
    for c in chunks:
        chunk_dim[c] = b.ora.chunks[c][1]
    tensors = []      # (id, chunk)
    w = b.add_tensor("weights", 4096, -1, -1, True)
    live_full = []
    used_in_closed_run = set()
    prev_chunk = -1
    for o in range(rng.randint(1, 14)):
        c = rng.choice([-1, -1] + chunks) if chunks else -1
        if c != prev_chunk and prev_chunk >= 0:
            used_in_closed_run |= {t for t, tc in tensors if tc == prev_chunk}
        # inputs: some earlier tensors that this operator may name
        usable = [t for t, tc in tensors if tc == -1 or (tc == c and t not in used_in_closed_run)]
        ins = rng.sample(usable, min(len(usable), rng.randint(0, 3))) + ([w] if rng.random() < 0.3 else [])
        outs = []
        for _ in range(rng.randint(1, 2)):
            if rng.random() < 0.5 and c >= 0:
                t = b.add_tensor(f"t{len(tensors)}", rng.randint(1, 600), chunk_dim[c], c)
                tensors.append((t, c))
            elif rng.random() < 0.2:
                t = b.add_tensor(f"t{len(tensors)}", rng.randint(1, 5000))
                tensors.append((t, -1))
            else:
                t = b.add_tensor(f"t{len(tensors)}", rng.randint(1, 600), rng.choice(dims))
                tensors.append((t, -1))
            outs.append(t)
        b.add_op(f"op{o}", ins, outs, c)
        prev_chunk = c
    for _ in range(rng.randint(0, 3)):
        t1, c1 = rng.choice(tensors)
        same = [t for t, tc in tensors if tc == c1 and t != t1]
        if same:
            b.add_alias(t1, rng.choice(same))
    for _ in range(rng.randint(0, 3)):
        if chunks:
            b.add_barrier(rng.choice(tensors)[0], rng.choice(chunks))
    return n_dims, len(chunks)


@pytest.mark.parametrize("seed", range(60))
def test_random_templates_match_the_oracle(seed):
    rng = random.Random(seed)
    b = Both()
    n_dims, n_chunks = random_template(rng, b)
    for _ in range(4):
        dims = [rng.choice([0, 1, 5, 100, 1000]) for _ in range(n_dims)]
        ks = [rng.choice([1, 2, 3, 7]) for _ in range(n_chunks)]
        b.check(dims, ks)
    dims = [rng.choice([12, 40]) for _ in range(n_dims)]      # small: the oracle re-plans in pure Python per increment
    _, top = b.check(dims, [1] * n_chunks)
    for frac in (1.0, 0.7, 0.4, 0.1):
        budget = int(top["peak_bytes"] * frac)
        assert b.lib.search(dims, budget) == po.search(b.ora, dims, budget)


@pytest.mark.parametrize("T,M", [(4096, 4096), (4096, 256), (32768, 4105), (700, 30)])
def test_search_matches_the_oracle_on_the_dllm_step(T, M):
    for logits in ("materialised", "fused"):
        b = Both()
        graph_templates.dllm_step(b, layers=2, d=64, d_ff=256, vocab=4096, logits=logits)
        _, top = b.check([T, M], [1, 1])
        for frac in (1.0, 0.75, 0.5, 0.3, 0.15, 0.05):
            budget = int(top["peak_bytes"] * frac)
            got = b.lib.search([T, M], budget)
            assert got == po.search(b.ora, [T, M], budget)
            ok, ks, summary, evals = got
            assert ok == (summary["peak_bytes"] <= budget)
            assert evals == sum(ks) - len(ks) + 1


def test_fused_reduction_takes_the_logits_out_of_the_search():
    """With materialised logits a tight budget raises K_logits at a high mask ratio; with the fused reduction the
    logits never become the bottleneck and only the feed-forward network is chunked."""
    mat, fus = GraphTemplate(), GraphTemplate()
    im = graph_templates.dllm_step(mat, layers=2, d=64, d_ff=256, vocab=8192, logits="materialised")
    graph_templates.dllm_step(fus, layers=2, d=64, d_ff=256, vocab=8192, logits="fused")
    T = M = 4096
    _, top_f = fus.plan([T, M], [1, 1], placements=False)
    budget = top_f["peak_bytes"]                       # what the fused graph needs without any chunking
    ok_m, ks_m, _, _ = mat.search([T, M], budget)
    ok_f, ks_f, _, evals_f = fus.search([T, M], budget)
    assert ok_f and ks_f == [1, 1] and evals_f == 1
    assert ok_m and ks_m[im["k_logits"]] > 1 and ks_m[im["k_ffn"]] == 1


def test_registrar_validates_its_arguments():
    L = binding.lib()
    INV = binding.MOSAIC_ERR_INVALID_ARG
    g = GraphTemplate()
    T = g.add_dim("T")
    M = g.add_dim("M")
    K = g.add_chunk_param("K", T)
    x = g.add_tensor("x", 10, T)
    xc = g.add_tensor("xc", 10, T, K)
    w = g.add_tensor("w", 10, -1, -1, True)
    assert L.mosaic_graph_add_dim(None, b"a") == INV
    assert L.mosaic_graph_add_chunk_param(g._g, b"k", 7) == INV
    assert L.mosaic_graph_add_tensor(g._g, b"t", -1, T, -1, 0) == INV
    assert L.mosaic_graph_add_tensor(g._g, b"t", 8, M, K, 0) == INV          # K chunks T, not M
    assert L.mosaic_graph_add_tensor(g._g, b"t", 8, T, K, 1) == INV          # persistent tensors are not chunked
    one = (ctypes.c_int32 * 1)
    assert L.mosaic_graph_add_op(g._g, b"o", one(99), 1, one(x), 1, -1) == INV
    assert L.mosaic_graph_add_op(g._g, b"o", one(xc), 1, one(x), 1, -1) == INV   # a chunk outside its loop
    assert L.mosaic_graph_add_alias(g._g, x, xc) == INV                      # different chunk parameters
    assert L.mosaic_graph_add_alias(g._g, x, w) == INV
    assert L.mosaic_graph_add_barrier(g._g, w, K) == INV
    assert L.mosaic_graph_add_barrier(g._g, x, 5) == INV
    g.add_op("make", [w], [x])
    g.add_op("loop", [x], [xc], K)
    g.add_op("other", [x], [x])
    assert L.mosaic_graph_add_op(g._g, b"again", one(xc), 1, one(x), 1, K) == INV   # xc belongs to the earlier loop
    s = binding.MosaicPlanSummary()
    d2 = (ctypes.c_int64 * 2)(10, 10)
    k1 = (ctypes.c_int32 * 1)(1)
    assert L.mosaic_graph_plan(g._g, d2, 1, k1, 1, None, 0, ctypes.byref(s)) == INV       # wrong number of dims
    assert L.mosaic_graph_plan(g._g, d2, 2, (ctypes.c_int32 * 1)(0), 1, None, 0, ctypes.byref(s)) == INV
    assert L.mosaic_graph_plan(g._g, (ctypes.c_int64 * 2)(-1, 3), 2, k1, 1, None, 0, ctypes.byref(s)) == INV
    assert L.mosaic_graph_plan(g._g, d2, 2, k1, 1, None, 0, None) == INV
    assert L.mosaic_graph_plan(g._g, d2, 2, k1, 1, None, 0, ctypes.byref(s)) == binding.MOSAIC_OK
    assert s.num_blocks == 2 and s.num_steps == 3
    assert L.mosaic_graph_search(g._g, d2, 2, -5, k1, 1, ctypes.byref(s), None) == INV
    ok, ks, summary, evals = g.search([10, 10], 0)
    assert not ok                                       # x itself cannot be chunked
    L.mosaic_graph_destroy(None)                        # accepted


def test_model_scale_search_is_fast_and_valid():
    """LLaDA-8B-sized template (32 layers, d = 4096, d_ff = 12288, V = 126464) at long context: the search must
    stay negligible next to a denoising step (section 4.4) and its plan must be valid and within the budget."""
    import time
    g = GraphTemplate()
    ids = graph_templates.dllm_step(g, layers=32, d=4096, d_ff=12288, vocab=126464, logits="materialised")
    T, M = 131072, 65536
    _, top = g.plan([T, M], [1, 1], placements=False)
    assert top["peak_chunk"] == ids["k_logits"]                 # 33 GB of fp32 logits dominate at this mask ratio
    budget = 8 << 30
    t0 = time.perf_counter()
    ok, ks, summary, evals = g.search([T, M], budget)
    dt = time.perf_counter() - t0
    assert ok and summary["peak_bytes"] <= budget and ks[ids["k_logits"]] > 1 and ks[ids["k_ffn"]] > 1
    assert dt < 0.25, dt
    placements, s2 = g.plan([T, M], ks)
    assert s2 == summary
    po.check_plan(placements)
    assert po.max_live_bytes(placements) <= summary["peak_bytes"]
    # one step less on either count no longer fits: the setting is minimal in both directions
    for c in (ids["k_logits"], ids["k_ffn"]):
        fewer = list(ks)
        fewer[c] -= 1
        _, s3 = g.plan([T, M], fewer, placements=False)
        assert s3["peak_bytes"] > budget
