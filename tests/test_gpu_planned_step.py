"""The paper's order of operations (section 4.1: template -> reserved address range -> chunk search -> reuse plan ->
bound pages -> execution) joined end to end on full-size workloads: the tail of a denoising step is registered as a
graph template (section 4.3), the search finds the K_logits a byte budget forces (section 4.4), the first-fit plan
gives every buffer an offset in one workspace (section 4.5), the VMM range is mapped up to the planned peak, and the
HIP path runs with its index list, scan scratch, partial results and outputs AT those offsets, in the searched
number of chunks, against the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

from gpu_helpers import check_against_oracle, oracle_rows
from oracle import planner_oracle as po
from paper_2601_06562_amd import binding, graph_templates, workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ROW_TILE = binding.ROW_TILE


@pytest.mark.parametrize("name,want_chunks", [("llada_first_step", 4), ("long_semi_ar", 3)])
def test_searched_plan_on_mapped_pages_runs_the_chunked_step(name, want_chunks):
    print(f"planned step: {name}, K_logits = {want_chunks}", flush=True)
    torch.cuda.set_device(0)
    wl = workloads.make(name, device=DEV)
    T, M, d, V = wl.T, wl.M, wl.d, wl.V
    R = -(-M // ROW_TILE)
    unbounded = binding.mosaic_plan_workspace(T, M, d, V, 0)
    S = unbounded.vocab_splits

    # (1) template, (3) search: the smallest budget that K_logits = want_chunks meets is the planned peak at that K
    g = binding.GraphTemplate()
    ids = graph_templates.mask_only_tail(g, S, binding.mosaic_compact_scratch_bytes(T), sync_bytes=binding.SYNC_BYTES)
    _, at_k = g.plan([T, R], [want_chunks], placements=False)
    _, below = g.plan([T, R], [want_chunks - 1], placements=False)
    budget = at_k["peak_bytes"]
    assert below["peak_bytes"] > budget
    ok, ks, summary, evals = g.search([T, R], budget)
    assert ok and ks == [want_chunks] and evals == want_chunks and summary["peak_bytes"] <= budget
    # (4) the plan
    placements, s2 = g.plan([T, R], ks)
    assert s2 == summary
    po.check_plan(placements)
    where = {(p["tensor"], p["iteration"]): p for p in placements}
    tiles_per_chunk = -(-R // want_chunks)
    C = tiles_per_chunk * ROW_TILE
    part = [where[(ids["partials"], it)] for it in range(want_chunks)]
    need = 12 * S * C + binding.SYNC_BYTES                  # what the fused call asks for
    assert all(need <= p["bytes"] <= need + tiles_per_chunk * binding.SYNC_BYTES for p in part)
    assert len({p["offset"] for p in part}) == 1            # consecutive chunks reuse one slot of the workspace
    naive = 12 * S * R * ROW_TILE + R * binding.SYNC_BYTES
    assert summary["peak_bytes"] <= budget < naive + 4 * T

    # (2) reserve once, (5) bind pages up to the planned peak
    try:
        vmm = binding.VmmWorkspace(1 << 30, device=0)
    except binding.MosaicError as e:
        if e.status == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE:
            pytest.skip("this device reports no virtual memory management")
        raise
    vmm.resize(summary["peak_bytes"])
    assert vmm.committed_bytes >= summary["peak_bytes"]

    def at(tensor, count, dtype):
        p = where[(ids[tensor], 0)]
        assert p["bytes"] >= count * torch.empty((), dtype=dtype).element_size()
        return vmm.tensor(p["offset"], count, dtype)
    idx = at("idx", T, torch.int32)
    count = at("count", 1, torch.int32)
    scratch = at("scratch", binding.mosaic_compact_scratch_bytes(T), torch.uint8)
    tok = at("out_token", M, torch.int32)
    conf = at("out_conf", M, torch.float32)
    lse = at("out_lse", M, torch.float32)
    partials = vmm.tensor(part[0]["offset"], part[0]["bytes"], torch.uint8)
    vmm.tensor(0, vmm.committed_bytes, torch.uint8).fill_(0xA5)

    # (6) execute: the kernel's plan is the searched chunking with the template's split count
    plan = binding.MosaicPlan.from_buffer_copy(unbounded)
    plan.num_chunks = -(-M // C)
    plan.rows_per_chunk = C
    plan.workspace_bytes = need
    plan.grid = min(256, tiles_per_chunk * S)
    assert plan.num_chunks == want_chunks
    binding.mosaic_mask_compact(wl.mask, idx, count, scratch)
    binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, idx, count, M, tok, conf, lse, plan, partials)
    torch.cuda.synchronize()
    assert int(count.item()) == M

    # against the oracle: a stratified sample with both sides of every chunk boundary and the ragged end
    rng = np.random.default_rng(7)
    edges = [r for c in range(1, want_chunks) for r in (c * C - 1, c * C) if r < M]
    rows = np.unique(np.concatenate([rng.choice(M, 64, replace=False), [0, M - 1], edges]))
    positions = idx[:M].cpu().numpy()[rows]
    want, logits = oracle_rows(wl.hidden, workloads.bf16_bits(wl.w), positions, return_logits=True)
    stats = check_against_oracle(dict(tok=tok.cpu().numpy()[rows], conf=conf.cpu().numpy()[rows],
                                      lse=lse.cpu().numpy()[rows]), want, logits, what=name + " planned")
    print(stats, flush=True)
    # against the unchunked run on ordinary buffers with the same split count: chunking changes nothing, bit for bit
    ref = binding.MaskOnlyLogits(T, d, V, max_rows=M, device=DEV)
    ref.step(wl.hidden, wl.w, wl.mask)
    torch.cuda.synchronize()
    assert ref.plan.vocab_splits == S and ref.plan.num_chunks == 1
    assert torch.equal(ref.idx[:M], idx[:M])
    assert torch.equal(ref.token[:M], tok) and torch.equal(ref.lse[:M], lse) and torch.equal(ref.conf[:M], conf)
    # nothing was written outside the planned blocks: the rest of the mapped range still holds the fill pattern
    used = np.zeros(vmm.committed_bytes, bool)
    for p in placements:
        used[p["offset"]:p["offset"] + p["bytes"]] = True
    whole = vmm.tensor(0, vmm.committed_bytes, torch.uint8).cpu().numpy()
    assert np.all(whole[~used] == 0xA5)
    del idx, count, scratch, tok, conf, lse, partials
    vmm.close()
