"""Host-side logic of libmosaic that needs no GPU: the library loads and exports every symbol the
header declares, the chunk-size selector against brute force, and argument validation (errors are
raised before anything is enqueued, so null device pointers are never dereferenced)."""
import ctypes
import os
import re

import pytest

from paper_2601_06562_amd import binding
from paper_2601_06562_amd.binding import MosaicPlan

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mosaic.h")).read()
    declared = set(re.findall(r"\b(mosaic_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    graph_header = open(os.path.join(ROOT, "include", "mosaic_graph.h")).read()
    graph_declared = set(re.findall(r"\b(mosaic_graph_[a-z_]+)\s*\(", graph_header))
    assert graph_declared == set(binding.GRAPH_EXPORTS)
    declared |= graph_declared
    L = binding.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert L.mosaic_version() >= 1000
    assert binding.status_string(0) == "MOSAIC_OK"
    assert binding.status_string(-3) == "MOSAIC_ERR_WORKSPACE_TOO_SMALL"


def workspace(C, S, per_partial=12):
    return per_partial * C * S + binding.SYNC_BYTES


def brute_force_min_chunks(max_rows, budget, per_partial=12):
    """Smallest K whose chunk fits with a single split, by enumeration (section 4.4: minimal K)."""
    rows = max(max_rows, 1)
    for K in range(1, rows + 1):
        C = -(-(-(-rows // K)) // 256) * 256
        if workspace(C, 1, per_partial) <= budget:
            return K, C
    return None


@pytest.mark.parametrize("rows", [1, 255, 256, 257, 4096, 6554, 58491, 131072])
def test_selector_unbounded_is_one_chunk(rows):
    plan = binding.mosaic_plan_workspace(131072, rows, 4096, 126464, 0)
    assert plan.num_chunks == 1 and plan.rows_per_chunk >= rows and plan.rows_per_chunk % 256 == 0
    assert plan.workspace_bytes == workspace(plan.rows_per_chunk, plan.vocab_splits)
    assert 1 <= plan.vocab_splits <= 256 and 1 <= plan.grid <= 256


@pytest.mark.parametrize("rows", [300, 4096, 5000, 58491])
@pytest.mark.parametrize("budget", [4096, 4097, 12 * 256 * 7, 12 * 1024 + 1024, 12 * 4096 + 1024, 100000, 10 ** 6])
def test_selector_matches_brute_force(rows, budget):
    plan = binding.mosaic_plan_workspace(131072, rows, 4096, 126464, budget)
    K, C = brute_force_min_chunks(rows, budget)
    assert plan.rows_per_chunk == C                      # minimal K <=> largest chunk that fits
    assert plan.num_chunks == -(-rows // C)
    assert plan.workspace_bytes <= budget
    assert plan.num_chunks * plan.rows_per_chunk >= rows
    # lazy: a roomier budget never needs more chunks
    roomy = binding.mosaic_plan_workspace(131072, rows, 4096, 126464, budget * 2)
    assert roomy.num_chunks <= plan.num_chunks


@pytest.mark.parametrize("rows", [300, 4096, 5000, 58491])
@pytest.mark.parametrize("budget", [6144, 6145, 20 * 256 * 7, 12 * 4096 + 1024, 20 * 4096 + 1024, 100000, 10 ** 6])
def test_selector_bounds_the_sampling_workspace(rows, budget):
    """A plan for a sampling step keeps 20 bytes per row and split; the budget bounds THAT (section 4.4: the search
    stops only at a configuration that fits), with the same minimal-K rule."""
    plan = binding.mosaic_plan_workspace(131072, rows, 4096, 126464, budget, sampling=True)
    assert plan.flags & binding.PLAN_SAMPLING
    K, C = brute_force_min_chunks(rows, budget, per_partial=20)
    assert plan.rows_per_chunk == C and plan.num_chunks == -(-rows // C)
    assert plan.workspace_bytes == workspace(plan.rows_per_chunk, plan.vocab_splits, 20) <= budget
    assert binding.mosaic_sample_workspace_bytes(plan) == plan.workspace_bytes
    greedy = binding.mosaic_plan_workspace(131072, rows, 4096, 126464, budget)
    assert not greedy.flags & binding.PLAN_SAMPLING and greedy.num_chunks <= plan.num_chunks
    assert greedy.workspace_bytes == workspace(greedy.rows_per_chunk, greedy.vocab_splits) <= budget


def test_sampling_selector_floor_and_unbounded_size():
    with pytest.raises(binding.MosaicError) as e:
        binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 6143, sampling=True)      # 20 * 256 + 1024 - 1
    assert e.value.status == binding.MOSAIC_ERR_WORKSPACE_TOO_SMALL
    assert binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 6144, sampling=True).rows_per_chunk == 256
    a = binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 0)
    b = binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 0, sampling=True)
    assert (a.num_chunks, a.rows_per_chunk, a.vocab_splits, a.grid) == (b.num_chunks, b.rows_per_chunk, b.vocab_splits, b.grid)
    assert (b.workspace_bytes - binding.SYNC_BYTES) * 12 == (a.workspace_bytes - binding.SYNC_BYTES) * 20


def test_selector_failure_is_exactly_the_non_chunkable_floor():
    with pytest.raises(binding.MosaicError) as e:
        binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 4095)
    assert e.value.status == binding.MOSAIC_ERR_WORKSPACE_TOO_SMALL
    assert binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 4096).rows_per_chunk == 256


def test_selector_split_choice_fills_the_chip():
    plan = binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 0)
    assert plan.vocab_splits == 16 and plan.grid == 256          # 16 row tiles x 16 splits = 256 CUs
    plan = binding.mosaic_plan_workspace(131072, 58491, 4096, 126464, 0)
    units = (plan.rows_per_chunk // 256) * plan.vocab_splits
    rounds = -(-units // 256)
    assert units / (rounds * 256) > 0.97


def test_selector_rejects_bad_arguments():
    L = binding.lib()
    plan = MosaicPlan()
    ok = lambda *a: L.mosaic_plan_workspace(*a, ctypes.byref(plan))
    assert ok(-1, 0, 4096, 1000, 0, 0, 0) == binding.MOSAIC_ERR_INVALID_ARG
    assert ok(10, 11, 4096, 1000, 0, 0, 0) == binding.MOSAIC_ERR_INVALID_ARG
    assert ok(10, 10, 4000, 1000, 0, 0, 0) == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE
    assert ok(2 ** 31, 10, 4096, 1000, 0, 0, 0) == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE
    assert L.mosaic_plan_workspace(10, 10, 4096, 1000, 0, 0, 0, None) == binding.MOSAIC_ERR_INVALID_ARG
    assert ok(10, 10, 4096, 1000, 0, 0, 2) == binding.MOSAIC_ERR_INVALID_ARG            # decode mode is 0 or 1
    assert ok(10, 10, 4096, 1000, 0, 0, -1) == binding.MOSAIC_ERR_INVALID_ARG
    assert ok(0, 0, 64, 1, 0, 0, 0) == binding.MOSAIC_OK and ok(0, 0, 64, 1, 0, 0, 1) == binding.MOSAIC_OK


def test_entry_points_validate_before_launch():
    L = binding.lib()
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(0x1000)        # never dereferenced: validation fails first
    assert L.mosaic_mask_compact(null, 16, fake, fake, fake, 1 << 20, null) == binding.MOSAIC_ERR_INVALID_ARG
    assert L.mosaic_mask_compact(fake, -1, fake, fake, fake, 1 << 20, null) == binding.MOSAIC_ERR_INVALID_ARG
    assert L.mosaic_mask_compact(fake, 2 ** 31, fake, fake, fake, 1 << 30, null) == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE
    assert L.mosaic_mask_compact(fake, 10 ** 6, fake, fake, fake, 8, null) == binding.MOSAIC_ERR_INVALID_ARG
    assert binding.mosaic_compact_scratch_bytes(0) >= 4 and binding.mosaic_compact_scratch_bytes(10 ** 6) >= 4 * 245
    plan = binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 0)
    P = ctypes.byref(plan)
    call = lambda **kw: L.mosaic_masked_logits_reduce(
        kw.get("hidden", fake), kw.get("T", 4096), kw.get("d", 4096), kw.get("ld_h", 4096), kw.get("w", fake),
        kw.get("V", 126464), fake, kw.get("count", fake), kw.get("max_rows", 4096), fake, fake, fake,
        kw.get("plan", P), kw.get("ws", fake), kw.get("ws_bytes", plan.workspace_bytes), null)
    assert call(hidden=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert call(count=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert call(hidden=ctypes.c_void_p(0x1008)) == binding.MOSAIC_ERR_INVALID_ARG          # misaligned
    assert call(d=4090) == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE
    assert call(ld_h=4000) == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE
    assert call(ld_h=4100) == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE
    assert call(ws_bytes=plan.workspace_bytes - 1) == binding.MOSAIC_ERR_WORKSPACE_TOO_SMALL
    assert call(max_rows=5000) == binding.MOSAIC_ERR_INVALID_ARG                            # > T
    assert call(max_rows=0) == binding.MOSAIC_OK                                            # nothing to do
    bad = MosaicPlan.from_buffer_copy(plan)
    bad.vocab_splits = 0
    assert call(plan=ctypes.byref(bad)) == binding.MOSAIC_ERR_INVALID_ARG
    small = binding.mosaic_plan_workspace(4096, 256, 4096, 126464, 0)                       # plan for fewer rows
    assert call(plan=ctypes.byref(small), ws_bytes=1 << 30) == binding.MOSAIC_ERR_INVALID_ARG


def test_static_workspace_entry_point_validates_before_touching_the_device():
    L = binding.lib()
    null, fake = ctypes.c_void_p(0), ctypes.c_void_p(0x1000)
    plan = binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 0)
    assert plan.workspace_bytes <= binding.STATIC_WORKSPACE_BYTES
    call = lambda **kw: L.mosaic_masked_logits_reduce_static(
        kw.get("hidden", fake), kw.get("T", 4096), kw.get("d", 4096), 4096, fake, 126464, fake, kw.get("count", fake),
        kw.get("max_rows", 4096), fake, fake, fake, kw.get("plan", ctypes.byref(plan)), null)
    assert call(hidden=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert call(count=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert call(d=4090) == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE
    assert call(max_rows=0) == binding.MOSAIC_OK
    # a plan beyond the fixed array is refused with a clear status, before any device call
    big = binding.mosaic_plan_workspace(131072, 58501, 4096, 126464, 0)
    assert big.workspace_bytes > binding.STATIC_WORKSPACE_BYTES
    assert L.mosaic_masked_logits_reduce_static(fake, 131072, 4096, 4096, fake, 126464, fake, fake, 58501, fake, fake,
                                                fake, ctypes.byref(big), null) == binding.MOSAIC_ERR_WORKSPACE_TOO_SMALL
    # ... and the selector, given the array's size as the budget, chunks the same rows to fit
    fits = binding.mosaic_plan_workspace(131072, 58501, 4096, 126464, binding.STATIC_WORKSPACE_BYTES)
    assert fits.workspace_bytes <= binding.STATIC_WORKSPACE_BYTES
    header = open(os.path.join(ROOT, "include", "mosaic.h")).read()
    assert "#define MOSAIC_STATIC_WORKSPACE_BYTES (4 << 20)" in header and binding.STATIC_WORKSPACE_BYTES == 4 << 20
    assert "#define MOSAIC_SYNC_BYTES 1024" in header and binding.SYNC_BYTES == 1024


def test_sampling_tail_entry_points_validate_before_launch():
    L = binding.lib()
    null, fake = ctypes.c_void_p(0), ctypes.c_void_p(0x1000)
    un = lambda **kw: L.mosaic_unmask_topn(kw.get("conf", fake), fake, fake, kw.get("count", fake),
                                           kw.get("max_rows", 100), kw.get("seq", fake), kw.get("B", 2), fake,
                                           kw.get("tokens", fake), fake, kw.get("T", 1000), null)
    assert un(count=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert un(seq=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert un(B=0) == binding.MOSAIC_ERR_INVALID_ARG
    assert un(max_rows=2000) == binding.MOSAIC_ERR_INVALID_ARG            # > T
    assert un(T=2 ** 31, max_rows=5) == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE
    assert un(conf=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert un(tokens=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert un(max_rows=0, conf=null) == binding.MOSAIC_OK                 # nothing to do
    sh = lambda **kw: L.mosaic_shift_indices(kw.get("idx", fake), kw.get("count", fake), kw.get("max_rows", 10),
                                             kw.get("seq", fake), kw.get("B", 1), kw.get("out", fake), null)
    assert sh(count=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert sh(B=0) == binding.MOSAIC_ERR_INVALID_ARG
    assert sh(out=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert sh(max_rows=-1) == binding.MOSAIC_ERR_INVALID_ARG
    assert sh(max_rows=0, idx=null) == binding.MOSAIC_OK


def test_sampling_entry_point_validates_before_launch():
    L = binding.lib()
    null, fake = ctypes.c_void_p(0), ctypes.c_void_p(0x1000)
    plan = binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 0)
    need = binding.mosaic_sample_workspace_bytes(plan)
    assert need == 20 * plan.rows_per_chunk * plan.vocab_splits + binding.SYNC_BYTES   # five planes per row and split
    assert need > plan.workspace_bytes
    assert L.mosaic_sample_workspace_bytes(None) == 0
    call = lambda **kw: L.mosaic_masked_logits_sample(
        kw.get("hidden", fake), 4096, kw.get("d", 4096), 4096, fake, 126464, fake, kw.get("noise_idx", null),
        kw.get("count", fake), kw.get("max_rows", 4096), kw.get("tau", 1.0), kw.get("seed", 7), fake, fake, fake,
        ctypes.byref(plan), fake, kw.get("ws_bytes", need), null)
    assert call(tau=-0.5) == binding.MOSAIC_ERR_INVALID_ARG
    assert call(tau=float("nan")) == binding.MOSAIC_ERR_INVALID_ARG
    assert call(tau=float("inf")) == binding.MOSAIC_ERR_INVALID_ARG
    assert call(ws_bytes=need - 1) == binding.MOSAIC_ERR_WORKSPACE_TOO_SMALL      # the greedy size is not enough
    assert call(ws_bytes=plan.workspace_bytes) == binding.MOSAIC_ERR_WORKSPACE_TOO_SMALL
    assert call(hidden=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert call(count=null) == binding.MOSAIC_ERR_INVALID_ARG
    assert call(d=4090) == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE
    assert call(max_rows=0) == binding.MOSAIC_OK                                   # nothing to do
    assert call(max_rows=0, noise_idx=fake) == binding.MOSAIC_OK                   # the optional list is accepted
    assert call(seed=2 ** 64 - 1, tau=-1.0) == binding.MOSAIC_ERR_INVALID_ARG      # a full 64-bit seed is accepted


def test_mfma_probe_validates_before_launch():
    L = binding.lib()
    null, fake = ctypes.c_void_p(0), ctypes.c_void_p(0x1000)
    assert L.mosaic_mfma_probe_flops(10, 256) == 10 * 256 * 4 * 64 * 16 * 16 * 32 * 2
    assert L.mosaic_mfma_probe_flops(-1, 256) == 0
    assert L.mosaic_mfma_probe(null, fake, 10, 256, null) == binding.MOSAIC_ERR_INVALID_ARG
    assert L.mosaic_mfma_probe(fake, null, 10, 256, null) == binding.MOSAIC_ERR_INVALID_ARG
    assert L.mosaic_mfma_probe(fake, fake, 0, 256, null) == binding.MOSAIC_ERR_INVALID_ARG
    assert L.mosaic_mfma_probe(fake, fake, 10, 0, null) == binding.MOSAIC_ERR_INVALID_ARG
    assert L.mosaic_mfma_probe(fake, fake, 10, 70000, null) == binding.MOSAIC_ERR_INVALID_ARG
    assert L.mosaic_mfma_probe(ctypes.c_void_p(0x1004), fake, 10, 256, null) == binding.MOSAIC_ERR_INVALID_ARG


def test_vmm_entry_points_validate_their_arguments():
    L = binding.lib()
    h = ctypes.c_void_p()
    assert L.mosaic_vmm_create(0, 1 << 20, None) == binding.MOSAIC_ERR_INVALID_ARG
    assert L.mosaic_vmm_create(-1, 1 << 20, ctypes.byref(h)) == binding.MOSAIC_ERR_INVALID_ARG and not h
    assert L.mosaic_vmm_create(0, 0, ctypes.byref(h)) == binding.MOSAIC_ERR_INVALID_ARG and not h
    assert L.mosaic_vmm_resize(None, 10) == binding.MOSAIC_ERR_INVALID_ARG
    assert L.mosaic_vmm_ptr(None) is None
    assert L.mosaic_vmm_committed_bytes(None) == 0 and L.mosaic_vmm_reserved_bytes(None) == 0
    assert L.mosaic_vmm_granularity(None) == 0 and L.mosaic_vmm_kept_contents(None) == 0
    assert L.mosaic_vmm_destroy(None) == binding.MOSAIC_OK


def test_selector_keeps_at_least_four_splits_for_cache_sharing():
    """Many row tiles would balance with a single split each, but the workgroups behind one L2 then share no hidden
    tile; the selector keeps four splits wherever the vocabulary has four tiles (a byte budget may still cut them)."""
    for rows in (65536, 131072, 16384 * 3):
        assert binding.mosaic_plan_workspace(rows, rows, 4096, 126464, 0).vocab_splits >= 4
    assert binding.mosaic_plan_workspace(65536, 65536, 4096, 512, 0).vocab_splits == 2        # only two tiles
    tight = binding.mosaic_plan_workspace(65536, 65536, 4096, 126464, 12 * 65536 + 1024)     # budget for one split
    assert tight.vocab_splits == 1 and tight.num_chunks == 1
