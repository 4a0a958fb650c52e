"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2601_06562_amd import binding, workloads

from gpu_helpers import check_against_oracle, oracle_rows, run_hip

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bf16(a):
    return torch.as_tensor(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).to(DEV)


# ------------------------------------------------------------------ a1: compaction, bit-exact
@pytest.mark.parametrize("T", [0, 1, 15, 16, 17, 63, 64, 65, 4095, 4096, 4097, 8192, 12345, 16384, 16385, 40000, 65535, 65536,
                               65537, 131072, 1000003])
@pytest.mark.parametrize("p", [0.0, 0.03, 0.5, 1.0])
def test_compaction_bit_exact(T, p):
    print(f"compaction T={T} p={p}", flush=True)
    rng = np.random.default_rng(T * 7 + int(p * 100))
    m = (rng.random(T) < p).astype(np.uint8) * rng.integers(1, 256, T, dtype=np.uint8)
    want = oracle.mask_select(m)
    mask = torch.from_numpy(m).to(DEV)
    idx = torch.full((max(T, 1) + 8,), -7, dtype=torch.int32, device=DEV)
    count = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    scratch = torch.empty(max(binding.mosaic_compact_scratch_bytes(T), 16), dtype=torch.uint8, device=DEV)
    binding.mosaic_mask_compact(mask, idx, count, scratch)
    torch.cuda.synchronize()
    got = idx.cpu().numpy()
    assert int(count.item()) == want.size
    assert np.array_equal(got[:want.size], want)
    assert np.all(got[want.size:] == -7)            # nothing written past M


def test_compaction_boundaries_and_unaligned_mask():
    T = 3 * 4096 + 5
    m = np.zeros(T + 3, np.uint8)
    for t in (0, 15, 16, 4095, 4096, 8191, 8192, T - 1):
        m[t + 3] = 200
    base = torch.from_numpy(m).to(DEV)
    mask = base[3:]                                  # data pointer not 16-byte aligned
    assert mask.data_ptr() % 16 != 0
    idx = torch.full((T,), -7, dtype=torch.int32, device=DEV)
    count = torch.zeros(1, dtype=torch.int32, device=DEV)
    scratch = torch.empty(binding.mosaic_compact_scratch_bytes(T), dtype=torch.uint8, device=DEV)
    binding.mosaic_mask_compact(mask, idx, count, scratch)
    torch.cuda.synchronize()
    assert idx[:int(count.item())].tolist() == [0, 15, 16, 4095, 4096, 8191, 8192, T - 1]


# ------------------------------------------------------------------ a2-a5: small shapes, element by element
SMALL = [
    # T, d, V, p  -- several row tiles with a ragged tail, vocabulary tails, K tails of the ring
    (1, 64, 1, 1.0),
    (7, 64, 33, 1.0),
    (300, 128, 1000, 0.9),
    (700, 192, 777, 0.5),
    (1024, 256, 2048, 1.0),
    (2000, 64, 5000, 0.4),
    (900, 448, 4099, 0.7),
    # vocabulary a multiple of 256: the hand-scheduled 4-wave kernel (1, 2, 3, 5, 8 K-tiles; 1..n vocab tiles)
    (300, 64, 256, 1.0),
    (520, 128, 512, 0.7),
    (700, 192, 768, 1.0),
    (1000, 320, 1280, 0.5),
    (130, 512, 2560, 1.0),
    (2100, 64, 4096, 0.9),
    # few rows against a wide vocabulary: one row tile spread over 128+ vocabulary splits
    (300, 256, 65536, 0.5),
    (600, 128, 50176, 0.6),
]


@pytest.mark.parametrize("T,d,V,p", SMALL)
def test_small_shapes_vs_oracle(T, d, V, p):
    print(f"small T={T} d={d} V={V} p={p}", flush=True)
    wl = workloads.small_random(T, d, V, p=p, seed=T + V, device=DEV)
    out = run_hip(wl.hidden, wl.w, wl.mask)
    idx_o, want = oracle.full_then_select(workloads.bf16_bits(wl.hidden), workloads.bf16_bits(wl.w),
                                          wl.mask.cpu().numpy())
    M = out["M"]
    assert M == idx_o.size and np.array_equal(out["idx"][:M], idx_o)
    _, logits = oracle.positions(workloads.bf16_bits(wl.hidden), workloads.bf16_bits(wl.w), idx_o, return_logits=True)
    rows = dict(tok=out["tok"][:M], conf=out["conf"][:M], lse=out["lse"][:M])
    check_against_oracle(rows, want, logits, what=wl.name)
    assert np.all(out["tok"][M:] == -7) and np.all(out["lse"][M:] == -7.0)   # rows >= count untouched


def test_integer_inputs_bit_exact():
    """Small-integer inputs: every logit is an integer reached exactly in any summation order, so the
    row maximum and arg-max must equal the oracle's exactly, on every row, ties included."""
    print("integer exact", flush=True)
    rng = np.random.default_rng(5)
    T, d, V = 600, 128, 1500
    H = rng.integers(-4, 5, (T, d)).astype(np.float32)
    W = rng.integers(-3, 4, (V, d)).astype(np.float32)
    mask = (rng.random(T) < 0.8).astype(np.uint8)
    out = run_hip(bf16(H), bf16(W), torch.from_numpy(mask).to(DEV))
    X = H.astype(np.int64) @ W.astype(np.int64).T
    idx = np.nonzero(mask)[0]
    M = idx.size
    assert out["M"] == M
    assert np.array_equal(out["tok"][:M], X[idx].argmax(1))           # numpy arg-max = lowest id on ties
    mx = X[idx].max(1).astype(np.float64)
    implied_max = out["lse"][:M].astype(np.float64) + np.log(out["conf"][:M].astype(np.float64))
    assert np.allclose(implied_max, mx, atol=2e-3)
    hb, wb = workloads.bf16_bits(bf16(H)), workloads.bf16_bits(bf16(W))
    want = oracle.positions(hb, wb, idx)
    assert np.array_equal(want.tok, out["tok"][:M])
    assert np.abs(out["lse"][:M] - want.lse).max() <= 2e-3


def test_tiny_workload_full_then_select():
    print("tiny workload", flush=True)
    wl = workloads.make("tiny", device=DEV)
    out = run_hip(wl.hidden, wl.w, wl.mask)
    idx_o, want = oracle.full_then_select(workloads.bf16_bits(wl.hidden), workloads.bf16_bits(wl.w),
                                          wl.mask.cpu().numpy())
    M = out["M"]
    assert M == idx_o.size and np.array_equal(out["idx"][:M], idx_o)
    rows = dict(tok=out["tok"][:M], conf=out["conf"][:M], lse=out["lse"][:M])
    stats = check_against_oracle(rows, want, what="tiny")
    print(stats, flush=True)


# ------------------------------------------------------------------ closed forms on the GPU path
def test_closed_forms_constant_and_planted():
    print("closed forms", flush=True)
    V, d, T = 8192, 64, 40
    H = np.zeros((T, d), np.float32)
    W = np.zeros((V, d), np.float32)
    vstars = [0, 1, 127, 128, 255, 256, 257, 4095, 4096, 8191]
    # rows 0..9: one dominant logit a=8 planted at vstars; rows 10..: all-zero hidden row
    W[:, 0] = 0.0
    for j, v in enumerate(vstars):
        H[j, j + 1] = 2.0
        W[v, j + 1] = 4.0
    out = run_hip(bf16(H), bf16(W), torch.ones(T, dtype=torch.uint8, device=DEV))
    a = 8.0
    for j, v in enumerate(vstars):
        s = math.exp(a) + V - 1 - (len(vstars) - 1) + (len(vstars) - 1)   # other planted ids see 0 on this row
        assert out["tok"][j] == v
        assert out["lse"][j] == pytest.approx(math.log(s), abs=2e-3)
        assert out["conf"][j] == pytest.approx(math.exp(a) / s, abs=2e-3)
    for j in range(len(vstars), T):
        assert out["tok"][j] == 0
        assert out["lse"][j] == pytest.approx(math.log(V), abs=1e-4)
        assert out["conf"][j] == pytest.approx(1.0 / V, rel=1e-4)


def test_duplicate_w_rows_tie_lowest_id():
    """Two identical LM-head rows accumulate in the same order, so their logits tie bitwise; the lower
    id must be reported, wherever the pair sits relative to tiles, waves and splits."""
    print("ties", flush=True)
    wl = workloads.small_random(300, 128, 4096, p=1.0, seed=77, device=DEV)
    w = wl.w.clone()
    h = wl.hidden.clone()
    pairs = [(3, 4000), (100, 131), (255, 256), (511, 2048), (1000, 1001)]
    boost = (h[:len(pairs)].float() * 0.5).to(torch.bfloat16)      # makes the planted rows dominate
    for j, (lo, hi) in enumerate(pairs):
        w[lo] = boost[j]
        w[hi] = boost[j]
    out = run_hip(h, w, wl.mask)
    want = oracle.positions(workloads.bf16_bits(h), workloads.bf16_bits(w), np.arange(len(pairs)))
    for j, (lo, hi) in enumerate(pairs):
        assert want.tok[j] == lo and want.gap[j] == 0.0
        assert out["tok"][j] == lo, (j, lo, hi, out["tok"][j])


# ------------------------------------------------------------------ invariances of the HIP path itself
def test_mask_only_equals_full_then_select_bitwise():
    """Observation #2 of the paper: computing only masked rows is pure redundancy elimination.  The same
    rows computed under a sparse mask, a full mask and with other rows zeroed must agree bit for bit."""
    print("mask-only == full-then-select", flush=True)
    wl = workloads.small_random(1500, 256, 3000, p=0.3, seed=3, device=DEV)
    sparse = run_hip(wl.hidden, wl.w, wl.mask)
    full = run_hip(wl.hidden, wl.w, torch.ones_like(wl.mask))
    idx = sparse["idx"][:sparse["M"]]
    for k in ("tok", "conf", "lse"):
        assert np.array_equal(sparse[k][:sparse["M"]], full[k][idx]), k
    h2 = wl.hidden.clone()
    h2[wl.mask == 0] = 0
    other = run_hip(h2, wl.w, wl.mask)
    for k in ("tok", "conf", "lse"):
        assert np.array_equal(sparse[k][:sparse["M"]], other[k][:sparse["M"]]), k


def test_chunking_is_a_bitwise_noop_and_deterministic():
    """Section 4.4: chunking along the sequence dimension must not change results.  Same vocabulary
    splits, K = 1, 2, 3, 5 chunks: bitwise equal; a repeat run: bitwise equal."""
    print("chunk invariance", flush=True)
    wl = workloads.small_random(1400, 128, 2500, p=0.9, seed=9, device=DEV)
    base = run_hip(wl.hidden, wl.w, wl.mask)
    again = run_hip(wl.hidden, wl.w, wl.mask)
    M = base["M"]
    S = base["op"].plan.vocab_splits
    for k in ("tok", "conf", "lse"):
        assert np.array_equal(base[k], again[k]), k
    for K in (2, 3, 5):
        def edit(plan, K=K):
            per = -(-1400 // K)
            plan.rows_per_chunk = -(-per // 256) * 256
            plan.num_chunks = -(-1400 // plan.rows_per_chunk)
            plan.vocab_splits = S
            plan.tile_panel = min(plan.tile_panel, plan.rows_per_chunk // 256)
        out = run_hip(wl.hidden, wl.w, wl.mask, plan_edit=edit)
        assert out["op"].plan.num_chunks >= 2
        for k in ("tok", "conf", "lse"):
            assert np.array_equal(base[k][:M], out[k][:M]), (K, k)


def test_fast_and_general_kernels_agree():
    """The 4-wave kernel (16x16x32 MFMAs) and the general kernel (32x32x16) sum the same products in a
    different association, so they agree to fp32 rounding, ragged last row tile included; each is checked
    against the oracle on its own elsewhere."""
    print("fast vs general kernel", flush=True)
    for (T, d, V, p) in [(1300, 256, 2048, 0.8), (257, 64, 256, 1.0), (600, 448, 1024, 0.33)]:
        wl = workloads.small_random(T, d, V, p=p, seed=T, device=DEV)
        fast = run_hip(wl.hidden, wl.w, wl.mask)

        def general(plan):
            plan.flags = binding.PLAN_GENERAL_KERNEL
        gen = run_hip(wl.hidden, wl.w, wl.mask, plan_edit=general)
        assert gen["op"].plan.flags == 1 and fast["op"].plan.flags == 0
        M = fast["M"]
        assert M == gen["M"]
        want = oracle.positions(workloads.bf16_bits(wl.hidden), workloads.bf16_bits(wl.w), fast["idx"][:M])
        clear = want.gap > 1e-4
        assert np.array_equal(fast["tok"][:M][clear], gen["tok"][:M][clear])
        assert np.allclose(fast["lse"][:M], gen["lse"][:M], atol=2e-5, rtol=0)
        assert np.allclose(fast["conf"][:M], gen["conf"][:M], rtol=1e-4, atol=0)
        assert np.array_equal(fast["tok"][M:], gen["tok"][M:])          # untouched tails


def test_budget_forces_chunks_and_bounds_workspace():
    print("budget", flush=True)
    wl = workloads.small_random(3000, 128, 2048, p=1.0, seed=4, device=DEV)
    free = run_hip(wl.hidden, wl.w, wl.mask)
    assert free["op"].plan.num_chunks == 1
    budget = 12 * 256 * 3 + binding.SYNC_BYTES               # room for one row tile x 3 splits
    tight = run_hip(wl.hidden, wl.w, wl.mask, budget_bytes=budget)
    plan = tight["op"].plan
    assert plan.workspace_bytes <= budget and plan.num_chunks == 4 and plan.rows_per_chunk == 768
    assert plan.vocab_splits == 1
    M = free["M"]
    assert np.array_equal(free["tok"][:M], tight["tok"][:M])
    assert np.allclose(free["lse"][:M], tight["lse"][:M], atol=1e-5)
    assert np.allclose(free["conf"][:M], tight["conf"][:M], rtol=1e-5)


def test_max_rows_bound_and_empty_mask():
    print("max_rows / empty", flush=True)
    wl = workloads.small_random(800, 64, 512, p=0.5, seed=6, device=DEV)
    out = run_hip(wl.hidden, wl.w, torch.zeros_like(wl.mask))
    assert out["M"] == 0 and np.all(out["tok"] == -7) and np.all(out["lse"] == -7.0)
    M = wl.M
    out = run_hip(wl.hidden, wl.w, wl.mask, max_rows=M)      # host knows M exactly
    ref = run_hip(wl.hidden, wl.w, wl.mask)                  # host only knows T
    assert out["M"] == M
    assert np.array_equal(out["tok"][:M], ref["tok"][:M])
    assert np.allclose(out["lse"][:M], ref["lse"][:M], atol=1e-5)


def test_strided_hidden_rows():
    print("strided hidden", flush=True)
    wl = workloads.small_random(500, 128, 700, p=0.6, seed=8, device=DEV)
    wide = torch.zeros((500, 192), dtype=torch.bfloat16, device=DEV)
    wide[:, :128] = wl.hidden
    a = run_hip(wl.hidden, wl.w, wl.mask)
    b = run_hip(wide[:, :128], wl.w, wl.mask)
    for k in ("tok", "conf", "lse"):
        assert np.array_equal(a[k], b[k]), k


def test_mfma_probe_runs_and_reports_its_flops():
    print("mfma probe", flush=True)
    operands = (torch.rand(32768, device=DEV) - 0.5).to(torch.bfloat16)
    sink = torch.full((65536,), float("nan"), dtype=torch.float32, device=DEV)
    flop = binding.mosaic_mfma_probe(operands, sink, 100, 256)
    torch.cuda.synchronize()
    assert flop == 100 * 256 * 4 * 64 * 16384
    assert bool(torch.isfinite(sink).all())            # every lane of every workgroup stored its sum


def test_large_common_offset_stays_within_tolerance():
    """All logits of a row shifted by a large constant (a hidden component along a direction every LM-head row
    shares): the exponent of exp(x - max) is formed from values of magnitude ~1000, where fp32 rounding of the
    products is largest; lse and conf must still meet the tolerances."""
    print("large offset", flush=True)
    rng = np.random.default_rng(12)
    T, d, V = 300, 128, 4096
    H = rng.standard_normal((T, d)).astype(np.float32)
    W = (rng.standard_normal((V, d)) * d ** -0.5).astype(np.float32)
    W[:, 0] = 1.0
    H[:, 0] = np.where(np.arange(T) % 2 == 0, 1024.0, -768.0)
    hidden, w = bf16(H), bf16(W)
    mask = torch.ones(T, dtype=torch.uint8, device=DEV)
    out = run_hip(hidden, w, mask)
    want = oracle.positions(workloads.bf16_bits(hidden), workloads.bf16_bits(w), np.arange(T))
    assert np.abs(want.lse).min() > 700
    stats = check_against_oracle(dict(tok=out["tok"][:T], conf=out["conf"][:T], lse=out["lse"][:T]), want,
                                 what="large offset")
    print(stats, flush=True)
