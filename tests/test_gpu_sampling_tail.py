"""GPU parity for the rows after mask-only logits: top-n unmasking (sampling tail, greedy reading of the
paper's section 2.1) and Dream-style shifted gather indices (section 4.5).  Integer and byte outputs:
bit-exact against the oracle; both sides decide on the same fp32 confidences."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_06562_amd import binding, workloads

from gpu_helpers import check_against_oracle, oracle_rows, run_hip

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a, dtype):
    a = np.asarray(a)
    if a.size == 0:                      # keep a real device pointer for empty inputs
        return torch.zeros(1, dtype=dtype, device=DEV)
    return torch.as_tensor(a, dtype=dtype).to(DEV)


def run_unmask(conf, tok, idx, seq_starts, n_per_seq, tokens, mask):
    M = len(idx)
    count = dev([M], torch.int32)
    d_tokens, d_mask = dev(tokens, torch.int32), dev(mask, torch.uint8)
    binding.mosaic_unmask_topn(dev(conf, torch.float32), dev(tok, torch.int32), dev(idx, torch.int32), count,
                               max(M, 1), dev(seq_starts, torch.int32), dev(n_per_seq, torch.int32), d_tokens, d_mask)
    torch.cuda.synchronize()
    return d_tokens.cpu().numpy(), d_mask.cpu().numpy()


@pytest.mark.parametrize("T,B,p,levels", [(64, 1, 0.5, 3), (1000, 3, 0.4, 5), (5000, 4, 0.9, 0), (40000, 2, 1.0, 7),
                                          (131072, 8, 0.3, 0), (2048, 2, 0.0, 0)])
def test_unmask_topn_bit_exact(T, B, p, levels):
    print(f"unmask T={T} B={B} p={p} levels={levels}", flush=True)
    rng = np.random.default_rng(T + B)
    cuts = np.sort(rng.choice(np.arange(1, T), B - 1, replace=False)) if B > 1 else np.array([], int)
    seq_starts = np.concatenate([[0], cuts, [T]]).astype(np.int32)
    mask = (rng.random(T) < p).astype(np.uint8)
    idx = np.nonzero(mask)[0].astype(np.int32)
    if levels:   # few distinct confidences: many exact ties, decided by position
        conf = rng.choice(np.linspace(0.05, 0.95, levels).astype(np.float32), idx.size)
    else:
        conf = rng.random(idx.size).astype(np.float32) * np.float32(1e-3)
    tok = rng.integers(0, 150000, idx.size).astype(np.int32)
    tokens = rng.integers(0, 150000, T).astype(np.int32)
    for trial in range(3):
        n_per_seq = rng.integers(0, max(2, int(1.3 * T * p / B) + 2), B).astype(np.int32)
        if trial == 0:
            n_per_seq[:] = 1
        want_tokens, want_mask, _ = oracle.unmask_topn(conf, tok, idx, seq_starts, n_per_seq, tokens, mask)
        got_tokens, got_mask = run_unmask(conf, tok, idx, seq_starts, n_per_seq, tokens, mask)
        assert np.array_equal(got_mask, want_mask), (trial, n_per_seq)
        assert np.array_equal(got_tokens, want_tokens), (trial, n_per_seq)


def test_shift_indices_bit_exact():
    print("shift indices", flush=True)
    rng = np.random.default_rng(2)
    T = 70000
    seq_starts = np.array([0, 1, 17, 4096, 4097, 30000, T], np.int32)
    mask = (rng.random(T) < 0.5).astype(np.uint8)
    mask[[0, 1, 17, 4096, 4097, 30000, T - 1]] = 1          # every sequence start is masked
    idx = np.nonzero(mask)[0].astype(np.int32)
    want = oracle.shift_indices(idx, seq_starts)
    out = torch.full((idx.size + 4,), -7, dtype=torch.int32, device=DEV)
    binding.mosaic_shift_indices(dev(idx, torch.int32), dev([idx.size], torch.int32), idx.size,
                                 dev(seq_starts, torch.int32), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[:idx.size], want) and np.all(got[idx.size:] == -7)


def test_shifted_prediction_end_to_end():
    """compact -> shift -> fused reduction on the shifted rows: equals the oracle evaluated at p-1."""
    print("shifted prediction", flush=True)
    wl = workloads.small_random(1200, 128, 1024, p=0.5, seed=31, device=DEV)
    seq_starts = np.array([0, 500, 1200], np.int32)
    op = binding.MaskOnlyLogits(wl.T, wl.d, wl.V, device=DEV)
    binding.mosaic_mask_compact(wl.mask, op.idx, op.count, op.scratch)
    gather = torch.empty_like(op.idx)
    binding.mosaic_shift_indices(op.idx, op.count, op.max_rows, dev(seq_starts, torch.int32), gather)
    binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, gather, op.count, op.max_rows, op.token, op.conf, op.lse,
                                        op.plan, op.workspace)
    torch.cuda.synchronize()
    M = int(op.count.item())
    idx = op.idx[:M].cpu().numpy()
    want_rows = oracle.shift_indices(idx, seq_starts)
    assert np.array_equal(gather[:M].cpu().numpy(), want_rows)
    want, logits = oracle_rows(wl.hidden, workloads.bf16_bits(wl.w), want_rows, return_logits=True)
    check_against_oracle(dict(tok=op.token[:M].cpu().numpy(), conf=op.conf[:M].cpu().numpy(),
                              lse=op.lse[:M].cpu().numpy()), want, logits, what="shifted")


def test_denoising_tail_loop_runs_to_completion():
    """Several denoising steps' tails back to back on one stream: compact -> mask-only logits -> unmask n per
    sequence -> next step sees the updated mask.  Every step's selection is checked against the oracle applied
    to that step's confidences; the loop must end with an empty mask after ceil(masked / n) steps."""
    print("denoising loop", flush=True)
    wl = workloads.small_random(900, 128, 2048, p=0.6, seed=41, device=DEV)
    seq_starts_h = np.array([0, 400, 900], np.int32)
    seq_starts = dev(seq_starts_h, torch.int32)
    n_h = np.array([37, 50], np.int32)
    n_per_seq = dev(n_h, torch.int32)
    mask = wl.mask.clone()
    tokens = torch.full((wl.T,), -1, dtype=torch.int32, device=DEV)
    op = binding.MaskOnlyLogits(wl.T, wl.d, wl.V, device=DEV)
    m0 = wl.mask.cpu().numpy()
    left = np.array([m0[:400].sum(), m0[400:].sum()])
    steps_needed = int(np.max(np.ceil(left / n_h)))
    steps = 0
    while True:
        mask_h, tokens_h = mask.cpu().numpy(), tokens.cpu().numpy()
        if mask_h.sum() == 0:
            break
        op.step(wl.hidden, wl.w, mask)
        binding.mosaic_unmask_topn(op.conf, op.token, op.idx, op.count, op.max_rows, seq_starts, n_per_seq, tokens, mask)
        torch.cuda.synchronize()
        M = int(op.count.item())
        assert M == int(mask_h.sum())
        want_tokens, want_mask, _ = oracle.unmask_topn(op.conf[:M].cpu().numpy(), op.token[:M].cpu().numpy(),
                                                       op.idx[:M].cpu().numpy(), seq_starts_h, n_h, tokens_h, mask_h)
        assert np.array_equal(mask.cpu().numpy(), want_mask) and np.array_equal(tokens.cpu().numpy(), want_tokens)
        steps += 1
        assert steps <= steps_needed
    assert steps == steps_needed
    final = tokens.cpu().numpy()
    assert np.all(final[m0 != 0] >= 0) and np.all(final[m0 == 0] == -1)      # exactly the masked positions were filled


def test_replanning_for_the_masks_that_remain_changes_the_schedule_not_the_results():
    """A scheduler that knows how many masks are left renews the plan (more vocabulary splits for fewer rows); the
    buffers stay, and the results are those of an object made for that bound."""
    print("replan", flush=True)
    T, d, V = 3000, 256, 16384
    wl = workloads.small_random(T, d, V, p=0.9, seed=5, device=DEV)
    op = binding.MaskOnlyLogits(T, d, V, device=DEV)
    mask = wl.mask.clone()
    splits = []
    for keep in (2500, 900, 200, 30):
        pos = torch.nonzero(mask).flatten()
        mask[pos[keep:]] = 0                                   # fewer masks each round
        M = int(mask.sum().item())
        op.replan(M)
        splits.append(op.plan.vocab_splits)
        op.step(wl.hidden, wl.w, mask)
        fresh = binding.MaskOnlyLogits(T, d, V, max_rows=M, device=DEV)
        fresh.step(wl.hidden, wl.w, mask)
        torch.cuda.synchronize()
        assert int(op.count.item()) == M == keep
        assert torch.equal(op.token[:M], fresh.token[:M]) and torch.equal(op.lse[:M], fresh.lse[:M])
        assert torch.equal(op.conf[:M], fresh.conf[:M])
    assert splits[-1] > splits[0]
    with pytest.raises(ValueError):
        op.replan(T + 1)
