"""GPU tests of the boundary's robustness, all through the C ABI: guard bytes behind every buffer an entry
point writes, gather entries outside [0, T), the sampling noise keyed by the predicted position under a shifted
gather list (paper section 4.5, last paragraph, with section 2.1), and the byte budget under sampling
(section 4.4: the search stops only at a configuration that fits)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_helpers import check_against_oracle
from paper_2601_06562_amd import binding, workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GUARD = 64          # canary bytes behind every buffer
CANARY = 0xA5


class Guarded:
    """A device buffer of `n` elements followed by GUARD canary bytes (and preceded by GUARD more)."""

    def __init__(self, n, dtype, fill=None):
        self.nbytes = int(n) * torch.empty((), dtype=dtype).element_size()
        self.raw = torch.full((GUARD + self.nbytes + GUARD,), CANARY, dtype=torch.uint8, device=DEV)
        self.t = self.raw[GUARD:GUARD + self.nbytes].view(dtype)
        if fill is not None:
            self.t.fill_(fill)

    def intact(self):
        front = bool((self.raw[:GUARD] == CANARY).all())
        back = bool((self.raw[GUARD + self.nbytes:] == CANARY).all())
        return front and back


class GuardedStep:
    """Every buffer of one denoising-step tail behind guard bytes, exactly as large as the entry points ask."""

    def __init__(self, T, d, V, max_rows, sampling, budget_bytes=0, plan_edit=None):
        self.plan = binding.mosaic_plan_workspace(T, max_rows, d, V, budget_bytes, sampling=sampling)
        if plan_edit is not None:
            plan_edit(self.plan)
            per = 20 if sampling else 12
            self.plan.workspace_bytes = per * self.plan.rows_per_chunk * self.plan.vocab_splits + binding.SYNC_BYTES
        self.max_rows = max_rows
        self.idx = Guarded(max(T, 1), torch.int32, -7)
        self.count = Guarded(1, torch.int32, 0)
        self.scratch = Guarded(binding.mosaic_compact_scratch_bytes(T), torch.uint8)
        self.workspace = Guarded(max(self.plan.workspace_bytes, 16), torch.uint8)
        self.token = Guarded(max(max_rows, 1), torch.int32, -7)
        self.conf = Guarded(max(max_rows, 1), torch.float32, -7.0)
        self.lse = Guarded(max(max_rows, 1), torch.float32, -7.0)
        self.gather = Guarded(max(max_rows, 1), torch.int32, -7)
        self.tokens = Guarded(max(T, 1), torch.int32, -1)
        self.all = [self.idx, self.count, self.scratch, self.workspace, self.token, self.conf, self.lse, self.gather,
                    self.tokens]

    def assert_intact(self, what):
        torch.cuda.synchronize()
        for name in ("idx", "count", "scratch", "workspace", "token", "conf", "lse", "gather", "tokens"):
            assert getattr(self, name).intact(), f"{what}: bytes around `{name}` were overwritten"


GUARD_SHAPES = [
    # T, d, V, p, what
    (300, 64, 256, 1.0, "4-wave kernel, one ragged row tile"),
    (1000, 128, 1280, 0.7, "4-wave kernel, several row tiles"),
    (700, 192, 777, 0.6, "general kernel, ragged vocabulary below one tile pair"),
    (900, 128, 1000, 0.9, "paired launch: 4-wave kernel + general kernel on the ragged last tile"),
    (70000, 64, 512, 0.03, "three-launch compaction (T > 65536)"),
    (513, 64, 512, 0.0, "empty mask"),
]


@pytest.mark.parametrize("T,d,V,p,what", GUARD_SHAPES)
@pytest.mark.parametrize("sampling", [False, True])
def test_no_entry_point_writes_outside_its_buffers(T, d, V, p, what, sampling):
    print(f"guard bytes: {what}, sampling={sampling}", flush=True)
    wl = workloads.small_random(T, d, V, p=p, seed=T + V, device=DEV)
    M = wl.M
    mask = Guarded(T, torch.uint8)
    mask.t.copy_(wl.mask)
    for chunks in (1, 3):
        def edit(plan, chunks=chunks):
            if chunks > 1 and plan.rows_per_chunk > 256:
                tiles = plan.rows_per_chunk // 256
                plan.rows_per_chunk = 256 * -(-tiles // chunks)
                plan.num_chunks = -(-max(M, 1) // plan.rows_per_chunk)
        g = GuardedStep(T, d, V, M, sampling, plan_edit=edit)
        binding.mosaic_mask_compact(mask.t, g.idx.t, g.count.t, g.scratch.t)
        g.assert_intact(what + ": compact")
        assert int(g.count.t.item()) == M
        seq_starts = torch.tensor([0, T // 3, T], dtype=torch.int32, device=DEV)
        binding.mosaic_shift_indices(g.idx.t, g.count.t, g.max_rows, seq_starts, g.gather.t)
        g.assert_intact(what + ": shift")
        if sampling:
            binding.mosaic_masked_logits_sample(wl.hidden, wl.w, g.gather.t, g.count.t, g.max_rows, 0.8, 99, g.token.t,
                                                g.conf.t, g.lse.t, g.plan, g.workspace.t, noise_idx=g.idx.t)
        else:
            binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, g.idx.t, g.count.t, g.max_rows, g.token.t, g.conf.t,
                                                g.lse.t, g.plan, g.workspace.t)
        g.assert_intact(what + f": fused pass, {g.plan.num_chunks} chunk(s)")
        assert bool((g.token.t[M:] == -7).all()) and bool((g.lse.t[M:] == -7.0).all())
        assert M == 0 or bool(((g.token.t[:M] >= 0) & (g.token.t[:M] < V)).all())
        n_per_seq = torch.tensor([5, 1 << 20], dtype=torch.int32, device=DEV)
        binding.mosaic_unmask_topn(g.conf.t, g.token.t, g.idx.t, g.count.t, g.max_rows, seq_starts, n_per_seq,
                                   g.tokens.t, mask.t)
        g.assert_intact(what + ": unmask")
        assert mask.intact()
        mask.t.copy_(wl.mask)


@pytest.mark.parametrize("V", [1024, 777])
def test_gather_entries_outside_the_tensor_are_clamped(V):
    """A caller-built gather list with entries outside [0, T): the rows read are 0 and T - 1, nothing else."""
    print(f"clamp V={V}", flush=True)
    T, d = 400, 128
    wl = workloads.small_random(T, d, V, p=1.0, seed=V, device=DEV)
    bad = np.array([-1, -(2 ** 31), T, T + 12345, 2 ** 31 - 1, 7, 0, T - 1], np.int32)
    expect_row = np.array([0, 0, T - 1, T - 1, T - 1, 7, 0, T - 1])
    n = bad.size
    idx = torch.as_tensor(bad, device=DEV)
    count = torch.tensor([n], dtype=torch.int32, device=DEV)
    plan = binding.mosaic_plan_workspace(T, n, d, V, sampling=True)
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=DEV)
    tok = torch.empty(n, dtype=torch.int32, device=DEV)
    conf = torch.empty(n, dtype=torch.float32, device=DEV)
    lse = torch.empty(n, dtype=torch.float32, device=DEV)
    binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, idx, count, n, tok, conf, lse, plan, ws)
    torch.cuda.synchronize()
    want, logits = oracle.positions(workloads.bf16_bits(wl.hidden), workloads.bf16_bits(wl.w), expect_row,
                                    return_logits=True)
    check_against_oracle(dict(tok=tok.cpu().numpy(), conf=conf.cpu().numpy(), lse=lse.cpu().numpy()), want, logits,
                         what="clamped gather")
    # sampling: the row read is clamped, the noise is keyed by the entry as given
    binding.mosaic_masked_logits_sample(wl.hidden, wl.w, idx, count, n, 0.7, 5, tok, conf, lse, plan, ws)
    torch.cuda.synchronize()
    got = tok.cpu().numpy()
    for j in range(n):
        tok_o, _, lse_o, gap_o = oracle.row_sample(logits[j], 0.7, 5, int(bad[j]))
        assert abs(float(lse[j]) - lse_o) <= 2e-3
        if gap_o > 2e-3:
            assert int(got[j]) == tok_o, (j, int(bad[j]))
    # the index helpers: the shift never emits an entry outside [0, T); unmasking skips such rows
    seq_starts = torch.tensor([0, T], dtype=torch.int32, device=DEV)
    gather = torch.full((n,), -7, dtype=torch.int32, device=DEV)
    binding.mosaic_shift_indices(idx, count, n, seq_starts, gather)
    torch.cuda.synchronize()
    g = gather.cpu().numpy()
    assert g.min() >= 0 and g.max() <= T - 1 and list(g[5:]) == [6, 0, T - 2]
    tokens = torch.full((T,), -1, dtype=torch.int32, device=DEV)
    mask = torch.ones(T, dtype=torch.uint8, device=DEV)
    srt = torch.as_tensor(np.sort(bad), device=DEV)               # the selection expects ascending entries
    cf = torch.linspace(0.1, 0.9, n, device=DEV)
    binding.mosaic_unmask_topn(cf, tok, srt, count, n, seq_starts, torch.tensor([n], dtype=torch.int32, device=DEV),
                               tokens, mask)
    torch.cuda.synchronize()
    written = np.nonzero(tokens.cpu().numpy() != -1)[0]
    assert set(written) == {0, 7, T - 1} and int(mask.sum().item()) == T - 3
    # an unsorted list (outside the contract) can bring an out-of-range entry into a sequence's span: it is skipped
    tokens.fill_(-1)
    mask.fill_(1)
    messy = torch.tensor([0, 2 ** 31 - 1, 7, T - 1], dtype=torch.int32, device=DEV)
    four = torch.tensor([4], dtype=torch.int32, device=DEV)
    binding.mosaic_unmask_topn(cf[:4].contiguous(), tok[:4].contiguous(), messy, four, 4, seq_starts, four, tokens, mask)
    torch.cuda.synchronize()
    assert set(np.nonzero(tokens.cpu().numpy() != -1)[0]) == {0, 7, T - 1} and int(mask.sum().item()) == T - 3


@pytest.mark.parametrize("V,kernel", [(1024, "4-wave"), (777, "general")])
def test_shifted_gather_draws_are_keyed_by_the_predicted_position(V, kernel):
    """Dream-style shifted prediction: a sequence start s and s + 1 both read hidden row s.  With noise_idx = the
    positions themselves their draws are independent (and equal the oracle's draw for each position); keyed by the
    row read they would always coincide."""
    print(f"noise_idx {kernel}", flush=True)
    T, d, n_seq, tau, seed = 1024, 128, 64, 1.0, 0xDEC0DE
    wl = workloads.small_random(T, d, V, p=1.0, seed=31 + V, device=DEV)
    starts = np.arange(0, T + 1, T // n_seq).astype(np.int32)
    seq_starts = torch.as_tensor(starts, device=DEV)
    op = binding.MaskOnlyLogits(T, d, V, device=DEV, sampling=True)
    binding.mosaic_mask_compact(wl.mask, op.idx, op.count, op.scratch)
    gather = torch.empty_like(op.idx)
    binding.mosaic_shift_indices(op.idx, op.count, op.max_rows, seq_starts, gather)
    binding.mosaic_masked_logits_sample(wl.hidden, wl.w, gather, op.count, op.max_rows, tau, seed, op.token, op.conf,
                                        op.lse, op.plan, op.workspace, noise_idx=op.idx)
    torch.cuda.synchronize()
    tok = op.token.cpu().numpy()
    rows_read = gather.cpu().numpy()
    assert np.array_equal(rows_read, oracle.shift_indices(np.arange(T, dtype=np.int32), starts))
    hb, wb = workloads.bf16_bits(wl.hidden), workloads.bf16_bits(wl.w)
    strict = same = 0
    for s in starts[:-1]:
        x = oracle.row_logits(hb[s], wb)                         # both positions read row s
        for p in (int(s), int(s) + 1):
            assert rows_read[p] == s
            tok_o, conf_o, lse_o, gap_o = oracle.row_sample(x, tau, seed, p)    # noise of the PREDICTED position
            assert abs(float(op.lse[p]) - lse_o) <= 2e-3
            if gap_o > 2e-3:
                strict += 1
                assert int(tok[p]) == tok_o, (p, int(tok[p]), tok_o)
                assert abs(float(op.conf[p]) - conf_o) <= 2e-3
        same += int(tok[s] == tok[s + 1])
    assert strict >= 0.9 * 2 * n_seq
    # identical logits, independent noise: P(same token) = sum_v softmax(x)_v^2, a few percent for these rows
    assert same <= n_seq // 4, same
    # without noise_idx the noise follows the row that is read and the two positions always coincide
    binding.mosaic_masked_logits_sample(wl.hidden, wl.w, gather, op.count, op.max_rows, tau, seed, op.token, op.conf,
                                        op.lse, op.plan, op.workspace)
    torch.cuda.synchronize()
    tok2 = op.token.cpu().numpy()
    assert all(tok2[s] == tok2[s + 1] for s in starts[:-1])


def test_budget_bounds_the_sampling_workspace_on_the_device():
    """A byte budget with sampling on: what is allocated stays within it, chunks are forced, results match the
    oracle and the unbounded run."""
    print("sampling budget", flush=True)
    T, d, V, tau, seed = 3000, 128, 2048, 0.9, 77
    wl = workloads.small_random(T, d, V, p=1.0, seed=4, device=DEV)
    budget = 20 * 256 * 3 + binding.SYNC_BYTES + 100           # one row tile x 3 splits x 20 bytes, the counters, a bit
    free = binding.MaskOnlyLogits(T, d, V, device=DEV, sampling=True)
    tight = binding.MaskOnlyLogits(T, d, V, device=DEV, sampling=True, budget_bytes=budget)
    assert free.plan.num_chunks == 1
    assert tight.workspace.numel() <= budget and tight.plan.workspace_bytes <= budget
    assert tight.plan.num_chunks == 4 and tight.plan.rows_per_chunk == 768 and tight.plan.vocab_splits == 1
    # the greedy selector would have cut fewer chunks under this budget: 20 bytes per partial is what binds here
    assert binding.mosaic_plan_workspace(T, T, d, V, budget).num_chunks < tight.plan.num_chunks
    outs = []
    for op in (free, tight):
        op.token.fill_(-7)
        op.sample_step(wl.hidden, wl.w, wl.mask, tau, seed)
        torch.cuda.synchronize()
        outs.append((op.token.cpu().numpy(), op.conf.cpu().numpy(), op.lse.cpu().numpy()))
    hb, wb = workloads.bf16_bits(wl.hidden), workloads.bf16_bits(wl.w)
    rows = np.unique(np.concatenate([np.arange(0, T, 37), np.arange(760, 776), np.arange(T - 8, T)]))
    strict = 0
    for p in rows:
        x = oracle.row_logits(hb[p], wb)
        tok_o, conf_o, lse_o, gap_o = oracle.row_sample(x, tau, seed, int(p))
        for tok, conf, lse in outs:
            assert abs(float(lse[p]) - lse_o) <= 2e-3
            if gap_o > 2e-3:
                assert int(tok[p]) == tok_o and abs(float(conf[p]) - conf_o) <= 2e-3
        strict += int(gap_o > 2e-3)
    assert strict >= 0.9 * rows.size
    assert np.array_equal(outs[0][0], outs[1][0])                # same draws whatever the chunking
