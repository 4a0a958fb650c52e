"""Full-size parity on the five benchmark workloads, in the launch configuration bench.py times:
sampled rows against the oracle (rows are independent, so a sample is the restriction of the full
oracle), plus properties that hold on every row."""
import math

import numpy as np
import pytest
import torch

from paper_2601_06562_amd import workloads

from gpu_helpers import check_against_oracle, oracle_rows, run_hip

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SAMPLE = 96


def sample_rows(M, rng, tile=256, extra=()):
    """Stratified sample of compacted row numbers: ends, tile boundaries, then random."""
    picks = {0, M - 1, *[e for e in extra if 0 <= e < M]}
    for b in range(tile, M, tile):
        if len(picks) < SAMPLE // 2:
            picks.update({b - 1, b})
    while len(picks) < min(SAMPLE, M):
        picks.add(int(rng.integers(0, M)))
    return np.array(sorted(picks), dtype=np.int64)


@pytest.mark.parametrize("name", ["llada_first_step", "long_semi_ar", "dream_late_step", "batched_mixed"])
def test_full_size_workload(name):
    print(f"full-size {name}: generating", flush=True)
    wl = workloads.make(name, device=DEV)
    M_true = wl.M
    print(f"full-size {name}: T={wl.T} d={wl.d} V={wl.V} M={M_true}; HIP path", flush=True)
    out = run_hip(wl.hidden, wl.w, wl.mask, max_rows=M_true)
    M = out["M"]
    assert M == M_true
    # compaction: bit-exact against the definition (ascending positions with a nonzero byte)
    want_idx = torch.nonzero(wl.mask.cpu(), as_tuple=False).flatten().numpy().astype(np.int32)
    assert np.array_equal(out["idx"][:M], want_idx)
    tok, conf, lse = out["tok"][:M], out["conf"][:M], out["lse"][:M]
    # whole-output properties
    assert np.all(np.isfinite(lse)) and np.all((conf > 0) & (conf <= 1.0 + 1e-6))
    assert np.all((tok >= 0) & (tok < wl.V))
    implied_max = lse + np.log(conf)
    assert np.all(implied_max > 1.0) and np.all(implied_max < 16.0)      # ~ sigma * sqrt(2 ln V), sigma in [0.5, 2]
    assert abs(float(np.mean(lse)) - (math.log(wl.V) + (0.5 if name != "batched_mixed" else 0.875))) < 0.2
    plan = out["op"].plan
    assert out["op"].workspace_bytes < 4 * M * wl.V / 50                 # nowhere near an [M,V] fp32 tensor
    print(f"full-size {name}: plan {plan}; oracle on {SAMPLE} rows", flush=True)
    rng = np.random.default_rng(11)
    extra = []
    if name == "batched_mixed":                                          # rows of every sequence, incl. the 2% one
        bounds = np.searchsorted(want_idx, np.arange(0, wl.T + 1, 16384))
        for b in range(8):
            extra += [int(bounds[b]), int(bounds[b + 1]) - 1, int((bounds[b] + bounds[b + 1]) // 2)]
    rows = sample_rows(M, rng, extra=extra)
    w_bits = workloads.bf16_bits(wl.w)
    want, logits = oracle_rows(wl.hidden, w_bits, want_idx[rows], return_logits=True)
    stats = check_against_oracle(dict(tok=tok[rows], conf=conf[rows], lse=lse[rows]), want, logits, what=name)
    print(f"full-size {name}: {stats}", flush=True)
    # "select": an unmasked position's row, computed by forcing it into a second mask, matches the oracle too
    if M < wl.T:
        unmasked = torch.nonzero(wl.mask == 0).flatten()[:8]
        m2 = torch.zeros_like(wl.mask)
        m2[unmasked] = 1
        out2 = run_hip(wl.hidden, wl.w, m2, max_rows=8)
        want2 = oracle_rows(wl.hidden, w_bits, unmasked.cpu().numpy())
        check_against_oracle(dict(tok=out2["tok"][:8], conf=out2["conf"][:8], lse=out2["lse"][:8]), want2,
                             what=name + " unmasked rows")


def span_flag(op):
    """The word the device-side span check leaves behind the round counters: 1 if some 64 consecutive rows of the
    list lay 4 GiB or more apart (the general kernel then did the work), 0 if the 4-wave kernel did."""
    return int(op.workspace[op.plan.workspace_bytes - 4:op.plan.workspace_bytes].view(torch.int32).item())


def test_hidden_tensor_beyond_4_gib():
    """A hidden tensor larger than 4 GiB, where a 32-bit byte offset from the start of the tensor wraps.  The 4-wave
    kernel addresses a wave's 64 rows from the lowest of them, so it serves such a tensor as long as no 64 consecutive
    rows of the list lie 4 GiB apart (decided on the device); a list with such a gap goes to the general kernel,
    which addresses rows with 64-bit pointers.  Both lists here, greedy and sampled, against the oracle."""
    import oracle
    from paper_2601_06562_amd import binding
    T, d, V = (1 << 19) + 4096, 4096, 1024                  # 4.03 GiB of bf16 hidden states
    print(f"beyond-4GiB hidden: T={T} d={d} V={V}", flush=True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(workloads.BASE_SEED + 77)
    hidden = workloads._normal_bf16(T, d, 1.0, gen, torch.device(DEV))
    w = workloads._normal_bf16(V, d, d ** -0.5, gen, torch.device(DEV))
    w_bits = workloads.bf16_bits(w)
    name = binding.mosaic_masked_logits_kernel_name(T, d, d, V, binding.mosaic_plan_workspace(T, 512, d, V), False)
    assert "masked_logits_kernel_w4<false>" in name and "masked_logits_kernel<3,2,false>" in name
    far = torch.cat([torch.arange(5, 40, 7), torch.arange((1 << 19) - 3, (1 << 19) + 300, 1), torch.tensor([T - 1])])
    near = torch.cat([torch.arange((1 << 19) - 350, (1 << 19) + 350, 1), torch.arange(T - 300, T, 1)])
    for what, pos, flag in (("a gap of 4 GiB inside one group of rows", far, 1), ("rows close together", near, 0)):
        print(f"beyond-4GiB hidden: {what}", flush=True)
        mask = torch.zeros(T, dtype=torch.uint8, device=DEV)
        mask[pos.to(DEV)] = 1
        assert int(pos.max()) * d * 2 > (1 << 32)
        out = run_hip(hidden, w, mask, max_rows=int(pos.numel()))
        M = out["M"]
        assert M == pos.numel() and np.array_equal(out["idx"][:M], np.sort(pos.numpy()).astype(np.int32))
        assert span_flag(out["op"]) == flag
        rows = np.arange(M) if M <= 320 else np.unique(np.concatenate([np.arange(0, M, 5), np.arange(690, 720)]))
        want = oracle_rows(hidden, w_bits, out["idx"][rows])
        stats = check_against_oracle(dict(tok=out["tok"][rows], conf=out["conf"][rows], lse=out["lse"][rows]), want,
                                     what="beyond 4 GiB, " + what)
        print(stats, flush=True)
        # the same list under sampling
        tau, seed = 0.9, 4321
        op = binding.MaskOnlyLogits(T, d, V, max_rows=M, device=DEV, sampling=True)
        op.sample_step(hidden, w, mask, tau, seed)
        torch.cuda.synchronize()
        assert span_flag(op) == flag
        tok, lse = op.token.cpu().numpy(), op.lse.cpu().numpy()
        strict = 0
        for j in rows[::4]:
            x = oracle.row_logits(workloads.bf16_bits(hidden[int(out["idx"][j])]), w_bits)
            tok_o, conf_o, lse_o, gap_o = oracle.row_sample(x, tau, seed, int(out["idx"][j]))
            assert abs(float(lse[j]) - lse_o) <= 2e-3
            if gap_o > 1e-3 * (1 + tau):
                strict += 1
                assert int(tok[j]) == tok_o, (what, j, int(tok[j]), tok_o, gap_o)
        assert strict >= 0.8 * len(rows[::4])
    del hidden
    torch.cuda.empty_cache()


def test_hidden_tensor_between_2_and_4_gib_on_the_fast_path():
    """Rows whose 32-bit byte offset has its top bit set: the 4-wave kernel adds the per-lane offset to a 64-bit
    base as an unsigned value (the documented behaviour of the scalar-base addressing form), so a hidden tensor
    of up to 4 GiB stays on the fast path."""
    T, d, V = 400000, 4096, 1024                            # 3.05 GiB of bf16 hidden states, V a multiple of 256
    print(f"2-4 GiB hidden: T={T} d={d} V={V}", flush=True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(workloads.BASE_SEED + 78)
    hidden = workloads._normal_bf16(T, d, 1.0, gen, torch.device(DEV))
    w = workloads._normal_bf16(V, d, d ** -0.5, gen, torch.device(DEV))
    mask = torch.zeros(T, dtype=torch.uint8, device=DEV)
    pos = torch.cat([torch.arange(3, 30, 9), torch.arange((1 << 18) - 2, (1 << 18) + 400, 1), torch.tensor([T - 1])])
    mask[pos.to(DEV)] = 1
    assert (1 << 31) < int(pos.max()) * d * 2 < (1 << 32)
    out = run_hip(hidden, w, mask, max_rows=int(pos.numel()))
    assert not (out["op"].plan.flags & 1)
    M = out["M"]
    assert M == pos.numel()
    want = oracle_rows(hidden, workloads.bf16_bits(w), out["idx"][:M])
    stats = check_against_oracle(dict(tok=out["tok"][:M], conf=out["conf"][:M], lse=out["lse"][:M]), want,
                                 what="2-4 GiB")
    print(stats, flush=True)
    del hidden
    torch.cuda.empty_cache()


def test_dream_shape_shifted_prediction_and_sampling():
    """The Dream-shaped workload end to end as Dream decodes: positions predicted from the hidden row before them
    (compact -> shifted gather list -> fused pass), greedy and with temperature sampling, on sampled rows."""
    import oracle
    from paper_2601_06562_amd import binding
    name = "dream_late_step"
    print(f"{name}: shifted + sampling, generating", flush=True)
    wl = workloads.make(name, device=DEV)
    M = wl.M
    seq_starts = torch.tensor([0, wl.T], dtype=torch.int32, device=DEV)
    op = binding.MaskOnlyLogits(wl.T, wl.d, wl.V, max_rows=M, device=DEV, sampling=True)
    binding.mosaic_mask_compact(wl.mask, op.idx, op.count, op.scratch)
    gather = torch.empty_like(op.idx)
    binding.mosaic_shift_indices(op.idx, op.count, op.max_rows, seq_starts, gather)
    binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, gather, op.count, op.max_rows, op.token, op.conf, op.lse,
                                        op.plan, op.workspace)
    torch.cuda.synchronize()
    assert int(op.count.item()) == M
    idx = op.idx[:M].cpu().numpy()
    rows_read = gather[:M].cpu().numpy()
    assert np.array_equal(rows_read, oracle.shift_indices(idx, np.array([0, wl.T], np.int32)))
    rng = np.random.default_rng(23)
    rows = sample_rows(M, rng)
    w_bits = workloads.bf16_bits(wl.w)
    want, logits = oracle_rows(wl.hidden, w_bits, rows_read[rows], return_logits=True)
    stats = check_against_oracle(dict(tok=op.token[:M].cpu().numpy()[rows], conf=op.conf[:M].cpu().numpy()[rows],
                                      lse=op.lse[:M].cpu().numpy()[rows]), want, logits, what=name + " shifted")
    print(f"{name} shifted: {stats}", flush=True)
    # the same gather list under sampling: the noise is keyed by the position that is PREDICTED (noise_idx)
    tau, seed = 0.7, 20260107
    binding.mosaic_masked_logits_sample(wl.hidden, wl.w, gather, op.count, op.max_rows, tau, seed, op.token, op.conf,
                                        op.lse, op.plan, op.workspace, noise_idx=op.idx)
    torch.cuda.synchronize()
    tok, conf, lse = op.token[:M].cpu().numpy(), op.conf[:M].cpu().numpy(), op.lse[:M].cpu().numpy()
    strict = 0
    for k, j in enumerate(rows):
        x = logits[k]
        tok_o, conf_o, lse_o, gap_o = oracle.row_sample(x, tau, seed, int(idx[j]))
        assert abs(float(lse[j]) - lse_o) <= 2e-3
        if gap_o > 1e-3 * (1 + tau):
            strict += 1
            assert int(tok[j]) == tok_o, (j, int(tok[j]), tok_o, gap_o)
            assert abs(float(conf[j]) - conf_o) <= 2e-3 and abs(float(conf[j]) - conf_o) <= 5e-3 * max(conf_o, 1e-30)
    assert strict >= 0.9 * len(rows)
    print(f"{name} shifted + sampling: {strict} strict rows of {len(rows)}", flush=True)


def test_batched_workload_under_sampling_in_several_rounds():
    """The batched workload under sampling: 229 row tiles, every workgroup takes 17 units one after the other (the
    running best, the bound on the generator's words and the candidate queues start afresh in each), rows of every
    sequence checked against the oracle's draw."""
    import oracle
    from paper_2601_06562_amd import binding
    name = "batched_mixed"
    print(f"{name}: sampling, generating", flush=True)
    wl = workloads.make(name, device=DEV)
    M = wl.M
    op = binding.MaskOnlyLogits(wl.T, wl.d, wl.V, max_rows=M, device=DEV, sampling=True)
    assert ((M + 255) // 256) * op.plan.vocab_splits > 4 * op.plan.grid
    tau, seed = 1.0, 0xABCDEF0123
    op.sample_step(wl.hidden, wl.w, wl.mask, tau, seed)
    torch.cuda.synchronize()
    assert int(op.count.item()) == M
    idx = op.idx[:M].cpu().numpy()
    tok, conf, lse = op.token[:M].cpu().numpy(), op.conf[:M].cpu().numpy(), op.lse[:M].cpu().numpy()
    assert np.all((tok >= 0) & (tok < wl.V)) and np.all(np.isfinite(lse)) and np.all((conf > 0) & (conf <= 1.0 + 1e-6))
    bounds = np.searchsorted(idx, np.arange(0, wl.T + 1, 16384))
    extra = []
    for b in range(8):
        extra += [int(bounds[b]), int(bounds[b + 1]) - 1, int((bounds[b] + bounds[b + 1]) // 2)]
    rows = sample_rows(M, np.random.default_rng(29), extra=extra)
    want, logits = oracle_rows(wl.hidden, workloads.bf16_bits(wl.w), idx[rows], return_logits=True)
    strict = 0
    for k, j in enumerate(rows):
        tok_o, conf_o, lse_o, gap_o = oracle.row_sample(logits[k], tau, seed, int(idx[j]))
        assert abs(float(lse[j]) - lse_o) <= 2e-3
        if gap_o > 1e-3 * (1 + tau):
            strict += 1
            assert int(tok[j]) == tok_o, (j, int(tok[j]), tok_o, gap_o)
            assert abs(float(conf[j]) - conf_o) <= 2e-3 and abs(float(conf[j]) - conf_o) <= 5e-3 * max(conf_o, 1e-30)
    assert strict >= 0.9 * len(rows)
    print(f"{name} sampling: {strict} strict rows of {len(rows)}", flush=True)
