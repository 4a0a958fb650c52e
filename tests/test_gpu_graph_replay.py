"""A whole denoising step (compaction, fused logits reduction, top-n unmasking) captured once into a HIP graph
and replayed: the masked-row count never visits the host, so the same graph serves every step of the loop while
the mask shrinks.  Each replay is checked against the eager loop, with eager work and synchronisations between
replays."""
import numpy as np
import pytest
import torch

from paper_2601_06562_amd import binding, workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def one_step(op, wl, mask, tokens, seq_starts, n_per_seq):
    op.step(wl.hidden, wl.w, mask)
    binding.mosaic_unmask_topn(op.conf, op.token, op.idx, op.count, op.max_rows, seq_starts, n_per_seq, tokens, mask)


@pytest.mark.parametrize("T,d,V", [(1500, 128, 2048), (900, 192, 777)])      # 4-wave kernel and general kernel
def test_denoising_loop_as_a_replayed_graph(T, d, V):
    print(f"graph replay T={T} d={d} V={V}", flush=True)
    wl = workloads.small_random(T, d, V, p=1.0, seed=77, device=DEV)
    seq_starts = torch.tensor([0, T // 3, T], dtype=torch.int32, device=DEV)
    n_per_seq = torch.tensor([T // 30, T // 12], dtype=torch.int32, device=DEV)
    steps = 6
    # eager loop
    op = binding.MaskOnlyLogits(T, d, V, device=DEV)
    mask = wl.mask.clone()
    tokens = torch.full((T,), -1, dtype=torch.int32, device=DEV)
    eager = []
    for _ in range(steps):
        one_step(op, wl, mask, tokens, seq_starts, n_per_seq)
        torch.cuda.synchronize()
        eager.append((mask.cpu().numpy().copy(), tokens.cpu().numpy().copy(), int(op.count.item())))
    per_step = T // 30 + T // 12
    assert [e[2] for e in eager] == [T - k * per_step for k in range(steps)]      # the count really changes per step
    # the same loop as one captured step, replayed
    gop = binding.MaskOnlyLogits(T, d, V, device=DEV)
    gmask = wl.mask.clone()
    gtokens = torch.full((T,), -1, dtype=torch.int32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up on the capture stream's side, then restore the state
        one_step(gop, wl, gmask, gtokens, seq_starts, n_per_seq)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gmask.copy_(wl.mask)
    gtokens.fill_(-1)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_step(gop, wl, gmask, gtokens, seq_starts, n_per_seq)
    torch.cuda.synchronize()
    gmask.copy_(wl.mask)                                # capture does not run the work, but start from a known state
    gtokens.fill_(-1)
    scratch = torch.zeros(1 << 16, device=DEV)
    for k in range(steps):
        graph.replay()
        torch.cuda.synchronize()
        scratch.add_(1.0)                               # eager work of the program's own between the replays
        assert float(scratch.sum().item()) == (k + 1) * (1 << 16)
        want_mask, want_tokens, want_count = eager[k]
        assert int(gop.count.item()) == want_count, k
        assert np.array_equal(gmask.cpu().numpy(), want_mask), k
        assert np.array_equal(gtokens.cpu().numpy(), want_tokens), k
