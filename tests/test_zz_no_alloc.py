"""mosaic_masked_logits_reduce_static (the entry point for callers that cannot allocate: partial results go to a
fixed array inside the library) against mosaic_masked_logits_reduce on a caller's workspace: bit-identical
outputs, on two calls in a row, the second with a smaller input, and on a plan that the selector cut down to fit
the array.  Through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2601_06562_amd import binding, workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def warm_up():
    """The first call on a device looks the array's address up, which makes the runtime materialise the library's
    device image (the array included): done once, before anything is measured."""
    wl = workloads.small_random(300, 64, 256, p=1.0, seed=9, device=DEV)
    op = binding.MaskOnlyLogits(300, 64, 256, device=DEV)
    binding.mosaic_mask_compact(wl.mask, op.idx, op.count, op.scratch)
    binding.mosaic_masked_logits_reduce_static(wl.hidden, wl.w, op.idx, op.count, op.max_rows, op.token, op.conf,
                                               op.lse, op.plan)
    torch.cuda.synchronize()


def both(T, d, V, p, seed, budget=0):
    warm_up()
    wl = workloads.small_random(T, d, V, p=p, seed=seed, device=DEV)
    op = binding.MaskOnlyLogits(T, d, V, max_rows=wl.M, budget_bytes=budget, device=DEV)
    op.step(wl.hidden, wl.w, wl.mask)
    torch.cuda.synchronize()
    M = int(op.count.item())
    ref = (op.token[:M].cpu().numpy().copy(), op.conf[:M].cpu().numpy().copy(), op.lse[:M].cpu().numpy().copy())
    tok = torch.full_like(op.token, -7)
    conf = torch.full_like(op.conf, -7.0)
    lse = torch.full_like(op.lse, -7.0)
    free0 = torch.cuda.mem_get_info()[0]
    binding.mosaic_masked_logits_reduce_static(wl.hidden, wl.w, op.idx, op.count, op.max_rows, tok, conf, lse, op.plan)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0                  # nothing was allocated on the device
    got = (tok[:M].cpu().numpy(), conf[:M].cpu().numpy(), lse[:M].cpu().numpy())
    for a, b, name in zip(ref, got, ("token", "conf", "lse")):
        assert np.array_equal(a, b), (name, T, d, V)
    assert bool((tok[M:] == -7).all()) and bool((lse[M:] == -7.0).all())
    return M, op.plan


def test_static_workspace_matches_the_callers_workspace_on_consecutive_calls():
    print("static workspace: large then small", flush=True)
    M1, plan1 = both(5000, 256, 4096, 0.9, seed=1)               # 18 row tiles
    M2, plan2 = both(700, 128, 1280, 0.5, seed=2)                # a smaller input on the array the first call used
    assert M2 < M1 and plan2.workspace_bytes < plan1.workspace_bytes
    both(300, 64, 777, 1.0, seed=3)                              # general kernel (ragged vocabulary)
    both(0 + 513, 64, 512, 0.0, seed=4)                          # empty mask: nothing runs


def test_static_workspace_with_a_plan_cut_down_to_fit_the_array():
    print("static workspace: budgeted plan", flush=True)
    T, d, V = 60000, 64, 65536                                   # unbounded: 235 row tiles x 8 splits > 4 MiB
    free = binding.mosaic_plan_workspace(T, T, d, V, 0)
    assert free.workspace_bytes > binding.STATIC_WORKSPACE_BYTES
    wl = workloads.small_random(T, d, V, p=1.0, seed=5, device=DEV)
    tok = torch.empty(T, dtype=torch.int32, device=DEV)
    conf = torch.empty(T, dtype=torch.float32, device=DEV)
    lse = torch.empty(T, dtype=torch.float32, device=DEV)
    idx = torch.arange(T, dtype=torch.int32, device=DEV)
    count = torch.tensor([T], dtype=torch.int32, device=DEV)
    with pytest.raises(binding.MosaicError) as e:
        binding.mosaic_masked_logits_reduce_static(wl.hidden, wl.w, idx, count, T, tok, conf, lse, free)
    assert e.value.status == binding.MOSAIC_ERR_WORKSPACE_TOO_SMALL
    M, plan = both(T, d, V, 1.0, seed=5, budget=binding.STATIC_WORKSPACE_BYTES)
    assert plan.workspace_bytes <= binding.STATIC_WORKSPACE_BYTES and M == T
