"""The VMM workspace on the GPU: the mapped prefix follows resize, the pointer never moves, memory is really
taken and given back, and the fused kernel produces bit-identical results on it."""
import numpy as np
import pytest
import torch

from paper_2601_06562_amd import binding, workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_vmm_workspace_grows_shrinks_and_serves_the_kernel():
    print("vmm workspace", flush=True)
    torch.cuda.set_device(0)
    torch.zeros(1, device=DEV)                              # context up
    try:
        ws = binding.VmmWorkspace(1 << 30, device=0)
    except binding.MosaicError as e:
        if e.status == binding.MOSAIC_ERR_UNSUPPORTED_SHAPE:
            pytest.skip("this device reports no virtual memory management")
        raise
    g = ws.granularity
    assert g > 0 and ws.reserved_bytes == -(-(1 << 30) // g) * g and ws.committed_bytes == 0
    base = ws.ptr
    assert base != 0 and base % g == 0
    free0, _ = torch.cuda.mem_get_info(0)
    assert free0 > (1 << 30)                                # reserving addresses took no memory worth noticing

    wl = workloads.small_random(1500, 256, 2048, p=0.9, seed=21, device=DEV)
    ref = binding.MaskOnlyLogits(wl.T, wl.d, wl.V, device=DEV)
    ref.step(wl.hidden, wl.w, wl.mask)
    torch.cuda.synchronize()
    M = int(ref.count.item())

    ws.resize(ref.plan.workspace_bytes)
    assert ws.ptr == base and ws.committed_bytes == -(-ref.plan.workspace_bytes // g) * g
    out = binding.MaskOnlyLogits(wl.T, wl.d, wl.V, device=DEV)
    binding.mosaic_mask_compact(wl.mask, out.idx, out.count, out.scratch)
    binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, out.idx, out.count, out.max_rows, out.token, out.conf, out.lse,
                                        out.plan, ws)
    torch.cuda.synchronize()
    assert torch.equal(out.token[:M], ref.token[:M])
    assert torch.equal(out.lse[:M], ref.lse[:M]) and torch.equal(out.conf[:M], ref.conf[:M])

    # grow by 64 MiB: more memory is held, the pointer stays; then the sampling variant with its larger workspace
    torch.cuda.synchronize()
    before, _ = torch.cuda.mem_get_info(0)
    ws.resize(64 << 20)
    after, _ = torch.cuda.mem_get_info(0)
    assert ws.ptr == base and ws.committed_bytes == -(-(64 << 20) // g) * g
    assert before - after >= (48 << 20)
    samp = binding.MaskOnlyLogits(wl.T, wl.d, wl.V, device=DEV, sampling=True)
    samp.sample_step(wl.hidden, wl.w, wl.mask, 1.0, 7)
    binding.mosaic_masked_logits_sample(wl.hidden, wl.w, out.idx, out.count, out.max_rows, 1.0, 7, out.token, out.conf,
                                        out.lse, out.plan, ws)
    torch.cuda.synchronize()
    assert torch.equal(out.token[:M], samp.token[:M])

    # shrink: the segment above the first one goes back to the driver
    torch.cuda.synchronize()
    before, _ = torch.cuda.mem_get_info(0)
    ws.resize(ref.plan.workspace_bytes)
    after, _ = torch.cuda.mem_get_info(0)
    assert ws.ptr == base and ws.committed_bytes == -(-ref.plan.workspace_bytes // g) * g
    assert after - before >= (48 << 20)
    binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, out.idx, out.count, out.max_rows, out.token, out.conf, out.lse,
                                        out.plan, ws)
    torch.cuda.synchronize()
    assert torch.equal(out.token[:M], ref.token[:M]) and torch.equal(out.lse[:M], ref.lse[:M])

    # too small a mapped prefix is refused by the entry point before anything runs; so is an over-large resize
    ws.resize(0)
    assert ws.committed_bytes == 0
    with pytest.raises(binding.MosaicError):
        binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, out.idx, out.count, out.max_rows, out.token, out.conf,
                                            out.lse, out.plan, ws)
    with pytest.raises(binding.MosaicError):
        ws.resize((1 << 30) + g + 1)
    ws.close()
    ws.close()                                              # idempotent
