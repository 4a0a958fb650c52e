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

    # grow by 64 MiB: more memory is held, the pointer stays, and -- when the driver lets pages be added behind the
    # ones already mapped -- what the range held is still there; then the sampling variant with its larger workspace
    torch.cuda.synchronize()
    first = ws.committed_bytes
    stamp = torch.arange(first // 4, dtype=torch.int32, device=DEV)
    ws.tensor(0, first // 4, torch.int32).copy_(stamp)
    torch.cuda.synchronize()
    before, _ = torch.cuda.mem_get_info(0)
    ws.resize(64 << 20)
    after, _ = torch.cuda.mem_get_info(0)
    assert ws.ptr == base and ws.committed_bytes == -(-(64 << 20) // g) * g
    assert before - after >= (48 << 20)
    print(f"vmm growth kept the contents: {ws.kept_contents}", flush=True)
    if ws.kept_contents:
        assert torch.equal(ws.tensor(0, first // 4, torch.int32), stamp)
    top = ws.tensor(ws.committed_bytes - 4096, 1024, torch.int32)        # the new pages take writes and give them back
    top.copy_(stamp[:1024])
    assert torch.equal(top, stamp[:1024])
    # several growths in a row, a kernel on the range after each
    for mib in (66, 70, 96):
        ws.resize(mib << 20)
        assert ws.ptr == base and ws.committed_bytes == -(-(mib << 20) // g) * g
        if ws.kept_contents:
            assert torch.equal(top, stamp[:1024])                        # written below the 64 MiB mark before
        binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, out.idx, out.count, out.max_rows, out.token, out.conf,
                                            out.lse, out.plan, ws)
        torch.cuda.synchronize()
        assert torch.equal(out.token[:M], ref.token[:M]) and torch.equal(out.lse[:M], ref.lse[:M])
    ws.resize(64 << 20)                                                  # back down: the plain path, one piece again
    assert not ws.kept_contents and ws.committed_bytes == -(-(64 << 20) // g) * g
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
