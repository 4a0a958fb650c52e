"""Seeded synthetic inputs for the mask-only logits path.

This module holds NO arithmetic of the method: it only draws hidden states, LM-head
weights and masks with the shapes and value distributions of the five benchmark
workloads, and is the one piece both the HIP path's tests and the CPU oracle's tests
read their inputs from.  The Mosaic paper itself measures on dummy inputs (section
5.1), so seeded random tensors stand in faithfully.

Every tensor is drawn in fp32 from a ``torch.Generator`` seeded with
``BASE_SEED + workload number`` on the requested device and rounded once to bf16
(round-to-nearest-even, torch's conversion).  The bits depend on the device the
generator lives on, so one run draws them once and hands the same bits to both sides.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

BASE_SEED = 20260106


@dataclass
class Workload:
    name: str
    T: int                 # flat number of positions (sum of the batch's sequence lengths)
    d: int                 # hidden size
    V: int                 # vocabulary size
    hidden: torch.Tensor   # bf16 [T, d]
    w: torch.Tensor        # bf16 [V, d]
    mask: torch.Tensor     # uint8 [T], nonzero = still masked
    seq_lens: list = field(default_factory=list)

    @property
    def M(self) -> int:
        return int((self.mask != 0).sum().item())


SPECS = {
    # name: (number, batch, L, d, V)
    "tiny": (1, 1, 512, 512, 8192),
    "llada_first_step": (2, 1, 4096, 4096, 126464),
    "long_semi_ar": (3, 1, 32768, 4096, 126464),
    "dream_late_step": (4, 1, 65536, 3584, 152064),
    "batched_mixed": (5, 8, 16384, 4096, 126464),
    # beyond the five benchmark configurations: the last steps of a block-wise decode, when few positions of the
    # block under generation are still masked (the regime where the LM head is read once for very few rows)
    "llada_block_tail": (6, 1, 4096, 4096, 126464),
}
BATCHED_RATIOS = (0.02, 0.05, 0.1, 0.25, 0.5, 0.75, 0.9, 1.0)


def _normal_bf16(rows, cols, std, gen, device, row_scale=None, block=8192):
    out = torch.empty((rows, cols), dtype=torch.bfloat16, device=device)
    for r0 in range(0, rows, block):
        r1 = min(rows, r0 + block)
        z = torch.randn((r1 - r0, cols), generator=gen, device=device, dtype=torch.float32)
        if std != 1.0:
            z *= std
        if row_scale is not None:
            z *= row_scale[r0:r1, None]
        out[r0:r1] = z.to(torch.bfloat16)
    return out


def _bernoulli(n, p, gen, device):
    if p >= 1.0:
        return torch.ones(n, dtype=torch.uint8, device=device)
    u = torch.rand(n, generator=gen, device=device, dtype=torch.float32)
    return (u < p).to(torch.uint8)


def make(name: str, device="cpu", scale_down: int = 1) -> Workload:
    """Draw workload ``name``.  ``scale_down`` > 1 divides L and V (kept multiples of 256) for
    quick checks of the same recipe at a smaller size; the benchmark and full-size parity
    tests use 1."""
    number, batch, L, d, V = SPECS[name]
    if scale_down > 1:
        L = max(256, L // scale_down)
        V = max(256, (V // scale_down) // 256 * 256)
    T = batch * L
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(BASE_SEED + number)

    w = _normal_bf16(V, d, d ** -0.5, gen, device)
    if name == "batched_mixed":
        row_scale = 0.5 + 1.5 * torch.rand(T, generator=gen, device=device, dtype=torch.float32)
        hidden = _normal_bf16(T, d, 1.0, gen, device, row_scale=row_scale)
    else:
        hidden = _normal_bf16(T, d, 1.0, gen, device)

    if name == "tiny":
        mask = _bernoulli(T, 0.5, gen, device)
    elif name == "llada_first_step":
        mask = torch.ones(T, dtype=torch.uint8, device=device)
    elif name == "long_semi_ar":
        prompt = (T * 3) // 4
        mask = torch.zeros(T, dtype=torch.uint8, device=device)
        mask[prompt:] = _bernoulli(T - prompt, 0.5, gen, device)
    elif name == "dream_late_step":
        mask = _bernoulli(T, 0.1, gen, device)
    elif name == "llada_block_tail":
        mask = torch.zeros(T, dtype=torch.uint8, device=device)
        block = min(512, T // 2)
        mask[T - block:] = _bernoulli(block, 0.4, gen, device)     # ~200 masked positions in the last block
    elif name == "batched_mixed":
        mask = torch.cat([_bernoulli(L, r, gen, device) for r in BATCHED_RATIOS])
    else:  # pragma: no cover
        raise KeyError(name)
    return Workload(name, T, d, V, hidden, w, mask, [L] * batch)


def small_random(T, d, V, p=0.5, seed=0, device="cpu", w_std=None) -> Workload:
    """A free-form small case with the same distributions (for tile/tail coverage)."""
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(BASE_SEED + 1000 + seed)
    w = _normal_bf16(V, d, (d ** -0.5) if w_std is None else w_std, gen, device)
    hidden = _normal_bf16(T, d, 1.0, gen, device) if T > 0 else torch.empty((0, d), dtype=torch.bfloat16,
                                                                             device=device)
    mask = _bernoulli(T, p, gen, device) if T > 0 else torch.empty(0, dtype=torch.uint8, device=device)
    return Workload(f"small_{T}x{d}x{V}_s{seed}", T, d, V, hidden, w, mask, [T])


def bf16_bits(t: torch.Tensor):
    """The uint16 bit patterns of a bf16 tensor, as a host numpy array (for the oracle)."""
    return t.detach().contiguous().cpu().view(torch.uint16).numpy()
