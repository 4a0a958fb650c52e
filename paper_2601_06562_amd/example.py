"""A denoising tail on synthetic data, as a user of the library would write it:

    python -m paper_2601_06562_amd.example [--steps 8] [--temperature 0.0]

Two sequences of a block-diffusion decoder share one flat batch; the last `block` positions of each are masked.  Every
step compacts the mask, runs the fused mask-only logits pass (greedy, or Gumbel-max sampling with --temperature) and
unmasks the most confident predictions of each sequence, until no mask is left; the plan is renewed every step for the
number of masks that remain.  The hidden states are random and do
not change between steps (no transformer runs here): the point is the order of the calls and what they cost.
Needs an MI355X and the built library; nothing here falls back to the CPU.
"""
import argparse
import time

import torch

from . import binding, workloads


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seq-len", type=int, default=16384)
    ap.add_argument("--block", type=int, default=2048, help="masked positions at the end of each sequence")
    ap.add_argument("--steps", type=int, default=8, help="denoising steps to empty the block")
    ap.add_argument("--temperature", type=float, default=0.0)
    ap.add_argument("--d", type=int, default=4096)
    ap.add_argument("--vocab", type=int, default=126464)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("this example needs the GPU")
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    L, B = args.seq_len, 2
    T = B * L
    hidden = workloads._normal_bf16(T, args.d, 1.0, gen, dev)
    w = workloads._normal_bf16(args.vocab, args.d, args.d ** -0.5, gen, dev)
    mask = torch.zeros(T, dtype=torch.uint8, device=dev)
    for b in range(B):
        mask[(b + 1) * L - args.block:(b + 1) * L] = 1
    tokens = torch.zeros(T, dtype=torch.int32, device=dev)
    seq_starts = torch.tensor([b * L for b in range(B + 1)], dtype=torch.int32, device=dev)
    n_step = -(-args.block // args.steps)
    per_step = torch.full((B,), n_step, dtype=torch.int32, device=dev)

    sampling = args.temperature > 0
    op = binding.MaskOnlyLogits(T, args.d, args.vocab, max_rows=B * args.block, device=dev, sampling=sampling)
    print(f"T = {T}, masked = {B * args.block}, workspace = {op.workspace_bytes} bytes "
          f"(fp32 logits of the masked rows alone would be {4 * B * args.block * args.vocab / 1e9:.2f} GB)")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    remaining = B * args.block
    for step in range(args.steps):
        op.replan(remaining)          # the scheduler knows how many masks are left: fewer rows, more vocabulary splits
        remaining = max(0, remaining - B * n_step)
        if sampling:
            op.sample_step(hidden, w, mask, args.temperature, 1234 + step)
        else:
            op.step(hidden, w, mask)
        binding.mosaic_unmask_topn(op.conf, op.token, op.idx, op.count, op.max_rows, seq_starts, per_step, tokens, mask)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    left = int(mask.sum().item())
    print(f"{args.steps} steps in {dt * 1e3:.2f} ms ({dt / args.steps * 1e3:.3f} ms per step), masks left: {left}")
    assert left == 0, "the block was not emptied"


if __name__ == "__main__":
    main()
