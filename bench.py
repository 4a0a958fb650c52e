"""Benchmark of the mask-only logits hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic input already resident in HBM:
mosaic_mask_compact (mask -> indices) followed by mosaic_masked_logits_reduce (gather-GEMM against
the LM head fused with the vocabulary reduction, then the split merge).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llada_first_step] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (2.5 PFLOP/s)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llada_first_step")
    ap.add_argument("--budget-bytes", type=int, default=0, help="workspace budget for the chunk-size selector")
    ap.add_argument("--cpu-rows", type=int, default=4096, help="rows of the workload the CPU oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one captured HIP graph of the step instead of eager launches (the count "
                         "stays on the device, so the step is capturable as it is); per-kernel events are then "
                         "taken around the whole step")
    ap.add_argument("--temperature", type=float, default=0.0,
                    help="> 0 times the Gumbel-max sampling variant of the fused kernel instead of the greedy one "
                         "(not the headline configuration)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device-to-device copy (for scaling rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this path is built and measured on ONE GPU; --gpus N with N > 1 is not supported "
                 "(rows are independent, so N GPUs would each run this same kernel on M/N rows)")

    import numpy as np
    import torch
    from paper_2601_06562_amd import MaskOnlyLogits, binding, workloads

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    binding.lib()   # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read": 1 << 30, "bytes_written": 1 << 30, "launches": 5}))
        return
    wl = workloads.make(args.workload, device=dev)
    M = wl.M
    torch.cuda.synchronize()
    mem0 = torch.cuda.memory_allocated(dev)
    op = MaskOnlyLogits(wl.T, wl.d, wl.V, max_rows=M, budget_bytes=args.budget_bytes, device=dev,
                        sampling=args.temperature > 0)
    mem_delta = torch.cuda.memory_allocated(dev) - mem0    # workspace + the three outputs, allocator-rounded
    stream = torch.cuda.current_stream()

    def step(ev=None):
        binding.mosaic_mask_compact(wl.mask, op.idx, op.count, op.scratch, stream)
        if ev is not None:
            ev[0].record(stream)
        if args.temperature > 0:
            binding.mosaic_masked_logits_sample(wl.hidden, wl.w, op.idx, op.count, op.max_rows, args.temperature,
                                                20260106 + (0 if ev is None else id(ev) & 0xFFFF), op.token, op.conf,
                                                op.lse, op.plan, op.workspace, stream)
        else:
            binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, op.idx, op.count, op.max_rows, op.token, op.conf,
                                                op.lse, op.plan, op.workspace, stream)
        if ev is not None:
            ev[1].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        eager_step = step
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            stream = side
            eager_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            stream = torch.cuda.current_stream()
            eager_step()
        stream = torch.cuda.current_stream()

        def step(ev=None):
            if ev is not None:
                ev[0].record(stream)
            graph.replay()
            if ev is not None:
                ev[1].record(stream)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert int(op.count.item()) == M
    sec_per_step = (t1 - t0) / args.steps
    kern_ms = float(np.mean([a.elapsed_time(b) for a, b in events]))   # fused kernel (+ the tiny merge)

    # What the matrix cores sustain on this chip right now: a register-only loop of the kernel's MFMA shape,
    # sized to run about as long as the fused kernel so the clock settles the same way.
    operands = (torch.rand(32768, device=dev) - 0.5).to(torch.bfloat16)
    sink = torch.empty(65536, dtype=torch.float32, device=dev)
    n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
    probe_iters = max(64, int(kern_ms * 1e-3 * 2.0e9 / 1024))          # 64 MFMAs x 16 cycles per iteration
    probe_ms = []
    for k in range(12):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        probe_flop = binding.mosaic_mfma_probe(operands, sink, probe_iters, n_cu, stream)
        b.record(stream)
        torch.cuda.synchronize()
        if k >= 2:
            probe_ms.append(a.elapsed_time(b))
    sustained_tflops = probe_flop / (float(np.mean(probe_ms)) * 1e-3) / 1e12

    flop = 2.0 * M * wl.d * wl.V
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        rec = json.load(open(tpath)).get(args.workload)
        if rec:
            traffic = rec["fetch_bytes"] + rec["write_bytes"]   # per launch, rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated
    tflops = flop / (kern_ms * 1e-3) / 1e12
    out = {
        "metric": "masked tokens/sec for mask-only logits (compact + fused gather-GEMM/vocab reduction)",
        "value": M / sec_per_step,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": args.workload, "T": wl.T, "d": wl.d, "V": wl.V, "masked_rows": M,
                   "num_chunks": op.plan.num_chunks, "rows_per_chunk": op.plan.rows_per_chunk,
                   "vocab_splits": op.plan.vocab_splits, "grid": op.plan.grid,
                   "decode": "greedy" if args.temperature <= 0 else f"gumbel-max tau={args.temperature}",
                   "launch": "hip-graph replay" if args.graph else "eager"},
        "tflops": flop / sec_per_step / 1e12,
        "pct_bf16_mfma_peak": 100.0 * flop / sec_per_step / 1e12 / PEAK_BF16_TFLOPS,
        "peak_workspace_bytes": op.workspace_bytes,
        "device_memory_delta_bytes": mem_delta,
        "logits_bytes_avoided": {"fp32_MxV": 4 * M * wl.V, "fp32_TxV": 4 * wl.T * wl.V},
        "roofline": {"bound": "mfma", "kernel": "masked_logits_kernel_w4", "achieved": tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tflops / PEAK_BF16_TFLOPS,
                     "kernel_ms": kern_ms, "flop_per_launch": flop, "traffic": traffic,
                     "algorithmic_bytes": 2 * wl.V * wl.d + 2 * M * wl.d + 12 * M,
                     "sustained_mfma_only": {"tflops": sustained_tflops, "frac_of_it": tflops / sustained_tflops,
                                             "what": "register-only v_mfma_f32_16x16x32_bf16 loop of equal duration "
                                                     "on all CUs (power-limited clock)"}},
    }

    if not args.no_cpu_baseline and args.temperature <= 0:
        import oracle
        rows = min(args.cpu_rows, M)
        rng = np.random.default_rng(0)
        pick = np.sort(rng.choice(M, size=rows, replace=False))
        pos = op.idx[:M][torch.as_tensor(pick, device=dev)].long()
        h_bits = workloads.bf16_bits(wl.hidden[pos])
        w_bits = workloads.bf16_bits(wl.w)
        oracle.positions(h_bits[:2], w_bits, np.arange(2))          # page in, build
        c0 = time.perf_counter()
        want = oracle.positions(h_bits, w_bits, np.arange(rows))
        c1 = time.perf_counter()
        got_tok = op.token[:M].cpu().numpy()[pick]
        got_lse = op.lse[:M].cpu().numpy()[pick]
        strict = want.gap > 1e-2
        out["cpu_baseline"] = {
            "value": rows / (c1 - c0), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{rows} of the {M} masked rows of {args.workload}, all {wl.V} logits each "
                      f"(fp64-accumulated), {c1 - c0:.1f} s",
            "parity_on_sample": {"max_abs_dlse": float(np.abs(got_lse - want.lse).max()),
                                 "argmax_equal_on_strict_rows": bool(np.array_equal(got_tok[strict], want.tok[strict])),
                                 "strict_rows": int(strict.sum())},
        }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
