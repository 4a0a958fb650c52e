"""Benchmark of the mask-only logits hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic input already resident in HBM:
mosaic_mask_compact (mask -> indices) followed by mosaic_masked_logits_reduce (gather-GEMM against
the LM head fused with the vocabulary reduction, then the split merge).  Prints ONE JSON line: the
headline fields are those of the workload the target is quoted on (llada_first_step); `workloads`
carries the same measurement, with an oracle check on a stratified sample of rows, for every benchmark
configuration.  Exit status 1 if any oracle check fails.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llada_first_step]
                    [--no-cpu-baseline] [--no-workloads]
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
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E (8 TB/s)
CONFIGS = ["tiny", "llada_first_step", "long_semi_ar", "dream_late_step", "batched_mixed"]   # the benchmark spec order
EXTRA = ["llada_block_tail"]                                                                 # few-rows regime
LSE_ATOL, CONF_ATOL, CONF_RTOL, GAP_STRICT = 2e-3, 2e-3, 5e-3, 1e-2


def stratified_rows(M, n, seq_bounds, rng):
    """n rows of the compacted list: the first and last rows, both sides of every row-tile boundary near the
    ends, a share from every sequence, the rest uniform."""
    import numpy as np
    if M <= n:
        return np.arange(M)
    picks = [0, 1, M - 2, M - 1]
    for edge in (256, 512, (M // 256) * 256, (M // 512) * 256):
        picks += [r for r in (edge - 1, edge) if 0 <= r < M]
    for lo, hi in seq_bounds:
        if hi > lo:
            picks += list(rng.choice(np.arange(lo, hi), size=min(16, hi - lo), replace=False))
    rest = rng.choice(M, size=n, replace=False)
    rows = np.unique(np.concatenate([np.asarray(picks, dtype=np.int64), rest]))
    return rows[:n] if rows.size > n else rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llada_first_step", help="the workload of the headline fields")
    ap.add_argument("--budget-bytes", type=int, default=0, help="workspace budget for the chunk-size selector")
    ap.add_argument("--cpu-rows", type=int, default=4096, help="rows of the headline workload the CPU oracle is timed on")
    ap.add_argument("--sample-rows", type=int, default=256, help="rows per workload checked against the oracle")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-workloads", action="store_true", help="skip the per-configuration array")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one captured HIP graph of the step instead of eager launches (the count "
                         "stays on the device, so the step is capturable as it is)")
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
    sampling = args.temperature > 0
    SAMPLING_SEED = 20260106
    traffic_db = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic_db = json.load(open(tpath))

    def measure(name, steps, warmup, budget=0, graph=False, temperature=None):
        """One workload: K timed steps on the current stream.  Returns the record and what the oracle check needs."""
        temperature = args.temperature if temperature is None else temperature
        sampling = temperature > 0
        wl = workloads.make(name, device=dev)
        M = wl.M
        torch.cuda.synchronize()
        mem0 = torch.cuda.memory_allocated(dev)
        op = MaskOnlyLogits(wl.T, wl.d, wl.V, max_rows=M, budget_bytes=budget, device=dev, sampling=sampling)
        mem_delta = torch.cuda.memory_allocated(dev) - mem0    # workspace + the three outputs, allocator-rounded
        stream = torch.cuda.current_stream()

        def step(ev=None, k=0):
            binding.mosaic_mask_compact(wl.mask, op.idx, op.count, op.scratch, stream)
            if ev is not None:
                ev[0].record(stream)
            if sampling:
                binding.mosaic_masked_logits_sample(wl.hidden, wl.w, op.idx, op.count, op.max_rows, temperature,
                                                    SAMPLING_SEED + k, op.token, op.conf, op.lse, op.plan,
                                                    op.workspace, stream)
            else:
                binding.mosaic_masked_logits_reduce(wl.hidden, wl.w, op.idx, op.count, op.max_rows, op.token, op.conf,
                                                    op.lse, op.plan, op.workspace, stream)
            if ev is not None:
                ev[1].record(stream)

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        if graph:
            eager_step = step
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            with torch.cuda.stream(side):
                stream = side
                eager_step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                stream = torch.cuda.current_stream()
                eager_step()
            stream = torch.cuda.current_stream()

            def step(ev=None, k=0):
                if ev is not None:
                    ev[0].record(stream)
                g.replay()
                if ev is not None:
                    ev[1].record(stream)
            for _ in range(warmup):
                step()
            torch.cuda.synchronize()
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for k in range(steps):
            step(events[k], k)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        assert int(op.count.item()) == M
        sec_per_step = (t1 - t0) / steps
        kern_ms = float(np.median([a.elapsed_time(b) for a, b in events]))   # fused kernel (+ the tiny merge)

        flop = 2.0 * M * wl.d * wl.V
        alg_bytes = 2 * wl.V * wl.d + 2 * M * wl.d + 12 * M
        tflops = flop / (kern_ms * 1e-3) / 1e12 if M else 0.0
        gbs = alg_bytes / (kern_ms * 1e-3) / 1e9
        kernel = binding.mosaic_masked_logits_kernel_name(wl.T, wl.d, wl.hidden.stride(0), wl.V, op.plan, sampling)
        rec = traffic_db.get(name) if not sampling else None
        traffic = rec["fetch_bytes"] + rec["write_bytes"] if rec else None
        if flop / alg_bytes >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
            roof = {"bound": "mfma", "kernel": kernel, "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": tflops / PEAK_BF16_TFLOPS}
        else:   # too few rows per byte of LM head: the bound is streaming W once from HBM
            roof = {"bound": "hbm", "kernel": kernel, "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": gbs / PEAK_HBM_GBS}
        roof.update({"kernel_ms": kern_ms, "flop_per_launch": flop, "algorithmic_bytes": alg_bytes, "traffic": traffic,
                     "traffic_source": ("profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE of this "
                                        "command in runs of their own, scaled by a 1 GiB copy; not a product of this run")
                     if traffic is not None else "null: no counter run is committed for this workload and decode mode"})
        out = {
            "workload": name, "T": wl.T, "d": wl.d, "V": wl.V, "masked_rows": M,
            "num_chunks": op.plan.num_chunks, "rows_per_chunk": op.plan.rows_per_chunk,
            "vocab_splits": op.plan.vocab_splits, "grid": op.plan.grid,
            "ms_per_step": sec_per_step * 1e3, "kernel_ms": kern_ms,
            "masked_tokens_per_s": M / sec_per_step, "tflops": flop / sec_per_step / 1e12,
            "pct_bf16_mfma_peak": 100.0 * flop / sec_per_step / 1e12 / PEAK_BF16_TFLOPS,
            "peak_workspace_bytes": op.workspace_bytes, "device_memory_delta_bytes": mem_delta,
            "logits_bytes_avoided": {"fp32_MxV": 4 * M * wl.V, "fp32_TxV": 4 * wl.T * wl.V},
            "roofline": roof,
        }
        if sampling:
            out["last_seed"] = SAMPLING_SEED + steps - 1
        return out, wl, op

    def sampling_check(wl, op, rows_wanted, tau, seed):
        """The draws of the last timed step against the oracle's Gumbel-max draw on a sample of rows: the same token
        wherever the oracle's two best perturbed scores are further apart than fp32 rounding can move them, else a
        token whose perturbed score is within that margin of the best."""
        import oracle
        M = wl.M
        rows = np.unique(np.random.default_rng(1).integers(0, M, rows_wanted))
        idx_host = op.idx[:M].cpu().numpy()
        pos = idx_host[rows].astype(np.int64)
        h_bits = workloads.bf16_bits(wl.hidden[torch.as_tensor(pos, device=dev)])
        w_bits = workloads.bf16_bits(wl.w)
        _, logits = oracle.positions(h_bits, w_bits, np.arange(rows.size), return_logits=True)
        tok = op.token[:M].cpu().numpy()[rows]
        lse = op.lse[:M].cpu().numpy()[rows].astype(np.float64)
        conf = op.conf[:M].cpu().numpy()[rows].astype(np.float64)
        margin = 1e-3 * (1.0 + tau)
        strict = equal = 0
        ok = True
        worst_lse = worst_conf = 0.0
        for k in range(rows.size):
            tok_o, conf_o, lse_o, gap_o = oracle.row_sample(logits[k], tau, seed, int(pos[k]))
            worst_lse = max(worst_lse, abs(lse[k] - lse_o))
            if not 0 <= tok[k] < wl.V:
                ok = False
                continue
            if tok[k] == tok_o:
                equal += 1
                worst_conf = max(worst_conf, abs(conf[k] - conf_o))
            if gap_o > margin:
                strict += 1
                ok = ok and tok[k] == tok_o
            elif tok[k] != tok_o:
                y_pick = float(logits[k][tok[k]]) + tau * oracle.gumbel(seed, int(pos[k]), int(tok[k]))
                y_best = float(logits[k][tok_o]) + tau * oracle.gumbel(seed, int(pos[k]), tok_o)
                ok = ok and y_pick >= y_best - margin
        ok = ok and worst_lse <= LSE_ATOL and worst_conf <= CONF_ATOL
        return {"rows": int(rows.size), "strict_rows": strict, "tokens_equal": equal, "max_abs_dlse": worst_lse,
                "max_abs_dconf_where_equal": worst_conf, "ok": bool(ok)}

    def oracle_check(wl, op, rows_wanted, with_logits=True):
        """Oracle on a stratified sample of the masked rows; the acceptance rule of the parity tests."""
        import oracle
        M = wl.M
        bounds, lo = [], 0
        idx_host = op.idx[:M].cpu().numpy()
        for L in wl.seq_lens:
            bounds.append((int(np.searchsorted(idx_host, lo)), int(np.searchsorted(idx_host, lo + L))))
            lo += L
        rows = stratified_rows(M, min(rows_wanted, M), bounds, np.random.default_rng(0))
        pos = torch.as_tensor(idx_host[rows].astype(np.int64), device=dev)
        h_bits = workloads.bf16_bits(wl.hidden[pos])
        w_bits = workloads.bf16_bits(wl.w)
        oracle.positions(h_bits[:2], w_bits, np.arange(min(2, rows.size)))          # page in, build
        c0 = time.perf_counter()
        if with_logits:     # the rows of logits themselves, to judge the ids picked on near-tie rows
            want, logits = oracle.positions(h_bits, w_bits, np.arange(rows.size), return_logits=True)
        else:
            want, logits = oracle.positions(h_bits, w_bits, np.arange(rows.size)), None
        c1 = time.perf_counter()
        tok = op.token[:M].cpu().numpy()[rows]
        conf = op.conf[:M].cpu().numpy()[rows].astype(np.float64)
        lse = op.lse[:M].cpu().numpy()[rows].astype(np.float64)
        strict = want.gap > GAP_STRICT
        dl = np.abs(lse - want.lse)
        dc = np.abs(conf - want.conf)
        rel = dc / np.maximum(want.conf, 1e-30)
        near_max = bool(np.all((tok >= 0) & (tok < wl.V)))
        if logits is not None:
            picked = logits[np.arange(rows.size), np.clip(tok, 0, wl.V - 1)]
            near_max = near_max and bool(np.all(picked >= want.rowmax - GAP_STRICT))
        res = {
            "rows": int(rows.size), "strict_rows": int(strict.sum()),
            "max_abs_dlse": float(dl.max(initial=0)), "max_abs_dconf": float(dc.max(initial=0)),
            "max_rel_dconf": float(rel.max(initial=0)),
            "argmax_equal_on_strict_rows": bool(np.array_equal(tok[strict], want.tok[strict])),
            "other_rows_within_1e-2_of_the_maximum": near_max if logits is not None else None,
        }
        res["ok"] = bool(res["max_abs_dlse"] <= LSE_ATOL and res["max_abs_dconf"] <= CONF_ATOL and
                         res["max_rel_dconf"] <= CONF_RTOL and res["argmax_equal_on_strict_rows"] and near_max)
        return res, rows.size, c1 - c0

    head, wl, op = measure(args.workload, args.steps, args.warmup, budget=args.budget_bytes, graph=args.graph)
    stream = torch.cuda.current_stream()

    # What the matrix cores sustain on this chip right now: a register-only loop of the kernel's MFMA shape,
    # sized to run about as long as the fused kernel so the clock settles the same way.
    operands = (torch.rand(32768, device=dev) - 0.5).to(torch.bfloat16)
    sink = torch.empty(65536, dtype=torch.float32, device=dev)
    n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
    probe_iters = max(64, int(head["kernel_ms"] * 1e-3 * 2.0e9 / 1024))          # 64 MFMAs x 16 cycles per iteration
    probe_ms = []
    for k in range(12):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        probe_flop = binding.mosaic_mfma_probe(operands, sink, probe_iters, n_cu, stream)
        b.record(stream)
        torch.cuda.synchronize()
        if k >= 2:
            probe_ms.append(a.elapsed_time(b))
    sustained_tflops = probe_flop / (float(np.median(probe_ms)) * 1e-3) / 1e12
    if head["roofline"]["bound"] == "mfma":
        head["roofline"]["sustained_mfma_only"] = {
            "tflops": sustained_tflops, "frac_of_it": head["roofline"]["achieved"] / sustained_tflops,
            "what": "register-only v_mfma_f32_16x16x32_bf16 loop of equal duration on all CUs (power-limited clock)"}

    out = {
        "metric": "masked tokens/sec for mask-only logits (compact + fused gather-GEMM/vocab reduction)",
        "value": head["masked_tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": args.workload, "T": head["T"], "d": head["d"], "V": head["V"],
                   "masked_rows": head["masked_rows"], "num_chunks": head["num_chunks"],
                   "rows_per_chunk": head["rows_per_chunk"], "vocab_splits": head["vocab_splits"], "grid": head["grid"],
                   "decode": "greedy" if not sampling else f"gumbel-max tau={args.temperature}",
                   "launch": "hip-graph replay" if args.graph else "eager",
                   "timing": "value and ms_per_step: wall clock over the K steps; kernel_ms: median of per-step HIP "
                             "events around the fused call on its stream"},
        "tflops": head["tflops"],
        "pct_bf16_mfma_peak": head["pct_bf16_mfma_peak"],
        "peak_workspace_bytes": head["peak_workspace_bytes"],
        "device_memory_delta_bytes": head["device_memory_delta_bytes"],
        "logits_bytes_avoided": head["logits_bytes_avoided"],
        "roofline": head["roofline"],
    }
    failed = []

    if not args.no_cpu_baseline and not sampling:
        import oracle
        res, rows, secs = oracle_check(wl, op, args.cpu_rows, with_logits=False)
        out["cpu_baseline"] = {
            "value": rows / secs, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{rows} of the {wl.M} masked rows of {args.workload}, all {wl.V} logits each "
                      f"(fp64-accumulated), {secs:.1f} s",
            "parity_on_sample": res,
        }
        if not res["ok"]:
            failed.append(args.workload)

    if not args.no_workloads and not sampling and not args.graph:
        del wl, op
        torch.cuda.empty_cache()
        arr = []
        for name in CONFIGS + EXTRA:
            steps = max(5, min(args.steps, 20))
            rec, wl_i, op_i = measure(name, steps, min(args.warmup, 3))
            rec["steps"] = steps
            if name in EXTRA:
                rec["extra"] = "not one of the benchmark configurations: the few-rows regime of the same kernel"
            if not args.no_cpu_baseline:
                res, _, _ = oracle_check(wl_i, op_i, args.sample_rows)
                rec["oracle_check"] = res
                if not res["ok"]:
                    failed.append(name)
            del rec["logits_bytes_avoided"], rec["device_memory_delta_bytes"]
            arr.append(rec)
            del wl_i, op_i
            torch.cuda.empty_cache()
        out["workloads"] = arr
        # the sampling variant of the fused kernel (Gumbel-max at temperature 1) on the headline workload, beside
        # the greedy kernel of this same run
        steps = max(5, min(args.steps, 20))
        rec, wl_s, op_s = measure(args.workload, steps, min(args.warmup, 3), budget=args.budget_bytes, temperature=1.0)
        out["sampling"] = {
            "workload": args.workload, "temperature": 1.0, "steps": steps, "kernel": rec["roofline"]["kernel"],
            "kernel_ms": rec["kernel_ms"], "greedy_kernel_ms": head["kernel_ms"],
            "ratio_to_greedy": rec["kernel_ms"] / head["kernel_ms"],
            "frac_of_bf16_mfma_peak": rec["roofline"]["frac"] if rec["roofline"]["bound"] == "mfma" else None,
            "peak_workspace_bytes": rec["peak_workspace_bytes"]}
        if not args.no_cpu_baseline:
            out["sampling"]["oracle_check"] = sampling_check(wl_s, op_s, min(args.sample_rows, 64), 1.0,
                                                             rec["last_seed"])
            if not out["sampling"]["oracle_check"]["ok"]:
                failed.append(args.workload + " (sampling)")
        del wl_s, op_s
    out["parity_failed"] = failed
    print(json.dumps(out), flush=True)
    if failed:
        sys.exit(1)


if __name__ == "__main__":
    main()
