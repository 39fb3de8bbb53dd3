#!/usr/bin/env python3
"""Benchmark of the drafter LM-head hot path on one MI355X.

One step = one call of the low-rank head (down-projection, vocabulary projection with the
fused running log-sum-exp / top-k, cross-workgroup merge) through the C ABI on one batch of
synthetic hidden states, with every input already resident in HBM.  The headline workload is
the single-row latency shape d=4096, r=512, V=128256, k=10 (C2); the 512-row throughput shape
(C4) and the full-head comparator are reported in the "extra" object of the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2|C3|C4|C5] [--quick]

Prints exactly one JSON line on stdout (progress goes to stderr).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = 2500.0      # dense bf16 / fp16 matrix peak
GEMV_MAX_ROWS = 4              # rows up to which the library streams (from 5 rows on: matrix cores)

# HBM bytes per launch of the dominant kernel from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/ (each scaled by the same counter's reading for a plain copy kernel of
# known size); None where not measured.
MEASURED_TRAFFIC_BYTES = {"C2": 131990491, "C4": 146981121}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes_low_rank(rows, d, r, V, k):
    """Bytes the method must move: every weight once, h once, outputs once."""
    return 2 * (d * r + r * V + rows * d) + rows * k * 8


def projection_kernel_bytes(rows, K, V):
    """Algorithmic bytes of one launch of the vocabulary-projection kernel: the [K, V] bf16 weight
    matrix once plus its [rows, K] input (fp32 when streaming, 16-bit on the matrix cores)."""
    return 2 * K * V + (4 if rows <= GEMV_MAX_ROWS else 2) * rows * K


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--copies", type=int, default=4,
                    help="distinct device copies of the weights rotated between steps so that every step "
                         "streams them from HBM rather than from the 256 MB last-level cache")
    ap.add_argument("--quick", action="store_true", help="skip the extra workloads and the CPU baseline")
    ap.add_argument("--no-extra", action="store_true", help="skip the extra workloads only")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch a plain elementwise copy of 128 MiB a few times: the reference a counter run "
                         "scales its FETCH_SIZE / WRITE_SIZE readings by")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_10453_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    binding.load_library()
    dev = torch.device("cuda:0")

    def upload(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    def null_event_pair_ms(n=50):
        """Elapsed time between two HIP events recorded back to back on an idle stream position:
        what an event pair reports around an empty interval."""
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        torch.cuda.synchronize()
        for a, b in pairs:
            a.record()
            b.record()
        torch.cuda.synchronize()
        v = sorted(a.elapsed_time(b) for a, b in pairs)
        return v[len(v) // 2]

    def _timed(step, steps, warmup, with_events):
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        kern_ms = None
        if with_events:
            # The same steps once more, with a HIP event pair recorded by the library around the
            # projection kernel of every call, on the call's own stream.
            pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                     for _ in range(steps)]
            for a, b in pairs:      # create the HIP handles
                a.record()
                b.record()
            torch.cuda.synchronize()
            for i, (a, b) in enumerate(pairs):
                binding.slimspec_set_timing_events(a, b)
                step(i)
            binding.slimspec_set_timing_events(None, None)
            torch.cuda.synchronize()
            kern_ms = sum(a.elapsed_time(b) for a, b in pairs) / steps
        return dt, kern_ms

    def time_low_rank(cfg, x, steps, warmup, copies, with_events=True):
        h = upload(x.h)
        As = [upload(x.A)]
        Bs = [upload(x.B)]
        for _ in range(copies - 1):
            As.append(As[0].clone())
            Bs.append(Bs[0].clone())
        ids = torch.empty((cfg.rows, cfg.k), dtype=torch.int32, device=dev)
        lp = torch.empty((cfg.rows, cfg.k), dtype=torch.float32, device=dev)
        ws = torch.empty(binding.slimspec_workspace_bytes(cfg.rows, cfg.d, cfg.r, cfg.V, cfg.k),
                         dtype=torch.uint8, device=dev)

        def step(i):
            binding.slimspec_head_topk(h, As[i % copies], Bs[i % copies], cfg.k,
                                       out_ids=ids, out_logprobs=lp, workspace=ws)

        return _timed(step, steps, warmup, with_events)

    def time_full(cfg, x, steps, warmup, copies, with_events=True):
        h = upload(x.h)
        Ws = [upload(x.W)]
        for _ in range(copies - 1):
            Ws.append(Ws[0].clone())
        ids = torch.empty((cfg.rows, cfg.k), dtype=torch.int32, device=dev)
        lp = torch.empty((cfg.rows, cfg.k), dtype=torch.float32, device=dev)
        ws = torch.empty(binding.slimspec_workspace_bytes(cfg.rows, cfg.d, cfg.r, cfg.V, cfg.k),
                         dtype=torch.uint8, device=dev)

        def step(i):
            binding.full_head_topk(h, Ws[i % copies], cfg.k, out_ids=ids, out_logprobs=lp, workspace=ws)

        return _timed(step, steps, warmup, with_events)

    def roofline_of(cfg, K, kern_ms, null_ms):
        """Roofline entry of the vocabulary-projection kernel of one call."""
        kbytes = projection_kernel_bytes(cfg.rows, K, cfg.V)
        flops = 2.0 * cfg.rows * K * cfg.V
        kern_s = kern_ms * 1e-3
        if cfg.rows > GEMV_MAX_ROWS:
            ach = flops / kern_s / 1e12
            out = {"bound": "mfma", "achieved": ach, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                   "frac": ach / MFMA_PEAK_TFLOPS,
                   "hbm_frac_same_kernel": kbytes / kern_s / 1e9 / HBM_PEAK_GBS}
        else:
            ach = kbytes / kern_s / 1e9
            out = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                   "frac": ach / HBM_PEAK_GBS}
        out.update({"traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name),
                    "kernel": "vocabulary projection + running log-sum-exp / top-k "
                              + ("(head_tile_kernel)" if cfg.rows > GEMV_MAX_ROWS else "(stream_topk_kernel)"),
                    "kernel_us": kern_ms * 1e3,
                    "kernel_us_minus_empty_event_pair": (kern_ms - null_ms) * 1e3,
                    "empty_event_pair_us": null_ms * 1e3,
                    "algorithmic_bytes_per_launch": kbytes,
                    "algorithmic_flops_per_launch": flops})
        return out

    # ------------------------------------------------------------------ headline workload
    cfg = synth.CONFIGS[args.workload]
    log(f"[bench] generating {cfg.name}: rows={cfg.rows} d={cfg.d} r={cfg.r} V={cfg.V} k={cfg.k}")
    x = synth.make_inputs(cfg, seed=0)
    copies = max(1, args.copies)
    null_ms = null_event_pair_ms()
    log(f"[bench] timing low-rank head: {args.warmup} warm-up + {args.steps} steps, {copies} weight copies")
    dt, kern_ms = time_low_rank(cfg, x, args.steps, args.warmup, copies)
    ms_per_step = dt / args.steps * 1e3
    rows_per_s = cfg.rows * args.steps / dt
    log(f"[bench] {ms_per_step * 1e3:.2f} us/call, {rows_per_s:.1f} rows/s, projection kernel {kern_ms * 1e3:.2f} us "
        f"(empty event pair {null_ms * 1e3:.2f} us)")

    out = {
        "metric": "LM-head rows/s (and us/call) at d=4096,r=512,V=128256; % HBM/MFMA peak",
        "value": rows_per_s, "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "us_per_call": ms_per_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights and hidden states, fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: low-rank head rows={cfg.rows} d={cfg.d} r={cfg.r} V={cfg.V} k={cfg.k}, "
                               f"{copies} rotating weight copies (cold last-level cache)",
                   "rows": cfg.rows, "d": cfg.d, "r": cfg.r, "V": cfg.V, "k": cfg.k},
        "roofline": roofline_of(cfg, cfg.r, kern_ms, null_ms),
        "call_hbm_frac": algorithmic_bytes_low_rank(cfg.rows, cfg.d, cfg.r, cfg.V, cfg.k)
                         / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
    }

    if args.copy_probe:
        src = torch.ones(32 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)       # one elementwise kernel: reads 128 MiB, writes 128 MiB
        torch.cuda.synchronize()
        out["copy_probe"] = {"kernel": "torch elementwise mul by 1.0", "bytes_read": src.numel() * 4,
                             "bytes_written": dst.numel() * 4, "launches": 5}
        del src, dst

    # ------------------------------------------------------------------ CPU baseline (the fp64 checker)
    if not args.quick:
        import oracle
        oracle.build(force=False)
        log("[bench] timing the CPU fp64 checker on the same inputs")
        sub_rows = min(cfg.rows, 8)
        hs = np.ascontiguousarray(x.h[:sub_rows])
        oracle.slimspec_head_topk(hs, x.A, x.B, cfg.k)          # warm the page cache / thread pool
        n, t0 = 0, time.perf_counter()
        while True:
            oracle.slimspec_head_topk(hs, x.A, x.B, cfg.k)
            n += 1
            el = time.perf_counter() - t0
            if el >= args.cpu_seconds and n >= 3:
                break
        out["cpu_baseline"] = {"value": n * sub_rows / el, "unit": "rows/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"{n} calls of the fp64 checker on the first {sub_rows} row(s) of the "
                                         f"same inputs, {el:.1f} s of wall time",
                               "us_per_call": el / n * 1e6}
    else:
        out["cpu_baseline"] = None

    # ------------------------------------------------------------------ extra workloads (context)
    if not (args.quick or args.no_extra):
        extra = {}
        log("[bench] full head on the same shape")
        xf = synth.make_inputs(cfg, seed=0, with_full_head=True)
        nf = max(10, args.steps // 4)
        fdt, fk = time_full(cfg, xf, nf, 5, 2)
        fms = fdt / nf * 1e3
        full_cfg_roof = roofline_of(cfg, cfg.d, fk, null_ms)
        extra["full_head"] = {"us_per_call": fms * 1e3, "projection_kernel_us": fk * 1e3,
                              "roofline_frac_kernel": full_cfg_roof["frac"], "bound": full_cfg_roof["bound"],
                              "low_rank_speedup": fms / ms_per_step,
                              "ideal_speedup": 1.0 / ((cfg.r / cfg.d) * (1 + cfg.d / cfg.V)),
                              "paper_relative_head_time_r_d8": 0.21,
                              "paper_hardware": "NVIDIA H200, vLLM 0.17.1 (context only; the paper's head time "
                                                "excludes softmax / top-k)"}
        w_bits = xf.W
        del xf
        torch.cuda.empty_cache()
        # six head calls (the paper's six draft steps, section 5.1) captured in one HIP graph: no host launch jitter
        try:
            hg = upload(x.h)
            Ag = [upload(x.A) for _ in range(2)]
            Bg = [upload(x.B) for _ in range(2)]
            idg = torch.empty((cfg.rows, cfg.k), dtype=torch.int32, device=dev)
            lpg = torch.empty((cfg.rows, cfg.k), dtype=torch.float32, device=dev)
            wsg = torch.empty(binding.slimspec_workspace_bytes(cfg.rows, cfg.d, cfg.r, cfg.V, cfg.k), dtype=torch.uint8, device=dev)
            binding.slimspec_head_topk(hg, Ag[0], Bg[0], cfg.k, out_ids=idg, out_logprobs=lpg, workspace=wsg)
            torch.cuda.synchronize()
            eager_ids, eager_lp = idg.clone(), lpg.clone()
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    for i in range(6):
                        binding.slimspec_head_topk(hg, Ag[i % 2], Bg[i % 2], cfg.k, out_ids=idg, out_logprobs=lpg, workspace=wsg)
            ok = True
            for _ in range(3):
                graph.replay()
                torch.cuda.synchronize()
                ok = ok and bool(torch.equal(idg, eager_ids)) and bool(torch.equal(lpg, eager_lp))
            nrep = 40
            t0 = time.perf_counter()
            for _ in range(nrep):
                graph.replay()
            torch.cuda.synchronize()
            extra["graph_of_6_calls"] = {"us_per_call": (time.perf_counter() - t0) / (6 * nrep) * 1e6,
                                         "replays_match_eager": ok, "weight_copies": 2}
            del graph
        except Exception as exc:                      # graph capture is a convenience figure only
            extra["graph_of_6_calls"] = {"error": repr(exc)[:200]}
        if cfg.name == "C2":
            c4 = synth.CONFIGS["C4"]
            log("[bench] 512-row throughput shape (C4)")
            x4 = synth.make_inputs(c4, seed=0)
            s4 = 50
            dt4, k4 = time_low_rank(c4, x4, s4, 5, 2)
            ms4 = dt4 / s4 * 1e3
            fl4 = 2.0 * c4.rows * (c4.d * c4.r + c4.r * c4.V)
            r4 = roofline_of(c4, c4.r, k4, null_ms)
            extra["C4_512_rows"] = {"us_per_call": ms4 * 1e3, "rows_per_s": c4.rows / (ms4 * 1e-3),
                                    "mfma_frac_call": fl4 / (ms4 * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                                    "roofline": r4}
            if c4.d == cfg.d and c4.V == cfg.V:
                # the full head on the same 512 rows (same kernel, contraction length d): the comparison of section 4.1
                import types
                log("[bench] full head, 512 rows")
                sf = 40          # (the first calls after idle run at lower clocks: ten warm-up calls)
                fdt4, fk4 = time_full(c4, types.SimpleNamespace(h=x4.h, W=w_bits), sf, 10, 2)
                fms4 = fdt4 / sf * 1e3
                rf4 = roofline_of(c4, c4.d, fk4, null_ms)
                extra["C4_512_rows"]["full_head"] = {"us_per_call": fms4 * 1e3, "projection_kernel_us": fk4 * 1e3,
                                                     "roofline_frac_kernel": rf4["frac"], "bound": rf4["bound"],
                                                     "low_rank_speedup": fms4 / ms4}
        out["extra"] = extra

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
