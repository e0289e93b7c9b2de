#!/usr/bin/env python3
"""Benchmark of the verify step on one MI355X.

A step = one duo_verify call (target pass over n*k draft tokens + speculative sampling + KV
commit) on seeded synthetic inputs already resident in HBM.  The default workload is the largest
Llama-2-7B-shaped configuration of the benchmark set: prefix 4096, 8 sequences x 8 tokens (64 rows).
Prints ONE JSON line: verified tokens/s and ms per step of that workload, the roofline entry of its
dominant kernel (timed live with HIP events on the launch stream), the CPU oracle timed beside it, and, on
the same weights, the step times of the other 7B configurations, the draft-length sweep at one
sequence, the Llama-3-8B GQA configuration and a 4096-token prompt prefill.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch from the hardware counters (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, each scaled by what
# the same counter reads for a copy of known size).  Counters cannot be read from inside the process, so the figures
# of the committed counter summaries are repeated here, keyed by the kernel's name WITH its template arguments as a
# kernel trace prints it; the library reports the name of the kernel it actually launched, and a kernel that is
# not in this table (a changed launch shape) gets `traffic: null` rather than another kernel's figure.
MEASURED_TRAFFIC_BYTES = {
    # (workload, kernel): bytes per launch, from profiles/<workload>_hbm_traffic.md
    ("C3", "gemm_wide_kernel<4, 2, 3, 1, 8, 4, EpiSwiGLU, false, true>"): 192648220,  # 189.83 MB read + 2.82 MB written
    ("C1", "gemm_wide_kernel<1, 2, 3, 1, 8, 4, EpiSwiGLU, true, true>"): 182106978,   # 181.75 MB read + 0.35 MB written
}

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C3", help="C0..C4 (default C3: Llama-2-7B shape, prefix 4096, 8 x 8 draft tokens)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a captured HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--also", default="auto", help="comma-separated other workloads to time after the main one and report under "
                    "\"configs\" (auto: C1,C2,C4 when the main workload is C3, else none; 'none' to skip)")
    ap.add_argument("--also-parity", type=int, default=1, help="1: also run the CPU oracle on each of the other workloads and "
                    "report the largest logit difference (0 to skip; adds about a minute)")
    ap.add_argument("--k-sweep", default="auto", help="comma-separated draft lengths: also time one sequence of k tokens on the "
                    "main workload's model and prefix (verify latency vs tokens verified); auto = 2,4,8,16 for C3, else none")
    ap.add_argument("--draft-step-ms", type=float, default=0.0,
                    help="with a k sweep: time of one draft-model step on the host; adds the cost coefficient c(k) and the "
                    "balanced draft budget gamma")
    ap.add_argument("--dtype", choices=["bf16", "fp16"], default="bf16", help="16-bit type of the weights and the KV cache "
                    "(bf16 is the configuration the metric is quoted on; fp16 is the paper's own precision)")
    ap.add_argument("--top-p", type=float, default=0.0, help="nucleus restriction of the target distributions in the timed step "
                    "(a variant; the headline number is quoted without it)")
    ap.add_argument("--prefill-tokens", type=int, default=-1,
                    help="also time the prefill of this many prompt tokens from an empty cache (time to first token of the "
                    "target model, Sec. 4.1) and add \"prefill\" to the line; default: 4096 for C3, else none")
    ap.add_argument("--prefill-chunk", type=int, default=1024, help="rows per prefill forward pass (at most 1024)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB elementwise copy (for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--main-only", action="store_true", help="the main workload's timing only: no other workloads, no sweep, "
                    "no prefill, no probe (for profiler runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the verify step of one model replica); "
              f"--gpus {args.gpus} is not supported.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2503_00784_amd import binding as B
    from paper_2503_00784_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if not os.path.exists(B.LIB_PATHS[args.dtype]):
        from paper_2503_00784_amd import build
        build.build(verbose=False)
    B.load(args.dtype)

    is_c3 = args.workload == "C3" and not args.main_only
    also = [] if args.main_only else (["C1", "C2", "C4"] if (args.also == "auto" and is_c3) else
                                      [t for t in args.also.split(",") if t and t not in ("auto", "none")])
    sweep = [] if args.main_only else ([2, 4, 8, 16] if (args.k_sweep == "auto" and is_c3) else
                                       [int(t) for t in args.k_sweep.split(",") if t and t not in ("auto", "none")])
    prefill_tokens = 0 if args.main_only else ((4096 if is_c3 else 0) if args.prefill_tokens < 0 else args.prefill_tokens)

    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    stream = torch.cuda.Stream()
    oracle = None
    if not args.no_cpu_baseline:
        from oracle import duo_oracle as oracle  # the reported CPU baseline and the parity figures; never in a timed region
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()

    class Loaded:
        """One workload resident on the GPU: engine, inputs, and the step that restores the cache state and verifies."""

        def __init__(self, wl, host_w, dev_w, extra_seq=0):
            self.wl, self.w = wl, host_w
            shape, P, n, k = wl.shape, wl.prefix_len, wl.n_seq, wl.k_draft
            self.max_seq = (max(P + n * k + 1, P + 65, extra_seq) + 31) // 32 * 32 + 32
            self.kb, self.vb, self.root = inputs.make_synthetic_cache(shape, P, self.max_seq, seed=args.seed, dtype=args.dtype)
            self.q, self.toks, self.u = inputs.make_draft(shape.vocab, n, k, seed=args.seed + 1, easy_rows=inputs.easy_rows_for(n, k))
            self.eng = B.VerifyEngine(shape, host_w, self.max_seq, weights=dev_w,
                                      max_prefill_rows=args.prefill_chunk if extra_seq else B.DUO_MAX_ROWS)
            self.eng.load_cache(self.kb, self.vb, P, self.root)
            self.d = (dev(self.toks), dev(self.q), dev(self.u))
            self.logits = torch.empty((n * k, shape.vocab), dtype=torch.float32, device="cuda")

        def step(self):
            # restore the cache state (the previous step's commit advanced the prefix length), then verify
            self.eng.set_prefix_len(self.wl.prefix_len)
            self.eng.verify(*self.d, logits_out=self.logits, top_p=args.top_p)

    def timed(step, warmup, steps):
        """(ms per step, run callable, launch kind): warm-up, then `steps` steps between device synchronisations."""
        with torch.cuda.stream(stream):
            for _ in range(3):
                step()
            stream.synchronize()
            if args.no_graph:
                run, kind = step, "eager"
            else:  # a capture failure is an error, not a reason to time something else
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    step()
                run, kind = graph.replay, "hip_graph_replay"
            for _ in range(warmup):
                run()
            stream.synchronize()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(steps):
                run()
            stream.synchronize()
            torch.cuda.synchronize()
            return (time.perf_counter() - t1) * 1e3 / steps, run, kind

    def oracle_step(ld):
        """The oracle's whole step on the workload's inputs: (seconds, result, fp32 logits)."""
        oshape = oracle.shape_from(ld.wl.shape)
        cache = oracle.OracleCache.from_bits(oshape, ld.kb, ld.vb, ld.wl.prefix_len, ld.root)
        t3 = time.perf_counter()
        ores, ol = oracle.oracle_verify(oshape, ld.w, cache, ld.toks, ld.q, ld.u, top_p=args.top_p)
        return time.perf_counter() - t3, ores, ol

    wl = inputs.WORKLOADS[args.workload]
    shape, P, n, k = wl.shape, wl.prefix_len, wl.n_seq, wl.k_draft
    t0 = time.time()
    log(f"[bench] workload {wl.name}: generating weights ({shape.weight_bytes() / 1e9:.2f} GB) ...")
    w = inputs.make_weights(shape, seed=args.seed, threads=16, dtype=args.dtype)
    dw = B.DeviceWeights(shape, w)
    main_ld = Loaded(wl, w, dw, extra_seq=prefill_tokens)
    eng = main_ld.eng
    log(f"[bench] inputs resident after {time.time() - t0:.1f}s")

    if args.calibration_copy:
        # A kernel of known traffic for the hardware counters: reads 256 MiB, writes 256 MiB, outside the timed region.
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    torch.cuda.synchronize()
    ms_per_step, run, launch_kind = timed(main_ld.step, args.warmup, args.steps)
    res = eng.results(n)
    assert res["status"] == 0, res
    main_logits = main_ld.logits.cpu().numpy()

    out_extra = {}
    with torch.cuda.stream(stream):
        if not args.main_only:
            # distribution of the step latency: one event pair per replay, outside the timed region
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(args.steps, 100))]
            for a, b in ev:
                a.record()
                run()
                b.record()
            stream.synchronize()
            lat = sorted(a.elapsed_time(b) for a, b in ev)
            pct = lambda f: lat[min(len(lat) - 1, int(f * len(lat)))]
            out_extra["latency_ms_p10_p50_p90"] = [round(pct(0.1), 4), round(pct(0.5), 4), round(pct(0.9), 4)]

            # what a plain streaming read reaches on this device: one 4 GiB buffer (far beyond the caches), five launches
            probe_buf = torch.empty(1 << 30, dtype=torch.int32, device="cuda")
            probe_buf.fill_(1)
            probe_bytes = probe_buf.numel() * 4
            sink = torch.zeros(2048, dtype=torch.int32, device="cuda")
            probe = {}
            for label, nt in (("GBps", False), ("GBps_nontemporal_loads", True)):
                B.stream_read_probe(probe_buf, sink, nt)
                pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
                for a, b in pe:
                    a.record()
                    B.stream_read_probe(probe_buf, sink, nt)
                    b.record()
                stream.synchronize()
                probe[label] = round(probe_bytes / (min(a.elapsed_time(b) for a, b in pe) * 1e-3) / 1e9, 1)
            out_extra["stream_read_probe"] = {**probe, "bytes": probe_bytes,
                                              "what": "one kernel of 16-byte loads over a 4 GiB buffer, best of five: ordinary loads, and "
                                                      "loads with the non-temporal hint that the projection kernels give their weight loads"}

            # the same step with every cache level evicted first (a 4 GiB read between the steps): the weights are far
            # larger than the last-level cache, so this should read the same as the back-to-back figure
            fe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
            for a, b in fe:
                B.stream_read_probe(probe_buf, sink)
                a.record()
                run()
                b.record()
            stream.synchronize()
            flushed = sorted(a.elapsed_time(b) for a, b in fe)
            out_extra["latency_ms_after_cache_flush_p50"] = round(flushed[len(flushed) // 2], 4)
            del probe_buf

        # per-kernel timing pass (eager launches, every dispatch with its own start/stop events on the same stream)
        B.profile_enable(True, args.dtype)
        prof_steps = min(args.steps, 20)
        for _ in range(prof_steps):
            main_ld.step()
        dropped = B.profile_dropped(args.dtype)
        names = B.profile_kernel_names(args.dtype)
        prof = B.profile_read(args.dtype)
        B.profile_enable(False, args.dtype)
        stream.synchronize()
        if dropped:
            raise RuntimeError(f"the per-kernel timer dropped {dropped} launches: fewer profiled steps are needed")

    algo_bytes = wl.algorithmic_bytes()
    tok_s = n * k / (ms_per_step * 1e-3)
    achieved = algo_bytes / (ms_per_step * 1e-3) / 1e9

    # roofline of the dominant kernel: algorithmic bytes of one launch over its average duration
    kernels = {}
    for name, v in prof.items():
        if v["launches"]:
            kernels[name] = {"avg_us": round(v["ms"] * 1e3 / v["launches"], 2), "launches_per_step": v["launches"] // prof_steps,
                             "ms_per_step": round(v["ms"] / prof_steps, 4)}
            if name in names:
                kernels[name]["kernel"] = names[name]
    per_launch = {"qkv_rope": 2 * (shape.q_dim + 2 * shape.kv_dim) * shape.d_model, "o_proj": 2 * shape.d_model * shape.q_dim,
                  "gate_up_swiglu": 2 * 2 * shape.d_ff * shape.d_model, "down_proj": 2 * shape.d_model * shape.d_ff,
                  "lm_head": 2 * shape.vocab * shape.d_model,
                  "attn": 2 * 2 * shape.kv_dim * P}
    # each projection's rate also as a fraction of what a read-only kernel with the same loads reaches on this device
    probe_ceiling = out_extra.get("stream_read_probe", {}).get("GBps_nontemporal_loads")
    for name, b in per_launch.items():
        if name in kernels:
            kernels[name]["algo_GBps"] = round(b / (kernels[name]["avg_us"] * 1e-6) / 1e9, 1)
            if probe_ceiling:
                kernels[name]["frac_of_stream_probe"] = round(kernels[name]["algo_GBps"] / probe_ceiling, 4)
    dom = max((nm for nm in per_launch if nm in kernels), key=lambda nm: kernels[nm]["ms_per_step"])
    dom_bytes = per_launch[dom]
    dom_gbps = dom_bytes / (kernels[dom]["avg_us"] * 1e-6) / 1e9
    dom_kernel = names.get(dom, "")
    traffic = MEASURED_TRAFFIC_BYTES.get((args.workload, dom_kernel))
    roofline = {"bound": "hbm", "kernel": dom, "kernel_name": dom_kernel, "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "traffic_source": (f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/{args.workload.lower()}_hbm_traffic.md"
                                   if traffic is not None else None),
                "algo_bytes_per_launch": dom_bytes, "avg_launch_us": kernels[dom]["avg_us"],
                "frac_of_stream_probe": (round(dom_gbps / probe_ceiling, 4) if probe_ceiling else None)}

    out = {"metric": "verified_tokens_per_s", "value": round(tok_s, 1), "unit": "tok/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
           "config": {"workload": wl.name, "prefix_len": P, "n_seq": n, "k_draft": k, "rows": n * k,
                      "launch": launch_kind, **({"top_p": args.top_p} if 0.0 < args.top_p < 1.0 else {})},
           "verify_latency_ms": round(ms_per_step, 4), "algorithmic_bytes": algo_bytes,
           "achieved_hbm_GBps": round(achieved, 1), "frac_hbm_peak": round(achieved / HBM_PEAK_GBPS, 4),
           "committed_tokens_per_s": round((int(res["commit_len"]) + 1) / (ms_per_step * 1e-3), 1),
           **out_extra, "roofline": roofline, "kernels": kernels}

    def other_workload(name, host_w, dev_w):
        """Step time of another configuration on weights already resident (fewer replays: it is a side figure)."""
        ld = Loaded(inputs.WORKLOADS[name], host_w, dev_w)
        ms, _, kind = timed(ld.step, 10, 40)
        r = ld.eng.results(ld.wl.n_seq)
        assert r["status"] == 0, r
        ab = ld.wl.algorithmic_bytes()
        entry = {"workload": ld.wl.name, "rows": ld.wl.n_seq * ld.wl.k_draft, "ms_per_step": round(ms, 4),
                 "verified_tokens_per_s": round(ld.wl.n_seq * ld.wl.k_draft / (ms * 1e-3), 1),
                 "achieved_hbm_GBps": round(ab / (ms * 1e-3) / 1e9, 1), "frac_hbm_peak": round(ab / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                 "launch": kind}
        if oracle is not None and args.also_parity:
            log(f"[bench] CPU oracle on {ld.wl.name} ...")
            secs, ores, ol = oracle_step(ld)
            entry["logits_max_abs_err"] = float(np.abs(ld.logits.cpu().numpy() - ol).max())
            entry["accept_len_equal"] = bool((r["accept_len"] == ores.accept_len).all())
            entry["oracle_seconds"] = round(secs, 2)
        return entry

    if sweep:
        from paper_2503_00784_amd import budget
        curve = []
        for kk in sweep:
            qk, tk, uk = inputs.make_draft(shape.vocab, 1, kk, seed=args.seed + 100 + kk)
            d_k = (dev(tk), dev(qk), dev(uk))

            def step_k():
                eng.set_prefix_len(P)
                eng.verify(*d_k)

            ms, _, _ = timed(step_k, 10, 40)
            curve.append((kk, ms))
        out["k_sweep"] = {"n_seq": 1, "prefix_len": P, "ms_by_k": {str(kk): round(ms, 4) for kk, ms in curve}}
        if args.draft_step_ms > 0:
            out["k_sweep"]["draft_step_ms"] = args.draft_step_ms
            out["k_sweep"]["cost_coefficient_by_k"] = {str(kk): round(c, 2)
                                                       for kk, c in budget.cost_coefficient(curve, args.draft_step_ms).items()}
            out["k_sweep"]["draft_budget"] = budget.draft_budget(curve, args.draft_step_ms)

    if prefill_tokens > 0:
        prompt = np.random.default_rng(args.seed + 7).integers(0, shape.vocab, size=prefill_tokens).tolist()
        with torch.cuda.stream(stream):
            times = []
            for _ in range(3):
                eng.set_prefix_len(0)
                stream.synchronize()
                t6 = time.perf_counter()
                eng.prefill(prompt, chunk=args.prefill_chunk)
                stream.synchronize()
                times.append(time.perf_counter() - t6)
            B.profile_enable(True, args.dtype)  # one more pass with per-kernel events
            eng.set_prefix_len(0)
            eng.prefill(prompt, chunk=args.prefill_chunk)
            pprof = B.profile_read(args.dtype)
            B.profile_enable(False, args.dtype)
            stream.synchronize()
        best = min(times)
        out["prefill"] = {"tokens": prefill_tokens, "chunk": args.prefill_chunk, "ms": round(best * 1e3, 3),
                          "tok_per_s": round(prefill_tokens / best, 1), "launch": "eager",
                          "kernel_ms": {nm: round(v["ms"], 3) for nm, v in pprof.items() if v["launches"]}}

    if oracle is not None:
        log("[bench] timing the CPU oracle on the same workload ...")
        secs, ores, ol = oracle_step(main_ld)
        err = float(np.abs(main_logits - ol).max())
        out["cpu_baseline"] = {"value": round(n * k / secs, 3), "unit": "tok/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"one full step of {wl.name} (numpy float64, BLAS threads = cores)",
                               "seconds": round(secs, 2)}
        out["parity"] = {"logits_max_abs_err": err,
                         "accept_len_equal": bool((res["accept_len"] == ores.accept_len).all()),
                         "accept_len": [int(a) for a in res["accept_len"]]}

    if also:
        configs = {}
        same_model = [nm for nm in also if inputs.WORKLOADS[nm].shape == shape]
        for nm in same_model:
            log(f"[bench] also: {nm}")
            configs[nm] = other_workload(nm, w, dw)
        del main_ld, eng
        others = [nm for nm in also if nm not in same_model]
        if others:  # another model: the main workload's parameters leave the GPU first
            del dw, w
            torch.cuda.empty_cache()
        for nm in others:
            oshape = inputs.WORKLOADS[nm].shape
            log(f"[bench] also: {nm}: generating weights ({oshape.weight_bytes() / 1e9:.2f} GB) ...")
            w2 = inputs.make_weights(oshape, seed=args.seed, threads=16, dtype=args.dtype)
            configs[nm] = other_workload(nm, w2, B.DeviceWeights(oshape, w2))
            del w2
        out["configs"] = configs
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
