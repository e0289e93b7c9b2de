#!/usr/bin/env python3
"""Benchmark of the verify step on one MI355X.

A step = one duo_verify call (target pass over n*k draft tokens + speculative sampling + KV
commit) on seeded synthetic inputs already resident in HBM.  The default workload is the
Llama-2-7B-shaped configuration the metric is quoted on (prefix 512, 1 sequence x 8 tokens).
Prints ONE JSON line: verified tokens/s, ms per step, the roofline entry of the dominant kernel
(measured live with HIP events on the launch stream) and the CPU oracle timed beside it.
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
# the same counter reads for a copy of known size): these cannot be read from inside the process, so the figures
# of the committed counter summary (profiles/c1_hbm_traffic.md) are repeated here, keyed by workload and kernel.
MEASURED_TRAFFIC_BYTES = {("C1", "gate_up_swiglu"): 181977918}

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C1", help="C0..C4 (default C1, the configuration the metric is quoted on)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a captured HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--k-sweep", default="", help="comma-separated draft lengths, e.g. 2,4,8,16: also time one sequence of k "
                    "tokens on the same model and prefix (verify latency vs tokens verified) and add \"k_sweep\" to the line")
    ap.add_argument("--draft-step-ms", type=float, default=0.0,
                    help="with --k-sweep: time of one draft-model step on the host; adds the cost coefficient c(k) and the "
                    "balanced draft budget gamma")
    ap.add_argument("--dtype", choices=["bf16", "fp16"], default="bf16", help="16-bit type of the weights and the KV cache "
                    "(bf16 is the configuration the metric is quoted on; fp16 is the paper's own precision)")
    ap.add_argument("--top-p", type=float, default=0.0, help="nucleus restriction of the target distributions in the timed step "
                    "(a variant; the headline number is quoted without it)")
    ap.add_argument("--prefill-tokens", type=int, default=0,
                    help="also time the prefill of this many prompt tokens from an empty cache (time to first token of the "
                    "target model, Sec. 4.1) and add \"prefill\" to the line")
    ap.add_argument("--prefill-chunk", type=int, default=512, help="rows per prefill forward pass (at most 1024)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB elementwise copy (for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
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

    wl = inputs.WORKLOADS[args.workload]
    shape, P, n, k = wl.shape, wl.prefix_len, wl.n_seq, wl.k_draft
    max_seq = (max(P + n * k + 1, args.prefill_tokens) + 31) // 32 * 32 + 32
    t0 = time.time()
    log(f"[bench] workload {wl.name}: generating weights ({shape.weight_bytes() / 1e9:.2f} GB) ...")
    w = inputs.make_weights(shape, seed=args.seed, threads=16, dtype=args.dtype)
    kb, vb, root = inputs.make_synthetic_cache(shape, P, max_seq, seed=args.seed, dtype=args.dtype)
    q, toks, u = inputs.make_draft(shape.vocab, n, k, seed=args.seed + 1, easy_rows=inputs.easy_rows_for(n, k))
    eng = B.VerifyEngine(shape, w, max_seq, max_prefill_rows=args.prefill_chunk if args.prefill_tokens > 0 else B.DUO_MAX_ROWS)
    eng.load_cache(kb, vb, P, root)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    d_toks, d_q, d_u = dev(toks), dev(q), dev(u)
    logits = torch.empty((n * k, shape.vocab), dtype=torch.float32, device="cuda")
    log(f"[bench] inputs resident after {time.time() - t0:.1f}s")

    def step():
        # restore the cache state (the previous step's commit advanced the prefix length), then verify
        eng.set_prefix_len(P)
        eng.verify(d_toks, d_q, d_u, logits_out=logits, top_p=args.top_p)

    if args.calibration_copy:
        # A kernel of known traffic for the hardware counters: reads 256 MiB, writes 256 MiB, outside the timed region.
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = None
    with torch.cuda.stream(stream):
        for _ in range(3):
            step()
        stream.synchronize()
        if not args.no_graph:
            try:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    step()
            except Exception as e:  # capture is an optimisation; fall back to eager launches
                log(f"[bench] graph capture failed ({e}); launching eagerly")
                graph = None
        run = (lambda: graph.replay()) if graph is not None else step
        for _ in range(args.warmup):
            run()
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            run()
        stream.synchronize()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        ms_per_step = (t2 - t1) * 1e3 / args.steps
        res = eng.results(n)
        assert res["status"] == 0, res

        # distribution of the step latency: one event pair per replay, outside the timed region
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(args.steps, 100))]
        for a, b in ev:
            a.record()
            run()
            b.record()
        stream.synchronize()
        lat = sorted(a.elapsed_time(b) for a, b in ev)
        pct = lambda f: lat[min(len(lat) - 1, int(f * len(lat)))]

        # what a plain streaming read reaches on this device: one 4 GiB buffer (far beyond the caches), five launches
        probe_buf = torch.empty(1 << 30, dtype=torch.int32, device="cuda")
        probe_buf.fill_(1)
        probe_bytes = probe_buf.numel() * 4
        sink = torch.zeros(2048, dtype=torch.int32, device="cuda")
        B.stream_read_probe(probe_buf, sink)
        pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        for a, b in pe:
            a.record()
            B.stream_read_probe(probe_buf, sink)
            b.record()
        stream.synchronize()
        probe_gbps = probe_bytes / (min(a.elapsed_time(b) for a, b in pe) * 1e-3) / 1e9

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
        del probe_buf

        # per-kernel timing pass (eager launches with HIP events between kernels on the same stream)
        B.profile_enable(True, args.dtype)
        prof_steps = min(args.steps, 20)
        for _ in range(prof_steps):
            step()
        prof = B.profile_read(args.dtype)
        B.profile_enable(False, args.dtype)
        stream.synchronize()

    algo_bytes = wl.algorithmic_bytes()
    tok_s = n * k / (ms_per_step * 1e-3)
    achieved = algo_bytes / (ms_per_step * 1e-3) / 1e9

    # roofline of the dominant kernel: the gate/up projection (2*F*d bf16 weights per launch)
    kernels = {}
    for name, v in prof.items():
        if v["launches"]:
            kernels[name] = {"avg_us": round(v["ms"] * 1e3 / v["launches"], 2), "launches_per_step": v["launches"] // prof_steps,
                             "ms_per_step": round(v["ms"] / prof_steps, 4)}
    per_launch = {"qkv_rope": 2 * (shape.q_dim + 2 * shape.kv_dim) * shape.d_model, "o_proj": 2 * shape.d_model * shape.q_dim,
                  "gate_up_swiglu": 2 * 2 * shape.d_ff * shape.d_model, "down_proj": 2 * shape.d_model * shape.d_ff,
                  "lm_head": 2 * shape.vocab * shape.d_model,
                  "attn": 2 * 2 * shape.kv_dim * P}
    for name, b in per_launch.items():
        if name in kernels:
            kernels[name]["algo_GBps"] = round(b / (kernels[name]["avg_us"] * 1e-6) / 1e9, 1)
    dom = max((nm for nm in per_launch if nm in kernels), key=lambda nm: kernels[nm]["ms_per_step"])
    dom_bytes = per_launch[dom]
    dom_gbps = dom_bytes / (kernels[dom]["avg_us"] * 1e-6) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, dom)),
                "algo_bytes_per_launch": dom_bytes, "avg_launch_us": kernels[dom]["avg_us"]}

    out = {"metric": "verified_tokens_per_s", "value": round(tok_s, 1), "unit": "tok/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
           "config": {"workload": wl.name, "prefix_len": P, "n_seq": n, "k_draft": k, "rows": n * k,
                      "launch": "hip_graph_replay" if graph is not None else "eager",
                      **({"top_p": args.top_p} if 0.0 < args.top_p < 1.0 else {})},
           "verify_latency_ms": round(ms_per_step, 4), "algorithmic_bytes": algo_bytes,
           "achieved_hbm_GBps": round(achieved, 1), "frac_hbm_peak": round(achieved / HBM_PEAK_GBPS, 4),
           "latency_ms_p10_p50_p90": [round(pct(0.1), 4), round(pct(0.5), 4), round(pct(0.9), 4)],
           "latency_ms_after_cache_flush_p50": round(flushed[len(flushed) // 2], 4),
           "committed_tokens_per_s": round((int(res["commit_len"]) + 1) / (ms_per_step * 1e-3), 1),
           "stream_read_probe": {"GBps": round(probe_gbps, 1), "bytes": probe_bytes,
                                 "what": "one kernel of plain 16-byte loads over a 4 GiB buffer, best of five"},
           "roofline": roofline, "kernels": kernels}

    if args.k_sweep:
        from paper_2503_00784_amd import budget
        curve = []
        for kk in [int(t) for t in args.k_sweep.split(",") if t]:
            qk, tk, uk = inputs.make_draft(shape.vocab, 1, kk, seed=args.seed + 100 + kk)
            d_tk, d_qk, d_uk = dev(tk), dev(qk), dev(uk)

            def step_k():
                eng.set_prefix_len(P)
                eng.verify(d_tk, d_qk, d_uk)

            with torch.cuda.stream(stream):
                for _ in range(3):
                    step_k()
                stream.synchronize()
                gk = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gk, stream=stream):
                    step_k()
                for _ in range(10):
                    gk.replay()
                stream.synchronize()
                t5 = time.perf_counter()
                for _ in range(50):
                    gk.replay()
                stream.synchronize()
                curve.append((kk, (time.perf_counter() - t5) * 1e3 / 50))
        out["k_sweep"] = {"n_seq": 1, "prefix_len": P, "ms_by_k": {str(kk): round(ms, 4) for kk, ms in curve}}
        if args.draft_step_ms > 0:
            out["k_sweep"]["draft_step_ms"] = args.draft_step_ms
            out["k_sweep"]["cost_coefficient_by_k"] = {str(kk): round(c, 2)
                                                       for kk, c in budget.cost_coefficient(curve, args.draft_step_ms).items()}
            out["k_sweep"]["draft_budget"] = budget.draft_budget(curve, args.draft_step_ms)

    if args.prefill_tokens > 0:
        prompt = np.random.default_rng(args.seed + 7).integers(0, shape.vocab, size=args.prefill_tokens).tolist()
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
        out["prefill"] = {"tokens": args.prefill_tokens, "chunk": args.prefill_chunk, "ms": round(best * 1e3, 3),
                          "tok_per_s": round(args.prefill_tokens / best, 1), "launch": "eager",
                          "kernel_ms": {nm: round(v["ms"], 3) for nm, v in pprof.items() if v["launches"]}}

    if not args.no_cpu_baseline:
        from oracle import duo_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        log("[bench] timing the CPU oracle on the same workload ...")
        oshape = O.shape_from(shape)
        cache = O.OracleCache.from_bits(oshape, kb, vb, P, root)
        t3 = time.perf_counter()
        ores, ol = O.oracle_verify(oshape, w, cache, toks, q, u, top_p=args.top_p)
        t4 = time.perf_counter()
        gl = logits.cpu().numpy()
        err = float(np.abs(gl - ol).max())
        out["cpu_baseline"] = {"value": round(n * k / (t4 - t3), 3), "unit": "tok/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"one full step of {wl.name} (numpy float64, BLAS threads = cores)",
                               "seconds": round(t4 - t3, 2)}
        out["parity"] = {"logits_max_abs_err": err,
                         "accept_len_equal": bool((res["accept_len"] == ores.accept_len).all()),
                         "accept_len": [int(a) for a in res["accept_len"]]}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
