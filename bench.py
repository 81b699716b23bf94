#!/usr/bin/env python3
"""Benchmark of the selective-recompute hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch of the 530B-class per-GPU shard
(h=20480, a=128, t=8, s=2048, b=1: 16 heads x head_dim 160; sequence-parallel rows 256 x 20480):
attn_core_fwd, attn_core_bwd_recompute (recompute-once form: delta, dK/dV + dS tiles, dQ from the tiles), ln_fwd, ln_bwd,
bias_dropout_add: seven launches per step, enqueued from the host (the host runs ahead of the GPU, so the stream never
drains; `--graph` replays one HIP graph per step instead, which measures about 10 us slower per step here).  `value` is the
attention core's algorithmic fwd+bwd FLOPs (14 d T N, causal: T = s(s+1)/2) per second of whole-step time.  On every 4th
timed step the dominant kernel (dK/dV pass) sits between two HIP events recorded on the launch stream; the other kernels'
durations come from a second, untimed pass with events between all launches (an event record costs stream time, so the
event-bracketed figures run a few microseconds above the rocprofv3 durations in profiles/).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="530B")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--spinup-ms", type=float, default=300.0,
                    help="untimed steps run for this long before the warm-up: from idle the GPU's clocks need some hundred ms of load to settle "
                         "(the first 10 ms after idle run about 8 %% slower), which 5 warm-up steps (1 ms) do not provide")
    ap.add_argument("--event-sample", type=int, default=4, help="the dominant kernel is bracketed by two HIP events on every n-th step of the timed region")
    ap.add_argument("--graph", action="store_true",
                    help="replay one HIP graph per step instead of launching the step's kernels from the host (measured slower here: a replay costs "
                         "about 10 us of launch latency, while host launches run ahead of the GPU and leave no gaps)")
    ap.add_argument("--two-pass", action="store_true", help="time the backward that recomputes the region twice (minimal workspace)")
    ap.add_argument("--stored-steps", type=int, default=20, help="steps of the stored-activation baseline (0 = skip)")
    ap.add_argument("--no-side", action="store_true", help="skip the rows-kernel, attainable-peak and neighbouring-kernel measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (known traffic) so that FETCH_SIZE / WRITE_SIZE of a rocprofv3 --pmc run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2205_05198_amd as sar
    from paper_2205_05198_amd.binding import SAR_BF16
    from paper_2205_05198_amd.workloads import WORKLOADS, attn_inputs, rows_inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    sar.load_library()   # raises if libsar.so is missing: there is no fallback path
    w = WORKLOADS[args.workload]
    s, b, A, d = w.s, w.b, w.A, w.d
    N = b * A

    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).cuda()

    q, k, v, do = attn_inputs(s, b, A, d, "bf16", seed=w.seed)
    desc = sar.AttnDesc.packed(s, b, w.a, w.h, t=w.t, rank=0, dtype=SAR_BF16, p=w.p, seed=w.seed, causal=w.causal)
    tq, tk, tv, tdo = (dev(x) for x in (q, k, v, do))
    o, dq, dk, dv = (torch.empty_like(tq) for _ in range(4))
    lse = torch.empty((b, A, s), dtype=torch.float32, device="cuda")
    ws_min = sar.attn_core_bwd_workspace_min(desc)
    ws_bytes = ws_min if args.two_pass else sar.attn_core_bwd_workspace(desc)
    once = ws_bytes > ws_min
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    rows, h = w.rows, w.rows_h
    inp = rows_inputs(rows, h, "bf16", seed=w.seed)
    rdesc = sar.RowsDesc.make(rows, h, dtype=SAR_BF16, p=w.p, seed=w.seed, offset=sar.attn_core_philox_count(desc))
    x, resid, dy, bias, gamma, beta = (dev(inp[n]) for n in ("x", "resid", "dy", "bias", "gamma", "beta"))
    y, dx, out = (torch.empty_like(x) for _ in range(3))
    mean = torch.empty(rows, dtype=torch.float32, device="cuda")
    rstd = torch.empty_like(mean)
    dgamma = torch.empty(h, dtype=torch.float32, device="cuda")
    dbeta = torch.empty_like(dgamma)
    ws2 = torch.empty(sar.ln_bwd_workspace(rdesc), dtype=torch.uint8, device="cuda")

    # the launches of one step, in order; DOM = the dominant kernel (dK/dV pass: 4 of the executed contractions)
    if once:
        names = ["attn_core_fwd", "attn_bwd_delta", "attn_bwd_dkdv", "attn_bwd_dq", "ln_fwd", "ln_bwd", "bias_dropout_add"]
        calls = [lambda: sar.attn_core_fwd(desc, tq, tk, tv, o, lse),
                 lambda: sar.attn_core_bwd_recompute_stages(desc, 1, tq, tk, tv, o, lse, tdo, dq, dk, dv, ws),
                 lambda: sar.attn_core_bwd_recompute_stages(desc, 2, tq, tk, tv, o, lse, tdo, dq, dk, dv, ws),
                 lambda: sar.attn_core_bwd_recompute_stages(desc, 4, tq, tk, tv, o, lse, tdo, dq, dk, dv, ws)]
        DOM = 2
    else:
        names = ["attn_core_fwd", "attn_bwd_dq", "attn_bwd_dkdv", "ln_fwd", "ln_bwd", "bias_dropout_add"]
        calls = [lambda: sar.attn_core_fwd(desc, tq, tk, tv, o, lse),
                 lambda: sar.attn_core_bwd_recompute_dq(desc, tq, tk, tv, o, lse, tdo, dq, ws),
                 lambda: sar.attn_core_bwd_recompute_dkdv(desc, tq, tk, tv, lse, tdo, dk, dv, ws)]
        DOM = 2
    calls += [lambda: sar.ln_fwd(rdesc, x, gamma, beta, y, mean, rstd),
              lambda: sar.ln_bwd(rdesc, dy, x, mean, rstd, gamma, dx, dgamma, dbeta, ws2),
              lambda: sar.bias_dropout_add(rdesc, x, bias, resid, out, None)]
    nk = len(calls)

    def step_eager(events=None):
        for i, call in enumerate(calls):
            if events is not None:
                events[i].record()
            call()
        if events is not None:
            events[nk].record()

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        sar.sar_bench_copy(src, dst)   # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # everything below runs on one side stream (graph capture needs a non-default stream; the events are recorded on it)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            step_eager()
        torch.cuda.synchronize()
        use_graph = args.graph
        if use_graph:
            def capture(lo, hi):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    for c in calls[lo:hi]:
                        c()
                return g
            g_all, g_head, g_tail = capture(0, nk), capture(0, DOM), capture(DOM + 1, nk)
            run_step = g_all.replay

            def run_step_sampled(e0, e1):
                g_head.replay()
                e0.record()
                calls[DOM]()
                e1.record()
                g_tail.replay()
        else:
            run_step = step_eager

            def run_step_sampled(e0, e1):
                for i, c in enumerate(calls):
                    if i == DOM:
                        e0.record()
                    c()
                    if i == DOM:
                        e1.record()
        t_spin = time.perf_counter()
        while (time.perf_counter() - t_spin) * 1e3 < args.spinup_ms:
            for _ in range(20):
                run_step()
            torch.cuda.synchronize()
        for _ in range(args.warmup):
            run_step()
        torch.cuda.synchronize()
        # Timed region: exactly `steps` steps.  An event record costs stream time, so only the dominant kernel is bracketed,
        # on every 4th step.
        SAMPLE = max(1, args.event_sample)
        nsamp = (args.steps + SAMPLE - 1) // SAMPLE
        dom_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nsamp)]
        for a, b_ in dom_ev:  # torch creates the underlying HIP event at the first record: not inside the timed region
            a.record()
            b_.record()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            if i % SAMPLE == 0:
                run_step_sampled(*dom_ev[i // SAMPLE])
            else:
                run_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / args.steps
        dom_ms = float(np.median([a.elapsed_time(b_) for a, b_ in dom_ev]))
        # second pass, untimed: events between all launches
        nb = min(max(args.steps, 10), 50)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(nk + 1)] for _ in range(nb)]
        for i in range(nb):
            step_eager(evs[i])
        torch.cuda.synchronize()
        # What two consecutive event records cost the stream when nothing lies between them, with kernels before and after
        # as in a step: an event-bracketed duration contains one such gap.
        gap_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for a, b_ in gap_ev:
            calls[DOM - 1]()
            a.record()
            b_.record()
            calls[DOM + 1]()
        torch.cuda.synchronize()
        event_gap_ms = float(np.median([a.elapsed_time(b_) for a, b_ in gap_ev]))
        kern_ms_raw = {n: float(np.median([evs[i][j].elapsed_time(evs[i][j + 1]) for i in range(nb)])) for j, n in enumerate(names)}
        kern_ms_raw[names[DOM]] = dom_ms
        kern_ms = {n: max(v - event_gap_ms, 0.0) for n, v in kern_ms_raw.items()}
        dom_ms_raw, dom_ms = dom_ms, kern_ms[names[DOM]]
        # whole steps without the sampling, for the line's context: graph replays only / host launches only
        def time_steps(fn, n):
            torch.cuda.synchronize()
            a = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - a) * 1e3 / n
        nctx = min(max(args.steps, 10), 100)
        ms_graph_only = time_steps(g_all.replay, nctx) if use_graph else None
        ms_host_launch = time_steps(step_eager, nctx)

    # algorithmic work (causal: T = s(s+1)/2 score pairs per head; every key: s^2)
    T = s * (s + 1) // 2 if w.causal else s * s
    one = 2 * d * T * N
    if once:
        flops = {"attn_core_fwd": 2 * one, "attn_bwd_dkdv": 4 * one, "attn_bwd_dq": one}   # executed = algorithmic contractions
        executed = 14 * d * T * N
    else:
        flops = {"attn_core_fwd": 2 * one, "attn_bwd_dq": 3 * one, "attn_bwd_dkdv": 4 * one}
        executed = 18 * d * T * N
    flops_alg_fwd_bwd = 14 * d * T * N                                                      # 2 fwd + 5 bwd contractions
    esz = 2
    bytes_alg = {
        "ln_fwd": rows * h * (esz + esz) + 8 * rows + 2 * esz * h,
        "ln_bwd": rows * h * 3 * esz + 8 * rows + esz * h + 8 * h,
        "bias_dropout_add": rows * h * 3 * esz + esz * h,
    }
    value = flops_alg_fwd_bwd / (ms_per_step * 1e-3) / 1e12
    attn_names = [n for n in names if n.startswith("attn")]
    attn_ms = sum(kern_ms[n] for n in attn_names)
    dom = names[DOM]
    achieved = flops[dom] / (dom_ms * 1e-3) / 1e12

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(args.workload, {}).get(dom + ("" if once else "_two_pass"))
        except Exception:
            traffic = None

    side_results = {}
    if not args.no_side:
        side_results = side_measurements(args, sar, torch, np, w, rdesc, rows, h, esz, bytes_alg,
                                         dict(x=x, resid=resid, dy=dy, bias=bias, gamma=gamma, beta=beta, y=y, dx=dx, out=out, mean=mean, rstd=rstd,
                                              dgamma=dgamma, dbeta=dbeta, ws2=ws2))

    # stored-activation baseline (Section 4.1) for the recompute-vs-stored ratio
    stored = None
    if args.stored_steps > 0:
        try:
            Pst = torch.empty((b, A, s, s), dtype=torch.bfloat16, device="cuda")
            Dst = torch.empty_like(Pst)
            Mst = torch.empty((b, A, s, s), dtype=torch.uint8, device="cuda")
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            for _ in range(2):
                sar.attn_core_fwd_stored(desc, tq, tk, tv, o, lse, Pst, Mst, Dst)
                sar.attn_core_bwd_stored(desc, tq, tk, tv, o, Pst, Mst, Dst, tdo, dq, dk, dv, ws)
            torch.cuda.synchronize()
            e[0].record()
            for _ in range(args.stored_steps):
                sar.attn_core_fwd_stored(desc, tq, tk, tv, o, lse, Pst, Mst, Dst)
            e[1].record()
            for _ in range(args.stored_steps):
                sar.attn_core_bwd_stored(desc, tq, tk, tv, o, Pst, Mst, Dst, tdo, dq, dk, dv, ws)
            e[2].record()
            torch.cuda.synchronize()
            st_fwd = e[0].elapsed_time(e[1]) / args.stored_steps
            st_bwd = e[1].elapsed_time(e[2]) / args.stored_steps
            st_ms = st_fwd + st_bwd
            extra = 2 * 5 * N * s * s   # P, M, D written by the forward and read by the backward (Section 4.1: 5 a s^2 b / t each way)
            mfma_stored = w.d in (64, 96, 128, 160) and s % 64 == 0
            stored = {"fwd_bwd_ms": st_ms, "fwd_ms": st_fwd, "bwd_ms": st_bwd, "recompute_over_stored": attn_ms / st_ms,
                      "kind": ("matrix-core kernels on the tiles of the recompute path: forward = recompute forward + a pass that writes P, M, D "
                               "(scores computed twice), backward reads P, M (row pass) and P, M, D (column pass)") if mfma_stored else
                              "plain fp32-arithmetic kernels that write/read P, M, D; not a tuned path",
                      "extra_hbm_bytes": extra, "extra_hbm_ms_at_peak": extra / (PEAK_HBM_GBS * 1e9) * 1e3,
                      "note": "P, M, D: 5 bytes per score element written once and read by both backward passes (M and P twice); host-launched, events around the batch"}
            del Pst, Dst, Mst
        except Exception as ex:  # noqa: BLE001
            stored = {"error": str(ex)}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sh = oracle.AttnShape(s=s, b=b, a=w.a, h=w.h, t=w.t, rank=0, p=w.p, seed=w.seed, causal=w.causal)
        nthreads = oracle.num_threads()
        nh = min(N, max(1, nthreads))
        c0 = time.perf_counter()
        oracle.attn_fwd(sh, q, k, v, heads=(0, nh))
        oracle.attn_bwd(sh, q, k, v, do, heads=(0, nh))
        oracle.ln_fwd(inp["x"], inp["gamma"], inp["beta"])
        oracle.ln_bwd(inp["dy"], inp["x"], inp["gamma"])
        oracle.bias_dropout_add(inp["x"], inp["bias"], inp["resid"], w.p, w.seed, 0)
        c1 = time.perf_counter()
        # one head alone runs on one thread (the oracle's threads split heads): the single-thread figure
        oracle.attn_fwd(sh, q, k, v, heads=(0, 1))
        oracle.attn_bwd(sh, q, k, v, do, heads=(0, 1))
        c2 = time.perf_counter()
        cpu = {"value": 14 * d * T * nh / (c1 - c0) / 1e12, "unit": "TFLOP/s", "cores": min(nthreads, nh), "kind": "oracle",
               "sample": f"{nh} of {N} heads of the {args.workload} attention core fwd+bwd (fp64, OpenMP over heads) + full LayerNorm fwd/bwd + "
                         f"bias-dropout-add, {c1 - c0:.1f} s", "seconds": c1 - c0,
               "single_thread": {"value": 14 * d * T / (c2 - c1) / 1e12, "unit": "TFLOP/s", "cores": 1, "seconds": c2 - c1,
                                 "sample": "1 head of the same attention core fwd+bwd on one thread"},
               "compiler_flags": " ".join(oracle.CFLAGS)}

    line = {
        "metric": "selective-recompute attn fwd+bwd TFLOP/s (% MFMA peak) at 1 GPU",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}-class per-GPU shard: attention core b={b} s={s} heads={A} head_dim={d} {'causal' if w.causal else 'no mask'} p={w.p}; "
                               f"LayerNorm fwd/bwd + bias-dropout-add on {rows}x{h} bf16", "t": w.t,
                   "backward": "region recomputed once (dS tiles in the workspace)" if once else "region recomputed twice (row pass + column pass)",
                   "launch": (f"one HIP graph replay per step (every {SAMPLE}th step: two graphs around the event-bracketed dominant kernel)" if use_graph
                              else f"host launches, asynchronous (every {SAMPLE}th step: two event records around the dominant kernel)"),
                   "spinup_ms": args.spinup_ms},
        "pct_mfma_peak": 100.0 * value / PEAK_BF16_MFMA_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_MFMA_TFLOPS, "traffic": traffic,
                     "duration_us": dom_ms * 1e3, "duration_us_events_raw": dom_ms_raw * 1e3, "event_gap_us": event_gap_ms * 1e3,
                     "duration_source": f"median of HIP events around the kernel on the launch stream, every {SAMPLE}th step of the timed region, minus the "
                                        "median of an empty event pair between the same neighbouring kernels (what the two records themselves cost)",
                     "flops_per_launch": flops[dom], "traffic_source": "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run, scaled by a copy of known size); not measured in this run"},
        "cpu_baseline": cpu,
        "kernels_ms": kern_ms, "kernels_ms_events_raw": kern_ms_raw,
        "step_ms": {"timed_region": ms_per_step, "graph_replays_only": ms_graph_only, "host_launches_only": ms_host_launch,
                    "sum_of_kernels": sum(kern_ms.values())},
        "attn_fwd_bwd": {"ms": attn_ms, "tflops_algorithmic_14dTN": flops_alg_fwd_bwd / (attn_ms * 1e-3) / 1e12,
                         "frac_mfma_peak": flops_alg_fwd_bwd / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
                         "tflops_model_12dTN": 12 * d * T * N / (attn_ms * 1e-3) / 1e12,
                         "executed_contraction_flops": executed, "workspace_bytes": ws_bytes},
        "stored_baseline": stored,
        "paper_context": {"full_recompute_overhead_pct": "30-40", "mfu_530B_2240_A100_pct": 54.2},
    }
    line.update(side_results)
    if "attainable_peaks" in line and line["attainable_peaks"].get("mfma_tflops"):
        ap_ = line["attainable_peaks"]
        line["roofline"]["frac_of_attainable"] = achieved / ap_["mfma_tflops"]
        line["attn_fwd_bwd"]["frac_attainable_mfma"] = line["attn_fwd_bwd"]["tflops_algorithmic_14dTN"] / ap_["mfma_tflops"]
    print(json.dumps(line))


def side_measurements(args, sar, torch, np, w, rdesc, rows, h, esz, bytes_alg, t):
    """Rows kernels cold and hot, attainable peaks, and the kernels next to the hot path.  None of it counts towards `value`."""
    from paper_2205_05198_amd.binding import SAR_BF16
    s, b = w.s, w.b
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())

    def timed_graph(fns, reps=5):
        """Median over `reps` replays of one HIP graph holding the launches `fns`; returns ms per launch."""
        with torch.cuda.stream(side):
            for f in fns[:2]:
                f()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for f in fns:
                    f()
            graph.replay()
            torch.cuda.synchronize()
            times = []
            for _ in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                graph.replay()
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1) / len(fns))
        return float(np.median(times))

    # hot: 20 launches on the same buffers (they stay in the caches); cold: consecutive launches rotate over NSETS distinct
    # buffer sets whose total exceeds 512 MB, so that every launch finds its inputs in HBM
    per_set = rows * h * esz
    NSETS = max(2, (600 << 20) // (3 * per_set) + 1)
    xs = [torch.randn((rows, h), device="cuda").to(torch.bfloat16) for _ in range(NSETS)]
    ys = [torch.randn((rows, h), device="cuda").to(torch.bfloat16) for _ in range(NSETS)]
    zs = [torch.empty((rows, h), dtype=torch.bfloat16, device="cuda") for _ in range(NSETS)]
    means = [torch.empty(rows, dtype=torch.float32, device="cuda") for _ in range(NSETS)]
    rstds = [torch.empty(rows, dtype=torch.float32, device="cuda") for _ in range(NSETS)]
    for i in range(NSETS):   # valid statistics for ln_bwd on every set
        sar.ln_fwd(rdesc, xs[i], t["gamma"], t["beta"], zs[i], means[i], rstds[i])
    torch.cuda.synchronize()
    kern = {
        "ln_fwd": lambda i: sar.ln_fwd(rdesc, xs[i], t["gamma"], t["beta"], zs[i], means[i], rstds[i]),
        "ln_bwd": lambda i: sar.ln_bwd(rdesc, ys[i], xs[i], means[i], rstds[i], t["gamma"], zs[i], t["dgamma"], t["dbeta"], t["ws2"]),
        "bias_dropout_add": lambda i: sar.bias_dropout_add(rdesc, xs[i], t["bias"], ys[i], zs[i], None),
        "copy_reference": lambda i: sar.sar_bench_copy(xs[i], zs[i]),
    }
    bytes_k = dict(bytes_alg)
    bytes_k["copy_reference"] = 2 * per_set
    hot, cold = {}, {}
    for n, f in kern.items():
        hot[n] = timed_graph([(lambda f=f: f(0))] * 20)
        cold[n] = timed_graph([(lambda f=f, i=i: f(i)) for i in range(NSETS)])
    del xs, ys, zs
    res = {
        "rows_kernels_ms_cold": cold, "rows_kernels_ms_hot": hot,
        "rows_kernels_gbs_cold": {n: bytes_k[n] / (cold[n] * 1e-3) / 1e9 for n in kern},
        "rows_kernels_gbs_hot": {n: bytes_k[n] / (hot[n] * 1e-3) / 1e9 for n in kern},
        "rows_kernels_frac_hbm_peak": {n: bytes_k[n] / (cold[n] * 1e-3) / 1e9 / PEAK_HBM_GBS for n in kern},
        "rows_kernels_note": f"cold = {NSETS} distinct buffer sets ({NSETS * 3 * per_set / 2**20:.0f} MiB) visited in turn inside one HIP graph, so no launch finds its "
                             "tensors in a cache; hot = the same buffers 20 times; frac_hbm_peak uses the cold figure; copy_reference = a plain copy kernel of "
                             "one [rows, h] tensor (read + write = ln_fwd's bytes)",
    }

    # attainable peaks: register-resident matrix-instruction loop; 1 GiB stream copy
    with torch.cuda.stream(side):
        sink = torch.zeros(4, dtype=torch.float32, device="cuda")
        sar.sar_bench_mfma(2000, sink)
        torch.cuda.synchronize()
        tm = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fl = sar.sar_bench_mfma(20000, sink)
            e1.record()
            torch.cuda.synchronize()
            tm.append(e0.elapsed_time(e1))
        mfma_tflops = fl / (float(np.median(tm)) * 1e-3) / 1e12
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        sar.sar_bench_copy(src, dst)
        torch.cuda.synchronize()
        tc = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            sar.sar_bench_copy(src, dst)
            e1.record()
            torch.cuda.synchronize()
            tc.append(e0.elapsed_time(e1))
        copy_gbs = 2 * (1 << 30) / (float(np.median(tc)) * 1e-3) / 1e9
        del src, dst
    res["attainable_peaks"] = {"mfma_tflops": mfma_tflops, "mfma_frac_of_datasheet": mfma_tflops / PEAK_BF16_MFMA_TFLOPS,
                               "hbm_copy_gbs": copy_gbs, "hbm_frac_of_datasheet": copy_gbs / PEAK_HBM_GBS,
                               "note": "register-resident loop of 32x32x16 bf16 matrix instructions, 8 waves per CU; copy of 1 GiB (read + write counted); medians of 5"}
    res["rows_kernels_frac_attainable_hbm"] = {n: res["rows_kernels_gbs_cold"][n] / copy_gbs for n in kern}

    # what an instruction costs the wave that issues it (one wave per SIMD; the two-wave probes give both waves' figures)
    with torch.cuda.stream(side):
        nwg, iters = 64, 200
        cyc = torch.zeros(nwg * 8, dtype=torch.int64, device="cuda")
        issue = {}
        for pi, pname in enumerate(sar.sar_bench_issue_names()):
            sar.sar_bench_issue(pi, iters, cyc, sink)       # once to warm the instruction cache
            ia, ib = sar.sar_bench_issue(pi, iters, cyc, sink)
            torch.cuda.synchronize()
            c = cyc.view(nwg, 8).double().cpu().numpy()
            val = [round(float(c[:, :4].mean()) / (iters * ia), 2)]
            if ib:
                val.append(round(float(c[:, 4:].mean()) / (iters * ib), 2))
            issue[pname] = val if len(val) > 1 else val[0]
    res["issue_cycles_per_instruction"] = issue

    # the kernels next to the hot path (not part of a step), hot-cache figures
    x, resid, dy, bias, gamma, beta, y, dx, out, mean, rstd = (t[n] for n in ("x", "resid", "dy", "bias", "gamma", "beta", "y", "dx", "out", "mean", "rstd"))
    dbias = torch.empty(h, dtype=torch.float32, device="cuda")
    ws3 = torch.empty(max(16, sar.bias_dropout_add_bwd_workspace(rdesc)), dtype=torch.uint8, device="cuda")
    extra_ms = {
        "bias_dropout_add_ln_fwd": timed_graph([lambda: sar.bias_dropout_add_ln_fwd(rdesc, x, bias, resid, gamma, beta, out, y, mean, rstd)] * 20),
        "bias_dropout_add_bwd": timed_graph([lambda: sar.bias_dropout_add_bwd(rdesc, dy, dx, dbias, ws3)] * 20),
    }
    g_rows, g_h = s * b, 4 * w.h // w.t   # bias + GeLU of the MLP block on one tensor-parallel rank: s*b rows of 4h/t columns
    gdesc = sar.RowsDesc.make(g_rows, g_h, dtype=SAR_BF16)
    gx = torch.randn((g_rows, g_h), device="cuda").to(torch.bfloat16)
    gdy = torch.randn((g_rows, g_h), device="cuda").to(torch.bfloat16)
    gb = (0.02 * torch.randn(g_h, device="cuda")).to(torch.bfloat16)
    gy, gdx = torch.empty_like(gx), torch.empty_like(gx)
    gdb = torch.empty(g_h, dtype=torch.float32, device="cuda")
    gws = torch.empty(max(16, sar.bias_gelu_bwd_workspace(gdesc)), dtype=torch.uint8, device="cuda")
    extra_ms["bias_gelu_fwd"] = timed_graph([lambda: sar.bias_gelu_fwd(gdesc, gx, gb, gy)] * 20)
    extra_ms["bias_gelu_bwd"] = timed_graph([lambda: sar.bias_gelu_bwd(gdesc, gdy, gx, gb, gdx, gdb, gws)] * 20)
    extra_bytes = {"bias_gelu_fwd": g_rows * g_h * 2 * esz + esz * g_h,                       # read x; write y
                   "bias_gelu_bwd": g_rows * g_h * 3 * esz + esz * g_h + 4 * g_h,             # read dy, x; write dx, dbias
                   "bias_dropout_add_ln_fwd": rows * h * 4 * esz + 8 * rows + 3 * esz * h,   # read x, resid; write out, y
                   "bias_dropout_add_bwd": rows * h * 2 * esz + 4 * h}                        # read dout; write dx, dbias
    res["next_rows_kernels"] = {n: {"ms": extra_ms[n], "gbs": extra_bytes[n] / (extra_ms[n] * 1e-3) / 1e9,
                                    "frac_hbm_peak": extra_bytes[n] / (extra_ms[n] * 1e-3) / 1e9 / PEAK_HBM_GBS, "cache": "hot"} for n in extra_ms}
    return res


if __name__ == "__main__":
    main()
