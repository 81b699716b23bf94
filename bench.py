#!/usr/bin/env python3
"""Benchmark of the selective-recompute hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch of the 530B-class per-GPU shard
(h=20480, a=128, t=8, s=2048, b=1: 16 heads x head_dim 160; sequence-parallel rows 256 x 20480):
attn_core_fwd, attn_core_bwd_recompute (row pass + column pass), ln_fwd, ln_bwd, bias_dropout_add.
`value` is the attention core's algorithmic fwd+bwd FLOPs (14 d T N, causal: T = s(s+1)/2) per second of
whole-step time.  The dominant kernel (dK/dV pass) is bracketed by HIP events inside the timed steps (every 4th
step: an event record costs stream time), on the stream the kernels run on; the other kernels' durations come
from a second, untimed pass with events between all launches.
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
    ap.add_argument("--stored-steps", type=int, default=20, help="steps of the stored-activation baseline (0 = skip)")
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
    ws = torch.empty(sar.attn_core_bwd_workspace(desc), dtype=torch.uint8, device="cuda")

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

    names = ["attn_core_fwd", "attn_bwd_dq", "attn_bwd_dkdv", "ln_fwd", "ln_bwd", "bias_dropout_add"]

    DOM = 2   # the dK/dV pass executes 4 of the 7 contractions: the dominant kernel, timed inside the timed region

    def step(events=None, marks=range(7)):
        calls = (lambda: sar.attn_core_fwd(desc, tq, tk, tv, o, lse),
                 lambda: sar.attn_core_bwd_recompute_dq(desc, tq, tk, tv, o, lse, tdo, dq, ws),
                 lambda: sar.attn_core_bwd_recompute_dkdv(desc, tq, tk, tv, lse, tdo, dk, dv, ws),
                 lambda: sar.ln_fwd(rdesc, x, gamma, beta, y, mean, rstd),
                 lambda: sar.ln_bwd(rdesc, dy, x, mean, rstd, gamma, dx, dgamma, dbeta, ws2),
                 lambda: sar.bias_dropout_add(rdesc, x, bias, resid, out, None))
        for i, call in enumerate(calls):
            if events is not None and i in marks:
                events[i].record()
            call()
        if events is not None and 6 in marks:
            events[6].record()

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)   # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Timed region: exactly `steps` steps.  An event record costs about 4 us of stream time here, so inside the timed
    # region only the dominant kernel is bracketed, on every 4th step; the other kernels are timed in a second pass
    # that does not count towards `value`.
    SAMPLE = 4
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i] if i % SAMPLE == 0 else None, marks=(DOM, DOM + 1))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    dom_ms = float(np.mean([evs[i][DOM].elapsed_time(evs[i][DOM + 1]) for i in range(0, args.steps, SAMPLE)]))
    nb = min(args.steps, 50)
    for i in range(nb):
        step(evs[i])
    torch.cuda.synchronize()
    kern_ms = {n: float(np.mean([evs[i][j].elapsed_time(evs[i][j + 1]) for i in range(nb)])) for j, n in enumerate(names)}
    kern_ms[names[DOM]] = dom_ms

    # algorithmic work (causal: T = s(s+1)/2 score pairs per head; every key: s^2)
    T = s * (s + 1) // 2 if w.causal else s * s
    one = 2 * d * T * N
    flops = {"attn_core_fwd": 2 * one, "attn_bwd_dq": 3 * one, "attn_bwd_dkdv": 4 * one}   # executed contractions
    flops_alg_fwd_bwd = 14 * d * T * N                                                      # 2 fwd + 5 bwd contractions
    esz = 2
    bytes_alg = {
        "ln_fwd": rows * h * (esz + esz) + 8 * rows + 2 * esz * h,
        "ln_bwd": rows * h * 3 * esz + 8 * rows + esz * h + 8 * h,
        "bias_dropout_add": rows * h * 3 * esz + esz * h,
    }
    value = flops_alg_fwd_bwd / (ms_per_step * 1e-3) / 1e12
    attn_ms = kern_ms["attn_core_fwd"] + kern_ms["attn_bwd_dq"] + kern_ms["attn_bwd_dkdv"]
    dom = names[DOM]
    achieved = flops[dom] / (dom_ms * 1e-3) / 1e12

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(args.workload, {}).get(dom)
        except Exception:
            traffic = None

    # The rows kernels last 6 - 14 us, less than a launch costs the host and about what an event record costs the stream.
    # Their own durations are therefore measured on the GPU's schedule: 20 launches captured in a HIP graph, events
    # around 5 replays.  Also timed this way: the kernels next to the hot path (not part of a step).
    def timed(fn, n=20, reps=5):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(n):
                    fn()
            graph.replay()
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev[0].record()
            for _ in range(reps):
                graph.replay()
            ev[1].record()
            torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / (n * reps)
    rows_ms = {
        "ln_fwd": timed(lambda: sar.ln_fwd(rdesc, x, gamma, beta, y, mean, rstd)),
        "ln_bwd": timed(lambda: sar.ln_bwd(rdesc, dy, x, mean, rstd, gamma, dx, dgamma, dbeta, ws2)),
        "bias_dropout_add": timed(lambda: sar.bias_dropout_add(rdesc, x, bias, resid, out, None)),
    }
    # context for the small sizes: a plain device copy of one [rows, h] tensor moves the bytes of ln_fwd (read + write)
    copy_ms = timed(lambda: y.copy_(x))
    dbias = torch.empty(h, dtype=torch.float32, device="cuda")
    ws3 = torch.empty(max(16, sar.bias_dropout_add_bwd_workspace(rdesc)), dtype=torch.uint8, device="cuda")
    extra_ms = {
        "bias_dropout_add_ln_fwd": timed(lambda: sar.bias_dropout_add_ln_fwd(rdesc, x, bias, resid, gamma, beta, out, y, mean, rstd)),
        "bias_dropout_add_bwd": timed(lambda: sar.bias_dropout_add_bwd(rdesc, dy, dx, dbias, ws3)),
    }
    # bias + GeLU of the MLP block on one tensor-parallel rank: s*b rows of 4h/t columns
    g_rows, g_h = s * b, 4 * w.h // w.t
    gdesc = sar.RowsDesc.make(g_rows, g_h, dtype=SAR_BF16)
    gx = torch.randn((g_rows, g_h), device="cuda").to(torch.bfloat16)
    gdy = torch.randn((g_rows, g_h), device="cuda").to(torch.bfloat16)
    gb = (0.02 * torch.randn(g_h, device="cuda")).to(torch.bfloat16)
    gy, gdx = torch.empty_like(gx), torch.empty_like(gx)
    gdb = torch.empty(g_h, dtype=torch.float32, device="cuda")
    gws = torch.empty(max(16, sar.bias_gelu_bwd_workspace(gdesc)), dtype=torch.uint8, device="cuda")
    extra_ms["bias_gelu_fwd"] = timed(lambda: sar.bias_gelu_fwd(gdesc, gx, gb, gy))
    extra_ms["bias_gelu_bwd"] = timed(lambda: sar.bias_gelu_bwd(gdesc, gdy, gx, gb, gdx, gdb, gws))
    extra_bytes = {"bias_gelu_fwd": g_rows * g_h * 2 * esz + esz * g_h,                       # read x; write y
                   "bias_gelu_bwd": g_rows * g_h * 3 * esz + esz * g_h + 4 * g_h,             # read dy, x; write dx, dbias
                   "bias_dropout_add_ln_fwd": rows * h * 4 * esz + 8 * rows + 3 * esz * h,   # read x, resid; write out, y
                   "bias_dropout_add_bwd": rows * h * 2 * esz + 4 * h}                        # read dout; write dx, dbias

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
                      "note": "P, M, D: 5 bytes per score element written once and read by both backward passes (M and P twice)"}
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
        cpu = {"value": 14 * d * T * nh / (c1 - c0) / 1e12, "unit": "TFLOP/s", "cores": min(nthreads, nh), "kind": "oracle",
               "sample": f"{nh} of {N} heads of the {args.workload} attention core fwd+bwd (fp64, OpenMP over heads) + full LayerNorm fwd/bwd + "
                         f"bias-dropout-add, {c1 - c0:.1f} s", "seconds": c1 - c0}

    line = {
        "metric": "selective-recompute attn fwd+bwd TFLOP/s (% MFMA peak) at 1 GPU",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}-class per-GPU shard: attention core b={b} s={s} heads={A} head_dim={d} {'causal' if w.causal else 'no mask'} p={w.p}; "
                               f"LayerNorm fwd/bwd + bias-dropout-add on {rows}x{h} bf16", "t": w.t},
        "pct_mfma_peak": 100.0 * value / PEAK_BF16_MFMA_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_MFMA_TFLOPS, "traffic": traffic},
        "cpu_baseline": cpu,
        "kernels_ms": kern_ms,
        "attn_fwd_bwd": {"ms": attn_ms, "tflops_algorithmic_14dTN": flops_alg_fwd_bwd / (attn_ms * 1e-3) / 1e12,
                         "tflops_model_12dTN": 12 * d * T * N / (attn_ms * 1e-3) / 1e12,
                         "tflops_executed_18dTN": 18 * d * T * N / (attn_ms * 1e-3) / 1e12},
        "rows_kernels_ms": rows_ms,
        "rows_copy_reference": {"ms": copy_ms, "gbs": 2 * rows * h * esz / (copy_ms * 1e-3) / 1e9,
                                "note": "torch copy of one [rows, h] tensor, timed the same way: what a dependency-free stream of ln_fwd's bytes reaches at this size"},
        "rows_kernels_gbs": {n: bytes_alg[n] / (rows_ms[n] * 1e-3) / 1e9 for n in bytes_alg},
        "rows_kernels_frac_hbm_peak": {n: bytes_alg[n] / (rows_ms[n] * 1e-3) / 1e9 / PEAK_HBM_GBS for n in bytes_alg},
        "next_rows_kernels": {n: {"ms": extra_ms[n], "gbs": extra_bytes[n] / (extra_ms[n] * 1e-3) / 1e9,
                                  "frac_hbm_peak": extra_bytes[n] / (extra_ms[n] * 1e-3) / 1e9 / PEAK_HBM_GBS} for n in extra_ms},
        "stored_baseline": stored,
        "paper_context": {"full_recompute_overhead_pct": "30-40", "mfu_530B_2240_A100_pct": 54.2},
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
