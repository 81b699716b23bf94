"""Sequence-length sweep of the attention core at the 530B head shape (16 heads of 160 on one tensor-parallel rank of 8):
bytes kept from forward to backward with and without selective recomputation (Section 5, Eq. 6: linear against quadratic
in s), the backward's scratch and form, and measured forward / backward time.

    python -m paper_2205_05198_amd.seq_sweep [--lengths 2048,4096,...] [--iters 10]

Prints a markdown table.  Needs a GPU; inputs are seeded synthetic draws as in bench.py.
"""
import argparse
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--lengths", default="2048,4096,8192,16384,32768")
    ap.add_argument("--iters", type=int, default=10)
    args = ap.parse_args()
    import torch

    import paper_2205_05198_amd as sar
    from paper_2205_05198_amd.binding import SAR_BF16

    a, t, h, b, p = 128, 8, 20480, 1, 0.1
    A, d = a // t, h // a
    print("| s | saved, selective (MB) | saved, stored (MB) | stored / selective | backward scratch (MB) | backward form | fwd (us) | bwd (us) | TFLOP/s (14dTN) |")
    print("|---|---|---|---|---|---|---|---|---|")
    for s in (int(x) for x in args.lengths.split(",")):
        desc = sar.AttnDesc.packed(s, b, a, h, t=t, rank=0, dtype=SAR_BF16, p=p, seed=1234)
        g = torch.Generator(device="cuda").manual_seed(1234 + s)
        q, k, v = ((torch.randn((s, b, A, d), device="cuda", generator=g) / np.sqrt(d)).to(torch.bfloat16) for _ in range(3))
        do = torch.randn((s, b, A, d), device="cuda", generator=g).to(torch.bfloat16)
        o, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
        lse = torch.empty((b, A, s), dtype=torch.float32, device="cuda")
        nws = sar.attn_core_bwd_workspace(desc)
        once = nws > sar.attn_core_bwd_workspace_min(desc)
        ws = torch.empty(nws, dtype=torch.uint8, device="cuda")

        def timed(fn):
            # untimed launches first, for 0.3 s: from idle the GPU's clocks take some hundred ms of load to settle
            t_spin = time.perf_counter()
            while time.perf_counter() - t_spin < 0.3:
                for _ in range(2):
                    fn()
                torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.iters * 1e3

        tf = timed(lambda: sar.attn_core_fwd(desc, q, k, v, o, lse))
        tb = timed(lambda: sar.attn_core_bwd_recompute(desc, q, k, v, o, lse, do, dq, dk, dv, ws))
        sel, sto = sar.attn_core_saved_bytes(desc, True), sar.attn_core_saved_bytes(desc, False)
        T = s * (s + 1) // 2
        tfl = 14 * d * T * b * A / ((tf + tb) * 1e-6) / 1e12
        print(f"| {s} | {sel / 1e6:.1f} | {sto / 1e6:.1f} | {sto / sel:.1f} | {nws / 1e6:.1f} | {'recompute once (dS tiles)' if once else 'recompute twice'} | "
              f"{tf:.1f} | {tb:.1f} | {tfl:.0f} |", flush=True)
        del q, k, v, do, o, dq, dk, dv, ws
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
