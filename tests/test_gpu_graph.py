"""GPU: the hot path captured in a HIP graph.  No entry point allocates, clears memory with a memset node or
synchronises, so a caller may capture a whole step; every replay must reproduce the eager results bit for bit."""
import pytest
import torch

import paper_2205_05198_amd as sar
from paper_2205_05198_amd.binding import SAR_BF16
from paper_2205_05198_amd.workloads import attn_inputs, rows_inputs

pytestmark = pytest.mark.gpu


def test_step_in_hip_graph_replays_bit_exact():
    from gpu_util import dev
    s, b, A, d, t = 320, 1, 2, 160, 2           # five 64-row blocks, two local heads (rank 1 of 2)
    q, k, v, do = attn_inputs(s, b, A, d, "bf16", seed=11)
    desc = sar.AttnDesc.packed(s, b, A * t, A * t * d, t=t, rank=1, dtype=SAR_BF16, p=0.1, seed=77)
    tq, tk, tv, tdo = (dev(a, "bf16") for a in (q, k, v, do))
    o, dq, dk, dv = (torch.zeros_like(tq) for _ in range(4))
    lse = torch.zeros((b, A, s), dtype=torch.float32, device="cuda")
    ws = torch.empty(sar.attn_core_bwd_workspace(desc), dtype=torch.uint8, device="cuda")
    rows, h = 96, 2048
    inp = rows_inputs(rows, h, "bf16", seed=12)
    rdesc = sar.RowsDesc.make(rows, h, dtype=SAR_BF16, p=0.1, seed=77, offset=sar.attn_core_philox_count(desc))
    x, resid, dy, bias, gamma, beta = (dev(inp[n], "bf16") for n in ("x", "resid", "dy", "bias", "gamma", "beta"))
    y, dx, out = (torch.zeros_like(x) for _ in range(3))
    mean = torch.zeros(rows, dtype=torch.float32, device="cuda")
    rstd = torch.zeros_like(mean)
    dgamma = torch.zeros(h, dtype=torch.float32, device="cuda")
    dbeta = torch.zeros_like(dgamma)
    ws2 = torch.empty(sar.ln_bwd_workspace(rdesc), dtype=torch.uint8, device="cuda")
    outputs = (o, lse, dq, dk, dv, y, mean, rstd, dx, dgamma, dbeta, out)

    def step():
        sar.attn_core_fwd(desc, tq, tk, tv, o, lse)
        sar.attn_core_bwd_recompute(desc, tq, tk, tv, o, lse, tdo, dq, dk, dv, ws)
        sar.ln_fwd(rdesc, x, gamma, beta, y, mean, rstd)
        sar.ln_bwd(rdesc, dy, x, mean, rstd, gamma, dx, dgamma, dbeta, ws2)
        sar.bias_dropout_add(rdesc, x, bias, resid, out, None)

    step()
    torch.cuda.synchronize()
    eager = [a.clone() for a in outputs]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capturing stream
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for replay in range(3):
        for a in outputs:                        # eager work between the replays: wipe every output
            a.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, ref in zip(("o", "lse", "dq", "dk", "dv", "y", "mean", "rstd", "dx", "dgamma", "dbeta", "out"), outputs, eager):
            assert torch.equal(a, ref), f"replay {replay}: {name} differs from the eager result"
