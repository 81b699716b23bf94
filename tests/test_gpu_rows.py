"""GPU parity: LayerNorm forward/backward and bias-dropout-add against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2205_05198_amd as sar
from paper_2205_05198_amd.workloads import WORKLOADS, rows_inputs

pytestmark = pytest.mark.gpu


def _run_ln(rows, h, dtype, inp, eps=1e-5):
    from gpu_util import DT, dev, host
    tdt, code = DT[dtype]
    desc = sar.RowsDesc.make(rows, h, dtype=code, eps=eps)
    x, dy, gamma, beta = (dev(inp[k], dtype) for k in ("x", "dy", "gamma", "beta"))
    y, dx = torch.empty_like(x), torch.empty_like(x)
    mean = torch.empty(rows, dtype=torch.float32, device="cuda")
    rstd = torch.empty_like(mean)
    dgamma = torch.empty(h, dtype=torch.float32, device="cuda")
    dbeta = torch.empty_like(dgamma)
    ws = torch.empty(sar.ln_bwd_workspace(desc), dtype=torch.uint8, device="cuda")
    sar.ln_fwd(desc, x, gamma, beta, y, mean, rstd)
    sar.ln_bwd(desc, dy, x, mean, rstd, gamma, dx, dgamma, dbeta, ws)
    torch.cuda.synchronize()
    return {k: host(v) for k, v in dict(y=y, mean=mean, rstd=rstd, dx=dx, dgamma=dgamma, dbeta=dbeta).items()}


@pytest.mark.parametrize("rows,h,dtype", [
    (128, 128, "f32"),            # tiny workload
    (37, 1032, "bf16"),           # ragged: h not a multiple of 64, rows not a multiple of 32
    (5, 8, "f32"),                # smallest row
    (3, 32768, "bf16"),           # widest supported row
    (1024, 6144, "bf16"), (256, 12288, "bf16"), (256, 20480, "bf16"), (256, 25600, "bf16"),  # 22B, 175B, 530B, 1T shards
])
def test_layernorm(rows, h, dtype):
    from gpu_util import BAR, err
    inp = rows_inputs(rows, h, dtype, seed=1234)
    print(f"ln rows={rows} h={h} {dtype}", flush=True)
    got = _run_ln(rows, h, dtype, inp)
    f = oracle.ln_fwd(inp["x"], inp["gamma"], inp["beta"], 1e-5)
    g = oracle.ln_bwd(inp["dy"], inp["x"], inp["gamma"], 1e-5)
    ref = {**f, **g}
    for nm in ("y", "dx"):
        e = err(got[nm], ref[nm], dtype)
        print(f"  {nm}: {e:.3e}", flush=True)
        assert e <= BAR[dtype], nm
    # statistics and parameter gradients are fp32 in both dtypes
    for nm in ("mean", "rstd", "dgamma", "dbeta"):
        e = err(got[nm], ref[nm], "f32")
        print(f"  {nm}: {e:.3e}", flush=True)
        assert e <= (1e-4 if nm in ("mean", "rstd") or dtype == "f32" else 1e-3), nm


def test_layernorm_large_mean():
    """Rows far from zero mean: the shifted single-pass variance must not cancel."""
    from gpu_util import err
    rows, h = 16, 4096
    inp = rows_inputs(rows, h, "f32", seed=5)
    inp["x"] = (inp["x"] * 0.5 + 300.0).astype(np.float32)
    got = _run_ln(rows, h, "f32", inp)
    f = oracle.ln_fwd(inp["x"], inp["gamma"], inp["beta"], 1e-5)
    assert err(got["y"], f["y"], "f32") < 1e-3
    assert err(got["rstd"], f["rstd"], "f32") < 1e-3


def _run_bda(rows, h, dtype, inp, p, seed, offset, row_offset=0, bias=True, mask=True, inplace=False):
    from gpu_util import DT, dev, host
    tdt, code = DT[dtype]
    desc = sar.RowsDesc.make(rows, h, dtype=code, p=p, seed=seed, offset=offset, row_offset=row_offset)
    x, resid = dev(inp["x"], dtype), dev(inp["resid"], dtype)
    b = dev(inp["bias"], dtype) if bias else None
    out = resid if inplace else torch.empty_like(x)
    m = torch.empty((rows, h), dtype=torch.uint8, device="cuda") if mask else None
    sar.bias_dropout_add(desc, x, b, resid, out, m)
    torch.cuda.synchronize()
    return host(out), (m.cpu().numpy() if mask else None)


@pytest.mark.parametrize("rows,h,dtype,p", [
    (128, 128, "f32", 0.1), (37, 1032, "bf16", 0.25), (9, 8, "bf16", 0.0),
    (1024, 6144, "bf16", 0.1), (256, 20480, "bf16", 0.1), (256, 25600, "bf16", 0.1),
])
def test_bias_dropout_add(rows, h, dtype, p):
    from gpu_util import BAR, err
    inp = rows_inputs(rows, h, dtype, seed=99)
    seed, offset, row_offset = 1234, (1 << 32) - 3, 7 * rows
    print(f"bda rows={rows} h={h} {dtype} p={p}", flush=True)
    ref = oracle.bias_dropout_add(inp["x"], inp["bias"], inp["resid"], p, seed, offset, row_offset)
    out, m = _run_bda(rows, h, dtype, inp, p, seed, offset, row_offset)
    assert np.array_equal(m, ref["mask"])              # bit-exact mask
    assert err(out, ref["out"], dtype) <= BAR[dtype]
    # no bias, no mask output, in-place residual
    ref2 = oracle.bias_dropout_add(inp["x"], None, inp["resid"], p, seed, offset, row_offset)
    out2, _ = _run_bda(rows, h, dtype, inp, p, seed, offset, row_offset, bias=False, mask=False, inplace=True)
    assert err(out2, ref2["out"], dtype) <= BAR[dtype]
