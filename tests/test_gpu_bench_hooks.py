"""GPU: the measurement hooks behind the C ABI return sane figures (they are what bench.py's attainable peaks and issue costs
come from): the matrix-instruction loop, the plain copy, and the per-instruction issue-cost probes."""
import pytest
import torch

import paper_2205_05198_amd as sar

pytestmark = pytest.mark.gpu


def test_copy_hook_copies():
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    sar.sar_bench_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_mfma_hook_reports_its_flops():
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    flops = sar.sar_bench_mfma(10, sink)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flops == cus * 8 * 4 * 10 * 2 * 32 * 32 * 16
    assert float(sink.abs().sum()) == 0.0          # never written


def test_issue_probes():
    """Every probe runs and gives cycles per instruction in a plausible range: a 32x32x16 matrix instruction occupies the
    pipe for 8 passes of 4 cycles, a vector instruction a 16-lane unit for 4, a dependent one waits for its operand."""
    names = sar.sar_bench_issue_names()
    assert len(names) >= 10 and len(set(names)) == len(names)
    nwg, iters = 8, 50
    cyc = torch.zeros(nwg * 8, dtype=torch.int64, device="cuda")
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    res = {}
    for i, n in enumerate(names):
        cyc.zero_()
        ia, ib = sar.sar_bench_issue(i, iters, cyc, sink)
        torch.cuda.synchronize()
        c = cyc.view(nwg, 8).double()
        assert ia > 0 and bool((c[:, :4] > 0).all()), n
        a = float(c[:, :4].mean()) / (iters * ia)
        assert 2.0 < a < 200.0, (n, a)
        if ib:
            assert bool((c[:, 4:] > 0).all()), n
        else:
            assert bool((c[:, 4:] == 0).all()), n   # no second wave was launched
        res[n] = a
        print(f"  {a:7.2f} cycles per instruction  {n}", flush=True)
    ind = res["vector instruction, independent"]
    assert 3.5 < ind < 8.0
    assert res["vector instruction, dependent on the one before"] > ind
    assert 28.0 < res["matrix instruction 32x32x16 bf16"] < 40.0
    with pytest.raises(sar.SarError):
        sar.sar_bench_issue(len(names), iters, cyc, sink)
