"""GPU: attn_core_bwd_recompute_noalloc (scratch built into the library) against attn_core_bwd_recompute with a caller's
workspace (the recompute-twice form it shares its kernels with): two calls in a row, the second on a smaller input, every
output bit for bit; and the size limit is an error, not a launch."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2205_05198_amd as sar
from paper_2205_05198_amd.binding import SAR_BF16, SarError
from paper_2205_05198_amd.workloads import attn_inputs

pytestmark = pytest.mark.gpu


def _both(s, b, A, d, seed):
    from gpu_util import dev
    q, k, v, do = attn_inputs(s, b, A, d, "bf16", seed=seed)
    desc = sar.AttnDesc.packed(s, b, A * 2, A * 2 * d, t=2, rank=1, dtype=SAR_BF16, p=0.1, seed=4321, offset=1000 + seed)
    tq, tk, tv, tdo = (dev(x, "bf16") for x in (q, k, v, do))
    o = torch.empty_like(tq)
    lse = torch.empty((b, A, s), dtype=torch.float32, device="cuda")
    sar.attn_core_fwd(desc, tq, tk, tv, o, lse)
    ref = [torch.full_like(tq, float("nan")) for _ in range(3)]
    ws = torch.empty(sar.attn_core_bwd_workspace_min(desc), dtype=torch.uint8, device="cuda")
    sar.attn_core_bwd_recompute(desc, tq, tk, tv, o, lse, tdo, *ref, ws)
    got = [torch.full_like(tq, float("nan")) for _ in range(3)]
    sar.attn_core_bwd_recompute_noalloc(desc, tq, tk, tv, o, lse, tdo, *got)
    torch.cuda.synchronize()
    for name, a, r in zip(("dq", "dk", "dv"), got, ref):
        assert not torch.isnan(r.float()).any(), name
        assert torch.equal(a, r), f"s={s} A={A} d={d}: {name} differs from the workspace form"


def test_noalloc_backward_matches_workspace_form_twice():
    print("noalloc s=328 then s=136", flush=True)
    _both(328, 2, 2, 160, seed=3)      # 1312 rows of scratch
    _both(136, 1, 3, 96, seed=4)       # a smaller input right after: 408 rows; the buffer still holds the first call's values


def test_noalloc_backward_size_limit():
    limit = sar.attn_core_bwd_noalloc_max_bytes()
    assert limit == 1 << 20
    s, b, A, d = 32768, 1, 16, 64      # 524 288 rows x 4 bytes = 2 MiB > 1 MiB: rejected on the host, nothing is launched
    desc = sar.AttnDesc.packed(s, b, A, A * d, dtype=SAR_BF16)
    fake = ctypes.c_void_p(0x10000)
    st = sar.load_library().attn_core_bwd_recompute_noalloc(ctypes.byref(desc), *([fake] * 9), ctypes.c_void_p(0))
    assert st == -3 and "built-in buffer" in sar.sar_last_error()
