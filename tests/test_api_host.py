"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares, reports
byte counts equal to the paper's accounting, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import oracle
import paper_2205_05198_amd as sar
from paper_2205_05198_amd import binding
from paper_2205_05198_amd.workloads import WORKLOADS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sar.library_path()):
        sar.build_library()
    return sar.load_library()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "sar.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = re.findall(r"\b(?:sar_status|size_t|uint64_t|void|const char\*)\s+(\w+)\s*\(", hdr)
    assert sorted(names) == sorted(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layout_matches_header():
    # 8 int32 + 2 float + 2 uint64 + 3 int64 with natural alignment
    assert ctypes.sizeof(sar.AttnDesc) == 8 * 4 + 2 * 4 + 2 * 8 + 3 * 8
    assert sar.AttnDesc.seed.offset == 40 and sar.AttnDesc.stride_s.offset == 56
    assert ctypes.sizeof(sar.RowsDesc) == 3 * 8 + 3 * 4 + 4 + 2 * 8 and sar.RowsDesc.seed.offset == 40


def test_saved_bytes_equal_paper_accounting(lib):
    for name in ("22B", "175B", "530B", "1T"):
        w = WORKLOADS[name]
        d = sar.AttnDesc.packed(w.s, w.b, w.a, w.h, t=w.t, p=w.p)
        for sel in (True, False):
            assert sar.attn_core_saved_bytes(d, sel) == oracle.accounting.attn_core_saved_bytes(w.s, w.b, w.h, w.a, w.t, sel)
        assert sar.attn_core_small_buffer_bytes(d) == oracle.accounting.attn_core_small_buffers(w.s, w.b, w.a, w.t)
        sh = oracle.AttnShape(s=w.s, b=w.b, a=w.a, h=w.h, t=w.t)
        assert sar.attn_core_philox_count(d) == oracle.attn_philox_count(sh)
        # the point of Section 5: no a*s^2*b term is left
        assert sar.attn_core_saved_bytes(d, False) - sar.attn_core_saved_bytes(d, True) == 5 * w.a * w.s * w.s * w.b // w.t
    w = WORKLOADS["tiny"]
    d = sar.AttnDesc.packed(w.s, w.b, w.a, w.h, dtype=binding.SAR_F32)
    assert sar.attn_core_saved_bytes(d, True) == 262144 and sar.attn_core_saved_bytes(d, False) - 262144 == 9 * 2 * 128 * 128


def _fake(n=1):
    return [ctypes.c_void_p(0x1000 * (i + 1)) for i in range(n)]


def test_attention_argument_errors(lib):
    good = dict(s=128, b=1, a=2, h=128)
    p = _fake(12)
    st = ctypes.c_void_p(0)

    def fwd(d, ptrs=p):
        return lib.attn_core_fwd(ctypes.byref(d), *ptrs[:5], st)

    assert lib.attn_core_fwd(None, *p[:5], st) == -1
    assert fwd(sar.AttnDesc.packed(**good), [None] + p[1:5]) == -1
    assert fwd(sar.AttnDesc.packed(s=0, b=1, a=2, h=128)) == -2
    assert fwd(sar.AttnDesc.packed(s=128, b=1, a=3, h=128 * 3, t=2)) == -2          # a % t
    d = sar.AttnDesc.packed(**good); d.rank = 1
    assert fwd(d) == -2
    assert fwd(sar.AttnDesc.packed(s=100, b=1, a=2, h=128)) == -3                   # s % 8
    assert fwd(sar.AttnDesc.packed(s=128, b=1, a=2, h=2 * 260)) == -3               # d > 256
    assert fwd(sar.AttnDesc.packed(**good, causal=2)) == -2                         # 0 (every key) and 1 (decoder mask) only
    assert fwd(sar.AttnDesc.packed(**good, dtype=7)) == -3
    assert fwd(sar.AttnDesc.packed(**good, p=1.0)) == -5
    assert fwd(sar.AttnDesc.packed(**good, p=-0.1)) == -5
    assert fwd(sar.AttnDesc.packed(**good), [ctypes.c_void_p(0x1008)] + p[1:5]) == -4
    d = sar.AttnDesc.packed(**good); d.stride_s = 130
    assert fwd(d) == -4
    assert "16" in sar.sar_last_error()
    # backward: workspace too small / missing, aliasing
    d = sar.AttnDesc.packed(**good)
    need = lib.attn_core_bwd_workspace_min(ctypes.byref(d))
    assert need >= 4 * 128 * 2
    # the once-form of the backward also holds the dS tiles: 3 causal 64 x 64 bf16 tiles per head here
    assert lib.attn_core_bwd_workspace(ctypes.byref(d)) == need + 2 * 3 * 64 * 64 * 2
    dn = sar.AttnDesc.packed(**good, causal=0)
    assert lib.attn_core_bwd_workspace(ctypes.byref(dn)) == need + 2 * 4 * 64 * 64 * 2
    df = sar.AttnDesc.packed(**good, dtype=binding.SAR_F32)   # plain kernels: two-pass form only
    assert lib.attn_core_bwd_workspace(ctypes.byref(df)) == lib.attn_core_bwd_workspace_min(ctypes.byref(df))
    # the stage calls need the full workspace of the once-form, and bf16 at a matrix-core head dimension
    assert lib.attn_core_bwd_recompute_stages(ctypes.byref(d), 7, *p[:9], p[9], need, st) == -6
    assert lib.attn_core_bwd_recompute_stages(ctypes.byref(d), 0, *p[:9], p[9], 1 << 30, st) == -2
    assert lib.attn_core_bwd_recompute_stages(ctypes.byref(df), 7, *p[:9], p[9], 1 << 30, st) == -3
    assert lib.attn_core_bwd_recompute(ctypes.byref(d), *p[:9], p[9], need - 1, st) == -6
    assert lib.attn_core_bwd_recompute(ctypes.byref(d), *p[:9], None, need, st) == -6
    assert lib.attn_core_bwd_recompute(ctypes.byref(d), *p[:6], p[0], p[7], p[8], p[9], need, st) == -2
    assert lib.attn_core_bwd_workspace(None) == 0
    assert lib.attn_core_saved_bytes(None, 1) == 0


def test_stored_baseline_argument_errors(lib):
    """attn_core_fwd_stored / attn_core_bwd_stored reject bad arguments before any launch."""
    p = _fake(14)
    st = ctypes.c_void_p(0)
    d = sar.AttnDesc.packed(s=128, b=1, a=2, h=128)
    # forward: desc, q, k, v, o, lse, P, M, D
    assert lib.attn_core_fwd_stored(None, *p[:8], st) == -1
    for missing in range(8):
        args = list(p[:8]); args[missing] = None
        assert lib.attn_core_fwd_stored(ctypes.byref(d), *args, st) == -1, missing
    args = list(p[:8]); args[5] = ctypes.c_void_p(0x1004)
    assert lib.attn_core_fwd_stored(ctypes.byref(d), *args, st) == -4
    assert lib.attn_core_fwd_stored(ctypes.byref(sar.AttnDesc.packed(s=100, b=1, a=2, h=128)), *p[:8], st) == -3
    # backward: desc, q, k, v, o, P, M, D, dO, dq, dk, dv, workspace, bytes
    need = lib.attn_core_bwd_workspace_min(ctypes.byref(d))
    for missing in range(11):
        args = list(p[:11]); args[missing] = None
        assert lib.attn_core_bwd_stored(ctypes.byref(d), *args, p[11], need, st) == -1, missing
    assert lib.attn_core_bwd_stored(ctypes.byref(d), *p[:11], p[11], need - 1, st) == -6
    assert lib.attn_core_bwd_stored(ctypes.byref(d), *p[:11], None, need, st) == -6
    assert lib.attn_core_bwd_stored(ctypes.byref(d), *p[:11], ctypes.c_void_p(0x20008), need, st) == -4


def test_rows_argument_errors(lib):
    p = _fake(10)
    st = ctypes.c_void_p(0)
    d = sar.RowsDesc.make(16, 128)
    assert lib.ln_fwd(None, *p[:6], st) == -1
    assert lib.ln_fwd(ctypes.byref(d), None, *p[1:6], st) == -1
    assert lib.ln_fwd(ctypes.byref(sar.RowsDesc.make(16, 100)), *p[:6], st) == -3    # h % 8
    assert lib.ln_fwd(ctypes.byref(sar.RowsDesc.make(16, 40000)), *p[:6], st) == -3  # h too wide
    assert lib.ln_fwd(ctypes.byref(sar.RowsDesc.make(0, 128)), *p[:6], st) == -2
    assert lib.ln_fwd(ctypes.byref(d), ctypes.c_void_p(0x1004), *p[1:6], st) == -4
    need = lib.ln_bwd_workspace(ctypes.byref(d))
    assert need > 0
    assert lib.ln_bwd(ctypes.byref(d), *p[:8], p[8], need - 1, st) == -6
    assert lib.bias_dropout_add(ctypes.byref(sar.RowsDesc.make(16, 128, p=1.5)), *p[:5], st) == -5
    assert lib.bias_dropout_add(ctypes.byref(d), p[0], None, p[1], p[0], None, st) == -2  # out aliases x
    assert lib.bias_dropout_add(ctypes.byref(d), None, None, p[1], p[2], None, st) == -1


def test_dropout_add_neighbours_argument_errors(lib):
    """bias_dropout_add_ln_fwd and bias_dropout_add_bwd reject bad arguments before any launch."""
    p = _fake(12)
    st = ctypes.c_void_p(0)
    d = sar.RowsDesc.make(16, 128, p=0.1)
    # fused forward: (desc, x, bias, resid, gamma, beta, out, y, mean, rstd, stream)
    assert lib.bias_dropout_add_ln_fwd(None, *p[:9], st) == -1
    assert lib.bias_dropout_add_ln_fwd(ctypes.byref(d), p[0], None, p[2], p[3], p[4], p[5], None, p[7], p[8], st) == -1   # y missing
    assert lib.bias_dropout_add_ln_fwd(ctypes.byref(d), p[0], None, p[2], p[3], p[4], p[0], p[6], p[7], p[8], st) == -2   # out aliases x
    assert lib.bias_dropout_add_ln_fwd(ctypes.byref(d), p[0], None, p[2], p[3], p[4], p[5], p[5], p[7], p[8], st) == -2   # y aliases out
    assert lib.bias_dropout_add_ln_fwd(ctypes.byref(d), p[0], ctypes.c_void_p(0x2004), p[2], p[3], p[4], p[5], p[6], p[7], p[8], st) == -4
    assert lib.bias_dropout_add_ln_fwd(ctypes.byref(sar.RowsDesc.make(16, 128, p=1.0)), *p[:9], st) == -5
    assert lib.bias_dropout_add_ln_fwd(ctypes.byref(sar.RowsDesc.make(16, 100)), *p[:9], st) == -3
    # backward: (desc, dout, dx, dbias, workspace, workspace_bytes, stream)
    assert lib.bias_dropout_add_bwd(None, p[0], p[1], None, None, 0, st) == -1
    assert lib.bias_dropout_add_bwd(ctypes.byref(d), None, p[1], None, None, 0, st) == -1
    assert lib.bias_dropout_add_bwd(ctypes.byref(d), ctypes.c_void_p(0x1008), p[1], None, None, 0, st) == -4
    tall = sar.RowsDesc.make(4096, 64, p=0.1)     # one column slab, many rows: the rows are split and partial sums need scratch
    need = lib.bias_dropout_add_bwd_workspace(ctypes.byref(tall))
    assert need >= 2 * 64 * 4
    assert lib.bias_dropout_add_bwd(ctypes.byref(tall), p[0], p[1], p[2], None, 0, st) == -6
    assert lib.bias_dropout_add_bwd(ctypes.byref(tall), p[0], p[1], p[2], p[3], need - 1, st) == -6
    wide = sar.RowsDesc.make(256, 20480, p=0.1)   # every slab sees every row: no scratch
    assert lib.bias_dropout_add_bwd_workspace(ctypes.byref(wide)) == 0


def test_bias_gelu_argument_errors(lib):
    p = _fake(8)
    st = ctypes.c_void_p(0)
    d = sar.RowsDesc.make(64, 256)
    assert lib.bias_gelu_fwd(None, p[0], p[1], p[2], st) == -1
    assert lib.bias_gelu_fwd(ctypes.byref(d), None, p[1], p[2], st) == -1
    assert lib.bias_gelu_fwd(ctypes.byref(d), p[0], p[1], None, st) == -1
    assert lib.bias_gelu_fwd(ctypes.byref(d), p[0], ctypes.c_void_p(0x3004), p[2], st) == -4
    assert lib.bias_gelu_fwd(ctypes.byref(sar.RowsDesc.make(64, 100)), p[0], p[1], p[2], st) == -3
    assert lib.bias_gelu_bwd(ctypes.byref(d), None, p[1], p[2], p[3], None, None, 0, st) == -1
    assert lib.bias_gelu_bwd(ctypes.byref(d), p[0], p[1], p[2], None, None, None, 0, st) == -1
    big = sar.RowsDesc.make(4096, 256)                       # rows split over several slab workgroups: dbias needs the workspace
    need = lib.bias_gelu_bwd_workspace(ctypes.byref(big))
    assert need > 0 and need == lib.bias_dropout_add_bwd_workspace(ctypes.byref(big))
    assert lib.bias_gelu_bwd(ctypes.byref(big), p[0], p[1], p[2], p[3], p[4], p[5], need - 1, st) == -6
    assert lib.bias_gelu_bwd_workspace(None) == 0

