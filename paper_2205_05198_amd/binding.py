"""ctypes binding of libsar.so: argument marshalling only, one Python function per C entry point.

Tensors are torch CUDA (ROCm) tensors used purely as device-memory handles (``data_ptr()``); kernels are
enqueued on torch's current stream.  No arithmetic of the method happens in Python.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_LIB_PATH = os.path.join(_HERE, "libsar.so")
# source file -> extra hipcc flags.  -amdgpu-mfma-vgpr-form keeps matrix-core accumulators in the VGPR file: with the
# default heuristics the compiler parks them in AGPRs and copies all of them through VGPRs on every trip of the tile
# loops.  The dK/dV pass needs both register files (2 accumulator sets) and pins its accumulators to AGPRs itself.
# The iterative-ilp scheduling strategy interleaves the Philox integer work with the matrix-core chains of the
# row-block kernels a little better than the default (about 5 % on the dQ pass, measured).
_SOURCES = {
    "sar_api.hip": [],
    "attn_simple.hip": [],
    "attn_mfma_rows.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-mllvm", "-amdgpu-sched-strategy=iterative-ilp"],
    "attn_mfma_cols.hip": [],
    "attn_mfma_cols_small.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "attn_mfma_cols_split.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "attn_mfma_stored.hip": [],
    "attn_mfma_dsgemm.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "rows.hip": [],
    "microbench.hip": [],
}
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wno-inline-asm", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

SAR_F32, SAR_BF16 = 0, 1


class SarError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libsar status {status}: {text}")
        self.status = status


class AttnDesc(ctypes.Structure):
    """sar_attn_desc of include/sar.h (paper notation: s, b, a, t, h; p = dropout probability)."""
    _fields_ = [
        ("s", ctypes.c_int32), ("b", ctypes.c_int32),
        ("a", ctypes.c_int32), ("t", ctypes.c_int32), ("rank", ctypes.c_int32),
        ("h", ctypes.c_int32), ("dtype", ctypes.c_int32), ("causal", ctypes.c_int32),
        ("scale", ctypes.c_float), ("p", ctypes.c_float),
        ("seed", ctypes.c_uint64), ("offset", ctypes.c_uint64),
        ("stride_s", ctypes.c_int64), ("stride_b", ctypes.c_int64), ("stride_a", ctypes.c_int64),
    ]

    @classmethod
    def packed(cls, s, b, a, h, t=1, rank=0, dtype=SAR_BF16, p=0.0, seed=0, offset=0, scale=None, causal=1):
        A, d = a // t, h // a
        if scale is None:
            scale = d ** -0.5
        return cls(s, b, a, t, rank, h, dtype, causal, scale, p, seed, offset, b * A * d, A * d, d)


class RowsDesc(ctypes.Structure):
    """sar_rows_desc of include/sar.h."""
    _fields_ = [
        ("rows", ctypes.c_int64), ("h", ctypes.c_int64), ("row_offset", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("eps", ctypes.c_float), ("p", ctypes.c_float),
        ("seed", ctypes.c_uint64), ("offset", ctypes.c_uint64),
    ]

    @classmethod
    def make(cls, rows, h, dtype=SAR_BF16, eps=1e-5, p=0.0, seed=0, offset=0, row_offset=0):
        return cls(rows, h, row_offset, dtype, eps, p, seed, offset)


def library_path() -> str:
    return _LIB_PATH


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source of the package for gfx950 and link libsar.so (hipcc cross-compiles without a GPU)."""
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = []
    procs = []
    for src, extra in _SOURCES.items():
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = ["hipcc", *HIPCC_FLAGS, *extra, "-c", os.path.join(_CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, pr in procs:
        out, _ = pr.communicate()
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", _LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
    return _LIB_PATH


_lib = None


def load_library():
    """dlopen libsar.so and declare the prototypes of include/sar.h.  Raises if the library is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} is missing: build it with __graft_entry__.build() "
                                "(there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, u64, sz = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_size_t
    ad, rd = ctypes.POINTER(AttnDesc), ctypes.POINTER(RowsDesc)
    protos = {
        "attn_core_fwd": (ctypes.c_int, [ad, vp, vp, vp, vp, vp, vp]),
        "attn_core_bwd_workspace": (sz, [ad]),
        "attn_core_bwd_workspace_min": (sz, [ad]),
        "attn_core_bwd_recompute_stages": (ctypes.c_int, [ad, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "sar_test_force_variants": (None, [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]),
        "attn_core_bwd_noalloc_max_bytes": (sz, []),
        "attn_core_bwd_recompute_noalloc": (ctypes.c_int, [ad, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "attn_core_bwd_recompute": (ctypes.c_int, [ad, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "attn_core_bwd_recompute_dq": (ctypes.c_int, [ad, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "attn_core_bwd_recompute_dkdv": (ctypes.c_int, [ad, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "attn_core_fwd_stored": (ctypes.c_int, [ad, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "attn_core_bwd_stored": (ctypes.c_int, [ad, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "attn_core_saved_bytes": (u64, [ad, ctypes.c_int]),
        "attn_core_small_buffer_bytes": (u64, [ad]),
        "attn_core_philox_count": (u64, [ad]),
        "ln_fwd": (ctypes.c_int, [rd, vp, vp, vp, vp, vp, vp, vp]),
        "ln_bwd_workspace": (sz, [rd]),
        "ln_bwd": (ctypes.c_int, [rd, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "bias_dropout_add": (ctypes.c_int, [rd, vp, vp, vp, vp, vp, vp]),
        "bias_dropout_add_ln_fwd": (ctypes.c_int, [rd, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "bias_dropout_add_bwd_workspace": (sz, [rd]),
        "bias_dropout_add_bwd": (ctypes.c_int, [rd, vp, vp, vp, vp, sz, vp]),
        "bias_gelu_fwd": (ctypes.c_int, [rd, vp, vp, vp, vp]),
        "bias_gelu_bwd_workspace": (sz, [rd]),
        "bias_gelu_bwd": (ctypes.c_int, [rd, vp, vp, vp, vp, vp, vp, sz, vp]),
        "sar_bench_mfma": (ctypes.c_int, [ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]),
        "sar_bench_copy": (ctypes.c_int, [vp, vp, sz, vp]),
        "sar_bench_issue_name": (ctypes.c_char_p, [ctypes.c_int]),
        "sar_bench_issue": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, vp, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int), vp]),
        "sar_last_error": (ctypes.c_char_p, []),
    }
    for name, (res, args) in protos.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


EXPORTS = ["attn_core_fwd", "attn_core_bwd_workspace", "attn_core_bwd_workspace_min", "attn_core_bwd_recompute",
           "attn_core_bwd_recompute_stages", "sar_test_force_variants", "attn_core_bwd_noalloc_max_bytes",
           "attn_core_bwd_recompute_noalloc", "attn_core_bwd_recompute_dq",
           "attn_core_bwd_recompute_dkdv", "attn_core_fwd_stored",
           "attn_core_bwd_stored", "attn_core_saved_bytes", "attn_core_small_buffer_bytes", "attn_core_philox_count",
           "ln_fwd", "ln_bwd_workspace", "ln_bwd", "bias_dropout_add", "bias_dropout_add_ln_fwd",
           "bias_dropout_add_bwd_workspace", "bias_dropout_add_bwd", "bias_gelu_fwd", "bias_gelu_bwd_workspace", "bias_gelu_bwd",
           "sar_bench_mfma", "sar_bench_copy", "sar_bench_issue_name", "sar_bench_issue", "sar_last_error"]


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int):
    if status != 0:
        raise SarError(status, sar_last_error())


def sar_last_error() -> str:
    return load_library().sar_last_error().decode()


def sar_bench_mfma(iters: int, sink) -> float:
    """Enqueue the matrix-core loop; returns the floating-point operations of the launch."""
    fl = ctypes.c_double(0.0)
    st = load_library().sar_bench_mfma(iters, _ptr(sink), ctypes.byref(fl), _stream())
    if st != 0:
        raise SarError(st, "sar_bench_mfma")
    return fl.value


def sar_bench_issue_names():
    """Names of the issue-cost probes, in probe order."""
    lib, out, i = load_library(), [], 0
    while True:
        n = lib.sar_bench_issue_name(i)
        if n is None:
            return out
        out.append(n.decode())
        i += 1


def sar_bench_issue(probe: int, iters: int, cycles, sink):
    """Enqueues one probe; cycles: int64 device tensor of workgroups * 8 elements.  Returns (insts_a, insts_b)."""
    ia, ib = ctypes.c_int(0), ctypes.c_int(0)
    st = load_library().sar_bench_issue(probe, iters, _ptr(cycles), cycles.numel() // 8, _ptr(sink), ctypes.byref(ia), ctypes.byref(ib), _stream())
    if st != 0:
        raise SarError(st, "sar_bench_issue")
    return ia.value, ib.value


def sar_bench_copy(src, dst):
    n = src.numel() * src.element_size()
    st = load_library().sar_bench_copy(_ptr(src), _ptr(dst), n, _stream())
    if st != 0:
        raise SarError(st, "sar_bench_copy")


def attn_core_fwd(desc: AttnDesc, q, k, v, o, lse):
    _check(load_library().attn_core_fwd(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _stream()))


def attn_core_bwd_workspace(desc: AttnDesc) -> int:
    return int(load_library().attn_core_bwd_workspace(ctypes.byref(desc)))


def attn_core_bwd_workspace_min(desc: AttnDesc) -> int:
    return int(load_library().attn_core_bwd_workspace_min(ctypes.byref(desc)))


def sar_test_force_variants(fwd_128_rows: int = -1, fwd_loader_waves: int = -1, dq_loader_waves: int = -1, dkdv_pipelined: int = -1):
    load_library().sar_test_force_variants(fwd_128_rows, fwd_loader_waves, dq_loader_waves, dkdv_pipelined)


def attn_core_bwd_recompute_stages(desc: AttnDesc, stages: int, q, k, v, o, lse, d_o, dq, dk, dv, workspace):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().attn_core_bwd_recompute_stages(ctypes.byref(desc), stages, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                                          _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace), nbytes, _stream()))


def attn_core_bwd_noalloc_max_bytes() -> int:
    return int(load_library().attn_core_bwd_noalloc_max_bytes())


def attn_core_bwd_recompute_noalloc(desc: AttnDesc, q, k, v, o, lse, d_o, dq, dk, dv):
    _check(load_library().attn_core_bwd_recompute_noalloc(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                                           _ptr(dq), _ptr(dk), _ptr(dv), _stream()))


def attn_core_bwd_recompute(desc: AttnDesc, q, k, v, o, lse, d_o, dq, dk, dv, workspace):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().attn_core_bwd_recompute(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                                   _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace), nbytes, _stream()))


def attn_core_bwd_recompute_dq(desc: AttnDesc, q, k, v, o, lse, d_o, dq, workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().attn_core_bwd_recompute_dq(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq),
                                                      _ptr(workspace), nbytes, _stream()))


def attn_core_bwd_recompute_dkdv(desc: AttnDesc, q, k, v, lse, d_o, dk, dv, workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().attn_core_bwd_recompute_dkdv(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(lse), _ptr(d_o), _ptr(dk), _ptr(dv),
                                                        _ptr(workspace), nbytes, _stream()))


def attn_core_fwd_stored(desc: AttnDesc, q, k, v, o, lse, P, M, D):
    _check(load_library().attn_core_fwd_stored(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(P), _ptr(M), _ptr(D), _stream()))


def attn_core_bwd_stored(desc: AttnDesc, q, k, v, o, P, M, D, d_o, dq, dk, dv, workspace):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().attn_core_bwd_stored(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(P), _ptr(M), _ptr(D), _ptr(d_o),
                                                _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace), nbytes, _stream()))


def attn_core_saved_bytes(desc: AttnDesc, selective: bool) -> int:
    return int(load_library().attn_core_saved_bytes(ctypes.byref(desc), 1 if selective else 0))


def attn_core_small_buffer_bytes(desc: AttnDesc) -> int:
    return int(load_library().attn_core_small_buffer_bytes(ctypes.byref(desc)))


def attn_core_philox_count(desc: AttnDesc) -> int:
    return int(load_library().attn_core_philox_count(ctypes.byref(desc)))


def ln_fwd(desc: RowsDesc, x, gamma, beta, y, mean, rstd):
    _check(load_library().ln_fwd(ctypes.byref(desc), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(mean), _ptr(rstd), _stream()))


def ln_bwd_workspace(desc: RowsDesc) -> int:
    return int(load_library().ln_bwd_workspace(ctypes.byref(desc)))


def ln_bwd(desc: RowsDesc, dy, x, mean, rstd, gamma, dx, dgamma, dbeta, workspace):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().ln_bwd(ctypes.byref(desc), _ptr(dy), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(dx), _ptr(dgamma), _ptr(dbeta),
                                  _ptr(workspace), nbytes, _stream()))


def bias_dropout_add(desc: RowsDesc, x, bias, resid, out, mask_out=None):
    _check(load_library().bias_dropout_add(ctypes.byref(desc), _ptr(x), _ptr(bias), _ptr(resid), _ptr(out), _ptr(mask_out), _stream()))


def bias_dropout_add_ln_fwd(desc: RowsDesc, x, bias, resid, gamma, beta, out, y, mean, rstd):
    _check(load_library().bias_dropout_add_ln_fwd(ctypes.byref(desc), _ptr(x), _ptr(bias), _ptr(resid), _ptr(gamma), _ptr(beta), _ptr(out),
                                                   _ptr(y), _ptr(mean), _ptr(rstd), _stream()))


def bias_dropout_add_bwd_workspace(desc: RowsDesc) -> int:
    return int(load_library().bias_dropout_add_bwd_workspace(ctypes.byref(desc)))


def bias_dropout_add_bwd(desc: RowsDesc, dout, dx, dbias=None, workspace=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().bias_dropout_add_bwd(ctypes.byref(desc), _ptr(dout), _ptr(dx), _ptr(dbias), _ptr(workspace), nbytes, _stream()))


def bias_gelu_fwd(desc: RowsDesc, x, bias, y):
    _check(load_library().bias_gelu_fwd(ctypes.byref(desc), _ptr(x), _ptr(bias), _ptr(y), _stream()))


def bias_gelu_bwd_workspace(desc: RowsDesc) -> int:
    return int(load_library().bias_gelu_bwd_workspace(ctypes.byref(desc)))


def bias_gelu_bwd(desc: RowsDesc, dy, x, bias, dx, dbias=None, workspace=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().bias_gelu_bwd(ctypes.byref(desc), _ptr(dy), _ptr(x), _ptr(bias), _ptr(dx), _ptr(dbias), _ptr(workspace), nbytes, _stream()))
