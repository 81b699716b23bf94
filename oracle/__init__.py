"""fp64 CPU oracle (TEST INFRASTRUCTURE ONLY).

Thin ctypes loader for ``sar_oracle.c`` plus the closed-form accounting of ``accounting.py``.
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package; the product path never does.  Nothing here imports the GPU package.

Arrays are numpy float64, C-contiguous.  Attention tensors use the paper's layout
``[s, b, A, d]`` (Section 3: activations are ``s x b x h``; one GPU holds ``A = a/t`` heads).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

from . import accounting  # noqa: F401  (re-export)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sar_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

CFLAGS = ["-O3", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math: fp64 arithmetic stays IEEE, in source order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Desc(ctypes.Structure):
    _fields_ = [
        ("s", ctypes.c_int32), ("b", ctypes.c_int32),
        ("a", ctypes.c_int32), ("t", ctypes.c_int32), ("rank", ctypes.c_int32),
        ("h", ctypes.c_int32),
        ("causal", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("p", ctypes.c_float),
        ("seed", ctypes.c_uint64), ("offset", ctypes.c_uint64),
        ("stride_s", ctypes.c_int64), ("stride_b", ctypes.c_int64), ("stride_a", ctypes.c_int64),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_num_threads.restype = ctypes.c_int
        _lib.orc_dropout_threshold.restype = ctypes.c_uint32
        _lib.orc_dropout_threshold.argtypes = [ctypes.c_float]
        _lib.orc_keep_bit.restype = ctypes.c_uint8
        _lib.orc_keep_bit.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32]
        _lib.orc_attn_philox_count.restype = ctypes.c_uint64
        _lib.orc_attn_fwd.restype = ctypes.c_int
        _lib.orc_attn_bwd.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


@dataclass
class AttnShape:
    """Paper notation (Table 1): s, b, a, h, t; this shard's rank; d = h/a; A = a/t local heads."""
    s: int
    b: int
    a: int
    h: int
    t: int = 1
    rank: int = 0
    causal: int = 1
    scale: float | None = None
    p: float = 0.0
    seed: int = 0
    offset: int = 0

    @property
    def A(self) -> int:
        return self.a // self.t

    @property
    def d(self) -> int:
        return self.h // self.a

    def alpha(self) -> float:
        return float(np.float32(1.0 / np.sqrt(self.d))) if self.scale is None else float(np.float32(self.scale))

    def _c(self) -> _Desc:
        A, d = self.A, self.d
        return _Desc(self.s, self.b, self.a, self.t, self.rank, self.h, self.causal, self.alpha(), float(np.float32(self.p)),
                     self.seed, self.offset, self.b * A * d, A * d, d)


def _dp(x):
    return x.ctypes.data_as(ctypes.c_void_p) if x is not None else None


def _f64(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    return x


def philox4x32_10(ctr, key):
    c = (ctypes.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    out = (ctypes.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, out)
    return [int(v) for v in out]


def dropout_threshold(p: float) -> int:
    return int(lib().orc_dropout_threshold(float(np.float32(p))))


def keep_bit(seed: int, offset: int, e: int, site: int, T: int) -> int:
    return int(lib().orc_keep_bit(seed, offset, e, site, T))


def attn_mask(sh: AttnShape) -> np.ndarray:
    """Raw softmax-dropout mask of this shard, uint8 [b, A, s, s] (also above the diagonal)."""
    M = np.empty((sh.b, sh.A, sh.s, sh.s), dtype=np.uint8)
    d = sh._c()
    lib().orc_attn_mask(ctypes.byref(d), _dp(M))
    return M


def attn_philox_count(sh: AttnShape) -> int:
    d = sh._c()
    return int(lib().orc_attn_philox_count(ctypes.byref(d)))


def attn_fwd(sh: AttnShape, q, k, v, materialise: bool = False, heads=None):
    """Returns dict(o [s,b,A,d], lse [b,A,s], and with materialise: P, M, D [b,A,s,s]).

    ``heads`` = (lo, hi) restricts the work to flattened (batch*A + head) indices in [lo, hi); the
    other entries of o and lse stay zero, and P, M, D then have shape [hi-lo, s, s]."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    assert q.shape == (sh.s, sh.b, sh.A, sh.d) == k.shape == v.shape
    o = np.zeros_like(q)
    lse = np.zeros((sh.b, sh.A, sh.s), dtype=np.float64)
    P = M = D = None
    lo, hi = heads if heads is not None else (0, sh.b * sh.A)
    if materialise:
        shape = (sh.b, sh.A, sh.s, sh.s) if heads is None else (hi - lo, sh.s, sh.s)
        P = np.zeros(shape, dtype=np.float64)
        D = np.zeros_like(P)
        M = np.zeros(P.shape, dtype=np.uint8)
    d = sh._c()
    rc = lib().orc_attn_fwd(ctypes.byref(d), _dp(q), _dp(k), _dp(v), _dp(o), _dp(lse), _dp(P), _dp(M), _dp(D),
                            ctypes.c_int(lo), ctypes.c_int(hi))
    if rc != 0:
        raise MemoryError("oracle attn_fwd: allocation failed")
    out = {"o": o, "lse": lse}
    if materialise:
        out.update(P=P, M=M, D=D)
    return out


def attn_bwd(sh: AttnShape, q, k, v, dO, extras: bool = False, heads=None):
    """Returns dict(dq, dk, dv [s,b,A,d]; with extras: delta [b,A,s], dS [b,A,s,s])."""
    q, k, v, dO = _f64(q), _f64(k), _f64(v), _f64(dO)
    assert q.shape == (sh.s, sh.b, sh.A, sh.d) == k.shape == v.shape == dO.shape
    dq, dk, dv = np.zeros_like(q), np.zeros_like(q), np.zeros_like(q)
    delta = dS = None
    lo, hi = heads if heads is not None else (0, sh.b * sh.A)
    if extras:
        delta = np.zeros((sh.b, sh.A, sh.s), dtype=np.float64)
        dS = np.zeros((sh.b, sh.A, sh.s, sh.s) if heads is None else (hi - lo, sh.s, sh.s), dtype=np.float64)
    d = sh._c()
    rc = lib().orc_attn_bwd(ctypes.byref(d), _dp(q), _dp(k), _dp(v), _dp(dO), _dp(dq), _dp(dk), _dp(dv), _dp(delta), _dp(dS),
                            ctypes.c_int(lo), ctypes.c_int(hi))
    if rc != 0:
        raise MemoryError("oracle attn_bwd: allocation failed")
    out = {"dq": dq, "dk": dk, "dv": dv}
    if extras:
        out.update(delta=delta, dS=dS)
    return out


def ln_fwd(x, gamma, beta, eps: float = 1e-5):
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    rows, h = x.shape
    y = np.empty_like(x)
    mean = np.empty(rows, dtype=np.float64)
    rstd = np.empty(rows, dtype=np.float64)
    lib().orc_ln_fwd(ctypes.c_int64(rows), ctypes.c_int64(h), ctypes.c_double(eps), _dp(x), _dp(gamma), _dp(beta), _dp(y), _dp(mean), _dp(rstd))
    return {"y": y, "mean": mean, "rstd": rstd}


def ln_bwd(dy, x, gamma, eps: float = 1e-5):
    dy, x, gamma = _f64(dy), _f64(x), _f64(gamma)
    rows, h = x.shape
    dx = np.empty_like(x)
    dgamma = np.empty(h, dtype=np.float64)
    dbeta = np.empty(h, dtype=np.float64)
    lib().orc_ln_bwd(ctypes.c_int64(rows), ctypes.c_int64(h), ctypes.c_double(eps), _dp(dy), _dp(x), _dp(gamma), _dp(dx), _dp(dgamma), _dp(dbeta))
    return {"dx": dx, "dgamma": dgamma, "dbeta": dbeta}


def bias_dropout_add(x, bias, resid, p: float, seed: int, offset: int, row_offset: int = 0):
    x, resid = _f64(x), _f64(resid)
    bias = _f64(bias) if bias is not None else None
    rows, h = x.shape
    out = np.empty_like(x)
    mask = np.empty((rows, h), dtype=np.uint8)
    lib().orc_bias_dropout_add(ctypes.c_int64(rows), ctypes.c_int64(h), ctypes.c_int64(row_offset), ctypes.c_float(float(np.float32(p))),
                               ctypes.c_uint64(seed), ctypes.c_uint64(offset), _dp(x), _dp(bias), _dp(resid), _dp(out), _dp(mask))
    return {"out": out, "mask": mask}


def bias_dropout_add_bwd(dout, p: float, seed: int, offset: int, row_offset: int = 0):
    dout = _f64(dout)
    rows, h = dout.shape
    dx = np.empty_like(dout)
    dresid = np.empty_like(dout)
    dbias = np.empty(h, dtype=np.float64)
    lib().orc_bias_dropout_add_bwd(ctypes.c_int64(rows), ctypes.c_int64(h), ctypes.c_int64(row_offset), ctypes.c_float(float(np.float32(p))),
                                   ctypes.c_uint64(seed), ctypes.c_uint64(offset), _dp(dout), _dp(dx), _dp(dresid), _dp(dbias))
    return {"dx": dx, "dresid": dresid, "dbias": dbias}


def bias_gelu_fwd(x, bias=None):
    """y = GeLU(x + bias), exact (erf) form; Section 4.1's MLP non-linearity."""
    x = _f64(x)
    bias = _f64(bias) if bias is not None else None
    rows, h = x.shape
    y = np.empty_like(x)
    lib().orc_bias_gelu_fwd(ctypes.c_int64(rows), ctypes.c_int64(h), _dp(x), _dp(bias), _dp(y))
    return y


def bias_gelu_bwd(dy, x, bias=None):
    """dx = dy GeLU'(x + bias), dbias = column sums of dx."""
    dy, x = _f64(dy), _f64(x)
    bias = _f64(bias) if bias is not None else None
    rows, h = x.shape
    dx = np.empty_like(x)
    dbias = np.empty(h, dtype=np.float64)
    lib().orc_bias_gelu_bwd(ctypes.c_int64(rows), ctypes.c_int64(h), _dp(dy), _dp(x), _dp(bias), _dp(dx), _dp(dbias))
    return {"dx": dx, "dbias": dbias}
