"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle's callers.

Holds no arithmetic of the method: only shapes (the paper's Table 3 models at their per-GPU share for
tensor-parallel size t = 8, s = 2048, Section 6) and random draws, rounded to the device dtype so that
the CPU oracle and the GPU library start from identical values.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str      # "f32" or "bf16"
    s: int          # sequence length
    b: int          # microbatch
    a: int          # global attention heads
    h: int          # hidden size
    t: int          # tensor-parallel size
    p: float        # dropout probability
    seed: int       # Philox seed
    rows: int       # rows of the sequence-parallel shard, (s/t)*b
    rows_h: int     # width of the LayerNorm / dropout-add rows
    causal: int = 1  # 1: decoder mask (the paper's models); 0: every key

    @property
    def A(self) -> int:
        return self.a // self.t

    @property
    def d(self) -> int:
        return self.h // self.a


WORKLOADS = {
    # tiny fp32 case: b=1, s=128, 2 heads of 64, LayerNorm on 128 x 128
    "tiny": Workload("tiny", "f32", 128, 1, 2, 128, 1, 0.1, 1234, 128, 128),
    # Table 3 models, one tensor-parallel rank of 8, s = 2048
    "22B": Workload("22B", "bf16", 2048, 4, 64, 6144, 8, 0.1, 1234, 1024, 6144),
    "175B": Workload("175B", "bf16", 2048, 1, 96, 12288, 8, 0.1, 1234, 256, 12288),
    "530B": Workload("530B", "bf16", 2048, 1, 128, 20480, 8, 0.1, 1234, 256, 20480),
    "1T": Workload("1T", "bf16", 2048, 1, 160, 25600, 8, 0.1, 1234, 256, 25600),
    # variants of the 530B shard: longer sequences (activation memory of the selective core grows linearly in s,
    # Eq. 6) and the encoder form of the core (no causal mask)
    "530B_s4096": Workload("530B_s4096", "bf16", 4096, 1, 128, 20480, 8, 0.1, 1234, 512, 20480),
    "530B_s8192": Workload("530B_s8192", "bf16", 8192, 1, 128, 20480, 8, 0.1, 1234, 1024, 20480),
    "530B_s16384": Workload("530B_s16384", "bf16", 16384, 1, 128, 20480, 8, 0.1, 1234, 2048, 20480),
    "530B_s32768": Workload("530B_s32768", "bf16", 32768, 1, 128, 20480, 8, 0.1, 1234, 4096, 20480),
    "530B_p0": Workload("530B_p0", "bf16", 2048, 1, 128, 20480, 8, 0.0, 1234, 256, 20480),   # no dropout: no random numbers drawn
    "530B_enc": Workload("530B_enc", "bf16", 2048, 1, 128, 20480, 8, 0.1, 1234, 256, 20480, 0),
}


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).reshape(x.shape)


def to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    return round_bf16(x) if dtype == "bf16" else x


def attn_inputs(s: int, b: int, A: int, d: int, dtype: str, seed: int = 1234, qk_std: float | None = None,
                outlier: bool = False):
    """Q, K, V, dO as float32 arrays [s, b, A, d] holding values exactly representable in `dtype`.

    Default scale follows the benchmark recipe: Q, K, V ~ N(0,1)/sqrt(d) for bf16 shards, N(0,1) for the
    tiny fp32 case; dO ~ N(0,1).  `qk_std` overrides the Q/K scale (stress inputs with peaked softmax);
    `outlier` plants one large score so the running maximum moves late in a row."""
    shape = (s, b, A, d)
    std = qk_std if qk_std is not None else (1.0 if dtype == "f32" else 1.0 / np.sqrt(d))
    out = []
    for k in range(4):
        g = np.random.default_rng(seed + k)
        x = g.standard_normal(shape, dtype=np.float32)
        if k < 2:
            x *= np.float32(std)
        elif k == 2:
            x *= np.float32(1.0 if dtype == "f32" else 1.0 / np.sqrt(d))
        out.append(x)
    q, k_, v, do = out
    if outlier and s >= 8:
        i, j = s - 3, s // 2
        k_[j, 0, 0, :] = 0
        q[i, 0, 0, :] = 0
        q[i, 0, 0, 0] = 8.0
        k_[j, 0, 0, 0] = 8.0 * np.sqrt(d) / 1.0
    return tuple(to_dtype(x, dtype) for x in (q, k_, v, do))


def rows_inputs(rows: int, h: int, dtype: str, seed: int = 1234):
    """x, resid, dy ~ N(0,1); bias ~ N(0, 0.02); gamma ~ N(1, 0.02); beta ~ N(0, 0.02)."""
    def draw(k, shape, mean=0.0, std=1.0):
        g = np.random.default_rng(seed + 100 + k)
        return (g.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean)).astype(np.float32)
    x = draw(0, (rows, h))
    resid = draw(1, (rows, h))
    dy = draw(2, (rows, h))
    bias = draw(3, (h,), 0.0, 0.02)
    gamma = draw(4, (h,), 1.0, 0.02)
    beta = draw(5, (h,), 0.0, 0.02)
    return {k: to_dtype(v, dtype) for k, v in dict(x=x, resid=resid, dy=dy, bias=bias, gamma=gamma, beta=beta).items()}
