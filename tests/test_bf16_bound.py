"""CPU: why the bf16 attention outputs are judged by |x - ref| <= 2e-2 RMS(ref) + 2^-8 (sum|terms| + |ref|).

An ideal pipeline is emulated in numpy on top of the oracle's exact fp64 tensors: exact scores and row sums, the
un-normalised probabilities rounded once to bf16 (they must be, to enter the matrix core), an exact product with V, the
result rounded once to bf16.  No implementation that stores bf16 can do better.  On the benchmark's input recipe it
  - misses the stated bar max|x - ref| <= 2e-2 RMS(ref) by a wide margin (first rows are ~sqrt(s) times the RMS),
  - also misses 2e-2 RMS + 2^-8 sum|terms| once s is large (unit roundoff of bf16 is 2^-8, and there are two roundings),
  - and always meets the bar the GPU tests use.
"""
import os
import sys

import numpy as np

import oracle
from paper_2205_05198_amd.workloads import attn_inputs, round_bf16

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def _ideal_forward(s, d, seed):
    sh = oracle.AttnShape(s=s, b=1, a=1, h=d, p=0.1, seed=1234, offset=5)
    q, k, v, _ = attn_inputs(s, 1, 1, d, "bf16", seed=seed)
    f = oracle.attn_fwd(sh, q, k, v, materialise=True, heads=(0, 1))
    M, D = f["M"][0].astype(np.float64), f["D"][0]
    Q, K, V = (np.asarray(a[:, 0, 0], dtype=np.float64) for a in (q, k, v))
    S = sh.alpha() * (Q @ K.T)
    S[np.triu_indices(s, 1)] = -np.inf
    Pt = np.exp(S - S.max(1, keepdims=True))
    l = Pt.sum(1, keepdims=True)
    Ptr = round_bf16(Pt.astype(np.float32)).astype(np.float64)
    c = 1.0 / (1.0 - float(np.float32(sh.p)))
    O = round_bf16(((Ptr * M) @ V * c / l).astype(np.float32)).astype(np.float64)
    return O, f["o"][:, 0, 0], D @ np.abs(V)


def test_ideal_bf16_pipeline_against_the_three_bars():
    from gpu_util import err_attn_bf16, err_attn_blocks
    worst_old = 0.0
    for s in (1024, 4096):
        O, ref, scale = _ideal_forward(s, 160, seed=67)
        rms = float(np.sqrt(np.mean(ref ** 2)))
        stated = float(np.max(np.abs(O - ref)) / rms)
        old = float(np.max(np.abs(O - ref) / (2e-2 * rms + 2.0 ** -8 * scale)))
        used = err_attn_bf16(O, ref, scale)
        blocks = err_attn_blocks(O, ref)
        print(f"s={s}: stated bar needs {stated:.3f} (bar 2e-2), one-rounding bound {old:.3f}, bound used {used:.3f}, block RMS {blocks:.2f} x 2^-9")
        assert stated > 2e-2          # the stated bar alone is out of reach of any bf16 store
        assert used <= 1.0            # two roundings at unit roundoff 2^-8 are covered
        assert 0.5 < blocks < 2.0     # and their RMS over a 64-row block is about 1.2 x 2^-9 of the block's RMS
        worst_old = max(worst_old, old)
    assert worst_old > 0.95           # a single rounding unit is (nearly) used up by the ideal pipeline already
