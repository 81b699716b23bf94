"""Host-side planner: how much activation memory and how many extra FLOPs each recomputation strategy of the
paper costs for a model and a parallel layout, and which strategy to pick under a memory budget.

Pure integer / rational arithmetic on the paper's closed forms (Sections 4, 5 and Appendix A); no GPU, no
dependency on the rest of the package.  Storage convention of Section 4: 2 bytes per activation element, 1 byte per
dropout-mask element, LayerNorm statistics and the like ignored.
"""
from __future__ import annotations

from dataclasses import dataclass
from fractions import Fraction

STRATEGIES = ("tp", "tp_sp", "tp_selective", "tp_sp_selective", "full")


@dataclass(frozen=True)
class Model:
    """Table 1 / Table 3 notation: hidden size, heads, layers, vocabulary, sequence length."""
    h: int
    a: int
    L: int
    v: int = 51200
    s: int = 2048


@dataclass(frozen=True)
class Layout:
    """b = microbatch, t = tensor-parallel size, p = pipeline-parallel size, m = interleaving stages (1 = none)."""
    b: int
    t: int
    p: int = 1
    m: int = 1


def layer_activation_bytes(mod: Model, lay: Layout, strategy: str) -> Fraction:
    """Per-layer activation bytes on one GPU (Table 2)."""
    s, b, h, a, t = mod.s, lay.b, mod.h, mod.a, lay.t
    sbh = s * b * h
    core = Fraction(5 * a * s * s * b, t)            # softmax output, its dropout mask, dropout output (Section 4.1)
    if strategy == "tp":                             # Eq. 2
        return 10 * sbh + Fraction(24 * sbh, t) + core
    if strategy == "tp_sp":                          # Eq. 4
        return Fraction(34 * sbh, t) + core
    if strategy == "tp_selective":                   # Table 2: Eq. 2 without the attention-core term
        return 10 * sbh + Fraction(24 * sbh, t)
    if strategy == "tp_sp_selective":                # Eq. 6 per layer
        return Fraction(34 * sbh, t)
    if strategy == "full":                           # only the layer input is kept
        return Fraction(2 * sbh)
    raise ValueError(f"unknown strategy {strategy!r}; one of {STRATEGIES}")


def first_stage_activation_bytes(mod: Model, lay: Layout, strategy: str) -> Fraction:
    """Activation bytes of the first pipeline stage, the one that holds the most (Section 4.2.3, Eq. 5 / 6):
    L layers' worth for the non-interleaved 1F1B schedule, L(1 + (p-1)/(pm)) with interleaving, plus the
    embedding dropout mask (sbhp/t) and, without pipeline parallelism, the output layer's extras (Section 4.3)."""
    s, b, h, t, p = mod.s, lay.b, mod.h, lay.t, lay.p
    layers = mod.L * (1 + Fraction(p - 1, p * lay.m)) if lay.m > 1 else Fraction(mod.L)
    total = layer_activation_bytes(mod, lay, strategy) * layers
    total += Fraction(s * b * h * p, t)
    if p == 1:
        total += Fraction(4 * s * b * h, t) * (1 + Fraction(mod.v, h))
    return total


def model_flops(mod: Model, B: int) -> int:
    """Eq. 7: forward + backward of L layers (24Bsh^2 + 4Bs^2h each, forward) and the logits (2Bshv)."""
    s, h = mod.s, mod.h
    return 3 * (mod.L * (24 * B * s * h * h + 4 * B * s * s * h) + 2 * B * s * h * mod.v)


def hardware_flops(mod: Model, B: int, strategy: str) -> int:
    """FLOPs actually executed: Eq. 7 without recomputation, Eq. 8 as printed with selective recomputation, and one
    more forward pass of every layer with full recomputation."""
    s, h = mod.s, mod.h
    base = model_flops(mod, B)
    if strategy in ("tp", "tp_sp"):
        return base
    if strategy in ("tp_selective", "tp_sp_selective"):
        return base + 12 * B * mod.L * s * s * h
    if strategy == "full":
        return base + mod.L * (24 * B * s * h * h + 4 * B * s * s * h)
    raise ValueError(f"unknown strategy {strategy!r}; one of {STRATEGIES}")


def flops_overhead(mod: Model, strategy: str) -> Fraction:
    """hardware / model FLOPs - 1 (independent of the batch size)."""
    return Fraction(hardware_flops(mod, 1, strategy), model_flops(mod, 1)) - 1


def plan(mod: Model, lay: Layout, activation_budget_bytes: int, sequence_parallel: bool = True) -> dict:
    """The cheapest strategy (in executed FLOPs) whose first-stage activations fit the budget: nothing recomputed,
    then the attention core only (Section 5), then everything.  Returns the choice with its bytes and overhead;
    'fits' is False if even full recomputation does not fit."""
    order = ("tp_sp", "tp_sp_selective", "full") if sequence_parallel else ("tp", "tp_selective", "full")
    rows = [{"strategy": st, "bytes": first_stage_activation_bytes(mod, lay, st), "flops_overhead": flops_overhead(mod, st)} for st in order]
    for r in rows:
        if r["bytes"] <= activation_budget_bytes:
            return {**r, "fits": True, "considered": rows}
    return {**rows[-1], "fits": False, "considered": rows}


def outstanding_microbatches(lay: Layout, stage: int) -> int:
    """Appendix C: microbatches whose back-propagation is still outstanding at pipeline stage `stage`
    (0 = first) in the non-interleaved 1F1B schedule: max(0, p - S)."""
    if stage < 0:
        raise ValueError("stage must be >= 0")
    return max(0, lay.p - stage)


def microbatch_level_plan(mod: Model, lay: Layout, stage: int, activation_budget_bytes: int,
                          checkpointed: str = "tp_sp_selective", stored: str = "tp_sp") -> dict:
    """Appendix C, microbatch-level recomputation: of the w = max(0, p - S) microbatches in flight at a stage, keep
    all activations of as many as the budget allows (`stored` strategy) and checkpoint the rest (`checkpointed`
    strategy); the stored ones form a moving window, so in steady state the same share of all microbatches runs
    without recomputation.  A stage holds L/p layers per microbatch (embedding and output-layer extras are left to
    first_stage_activation_bytes).  Returns the window, the number stored in full, the bytes used, the share of
    microbatches that recompute and the resulting executed-FLOPs overhead; 'fits' is False if even checkpointing
    every microbatch exceeds the budget."""
    if lay.m != 1:
        raise ValueError("Appendix C describes the non-interleaved schedule (m = 1)")
    w = outstanding_microbatches(lay, stage)
    layers = Fraction(mod.L, lay.p)
    full = layer_activation_bytes(mod, lay, stored) * layers
    ckpt = layer_activation_bytes(mod, lay, checkpointed) * layers
    if full < ckpt:
        raise ValueError("the stored strategy must keep at least what the checkpointed one keeps")
    over = flops_overhead(mod, checkpointed)
    if w == 0:
        return {"window": 0, "stored_in_full": 0, "bytes": Fraction(0), "recompute_share": Fraction(0), "flops_overhead": Fraction(0), "fits": True}
    if w * ckpt > activation_budget_bytes:
        return {"window": w, "stored_in_full": 0, "bytes": w * ckpt, "recompute_share": Fraction(1), "flops_overhead": over, "fits": False}
    k = w if full == ckpt else min(w, int((activation_budget_bytes - w * ckpt) // (full - ckpt)))
    share = Fraction(w - k, w)
    return {"window": w, "stored_in_full": k, "bytes": k * full + (w - k) * ckpt, "recompute_share": share, "flops_overhead": share * over, "fits": True}
