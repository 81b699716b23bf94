"""Activation-byte and FLOP accounting of the paper, written out term by term (TEST INFRASTRUCTURE ONLY).

All byte counts assume the paper's storage convention (Section 4): 2 bytes per activation element,
1 byte per dropout-mask element, small buffers (LayerNorm statistics) ignored.  Integers throughout,
so that results can be compared bit for bit with what the GPU library reports.
"""
from __future__ import annotations

from fractions import Fraction


# ------------------------------------------------------------------ per-layer activation bytes
def attention_block_items(s: int, b: int, h: int, a: int, elem: int = 2) -> dict:
    """Itemised storage of the attention block without parallelism (Section 4.1, "Attention block")."""
    sbh = s * b * h
    as2b = a * s * s * b
    return {
        "qkv_input": elem * sbh,            # shared input of the Q, K, V matrix multiplies
        "qk_t": 2 * elem * sbh,             # Q and K
        "softmax_out": elem * as2b,         # softmax output
        "softmax_dropout_mask": as2b,       # 1 byte per element
        "dropout_out": elem * as2b,         # input of the product with V
        "values": elem * sbh,               # V
        "projection_input": elem * sbh,     # linear projection stores its input
        "attention_dropout_mask": sbh,      # 1 byte per element
    }


def mlp_block_items(s: int, b: int, h: int, elem: int = 2) -> dict:
    """Section 4.1, "MLP": two linear inputs, GeLU input, dropout mask."""
    sbh = s * b * h
    return {"linear1_input": elem * sbh, "linear2_input": 4 * elem * sbh, "gelu_input": 4 * elem * sbh, "dropout_mask": sbh}


def layernorm_items(s: int, b: int, h: int, elem: int = 2) -> dict:
    """Section 4.1, "Layer norm": two layer norms, each stores its input."""
    sbh = s * b * h
    return {"ln1_input": elem * sbh, "ln2_input": elem * sbh}


def act_bytes_no_parallel(s, b, h, a) -> int:
    """Eq. 1: sbh(34 + 5as/h)."""
    return 34 * s * b * h + 5 * a * s * s * b


def act_bytes_tp(s, b, h, a, t) -> Fraction:
    """Eq. 2: sbh(10 + 24/t + 5as/(ht))."""
    return Fraction(10 * s * b * h) + Fraction(24 * s * b * h, t) + Fraction(5 * a * s * s * b, t)


def act_bytes_tp_sp(s, b, h, a, t) -> Fraction:
    """Eq. 4: (sbh/t)(34 + 5as/h)."""
    return Fraction(34 * s * b * h + 5 * a * s * s * b, t)


def act_bytes_tp_selective(s, b, h, a, t) -> Fraction:
    """Table 2, tensor parallel + selective recomputation: sbh(10 + 24/t)."""
    return Fraction(10 * s * b * h) + Fraction(24 * s * b * h, t)


def act_bytes_tp_sp_selective(s, b, h, a, t) -> Fraction:
    """Table 2 / Eq. 6 per layer: 34 sbh/t."""
    return Fraction(34 * s * b * h, t)


def act_bytes_full_recompute(s, b, h) -> int:
    """Table 2, full activation recomputation: 2 sbh (layer input only)."""
    return 2 * s * b * h


def interleave_factor(p: int, m: int) -> Fraction:
    """Section 4.2.3: interleaved schedule stores L(1 + (p-1)/(pm)) layers of activations."""
    return 1 + Fraction(p - 1, p * m)


def total_act_bytes_first_stage(s, b, h, a, L, t, p, v, selective: bool = False) -> Fraction:
    """Eq. 5 (or Eq. 6 with selective recomputation) plus the embedding / head extras of Section 4.3."""
    per_layer = act_bytes_tp_sp_selective(s, b, h, a, t) if selective else act_bytes_tp_sp(s, b, h, a, t)
    extra = Fraction(s * b * h * p, t)
    if p == 1:
        extra += Fraction(4 * s * b * h, t) * (1 + Fraction(v, h))
    return per_layer * L + extra


# ------------------------------------------------------------------ attention core, one GPU's share
def attn_core_saved_bytes(s, b, h, a, t, selective: bool, elem: int = 2) -> int:
    """Bytes the attention core keeps from forward to backward on one tensor-parallel rank.

    Stored path (Section 4.1): Q, K, V (6sbh/t), the core's output = projection input (2sbh/t), softmax
    output, mask, dropout output (5 a s^2 b / t).  Selective path (Section 5): the s^2 terms vanish.
    """
    A = a // t
    d = h // a
    qkvo = 4 * elem * s * b * A * d
    if selective:
        return qkvo
    return qkvo + (2 * elem + 1) * A * s * s * b


def attn_core_small_buffers(s, b, a, t) -> int:
    """Not in the paper's count ("small buffers", Section 4): fp32 log-sum-exp per row + 16 B seed/offset."""
    return 4 * (a // t) * s * b + 16


# ------------------------------------------------------------------ FLOPs (Appendix A)
def layer_forward_flops(B, s, h) -> int:
    """Appendix A: 24 B s h^2 + 4 B s^2 h per layer, forward."""
    return 24 * B * s * h * h + 4 * B * s * s * h


def model_flops(B, L, s, h, v) -> int:
    """Eq. 7 = 3 x (L layers forward + logits 2Bshv)."""
    return 3 * (L * layer_forward_flops(B, s, h) + 2 * B * s * h * v)


def hardware_flops(B, L, s, h, v) -> int:
    """Eq. 8 as printed: 72BLsh^2 (1 + s/3h + v/12hL), i.e. Eq. 7 + 12 B L s^2 h.

    The sentence before Eq. 8 counts the recomputation as one extra attention forward (4 B s^2 h per
    layer), which would add only s/18h inside the bracket; the printed equation adds s/6h, three times
    that.  The printed form is the one that reproduces the HFU column of Table 5 and the 2.7 % / 1.6 %
    overheads of Section 5, so it is the one taken here."""
    return model_flops(B, L, s, h, v) + 12 * B * L * s * s * h


def hardware_flops_text_reading(B, L, s, h, v) -> int:
    """The other reading: Eq. 7 plus exactly one more QK^T and attention-over-V product per layer."""
    return model_flops(B, L, s, h, v) + L * 4 * B * s * s * h


def model_flops_closed_form(B, L, s, h, v) -> Fraction:
    return 72 * B * L * s * h * h * (1 + Fraction(s, 6 * h) + Fraction(v, 12 * h * L))


def hardware_flops_closed_form(B, L, s, h, v) -> Fraction:
    return 72 * B * L * s * h * h * (1 + Fraction(s, 3 * h) + Fraction(v, 12 * h * L))


# ------------------------------------------------------------------ attention core FLOPs on one GPU, causal
def attn_core_flops(s, b, A, d, causal: bool = True) -> dict:
    """Dense-contraction FLOPs of the core on N = b*A heads; a causal core touches T = s(s+1)/2 pairs.

    forward: QK^T and PV (2 contractions); backward with recomputation as a fused kernel needs 5
    (QK^T again, dO V^T, D^T dO, dS K, dS^T Q); the paper's convention (Appendix A, Eq. 8) counts the
    recomputation as a whole extra forward, i.e. 6."""
    N = b * A
    pairs = s * (s + 1) // 2 if causal else s * s
    one = 2 * d * pairs * N
    return {"fwd": 2 * one, "bwd_fused": 5 * one, "bwd_paper": 6 * one, "bwd_stored": 4 * one}
