"""Pins for the accounting oracle: every figure is one the paper prints (tests/golden/paper_numbers.txt)
or a per-GPU byte count that follows from its Table 2 rows."""
import os
from fractions import Fraction

from oracle import accounting as acc

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_numbers.txt")


def _load():
    vals, models = {}, {}
    for line in open(GOLD):
        line = line.split("#")[0].split()
        if not line:
            continue
        if line[0] == "model":
            name = line[1]
            a, h, L, t, p, gpus, gb, mb = map(int, line[2:10])
            it, mfu, hfu = map(float, line[10:13])
            models[name] = dict(a=a, h=h, L=L, t=t, p=p, gpus=gpus, B=gb, b=mb, iter_s=it, mfu=mfu, hfu=hfu)
        else:
            vals[line[0]] = float(line[1])
    return vals, models


V, MODELS = _load()
S, VOCAB = int(V["seq_len"]), int(V["vocab"])


def test_itemised_sums_equal_closed_forms():
    s, b, h, a = 2048, 4, 6144, 64
    att = acc.attention_block_items(s, b, h, a)
    assert sum(att.values()) == 11 * s * b * h + 5 * a * s * s * b          # Section 4.1
    assert sum(acc.mlp_block_items(s, b, h).values()) == 19 * s * b * h       # Section 4.1
    assert sum(acc.layernorm_items(s, b, h).values()) == 4 * s * b * h        # Section 4.1
    total = sum(att.values()) + 19 * s * b * h + 4 * s * b * h
    assert total == acc.act_bytes_no_parallel(s, b, h, a)                     # Eq. 1
    t = 8
    assert acc.act_bytes_tp(s, b, h, a, 1) == acc.act_bytes_no_parallel(s, b, h, a)
    assert acc.act_bytes_tp_sp(s, b, h, a, t) * t == acc.act_bytes_no_parallel(s, b, h, a)  # Eq. 4 = Eq. 1 / t
    # the 10 sbh of Eq. 2 is exactly the replicated LayerNorm inputs and the two dropout masks
    assert acc.act_bytes_tp(s, b, h, a, t) - acc.act_bytes_tp_sp(s, b, h, a, t) == Fraction(10 * s * b * h * (t - 1), t)
    # selective recomputation removes exactly the 5 a s^2 b / t term
    assert acc.act_bytes_tp_sp(s, b, h, a, t) - acc.act_bytes_tp_sp_selective(s, b, h, a, t) == Fraction(5 * a * s * s * b, t)
    assert acc.act_bytes_tp(s, b, h, a, t) - acc.act_bytes_tp_selective(s, b, h, a, t) == Fraction(5 * a * s * s * b, t)


def test_worked_examples_of_section5():
    g, m = MODELS["175B"], MODELS["530B"]
    assert Fraction(5 * g["a"] * S, g["h"]) == V["gpt3_5as_over_h"]
    assert Fraction(5 * m["a"] * S, m["h"]) == V["mtnlg_5as_over_h"]
    for mod, key in ((g, "gpt3"), (m, "mtnlg")):
        full = acc.act_bytes_tp_sp(S, 1, mod["h"], mod["a"], 8)
        sel = acc.act_bytes_tp_sp_selective(S, 1, mod["h"], mod["a"], 8)
        assert round(float(100 * (1 - sel / full))) == V[key + "_selective_saving_pct"]
        # FLOPs overhead ~ s/6h (Eq. 9); the paper truncates 2.78 -> 2.7 and 1.67 -> 1.6
        ratio = acc.hardware_flops(1, mod["L"], S, mod["h"], VOCAB) / acc.model_flops(1, mod["L"], S, mod["h"], VOCAB)
        assert abs(100 * (ratio - 1) - V[key + "_flops_overhead_pct"]) < 0.1
        assert abs(float(ratio) - (1 + S / (6 * mod["h"]))) < 2e-3


def test_flops_closed_forms_and_table5_utilisation():
    for name, m in MODELS.items():
        B, L, h = m["B"], m["L"], m["h"]
        assert acc.model_flops(B, L, S, h, VOCAB) == acc.model_flops_closed_form(B, L, S, h, VOCAB)        # Eq. 7
        assert acc.hardware_flops(B, L, S, h, VOCAB) == acc.hardware_flops_closed_form(B, L, S, h, VOCAB)  # Eq. 8
        peak = V["a100_peak_tflops"] * 1e12 * m["gpus"]
        mfu = 100 * acc.model_flops(B, L, S, h, VOCAB) / m["iter_s"] / peak
        hfu = 100 * acc.hardware_flops(B, L, S, h, VOCAB) / m["iter_s"] / peak
        assert abs(mfu - m["mfu"]) < 0.25, (name, mfu)   # Table 5 (22B differs by 0.2 pt: 1.10 s is rounded)
        assert abs(hfu - m["hfu"]) < 0.25, (name, hfu)


def test_output_deallocation_and_figure7():
    m = MODELS["530B"]
    assert abs(2 * S * m["b"] * m["h"] * m["p"] / 2 ** 30 - V["out_dealloc_530b_gb"]) < 0.01   # Appendix B
    for name, mod in MODELS.items():
        base = acc.act_bytes_tp(S, mod["b"], mod["h"], mod["a"], 8)
        both = acc.act_bytes_tp_sp_selective(S, mod["b"], mod["h"], mod["a"], 8)
        assert float(100 * both / base) < V["both_techniques_pct_max"]                           # Section 6.1
        assert 4.5 < float(base / both) < 6.5                                                    # "5x"
        full = acc.act_bytes_full_recompute(S, mod["b"], mod["h"])
        assert 6 < float(100 * full / base) < 11                                                 # "about 10%"
        for one in (acc.act_bytes_tp_sp, acc.act_bytes_tp_selective):
            assert 0.4 < float(one(S, mod["b"], mod["h"], mod["a"], 8) / base) < 0.75            # "nearly in half"
    assert acc.interleave_factor(8, 3) == 1 + Fraction(7, 24)                                    # Section 4.2.3


# per-GPU byte counts at the benchmark shapes (t = 8, s = 2048), from the Table 2 rows
TABLE = {
    "22B": (1325400064, 884998144, 654311424, 213909504, 100663296, 721420288, 50331648),
    "175B": (578813952, 358612992, 327155712, 106954752, 50331648, 276824064, 25165824),
    "530B": (880803840, 513802240, 545259520, 178257920, 83886080, 377487360, 41943040),
    "1T": (1101004800, 642252800, 681574400, 222822400, 104857600, 471859200, 52428800),
}


def test_per_gpu_bytes_at_benchmark_shapes():
    for name, want in TABLE.items():
        m = MODELS[name]
        s, b, h, a, t = S, m["b"], m["h"], m["a"], 8
        got = (acc.act_bytes_tp(s, b, h, a, t), acc.act_bytes_tp_sp(s, b, h, a, t), acc.act_bytes_tp_selective(s, b, h, a, t),
               acc.act_bytes_tp_sp_selective(s, b, h, a, t), acc.act_bytes_full_recompute(s, b, h),
               acc.attn_core_saved_bytes(s, b, h, a, t, False), acc.attn_core_saved_bytes(s, b, h, a, t, True))
        assert tuple(int(x) for x in got) == want, name
        # the attention core's share: 8 sbh/t stored + 5 a s^2 b / t avoided
        assert got[5] - got[6] == 5 * a * s * s * b // t
        assert got[6] == 8 * s * b * h // t
    assert acc.attn_core_small_buffers(2048, 1, 128, 8) == 131072 + 16


def test_attn_core_flops():
    f = acc.attn_core_flops(2048, 1, 16, 160)
    T = 2048 * 2049 // 2
    assert f["fwd"] == 4 * 160 * T * 16 and f["bwd_fused"] == 10 * 160 * T * 16 and f["bwd_paper"] == 12 * 160 * T * 16
    # without the causal discount the forward count is Appendix A's 4 B s^2 h for this GPU's heads
    f2 = acc.attn_core_flops(2048, 1, 16, 160, causal=False)
    assert f2["fwd"] == 4 * 1 * 2048 * 2048 * (16 * 160)


def test_first_stage_total_against_section_4_3_items_and_appendix_b():
    """total_act_bytes_first_stage = L layers of Eq. 5 / Eq. 6 plus the extras that Section 4.3 itemises, checked against
    the items themselves (not the closed form the function uses) and against the number Appendix B prints."""
    # p > 1 (530B: p = 35): the only extra is the embedding dropout, sbhp/t bytes.  Appendix B prints sbhp = 2.73 GB at
    # 2 bytes per element for this model, so the extra is 2.73 GiB / (2 t).
    m = MODELS["530B"]
    for sel, per_layer in ((False, acc.act_bytes_tp_sp), (True, acc.act_bytes_tp_sp_selective)):
        tot = acc.total_act_bytes_first_stage(S, m["b"], m["h"], m["a"], m["L"], 8, m["p"], VOCAB, selective=sel)
        extra = tot - m["L"] * per_layer(S, m["b"], m["h"], m["a"], 8)
        assert abs(float(extra) * 2 * 8 / 2 ** 30 - V["out_dealloc_530b_gb"]) < 0.01
    # p = 1 (22B): besides the embedding dropout (sbh/t), the final LayerNorm input (2sbh/t), the output projection's
    # input (2sbh/t) and the fp32 logits (4sbv/t), as Section 4.3 lists them one by one
    m = MODELS["22B"]
    assert m["p"] == 1
    s, b, h, t = S, m["b"], m["h"], 8
    items = Fraction(s * b * h, t) + Fraction(2 * s * b * h, t) + Fraction(2 * s * b * h, t) + Fraction(4 * s * b * VOCAB, t)
    tot = acc.total_act_bytes_first_stage(s, b, h, m["a"], m["L"], t, 1, VOCAB)
    assert tot - m["L"] * acc.act_bytes_tp_sp(s, b, h, m["a"], t) == items
    # the extras are small beside the layers (the section's point; its "0.01 %" does not follow from its own formula)
    assert float(items / tot) < 0.01


def test_the_other_reading_of_eq8_does_not_reproduce_the_printed_overheads():
    """Eq. 8 as printed adds 12 B L s^2 h; the sentence before it (one more QK^T and attention-over-V per layer) adds
    4 B L s^2 h.  Only the printed equation gives Section 5's 2.7 % / 1.6 % and Table 5's HFU column; the other reading
    is kept as hardware_flops_text_reading and is exactly a third of the way from Eq. 7 to Eq. 8."""
    for key, name in (("gpt3", "175B"), ("mtnlg", "530B")):
        m = MODELS[name]
        mf = acc.model_flops(1, m["L"], S, m["h"], VOCAB)
        hf = acc.hardware_flops(1, m["L"], S, m["h"], VOCAB)
        tf = acc.hardware_flops_text_reading(1, m["L"], S, m["h"], VOCAB)
        assert 3 * (tf - mf) == hf - mf
        assert tf - mf == m["L"] * 4 * S * S * m["h"]                                  # one QK^T + one PV forward per layer, Appendix A's 4 B s^2 h
        assert abs(100 * (tf / mf - 1) - V[key + "_flops_overhead_pct"]) > 1.0         # 0.9 % / 0.6 %: not what the paper prints
    m = MODELS["530B"]
    peak = V["a100_peak_tflops"] * 1e12 * m["gpus"]
    hfu_text = 100 * acc.hardware_flops_text_reading(m["B"], m["L"], S, m["h"], VOCAB) / m["iter_s"] / peak
    assert abs(hfu_text - m["hfu"]) > 0.25                                             # Table 5's HFU needs the printed equation
