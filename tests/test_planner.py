"""The package's host-side planner against the paper's printed numbers and against the accounting oracle
(two independent write-ups of the same closed forms)."""
from fractions import Fraction
import os

from oracle import accounting as acc
from paper_2205_05198_amd import planner as pl

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    vals, models = {}, {}
    for line in open(os.path.join(HERE, "golden", "paper_numbers.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        if line[0] == "model":
            name, a, h, L, t, p, gpus, gb, mb = line[1], *map(int, line[2:10])
            models[name] = dict(a=a, h=h, L=L, t=t, p=p, b=mb)
        else:
            vals[line[0]] = float(line[1])
    return vals, models


def test_table2_and_equations_against_the_oracle():
    vals, models = _golden()
    for name, c in models.items():
        mod = pl.Model(h=c["h"], a=c["a"], L=c["L"], v=int(vals["vocab"]), s=int(vals["seq_len"]))
        lay = pl.Layout(b=c["b"], t=c["t"], p=c["p"])
        s, b, h, a, t = mod.s, lay.b, mod.h, mod.a, lay.t
        assert pl.layer_activation_bytes(mod, lay, "tp") == acc.act_bytes_tp(s, b, h, a, t)
        assert pl.layer_activation_bytes(mod, lay, "tp_sp") == acc.act_bytes_tp_sp(s, b, h, a, t)
        assert pl.layer_activation_bytes(mod, lay, "tp_selective") == acc.act_bytes_tp_selective(s, b, h, a, t)
        assert pl.layer_activation_bytes(mod, lay, "tp_sp_selective") == acc.act_bytes_tp_sp_selective(s, b, h, a, t)
        assert pl.layer_activation_bytes(mod, lay, "full") == acc.act_bytes_full_recompute(s, b, h)
        for sel, st in ((False, "tp_sp"), (True, "tp_sp_selective")):
            assert pl.first_stage_activation_bytes(mod, lay, st) == acc.total_act_bytes_first_stage(s, b, h, a, mod.L, t, lay.p, mod.v, sel)
        assert pl.model_flops(mod, 7) == acc.model_flops(7, mod.L, s, h, mod.v)
        assert pl.hardware_flops(mod, 7, "tp_sp_selective") == acc.hardware_flops(7, mod.L, s, h, mod.v)
    # t = 1 is Eq. 1
    mod, lay = pl.Model(h=1024, a=16, L=2, s=512), pl.Layout(b=3, t=1)
    assert pl.layer_activation_bytes(mod, lay, "tp") == acc.act_bytes_no_parallel(512, 3, 1024, 16) == pl.layer_activation_bytes(mod, lay, "tp_sp")


def test_printed_numbers_of_sections_5_and_6():
    vals, models = _golden()
    gpt3 = pl.Model(h=12288, a=96, L=96, v=int(vals["vocab"]))
    mtnlg = pl.Model(h=20480, a=128, L=105, v=int(vals["vocab"]))
    # Section 5: the attention-core term is 5as/h of the 34 + 5as/h; dropping it saves 70 % / 65 %
    for mod, key in ((gpt3, "gpt3"), (mtnlg, "mtnlg")):
        lay = pl.Layout(b=1, t=8)
        full_, sel = pl.layer_activation_bytes(mod, lay, "tp_sp"), pl.layer_activation_bytes(mod, lay, "tp_sp_selective")
        assert (full_ - sel) / sel * 34 == vals[f"{key}_5as_over_h"]
        assert round(float(1 - sel / full_) * 100) == vals[f"{key}_selective_saving_pct"]
        assert round(float(pl.flops_overhead(mod, "tp_sp_selective")) * 100, 1) == vals[f"{key}_flops_overhead_pct"]
        # full recomputation: one more forward on top of forward + 2 x backward = about a third more
        assert Fraction(30, 100) < pl.flops_overhead(mod, "full") < Fraction(34, 100)
    # Section 6.1 / Figure 7: both techniques together need under a fifth of the tensor-parallel baseline; full
    # recomputation about a tenth
    for name, c in models.items():
        mod, lay = pl.Model(h=c["h"], a=c["a"], L=c["L"], v=int(vals["vocab"])), pl.Layout(b=c["b"], t=c["t"], p=c["p"])
        base = pl.layer_activation_bytes(mod, lay, "tp")
        assert float(pl.layer_activation_bytes(mod, lay, "tp_sp_selective") / base) * 100 <= vals["both_techniques_pct_max"]
        assert 2 <= float(pl.layer_activation_bytes(mod, lay, "full") / base) * 100 <= vals["full_recompute_pct"] + 2


def test_interleaving_and_plan():
    mod, lay = pl.Model(h=20480, a=128, L=105), pl.Layout(b=1, t=8, p=35)
    plain = pl.first_stage_activation_bytes(mod, lay, "tp_sp_selective")
    inter = pl.first_stage_activation_bytes(mod, pl.Layout(b=1, t=8, p=35, m=3), "tp_sp_selective")
    extra = Fraction(mod.s * 1 * mod.h * 35, 8)
    assert (inter - extra) == (plain - extra) * acc.interleave_factor(35, 3)
    # a budget between the selective and the no-recompute footprint picks selective; a tiny one falls back to full
    lo, hi = pl.first_stage_activation_bytes(mod, lay, "tp_sp_selective"), pl.first_stage_activation_bytes(mod, lay, "tp_sp")
    assert pl.plan(mod, lay, int(hi) + 1)["strategy"] == "tp_sp"
    got = pl.plan(mod, lay, int((lo + hi) / 2))
    assert got["strategy"] == "tp_sp_selective" and got["fits"] and got["flops_overhead"] == pl.flops_overhead(mod, "tp_sp_selective")
    assert pl.plan(mod, lay, int(lo) - 1)["strategy"] == "full"
    assert not pl.plan(mod, lay, 1000)["fits"]
    assert pl.plan(mod, lay, int((lo + hi) / 2), sequence_parallel=False)["strategy"] in ("tp_selective", "full")


def test_microbatch_level_window_and_share():
    """Appendix C: max(0, p - S) microbatches are in flight at stage S; the figure's example (p = 4) keeps one of
    the first stage's four microbatches in full when the memory left over after checkpointing all four holds
    exactly one more full set; later stages need less and the last ones nothing."""
    from paper_2205_05198_amd.planner import Layout, Model, layer_activation_bytes, microbatch_level_plan, outstanding_microbatches, flops_overhead
    mod, lay = Model(h=12288, a=96, L=96), Layout(b=1, t=8, p=4)
    assert [outstanding_microbatches(lay, S) for S in range(6)] == [4, 3, 2, 1, 0, 0]
    layers = mod.L // lay.p
    full = layer_activation_bytes(mod, lay, "tp_sp") * layers
    ck = layer_activation_bytes(mod, lay, "tp_sp_selective") * layers
    budget = int(4 * ck + (full - ck))            # all four checkpointed + room to keep one of them in full
    r = microbatch_level_plan(mod, lay, 0, budget)
    assert (r["window"], r["stored_in_full"], r["fits"]) == (4, 1, True)
    assert r["bytes"] == full + 3 * ck and r["bytes"] <= budget
    assert r["recompute_share"] == Fraction(3, 4) and r["flops_overhead"] == Fraction(3, 4) * flops_overhead(mod, "tp_sp_selective")
    assert microbatch_level_plan(mod, lay, 0, budget - 1)["stored_in_full"] == 0      # one byte short: none fits in full
    # the same budget stores more microbatches in full at later stages, and every one from some stage on
    ks = [microbatch_level_plan(mod, lay, S, budget) for S in range(5)]
    assert [k["window"] - k["stored_in_full"] for k in ks] == sorted((k["window"] - k["stored_in_full"] for k in ks), reverse=True)
    assert ks[3]["recompute_share"] == 0 and ks[4] == {"window": 0, "stored_in_full": 0, "bytes": 0, "recompute_share": 0, "flops_overhead": 0, "fits": True}
    # too small even for checkpointing everything
    assert microbatch_level_plan(mod, lay, 0, int(4 * ck) - 1)["fits"] is False
    # first-stage bytes with nothing stored in full are the L-layer figure of Eq. 6 without the embedding terms
    assert microbatch_level_plan(mod, lay, 0, int(4 * ck))["bytes"] == layer_activation_bytes(mod, lay, "tp_sp_selective") * mod.L
