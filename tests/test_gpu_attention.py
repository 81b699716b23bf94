"""GPU parity: the HIP attention core against the fp64 oracle, through the C ABI.

Bars: fp32 path 1e-4 in max_e |x-ref| / max(|ref_e|, RMS(ref)).  bf16 attention outputs and gradients, per (batch, head):
elementwise |x - ref|_e <= 2e-2 RMS(ref) + 2^-8 (scale_e + |ref_e|), scale_e = the sum of the magnitudes of the terms that
make up element e: one bf16 rounding (unit roundoff 2^-8) of every term and one of the result (the stated 2e-2 RMS alone
cannot hold for any bf16 store on causal near-uniform rows, whose first rows are ~sqrt(s) times the tensor RMS), AND per
block of 64 rows RMS(x - ref) <= 4 x 2^-9 RMS(ref of the block), which judges late rows by their own size (stress inputs
with a peaked softmax, whose gradients are differences of large terms: <= 3 x 2^-9 RMS(scale of the block)).  Dropout masks and byte counts bit-exact (tests/test_gpu_attention_masks.py observes the
masks of the fused kernels directly)."""
import sys

import numpy as np
import pytest

import oracle
from paper_2205_05198_amd.workloads import WORKLOADS, attn_inputs

pytestmark = pytest.mark.gpu


def _check(tag, got, ref, dtype, names):
    from gpu_util import BAR, err
    for nm in names:
        e = err(got[nm], ref[nm], dtype)
        print(f"  {tag} {nm}: err {e:.3e} (bar {BAR[dtype]:.0e})", flush=True)
        assert e <= BAR[dtype], (tag, nm, e)


def _oracle(sh, q, k, v, do, heads=None):
    f = oracle.attn_fwd(sh, q, k, v, heads=heads)
    g = oracle.attn_bwd(sh, q, k, v, do, heads=heads)
    return {**f, **g}


@pytest.fixture(autouse=True)
def _library_picks_variants():
    """Every test starts and ends with the library choosing its kernel variants."""
    import paper_2205_05198_amd as sar
    sar.sar_test_force_variants(-1, -1, -1, -1)
    yield
    sar.sar_test_force_variants(-1, -1, -1, -1)


def _check_bf16_heads(tag, sh, q, k, v, do, got, heads, peaked=False):
    """bf16 attention bar per (batch, head): |x - ref| <= 2e-2 RMS(ref) + 2^-8 * forward-error magnitude, and the
    64-row-block RMS guard (against the block's own RMS, or, for `peaked` stress inputs, against the RMS of the terms'
    magnitudes).  The oracle runs on groups of consecutive heads at once (one thread per head)."""
    from gpu_util import BLOCK_GUARD, BLOCK_GUARD_TERMS, attn_scales, err_attn_blocks, err_attn_bf16
    heads = sorted(heads)
    group = max(1, oracle.num_threads())
    runs = []   # maximal runs of consecutive (batch, head) indices, at most `group` long
    for bn in heads:
        if runs and runs[-1][1] == bn and bn - runs[-1][0] < group:
            runs[-1][1] = bn + 1
        else:
            runs.append([bn, bn + 1])
    for lo, hi in runs:
        f = oracle.attn_fwd(sh, q, k, v, materialise=True, heads=(lo, hi))
        g = oracle.attn_bwd(sh, q, k, v, do, heads=(lo, hi))
        ref = {**f, **g}
        for bn in range(lo, hi):
            be, n = bn // sh.A, bn % sh.A
            sc = attn_scales(sh, q, k, v, do, be, n, f["P"][bn - lo], f["M"][bn - lo].astype(np.float64), f["D"][bn - lo])
            for nm in ("o", "dq", "dk", "dv"):
                e = err_attn_bf16(got[nm][:, be, n], ref[nm][:, be, n], sc[nm])
                eb = err_attn_blocks(got[nm][:, be, n], ref[nm][:, be, n])
                et = err_attn_blocks(got[nm][:, be, n], ref[nm][:, be, n], sc[nm])
                print(f"  {tag}[{bn}] {nm}: {e:.3f} of the bound, block RMS error {eb:.2f} x 2^-9 of the block, {et:.3f} x 2^-9 of its terms", flush=True)
                assert e <= 1.0, (tag, bn, nm, e)
                if peaked:
                    assert et <= BLOCK_GUARD_TERMS, (tag, bn, nm, et)
                else:
                    assert eb <= BLOCK_GUARD, (tag, bn, nm, eb)
            lref = ref["lse"][be, n]
            assert np.max(np.abs(got["lse"][be, n] - lref)) < 2e-3 * (1.0 + np.max(np.abs(lref)))


def test_tiny_fp32_workload():
    """b=1, s=128, 2 heads of 64, p=0.1, seed 1234, Q,K,V,dO ~ N(0,1)."""
    from gpu_util import run_attn
    w = WORKLOADS["tiny"]
    sh = oracle.AttnShape(s=w.s, b=w.b, a=w.a, h=w.h, t=w.t, p=w.p, seed=w.seed)
    q, k, v, do = attn_inputs(w.s, w.b, w.A, w.d, "f32", seed=w.seed)
    print("tiny fp32", flush=True)
    got = run_attn(sh, "f32", q, k, v, do)
    ref = _oracle(sh, q, k, v, do)
    _check("tiny", got, ref, "f32", ["o", "dq", "dk", "dv"])
    assert np.max(np.abs(got["lse"] - ref["lse"]) / (1.0 + np.abs(ref["lse"]))) < 1e-5


@pytest.mark.parametrize("s,b,a,t,rank,d,p,std,outlier", [
    (40, 2, 3, 1, 0, 32, 0.2, 1.0, False),     # ragged: s not a multiple of the wave/block sizes
    (136, 1, 4, 2, 1, 64, 0.1, 4.0, True),     # peaked softmax, late-moving maximum, second TP rank
    (64, 1, 1, 1, 0, 8, 0.0, 1.0, False),      # p = 0, smallest head dimension
    (8, 1, 2, 1, 0, 256, 0.5, 1.0, False),     # one block, largest head dimension
    (-104, 1, 2, 1, 0, 64, 0.1, 1.0, False),   # negative s: the same without the causal mask (encoder), ragged
    (-40, 2, 3, 1, 0, 32, 0.0, 4.0, True),
])
def test_fp32_shapes(s, b, a, t, rank, d, p, std, outlier):
    from gpu_util import run_attn
    causal, s = int(s > 0), abs(s)
    sh = oracle.AttnShape(s=s, b=b, a=a, h=a * d, t=t, rank=rank, p=p, seed=77, offset=123456789012, causal=causal)
    q, k, v, do = attn_inputs(s, b, sh.A, d, "f32", seed=5, qk_std=std, outlier=outlier)
    print(f"fp32 s={s} b={b} A={sh.A} d={d} p={p}", flush=True)
    got = run_attn(sh, "f32", q, k, v, do)
    ref = _oracle(sh, q, k, v, do)
    _check("fp32", got, ref, "f32", ["o", "dq", "dk", "dv"])
    assert np.max(np.abs(got["lse"] - ref["lse"]) / (1.0 + np.abs(ref["lse"]))) < 1e-5


@pytest.mark.parametrize("two_pass", [False, True])
@pytest.mark.parametrize("d", [64, 96, 128, 160])
@pytest.mark.parametrize("s,b,A,p,std,causal", [(200, 2, 2, 0.1, None, 1), (328, 1, 3, 0.25, 1.0, 1), (200, 1, 2, 0.1, None, 0), (264, 1, 1, 0.0, 1.0, 0),
                                                 (200, 1, 2, 0.0, None, 1), (256, 1, 2, 0.1, 4.0, 1)])
def test_bf16_matrix_core_path_small(d, s, b, A, p, std, causal, two_pass):
    """Several 64-key tiles and 64-row blocks plus a ragged tail (s % 64 = 8), every benchmark head dimension, both forms
    of the backward (region recomputed once / twice); causal = 0 is the encoder variant (every key), including p = 0;
    std = 4 is the stress input on the matrix cores (Q, K ~ 4 N(0,1): a peaked softmax, plus one planted outlier score)."""
    from gpu_util import run_attn
    sh = oracle.AttnShape(s=s, b=b, a=A * 2, h=A * 2 * d, t=2, rank=1, p=p, seed=1234, offset=(1 << 33) + 5, causal=causal)
    q, k, v, do = attn_inputs(s, b, A, d, "bf16", seed=9, qk_std=std, outlier=std is not None)
    print(f"bf16 s={s} b={b} A={A} d={d} p={p} std={std} two_pass={two_pass}", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do, two_pass=two_pass)
    _check_bf16_heads("bf16", sh, q, k, v, do, got, range(b * A), peaked=std is not None)


@pytest.mark.parametrize("d,s,causal", [(64, 328, 1), (160, 328, 1), (160, 200, 0), (128, 136, 1)])
def test_forward_with_128_row_workgroups(d, s, causal):
    """The forward kernel with 128 query rows per workgroup (chosen by the library for long sequences) forced on small
    ragged shapes: lower and upper row groups end on different tiles under the mask, the last block is partly empty."""
    import paper_2205_05198_amd as sar
    from gpu_util import run_attn
    sar.sar_test_force_variants(1, -1, -1)
    sh = oracle.AttnShape(s=s, b=1, a=2, h=2 * d, p=0.1, seed=5, causal=causal)
    q, k, v, do = attn_inputs(s, 1, 2, d, "bf16", seed=17)
    print(f"fwd128 d={d} s={s} causal={causal}", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do)
    _check_bf16_heads("fwd128", sh, q, k, v, do, got, range(2))


@pytest.mark.parametrize("lw", [0, 1, 2])
@pytest.mark.parametrize("d,s,causal", [(64, 328, 1), (96, 200, 1), (160, 328, 1), (160, 200, 0), (128, 136, 1), (160, 40, 1)])
def test_forward_with_and_without_loader_waves(d, s, causal, lw):
    """The 64-row forward kernel and the dQ pass with (1: 8 waves) and without (0: 4 waves) their tile-fetching waves, and
    the forward as producer / consumer wave pairs (2), each forced whatever the library would pick for the head dimension,
    on ragged shapes (the last tile is fetched with clamped rows; s = 40: a single tile)."""
    import paper_2205_05198_amd as sar
    from gpu_util import run_attn
    sar.sar_test_force_variants(0, lw, lw)
    sh = oracle.AttnShape(s=s, b=1, a=2, h=2 * d, p=0.1, seed=5, causal=causal)
    q, k, v, do = attn_inputs(s, 1, 2, d, "bf16", seed=19)
    print(f"fwd loader waves={lw} d={d} s={s} causal={causal}", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do, two_pass=True)   # the row pass with loader waves belongs to the two-pass backward
    _check_bf16_heads(f"fwd-lw{lw}", sh, q, k, v, do, got, range(2))


@pytest.mark.parametrize("two_pass", [False, True])
@pytest.mark.parametrize("d,s,b,A,causal,p", [(160, 320, 3, 44, 1, 0.1), (128, 768, 1, 44, 1, 0.1), (64, 256, 2, 66, 0, 0.1), (64, 128, 5, 60, 1, 0.1), (160, 384, 1, 132, 1, 0.0)])
def test_column_pass_persistent_workgroups(d, s, b, A, causal, p, two_pass):
    """The producer / consumer column pass with persistent workgroups (forced), at head counts where a workgroup really gets
    several key blocks: 132 heads (one workgroup per head takes all its key blocks in turn) and 44 heads (five workgroups per
    head: key blocks wq, 9 - wq, 10 + wq of 12).  A later block of a list starts from K, V and a first (Q, dO) tile requested
    during the last step of the block before it, in LDS stages that rotate from block to block.  300 heads: more heads than
    compute units, the request falls back to one key block per workgroup."""
    import paper_2205_05198_amd as sar
    from gpu_util import run_attn
    sar.sar_test_force_variants(-1, -1, -1, 3)
    sh = oracle.AttnShape(s=s, b=b, a=A, h=A * d, p=p, seed=78, offset=(1 << 32) - 54321, causal=causal)
    q, k, v, do = attn_inputs(s, b, A, d, "bf16", seed=37)
    print(f"column pass persistent d={d} s={s} b={b} A={A} causal={causal} two_pass={two_pass}", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do, two_pass=two_pass)
    N = b * A
    _check_bf16_heads("cols-pers", sh, q, k, v, do, got, [0, 1, N // 2, N - 1])


@pytest.mark.parametrize("d,s,b,A,causal,p", [(160, 328, 3, 44, 1, 0.1), (128, 776, 1, 44, 1, 0.1), (160, 264, 2, 66, 0, 0.1), (128, 136, 5, 60, 1, 0.1), (160, 392, 1, 132, 1, 0.0)])
def test_forward_persistent_workgroups(d, s, b, A, causal, p):
    """The forward with persistent workgroups (forced), at head counts where a workgroup really gets several row blocks: 132
    heads (one workgroup per head takes all its row blocks in turn) and 44 heads (five workgroups per head: ranks wq, 9 - wq,
    10 + wq of 13 row blocks, the last one ragged).  A later block of a list starts from Q operands, Philox words and K / V
    tiles requested during the block before it.  300 heads: more heads than compute units, the request falls back to one
    row block per workgroup."""
    import paper_2205_05198_amd as sar
    from gpu_util import run_attn
    sar.sar_test_force_variants(0, 3, -1, -1)
    sh = oracle.AttnShape(s=s, b=b, a=A, h=A * d, p=p, seed=77, offset=(1 << 32) - 12345, causal=causal)
    q, k, v, do = attn_inputs(s, b, A, d, "bf16", seed=31)
    print(f"fwd persistent d={d} s={s} b={b} A={A} causal={causal}", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do)
    N = b * A
    _check_bf16_heads("fwd-pers", sh, q, k, v, do, got, [0, 1, N // 2, N - 1])


@pytest.mark.parametrize("two_pass", [False, True])
@pytest.mark.parametrize("d,s,causal", [(160, 8, 1), (64, 24, 1), (128, 64, 1), (160, 72, 1), (96, 40, 0), (160, 56, 0)])
def test_bf16_matrix_core_path_short_sequences(d, s, causal, two_pass):
    """Sequences of at most one or two tiles on the matrix-core kernels: the only tile is ragged (rows past the end are
    fetched clamped and masked), a workgroup has a single step, three of four waves may have nothing but masked keys."""
    from gpu_util import run_attn
    sh = oracle.AttnShape(s=s, b=2, a=2, h=2 * d, p=0.1, seed=9, causal=causal)
    q, k, v, do = attn_inputs(s, 2, 2, d, "bf16", seed=23)
    print(f"short d={d} s={s} causal={causal} two_pass={two_pass}", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do, two_pass=two_pass)
    _check_bf16_heads("short", sh, q, k, v, do, got, range(4))


def test_random_shapes_and_kernel_variants():
    """A seeded sweep: head dimension, sequence length (any multiple of 8 up to 560), batch, heads, TP rank, p, mask, the
    form of the backward (region recomputed once or twice) and the kernel variants (128-row forward, loader waves in the
    forward and in the row pass: forced on, forced off or left to the library) drawn at random; every (batch, head) of
    every case against the oracle."""
    import random
    import paper_2205_05198_amd as sar
    from gpu_util import run_attn
    rng = random.Random(20240611)
    for case in range(16):
        d = rng.choice([64, 96, 128, 160])
        s = 8 * rng.randint(1, 70)
        b, A, t = rng.choice([1, 2]), rng.choice([1, 2, 3]), rng.choice([1, 2])
        rank = rng.randrange(t)
        p, causal = rng.choice([0.0, 0.1, 0.3]), rng.choice([0, 1, 1])
        env = [rng.choice([-1, 0, 1]), rng.choice([-1, 0, 1, 2, 3]), rng.choice([-1, 0, 1]), rng.choice([-1, 0, 1, 2, 3])]
        if s < 128:
            env[0] = -1
        sar.sar_test_force_variants(*env)
        two_pass = case % 2 == 1
        sh = oracle.AttnShape(s=s, b=b, a=A * t, h=A * t * d, t=t, rank=rank, p=p, seed=1000 + case, offset=7 * case, causal=causal)
        q, k, v, do = attn_inputs(s, b, A, d, "bf16", seed=500 + case)
        print(f"case {case}: d={d} s={s} b={b} A={A} t={t} rank={rank} p={p} causal={causal} variants={env} two_pass={two_pass}", flush=True)
        got = run_attn(sh, "bf16", q, k, v, do, two_pass=two_pass)
        _check_bf16_heads(f"sweep{case}", sh, q, k, v, do, got, range(b * A))


@pytest.mark.parametrize("pipe", [0, 1, 2, 3])
@pytest.mark.parametrize("two_pass", [False, True])
@pytest.mark.parametrize("d,s,b,A,p,causal", [(160, 320, 1, 2, 0.1, 1), (128, 256, 2, 1, 0.25, 1), (160, 192, 1, 2, 0.1, 0), (128, 64, 1, 2, 0.0, 1), (160, 128, 1, 1, 0.0, 0),
                                              (64, 320, 2, 1, 0.1, 1), (96, 192, 1, 2, 0.25, 0), (64, 64, 1, 1, 0.0, 1)])
def test_column_pass_pipelined_and_plain(d, s, b, A, p, causal, two_pass, pipe):
    """The column pass in its plain form (0), its software-pipelined form (1: three query-tile stages, K operands in
    registers) and its producer / consumer form (2: two waves per SIMD), each forced, on sequences of one to five full
    tiles: with and without the mask, with and without dropout, in both forms of the backward."""
    import paper_2205_05198_amd as sar
    from gpu_util import run_attn
    sar.sar_test_force_variants(-1, -1, -1, pipe)
    sh = oracle.AttnShape(s=s, b=b, a=A * 2, h=A * 2 * d, t=2, rank=1, p=p, seed=77, offset=(1 << 32) - 1000, causal=causal)
    q, k, v, do = attn_inputs(s, b, A, d, "bf16", seed=29)
    print(f"column pass pipelined={pipe} d={d} s={s} causal={causal} p={p} two_pass={two_pass}", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do, two_pass=two_pass)
    _check_bf16_heads(f"cols-pipe{pipe}", sh, q, k, v, do, got, range(b * A))


def test_bf16_generic_path_other_head_dim():
    from gpu_util import run_attn
    sh = oracle.AttnShape(s=72, b=1, a=2, h=2 * 40, p=0.1, seed=3)
    q, k, v, do = attn_inputs(72, 1, 2, 40, "bf16", seed=21)
    got = run_attn(sh, "bf16", q, k, v, do)
    _check_bf16_heads("bf16-d40", sh, q, k, v, do, got, range(2))


@pytest.mark.parametrize("dtype,d,causal", [("f32", 64, 1), ("bf16", 96, 1), ("bf16", 96, 0)])
def test_stored_baseline_mask_bit_exact(dtype, d, causal):
    """The stored path exposes P, M, D: M must equal the oracle's mask bit for bit (0 above the diagonal when causal)."""
    from gpu_util import BAR, err, run_attn
    sh = oracle.AttnShape(s=128, b=2, a=4, h=4 * d, t=2, rank=1, p=0.1, seed=1234, offset=77, causal=causal)
    q, k, v, do = attn_inputs(128, 2, 2, d, dtype, seed=31)
    got = run_attn(sh, dtype, q, k, v, do, stored=True)
    f = oracle.attn_fwd(sh, q, k, v, materialise=True)
    g = oracle.attn_bwd(sh, q, k, v, do)
    assert np.array_equal(got["M"], f["M"])
    assert np.array_equal(got["M"], np.tril(oracle.attn_mask(sh)) if causal else oracle.attn_mask(sh))
    for nm in ("P", "D"):
        assert np.max(np.abs(got[nm] - f[nm])) <= (1e-6 if dtype == "f32" else 2.0 ** -8), nm
    if dtype == "f32":
        _check("stored", got, {**f, **g}, dtype, ["o", "dq", "dk", "dv"])
    else:
        _check_bf16_heads("stored", sh, q, k, v, do, got, range(4))


@pytest.mark.parametrize("d,causal", [(64, 1), (160, 1), (160, 0)])
def test_stored_baseline_matrix_core_shapes(d, causal):
    """The stored baseline on the matrix cores (bf16, s a multiple of 64) over several 64-row blocks: M bit-exact, P and D
    within one bf16 rounding, O, LSE and the gradients to the bf16 bar."""
    from gpu_util import run_attn
    s = 320
    sh = oracle.AttnShape(s=s, b=1, a=2, h=2 * d, p=0.1, seed=99, offset=8, causal=causal)
    q, k, v, do = attn_inputs(s, 1, 2, d, "bf16", seed=33)
    print(f"stored mfma d={d} causal={causal}", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do, stored=True)
    f = oracle.attn_fwd(sh, q, k, v, materialise=True)
    assert np.array_equal(got["M"], f["M"])
    for nm in ("P", "D"):
        assert np.max(np.abs(got[nm] - f[nm])) <= 2.0 ** -8, nm
    _check_bf16_heads("stored-mfma", sh, q, k, v, do, got, range(2))


def test_recompute_equals_stored_and_is_deterministic():
    """Selective recomputation is an exact rewrite (Section 5): same mask, same gradients up to rounding, run to run bit-identical."""
    from gpu_util import run_attn
    sh = oracle.AttnShape(s=192, b=1, a=2, h=2 * 128, p=0.1, seed=1234)
    q, k, v, do = attn_inputs(192, 1, 2, 128, "bf16", seed=41)
    r1 = run_attn(sh, "bf16", q, k, v, do)
    r2 = run_attn(sh, "bf16", q, k, v, do)
    for nm in ("o", "lse", "dq", "dk", "dv"):
        assert np.array_equal(r1[nm], r2[nm]), nm
    st = run_attn(sh, "bf16", q, k, v, do, stored=True)
    _check_bf16_heads("recompute", sh, q, k, v, do, r1, range(2))
    _check_bf16_heads("stored", sh, q, k, v, do, st, range(2))
    # a different offset gives a different mask, hence a different O
    sh2 = oracle.AttnShape(s=192, b=1, a=2, h=2 * 128, p=0.1, seed=1234, offset=oracle.attn_philox_count(sh))
    r3 = run_attn(sh2, "bf16", q, k, v, do)
    assert not np.array_equal(r1["o"], r3["o"])


@pytest.mark.parametrize("name,two_pass", [("530B", False), ("530B", True), ("22B", False), ("175B", False), ("1T", False)])
def test_full_size_every_head(name, two_pass):
    """Benchmark shapes in the launch configuration the benchmark times: every (batch, head) of the shard against the
    oracle (16 at 530B, 32 at 22B, 12 at 175B, 20 at 1T); at 530B both forms of the backward."""
    from gpu_util import run_attn
    w = WORKLOADS[name]
    sh = oracle.AttnShape(s=w.s, b=w.b, a=w.a, h=w.h, t=w.t, rank=3, p=w.p, seed=w.seed)
    q, k, v, do = attn_inputs(w.s, w.b, w.A, w.d, "bf16", seed=w.seed)
    print(f"{name}: s={w.s} b={w.b} A={w.A} d={w.d} two_pass={two_pass}", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do, two_pass=two_pass)
    _check_bf16_heads(name, sh, q, k, v, do, got, range(w.b * w.A))
    sys.stdout.flush()


def test_stress_inputs_full_length():
    """The stress input at the benchmark's sequence length on the matrix cores: Q, K ~ 4 N(0,1) (score std ~ 16 sqrt(d) alpha:
    a sharply peaked softmax whose running maximum moves many times) plus a planted outlier, two heads of 160."""
    from gpu_util import run_attn
    s, d = 2048, 160
    sh = oracle.AttnShape(s=s, b=1, a=2, h=2 * d, p=0.1, seed=4321, offset=17)
    q, k, v, do = attn_inputs(s, 1, 2, d, "bf16", seed=71, qk_std=4.0, outlier=True)
    print("bf16 stress s=2048 d=160", flush=True)
    for two_pass in (False, True):
        got = run_attn(sh, "bf16", q, k, v, do, two_pass=two_pass)
        _check_bf16_heads(f"stress-{'twice' if two_pass else 'once'}", sh, q, k, v, do, got, range(2), peaked=True)


def test_sequence_8192_single_head():
    """s = 8192 at the 530B head dimension (128 tiles per row block, 128-row forward workgroups): one head against the oracle."""
    from gpu_util import run_attn
    s, d = 8192, 160
    sh = oracle.AttnShape(s=s, b=1, a=8, h=8 * d, t=8, rank=2, p=0.1, seed=1234, offset=5)
    q, k, v, do = attn_inputs(s, 1, 1, d, "bf16", seed=67)
    print("bf16 s=8192 one head", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do)
    _check_bf16_heads("s8192", sh, q, k, v, do, got, range(1))


def test_longer_sequence_single_head():
    """s = 4096 at the 530B head dimension (64 tiles per row block): one head against the oracle."""
    from gpu_util import run_attn
    s, d = 4096, 160
    sh = oracle.AttnShape(s=s, b=1, a=8, h=8 * d, t=8, rank=5, p=0.1, seed=1234, offset=99)
    q, k, v, do = attn_inputs(s, 1, 1, d, "bf16", seed=61)
    print("bf16 s=4096 one head", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do)
    _check_bf16_heads("s4096", sh, q, k, v, do, got, range(1))


def test_longer_sequence_single_head_128_row_workgroups():
    """The same with the forward's 128-row workgroups (what the library picks at this head dimension once there are more
    row blocks than CUs): 32 row blocks, up to 64 tiles each."""
    import paper_2205_05198_amd as sar
    from gpu_util import run_attn
    sar.sar_test_force_variants(1, -1, -1)
    s, d = 4096, 160
    sh = oracle.AttnShape(s=s, b=1, a=8, h=8 * d, t=8, rank=5, p=0.1, seed=1234, offset=99)
    q, k, v, do = attn_inputs(s, 1, 1, d, "bf16", seed=61)
    print("bf16 s=4096 one head, 128-row forward", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do)
    _check_bf16_heads("s4096-128", sh, q, k, v, do, got, range(1))


def test_stored_baseline_full_size_sampled_head():
    """The stored-activation baseline at the benchmark's shape (530B shard): mask of one head bit for bit, P and D within one
    bf16 rounding, outputs and gradients of that head to the bf16 bar."""
    from gpu_util import run_attn
    w = WORKLOADS["530B"]
    sh = oracle.AttnShape(s=w.s, b=w.b, a=w.a, h=w.h, t=w.t, rank=3, p=w.p, seed=w.seed)
    q, k, v, do = attn_inputs(w.s, w.b, w.A, w.d, "bf16", seed=w.seed)
    print("stored 530B", flush=True)
    got = run_attn(sh, "bf16", q, k, v, do, stored=True)
    n = 9
    f = oracle.attn_fwd(sh, q, k, v, materialise=True, heads=(n, n + 1))
    assert np.array_equal(got["M"][0, n], f["M"][0])
    for nm in ("P", "D"):
        assert np.max(np.abs(got[nm][0, n] - f[nm][0])) <= 2.0 ** -8, nm
    _check_bf16_heads("stored-530B", sh, q, k, v, do, got, (n,))



def test_sequence_16384_sampled_rows_and_both_backward_forms():
    """s = 16384 (256 tiles per row block; the oracle would need minutes per head): sampled rows of O, LSE and dQ against the
    definition written out in fp64 for those rows (row i needs only its own scores), the mask from the oracle's Philox; and
    the two forms of the backward against each other on every element (same arithmetic, different kernels for dQ)."""
    import paper_2205_05198_amd as sar
    import torch
    from gpu_util import dev, host
    from paper_2205_05198_amd.binding import SAR_BF16
    s, d, p = 16384, 160, 0.1
    sh = oracle.AttnShape(s=s, b=1, a=1, h=d, p=p, seed=1234, offset=3)
    q, k, v, do = attn_inputs(s, 1, 1, d, "bf16", seed=73)
    desc = sar.AttnDesc.packed(s, 1, 1, d, dtype=SAR_BF16, p=p, seed=1234, offset=3, scale=sh.alpha())
    tq, tk, tv, tdo = (dev(x, "bf16") for x in (q, k, v, do))
    o = torch.empty_like(tq)
    lse = torch.empty((1, 1, s), dtype=torch.float32, device="cuda")
    print("bf16 s=16384 one head", flush=True)
    sar.attn_core_fwd(desc, tq, tk, tv, o, lse)
    res = {}
    for form, nbytes in (("once", sar.attn_core_bwd_workspace(desc)), ("twice", sar.attn_core_bwd_workspace_min(desc))):
        dq, dk, dv = (torch.empty_like(tq) for _ in range(3))
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        sar.attn_core_bwd_recompute(desc, tq, tk, tv, o, lse, tdo, dq, dk, dv, ws)
        torch.cuda.synchronize()
        res[form] = {n: host(x)[:, 0, 0] for n, x in (("dq", dq), ("dk", dk), ("dv", dv))}
        del ws
    assert sar.attn_core_bwd_workspace(desc) > sar.attn_core_bwd_workspace_min(desc)
    # the column pass is the same kernel in both forms: dV (which does not involve delta) agrees bit for bit; delta is summed
    # in a different order by the two forms (fp32), so dK and dQ agree to a rounding of the result
    assert np.array_equal(res["once"]["dv"], res["twice"]["dv"])
    for n in ("dk", "dq"):
        r = float(np.sqrt(np.mean(res["twice"][n] ** 2)))
        assert np.max(np.abs(res["once"][n] - res["twice"][n]) / (2e-2 * r + 2.0 ** -7 * np.abs(res["twice"][n]))) <= 1.0, n
    rms = float(np.sqrt(np.mean(res["twice"]["dq"] ** 2)))
    # sampled rows, fp64
    Q, K, V, DO = (np.asarray(x[:, 0, 0], dtype=np.float64) for x in (q, k, v, do))
    O, L = host(o)[:, 0, 0], host(lse)[0, 0]
    c, T = 1.0 / (1.0 - float(np.float32(p))), oracle.dropout_threshold(p)
    rows = [0, 1, 63, 64, 1000, 4095, 4096, 8191, 12345, s - 65, s - 1]
    o_rms, dq_rms = float(np.sqrt(np.mean(O ** 2))), rms
    for i in rows:
        sc = sh.alpha() * (K[:i + 1] @ Q[i])
        m = sc.max()
        e = np.exp(sc - m)
        P = e / e.sum()
        M = np.array([oracle.keep_bit(sh.seed, sh.offset, i * s + j, 0, T) for j in range(i + 1)], dtype=np.float64)
        D = P * M * c
        o_ref = D @ V[:i + 1]
        assert abs(L[i] - (m + np.log(e.sum()))) < 2e-3 * (1 + abs(m)), i
        assert np.all(np.abs(O[i] - o_ref) <= 2e-2 * o_rms + 2.0 ** -8 * (D @ np.abs(V[:i + 1]) + np.abs(o_ref))), i
        dP = (V[:i + 1] @ DO[i]) * M * c
        delta = float(P @ dP)
        dS = P * (dP - delta)
        dq_ref = sh.alpha() * (dS @ K[:i + 1])
        dabs = float(np.abs(DO[i]) @ (D @ np.abs(V[:i + 1])))
        scale = sh.alpha() * ((P * (np.abs(dP) + dabs)) @ np.abs(K[:i + 1]))
        for form in ("once", "twice"):
            assert np.all(np.abs(res[form]["dq"][i] - dq_ref) <= 2e-2 * dq_rms + 2.0 ** -8 * (scale + np.abs(dq_ref))), (form, i)
