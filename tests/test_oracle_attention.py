"""Pins for the oracle's attention core (CPU only): library special cases, closed forms, invariants,
brute-force finite differences.  None of them re-uses the oracle's own formulas."""
import numpy as np
import torch

import oracle


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def _to_bhsd(x):  # [s,b,A,d] -> torch [b,A,s,d]
    return torch.from_numpy(np.ascontiguousarray(x.transpose(1, 2, 0, 3)))


def _from_bhsd(t):
    return t.detach().numpy().transpose(2, 0, 1, 3)


def test_p0_forward_matches_library_attention_and_logsumexp():
    sh = oracle.AttnShape(s=37 + 3, b=2, a=3, h=3 * 10, p=0.0)
    q, k, v = (_rand((sh.s, sh.b, sh.A, sh.d), i) for i in range(3))
    out = oracle.attn_fwd(sh, q, k, v, materialise=True)
    ref = torch.nn.functional.scaled_dot_product_attention(_to_bhsd(q), _to_bhsd(k), _to_bhsd(v), is_causal=True, scale=sh.alpha())
    assert np.abs(out["o"] - _from_bhsd(ref)).max() < 1e-13
    S = torch.einsum("bhid,bhjd->bhij", _to_bhsd(q), _to_bhsd(k)) * sh.alpha()
    S = S.masked_fill(torch.triu(torch.ones(sh.s, sh.s, dtype=torch.bool), 1), float("-inf"))
    assert np.abs(out["lse"] - torch.logsumexp(S, -1).numpy()).max() < 1e-13
    assert np.abs(out["P"].sum(-1) - 1.0).max() < 1e-14
    assert (np.triu(out["P"], 1) == 0).all()
    assert np.array_equal(out["D"], out["P"])  # p = 0: dropout is the identity


def test_p0_backward_matches_autograd():
    sh = oracle.AttnShape(s=24, b=1, a=2, h=2 * 12, p=0.0)
    q, k, v, do = (_rand((sh.s, sh.b, sh.A, sh.d), 10 + i) for i in range(4))
    tq, tk, tv = (_to_bhsd(x).requires_grad_(True) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=sh.alpha())
    ref.backward(_to_bhsd(do))
    g = oracle.attn_bwd(sh, q, k, v, do)
    for name, t in (("dq", tq), ("dk", tk), ("dv", tv)):
        assert np.abs(g[name] - _from_bhsd(t.grad)).max() < 1e-12, name


def test_row0_and_zero_query_closed_forms_with_dropout():
    sh = oracle.AttnShape(s=40, b=2, a=2, h=16, p=0.3, seed=77, offset=5)
    q, k, v = (_rand((sh.s, sh.b, sh.A, sh.d), 20 + i) for i in range(3))
    M = oracle.attn_mask(sh)
    c = 1.0 / (1.0 - float(np.float32(0.3)))
    out = oracle.attn_fwd(sh, q, k, v, materialise=True)
    # row 0 attends only to itself: O_0 = M_00 v_0 / (1-p)
    for be in range(sh.b):
        for n in range(sh.A):
            assert np.allclose(out["o"][0, be, n], M[be, n, 0, 0] * v[0, be, n] * c, rtol=0, atol=1e-15)
    # stored mask = raw mask on and below the diagonal, zero above
    assert np.array_equal(out["M"], np.tril(M))
    assert 0.6 < out["M"][np.tril(np.ones((sh.s, sh.s), bool))[None, None].repeat(2, 0).repeat(2, 1)].mean() < 0.8
    # Q = 0: uniform softmax over the prefix, O_i = c/(i+1) sum_{j<=i} M_ij v_j
    out0 = oracle.attn_fwd(sh, np.zeros_like(q), k, v)
    for i in (0, 1, 7, 39):
        want = c / (i + 1) * np.einsum("bnj,jbnd->bnd", M[:, :, i, : i + 1].astype(float), v[: i + 1])
        assert np.abs(out0["o"][i] - want).max() < 1e-14
        assert np.allclose(out0["lse"][:, :, i], np.log(i + 1.0), atol=1e-14)
    # O(p) = c (P o M) V with P from the p = 0 run
    P0 = oracle.attn_fwd(oracle.AttnShape(s=40, b=2, a=2, h=16, p=0.0), q, k, v, materialise=True)["P"]
    want = c * np.einsum("bnij,jbnd->ibnd", P0 * np.tril(M), v)
    assert np.abs(out["o"] - want).max() < 1e-13
    assert np.abs(out["D"] - c * P0 * np.tril(M)).max() < 1e-15


def test_noncausal_matches_library():
    sh = oracle.AttnShape(s=16, b=1, a=2, h=8, p=0.0, causal=0)
    q, k, v = (_rand((sh.s, sh.b, sh.A, sh.d), 30 + i) for i in range(3))
    ref = torch.nn.functional.scaled_dot_product_attention(_to_bhsd(q), _to_bhsd(k), _to_bhsd(v), is_causal=False, scale=sh.alpha())
    assert np.abs(oracle.attn_fwd(sh, q, k, v)["o"] - _from_bhsd(ref)).max() < 1e-13


def test_noncausal_backward_matches_autograd_and_mask_is_full():
    """Encoder variant: every key; gradients against autograd at p = 0, and with dropout every (i, j) draws a bit."""
    sh = oracle.AttnShape(s=24, b=1, a=2, h=2 * 12, p=0.0, causal=0)
    q, k, v, do = (_rand((sh.s, sh.b, sh.A, sh.d), 70 + i) for i in range(4))
    tq, tk, tv = (_to_bhsd(x).requires_grad_(True) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=False, scale=sh.alpha())
    ref.backward(_to_bhsd(do))
    g = oracle.attn_bwd(sh, q, k, v, do)
    for name, t in (("dq", tq), ("dk", tk), ("dv", tv)):
        assert np.abs(g[name] - _from_bhsd(t.grad)).max() < 1e-12, name
    shd = oracle.AttnShape(s=24, b=1, a=2, h=2 * 12, p=0.4, seed=11, causal=0)
    f = oracle.attn_fwd(shd, q, k, v, materialise=True)
    assert np.array_equal(f["M"], oracle.attn_mask(shd))           # nothing is cut away above the diagonal
    assert np.allclose(f["P"].sum(-1), 1.0) and (f["P"] > 0).all()  # full rows
    assert np.allclose(f["D"], f["P"] * f["M"] / (1.0 - float(np.float32(0.4))))


def test_backward_finite_differences_with_dropout():
    sh = oracle.AttnShape(s=8, b=1, a=2, h=8, p=0.25, seed=3, offset=17)
    q, k, v, do = (_rand((sh.s, sh.b, sh.A, sh.d), 40 + i) for i in range(4))
    g = oracle.attn_bwd(sh, q, k, v, do)

    def loss(q_, k_, v_):
        return float((oracle.attn_fwd(sh, q_, k_, v_)["o"] * do).sum())

    eps = 1e-6
    for name, idx in (("dq", 0), ("dk", 1), ("dv", 2)):
        base = [q, k, v]
        num = np.zeros_like(q)
        it = np.nditer(q, flags=["multi_index"])
        for _ in it:
            mi = it.multi_index
            xp = [x.copy() for x in base]
            xm = [x.copy() for x in base]
            xp[idx][mi] += eps
            xm[idx][mi] -= eps
            num[mi] = (loss(*xp) - loss(*xm)) / (2 * eps)
        scale = max(1.0, np.abs(num).max())
        assert np.abs(g[name] - num).max() / scale < 1e-7, name


def test_backward_invariants():
    sh = oracle.AttnShape(s=48, b=2, a=2, h=2 * 6, p=0.1, seed=5)
    q, k, v, do = (_rand((sh.s, sh.b, sh.A, sh.d), 50 + i) for i in range(4))
    f = oracle.attn_fwd(sh, q, k, v)
    g = oracle.attn_bwd(sh, q, k, v, do, extras=True)
    # delta_i (from P and dP) equals sum_k dO_ik O_ik (what a fused kernel uses)
    want = np.einsum("ibnd,ibnd->bni", do, f["o"])
    assert np.abs(g["delta"] - want).max() < 1e-12
    # rows of dS sum to zero (softmax Jacobian annihilates constants)
    assert np.abs(g["dS"].sum(-1)).max() < 1e-12
    assert (np.triu(g["dS"], 1) == 0).all()
    # a constant shift of all of K's rows by a vector u leaves O unchanged => sum_j dK_j = 0 exactly in theory
    assert np.abs(g["dk"].sum(0)).max() < 1e-12


def test_head_subset():
    sh = oracle.AttnShape(s=16, b=2, a=3, h=12, p=0.2, seed=9)
    q, k, v, do = (_rand((sh.s, sh.b, sh.A, sh.d), 60 + i) for i in range(4))
    full = oracle.attn_fwd(sh, q, k, v)
    part = oracle.attn_fwd(sh, q, k, v, heads=(4, 5))  # batch 1, head 1
    assert np.array_equal(part["o"][:, 1, 1], full["o"][:, 1, 1]) and (part["o"][:, 0] == 0).all()
    gfull = oracle.attn_bwd(sh, q, k, v, do)
    gpart = oracle.attn_bwd(sh, q, k, v, do, heads=(4, 5))
    assert np.array_equal(gpart["dk"][:, 1, 1], gfull["dk"][:, 1, 1]) and (gpart["dk"][:, 0] == 0).all()
