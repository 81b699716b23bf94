"""Pins for the oracle's LayerNorm and bias-dropout-add (CPU only)."""
import numpy as np
import torch

import oracle


def _rand(shape, seed, scale=1.0, mean=0.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale + mean


def test_ln_matches_library_and_autograd():
    rows, h = 12, 40
    x, dy = _rand((rows, h), 1, 2.0, 0.5), _rand((rows, h), 2)
    gamma, beta = _rand(h, 3, 0.3, 1.0), _rand(h, 4, 0.3)
    f = oracle.ln_fwd(x, gamma, beta, 1e-5)
    tx, tg, tb = (torch.from_numpy(a).requires_grad_(True) for a in (x, gamma, beta))
    ref = torch.nn.functional.layer_norm(tx, (h,), tg, tb, 1e-5)
    ref.backward(torch.from_numpy(dy))
    assert np.abs(f["y"] - ref.detach().numpy()).max() < 1e-13
    assert np.abs(f["mean"] - x.mean(1)).max() < 1e-14
    assert np.abs(f["rstd"] - 1.0 / np.sqrt(x.var(1) + 1e-5)).max() < 1e-12
    g = oracle.ln_bwd(dy, x, gamma, 1e-5)
    assert np.abs(g["dx"] - tx.grad.numpy()).max() < 1e-12
    assert np.abs(g["dgamma"] - tg.grad.numpy()).max() < 1e-12
    assert np.abs(g["dbeta"] - tb.grad.numpy()).max() < 1e-12


def test_ln_invariants():
    rows, h = 6, 64
    x, dy = _rand((rows, h), 5, 3.0), _rand((rows, h), 6)
    gamma = _rand(h, 7, 0.1, 1.0)
    f = oracle.ln_fwd(x, np.ones(h), np.zeros(h), 1e-5)
    var = x.var(1)
    assert np.abs(f["y"].mean(1)).max() < 1e-14
    assert np.abs((f["y"] ** 2).mean(1) - var / (var + 1e-5)).max() < 1e-12
    g = oracle.ln_bwd(dy, x, gamma, 1e-5)
    assert np.abs(g["dx"].sum(1)).max() < 1e-12  # dx is orthogonal to constants


def test_ln_finite_differences():
    rows, h = 4, 8
    x, dy = _rand((rows, h), 8), _rand((rows, h), 9)
    gamma, beta = _rand(h, 10, 0.5, 1.0), _rand(h, 11)
    g = oracle.ln_bwd(dy, x, gamma, 1e-5)
    eps = 1e-6
    num = np.zeros_like(x)
    for r in range(rows):
        for c in range(h):
            xp, xm = x.copy(), x.copy()
            xp[r, c] += eps
            xm[r, c] -= eps
            num[r, c] = ((oracle.ln_fwd(xp, gamma, beta)["y"] - oracle.ln_fwd(xm, gamma, beta)["y"]) * dy).sum() / (2 * eps)
    assert np.abs(g["dx"] - num).max() < 1e-7


def test_bias_dropout_add():
    rows, h = 10, 24
    x, resid, bias = _rand((rows, h), 12), _rand((rows, h), 13), _rand(h, 14)
    # p = 0: plain sum
    r0 = oracle.bias_dropout_add(x, bias, resid, 0.0, 1, 0)
    assert np.array_equal(r0["out"], resid + (x + bias)) and r0["mask"].all()
    # no bias: the paper's Dropout(W) + residual
    r = oracle.bias_dropout_add(x, None, resid, 0.25, 42, 8)
    c = 1.0 / (1.0 - 0.25)
    assert np.abs(r["out"] - (resid + r["mask"] * x * c)).max() < 1e-15
    rb = oracle.bias_dropout_add(x, bias, resid, 0.25, 42, 8)
    assert np.array_equal(rb["mask"], r["mask"])
    assert np.abs(rb["out"] - (resid + r["mask"] * (x + bias) * c)).max() < 1e-15
    # a shard's mask is the matching slice of the global one
    lo = oracle.bias_dropout_add(x[4:], bias, resid[4:], 0.25, 42, 8, row_offset=4)
    assert np.array_equal(lo["mask"], r["mask"][4:])
    # element index (row_offset + r)*h + c in site 1, against an independent statement
    from test_oracle_philox import keep_bigint
    for (rr, cc) in [(0, 0), (3, 23), (9, 8)]:
        assert r["mask"][rr, cc] == keep_bigint(42, 8, rr * h + cc, 1, 0.25)
    # backward by autograd on the definition
    dout = _rand((rows, h), 15)
    g = oracle.bias_dropout_add_bwd(dout, 0.25, 42, 8)
    tx, tb, tr = (torch.from_numpy(a).requires_grad_(True) for a in (x, bias, resid))
    (tr + torch.from_numpy(r["mask"].astype(np.float64)) * (tx + tb) * c).backward(torch.from_numpy(dout))
    assert np.abs(g["dx"] - tx.grad.numpy()).max() < 1e-15
    assert np.abs(g["dbias"] - tb.grad.numpy()).max() < 1e-13
    assert np.array_equal(g["dresid"], dout)
