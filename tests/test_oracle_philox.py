"""Pins for the oracle's Philox generator and the dropout-mask mapping (CPU only)."""
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK32 = (1 << 32) - 1


def philox_bigint(ctr, key):
    """Independent re-statement of Philox4x32-10 with Python integers (Salmon et al., SC'11)."""
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        p0 = M0 * c[0]
        p1 = M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & MASK32, p1 & MASK32, ((p0 >> 32) ^ c[3] ^ k[1]) & MASK32, p0 & MASK32]
        k = [(k[0] + W0) & MASK32, (k[1] + W1) & MASK32]
    return c


def keep_bigint(seed, offset, e, site, p):
    T = int(np.floor(float(np.float32(p)) * 65536.0 + 0.5))
    G = (offset + (e >> 3)) & ((1 << 64) - 1)
    out = philox_bigint([G & MASK32, G >> 32, 0, site], [seed & MASK32, seed >> 32])
    r = e & 7
    u = (out[r >> 1] >> (16 * (r & 1))) & 0xFFFF
    return int(u >= T)


def test_known_answer_vectors():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert oracle.philox4x32_10(v[0:4], v[4:6]) == v[6:10]
        assert philox_bigint(v[0:4], v[4:6]) == v[6:10]


def test_c_matches_bigint_random():
    g = np.random.default_rng(7)
    for _ in range(2000):
        ctr = [int(x) for x in g.integers(0, 1 << 32, 4)]
        key = [int(x) for x in g.integers(0, 1 << 32, 2)]
        assert oracle.philox4x32_10(ctr, key) == philox_bigint(ctr, key)


def test_threshold():
    assert oracle.dropout_threshold(0.1) == 6554
    assert oracle.dropout_threshold(0.0) == 0
    assert oracle.dropout_threshold(0.5) == 32768


def test_mask_mapping_matches_bigint():
    g = np.random.default_rng(11)
    for _ in range(500):
        seed = int(g.integers(0, 1 << 63)) * 2 + 1
        offset = int(g.integers(0, 1 << 62))
        e = int(g.integers(0, 1 << 40))
        site = int(g.integers(0, 2))
        T = oracle.dropout_threshold(0.1)
        assert oracle.keep_bit(seed, offset, e, site, T) == keep_bigint(seed, offset, e, site, 0.1)
    # 64-bit wrap of the call counter and carry into the high counter word
    T = oracle.dropout_threshold(0.3)
    for e in (0, 7, 8, 15, 16):
        assert oracle.keep_bit(5, (1 << 64) - 1, e, 0, T) == keep_bigint(5, (1 << 64) - 1, e, 0, 0.3)
        assert oracle.keep_bit(5, (1 << 32) - 1, e, 0, T) == keep_bigint(5, (1 << 32) - 1, e, 0, 0.3)


def test_attn_mask_indexing_and_sharding():
    # global a=4 heads, t=2: the two ranks' masks are the halves of the t=1 mask
    full = oracle.attn_mask(oracle.AttnShape(s=16, b=2, a=4, h=32, t=1, p=0.25, seed=99, offset=1000))
    r0 = oracle.attn_mask(oracle.AttnShape(s=16, b=2, a=4, h=32, t=2, rank=0, p=0.25, seed=99, offset=1000))
    r1 = oracle.attn_mask(oracle.AttnShape(s=16, b=2, a=4, h=32, t=2, rank=1, p=0.25, seed=99, offset=1000))
    assert np.array_equal(full[:, 0:2], r0) and np.array_equal(full[:, 2:4], r1)
    # element index ((beta*a + n)*s + i)*s + j, checked against the big-int statement
    for (be, n, i, j) in [(0, 0, 0, 0), (1, 3, 15, 15), (1, 2, 7, 9), (0, 1, 8, 0)]:
        e = ((be * 4 + n) * 16 + i) * 16 + j
        assert full[be, n, i, j] == keep_bigint(99, 1000, e, 0, 0.25)


def test_keep_rate_and_special_cases():
    sh = oracle.AttnShape(s=256, b=1, a=4, h=64, p=0.1, seed=1234)
    M = oracle.attn_mask(sh)
    n = M.size
    T = oracle.dropout_threshold(0.1)
    q = 1.0 - T / 65536.0
    assert abs(M.mean() - q) < 4.0 * np.sqrt(q * (1 - q) / n)
    assert oracle.attn_mask(oracle.AttnShape(s=32, b=1, a=2, h=16, p=0.0, seed=1)).all()
    # a different offset window gives an (almost) independent mask
    M2 = oracle.attn_mask(oracle.AttnShape(s=256, b=1, a=4, h=64, p=0.1, seed=1234, offset=oracle.attn_philox_count(sh)))
    agree = (M == M2).mean()
    expect = q * q + (1 - q) * (1 - q)
    assert abs(agree - expect) < 0.01
    # and a different site too
    x = np.zeros((8, 64))
    m_site1 = oracle.bias_dropout_add(x, None, x, 0.1, 1234, 0)["mask"]
    assert not np.array_equal(m_site1.ravel()[:512], M.ravel()[:512])
    assert oracle.attn_philox_count(sh) == 1 * 4 * 256 * 256 // 8
