"""GPU: the dropout masks that the fused attention kernels draw, observed bit for bit through the C ABI.

The recompute kernels never write a mask (Section 5: nothing of size s x s leaves the region), so each kernel's own mask is
made visible through its ordinary outputs by probe inputs; every extracted mask must equal the oracle's Philox mask
(np.array_equal), which also shows that forward and backward use the same one.

  forward     Q = 0 makes every allowed probability of row i equal (1/(i+1) under the causal mask); V_j = e_(j - j0) for
              the d keys of one block [j0, j0 + d) and 0 elsewhere  =>  O_i[x] != 0  <=>  key j0 + x is kept (and allowed).
  column pass dO_i = e_(i - i0) for the d rows of one block and 0 elsewhere  =>  dV_j[x] = D_(i0 + x, j) != 0  <=>  kept.
  dQ          K_j = e_(j - j0) on one block, V_j = e_0, dO_i = e_0 (so dO_i . V_j = 1 everywhere), O = 0 (so the per-row
              term is 0)  =>  dQ_i[x] = alpha dS_(i, j0 + x) != 0  <=>  kept.  In the two-pass backward this is the mask of
              the row pass; in the recompute-once backward it is the mask that went into the stored dS tiles.
ceil(s / d) calls per probe give the whole mask of every head of the shard.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2205_05198_amd as sar
from paper_2205_05198_amd.binding import SAR_BF16

pytestmark = pytest.mark.gpu


def _one_hot_block(s, b, A, d, blk):
    """[s, b, A, d] with row r = e_(r - blk d) for the rows of block blk, 0 elsewhere."""
    x = torch.zeros((s, b, A, d), dtype=torch.bfloat16, device="cuda")
    r = torch.arange(blk * d, min(s, (blk + 1) * d), device="cuda")
    x[r, :, :, r - blk * d] = 1.0
    return x


def _e0(s, b, A, d):
    x = torch.zeros((s, b, A, d), dtype=torch.bfloat16, device="cuda")
    x[..., 0] = 1.0
    return x


def _expected(sh):
    M = oracle.attn_mask(sh)                       # [b, A, s, s], also above the diagonal
    return np.tril(M) if sh.causal else M


def _extract(sh, which, two_pass=False):
    """Mask of every (batch, head) of the shard as drawn by one kernel: uint8 [b, A, s, s]."""
    s, b, A, d = sh.s, sh.b, sh.A, sh.d
    desc = sar.AttnDesc.packed(s, b, sh.a, sh.h, t=sh.t, rank=sh.rank, dtype=SAR_BF16, p=sh.p, seed=sh.seed, offset=sh.offset,
                               scale=sh.alpha(), causal=sh.causal)
    zeros = torch.zeros((s, b, A, d), dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(zeros)
    lse = torch.empty((b, A, s), dtype=torch.float32, device="cuda")
    dq, dk, dv = (torch.empty_like(zeros) for _ in range(3))
    nbytes = sar.attn_core_bwd_workspace_min(desc) if two_pass else sar.attn_core_bwd_workspace(desc)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    got = np.zeros((b, A, s, s), dtype=np.uint8)
    nblk = (s + d - 1) // d
    if which != "fwd":
        # LSE of the all-zero scores: ln(number of allowed keys), from the forward itself
        sar.attn_core_fwd(desc, zeros, zeros, _e0(s, b, A, d), o, lse)
    for blk in range(nblk):
        lo, hi = blk * d, min(s, (blk + 1) * d)
        hot = _one_hot_block(s, b, A, d, blk)
        if which == "fwd":
            sar.attn_core_fwd(desc, zeros, zeros, hot, o, lse)
            torch.cuda.synchronize()
            nz = (o != 0).cpu().numpy()                                     # [i, b, A, x]
            got[:, :, :, lo:hi] = np.transpose(nz, (1, 2, 0, 3))[..., :hi - lo]
        elif which == "dv":
            sar.attn_core_bwd_recompute(desc, zeros, zeros, _e0(s, b, A, d), zeros, lse, hot, dq, dk, dv, ws)
            torch.cuda.synchronize()
            nz = (dv != 0).cpu().numpy()                                    # [j, b, A, x]  ->  M[i0 + x, j]
            got[:, :, lo:hi, :] = np.transpose(nz, (1, 2, 3, 0))[:, :, :hi - lo, :]
        else:
            e0 = _e0(s, b, A, d)
            sar.attn_core_bwd_recompute(desc, zeros, hot, e0, zeros, lse, e0, dq, dk, dv, ws)
            torch.cuda.synchronize()
            nz = (dq != 0).cpu().numpy()                                    # [i, b, A, x]
            got[:, :, :, lo:hi] = np.transpose(nz, (1, 2, 0, 3))[..., :hi - lo]
    return got


def _compare(sh, which, two_pass=False):
    want = _expected(sh)
    got = _extract(sh, which, two_pass)
    bad = int(np.count_nonzero(got != want))
    kept = float(want.sum()) / (want.size / 2 if sh.causal else want.size)
    print(f"  {which} two_pass={two_pass}: {want.size} mask bits, kept fraction of the allowed ones {kept:.4f}, mismatches {bad}", flush=True)
    assert bad == 0, (which, two_pass, bad, np.argwhere(got != want)[:5])


@pytest.mark.parametrize("d,s,causal", [(64, 200, 1), (96, 328, 1), (128, 264, 0), (160, 328, 1), (160, 200, 0)])
def test_fused_kernel_masks_small(d, s, causal):
    """Ragged shapes, every head dimension, with and without the causal mask: forward, column pass and dQ of both forms of the
    backward.  The offset puts the carry of the low counter word inside the tensor."""
    t, A = 2, 2
    count = 2 * t * A * s * s // 8            # Philox calls of the global tensor (b = 2)
    sh = oracle.AttnShape(s=s, b=2, a=A * t, h=A * t * d, t=t, rank=1, p=0.1, seed=1234, offset=(1 << 32) - count + count // 8, causal=causal)   # overflows 7/8 into the global tensor: batch 1 of this rank
    print(f"masks d={d} s={s} causal={causal}", flush=True)
    _compare(sh, "fwd")
    for two_pass in (False, True):
        _compare(sh, "dv", two_pass)
        _compare(sh, "dq", two_pass)


def test_fused_kernel_masks_kernel_variants():
    """The forward's other variants (128-row workgroups; without loader waves; producer / consumer pairs; persistent workgroups)
    and the forms of the column pass draw the same mask."""
    sh = oracle.AttnShape(s=328, b=1, a=4, h=4 * 160, t=2, rank=1, p=0.25, seed=99, offset=12345)
    try:
        for variant in ((1, -1, -1, -1), (0, 0, 0, -1), (0, 1, 1, -1), (0, 2, -1, -1)):
            sar.sar_test_force_variants(*variant)
            print(f"masks variants={variant}", flush=True)
            _compare(sh, "fwd")
            _compare(sh, "dq", two_pass=True)
        # the forward with persistent workgroups, 132 heads: every workgroup takes the three row blocks of its head in turn
        sar.sar_test_force_variants(0, 3, -1, -1)
        print("masks persistent forward", flush=True)
        _compare(oracle.AttnShape(s=328, b=3, a=44, h=44 * 160, p=0.25, seed=99, offset=(1 << 32) - 70000), "fwd")
        # the column pass with persistent workgroups, 132 heads: every workgroup takes the five key blocks of its head in turn
        sar.sar_test_force_variants(-1, -1, -1, 3)
        print("masks persistent column pass", flush=True)
        shp = oracle.AttnShape(s=320, b=3, a=44, h=44 * 160, p=0.25, seed=99, offset=(1 << 32) - 70000)
        for two_pass in (False, True):
            _compare(shp, "dv", two_pass)
        _compare(shp, "dq", False)
        # the column pass in its three forms at a length of full tiles (s % 64 == 0), every head dimension (a form that does not
        # exist at a head dimension falls back to the plain one)
        for d in (64, 96, 128, 160):
            sh2 = oracle.AttnShape(s=320, b=1, a=4, h=4 * d, t=2, rank=1, p=0.25, seed=99, offset=(1 << 32) - 4000)
            for pipe in (0, 1, 2, 3):
                sar.sar_test_force_variants(-1, -1, -1, pipe)
                print(f"masks column pass form={pipe} d={d}", flush=True)
                for two_pass in (False, True):
                    _compare(sh2, "dv", two_pass)
                    _compare(sh2, "dq", two_pass)
    finally:
        sar.sar_test_force_variants(-1, -1, -1, -1)


def test_fused_kernel_masks_530B_shard():
    """The benchmark's shape (530B shard: s = 2048, 16 heads of 160) as rank 3 of 8, every head, in the launch configuration
    that is timed; the offset is chosen so that the low 32-bit word of the Philox counter overflows inside this rank's
    heads (inside head 9 of 16)."""
    s, a, t, rank, d = 2048, 128, 8, 3, 160
    A = a // t
    first = (rank * A) * s * s // 8                 # call index of this rank's first element
    per_head = s * s // 8
    offset = (1 << 32) - first - 9 * per_head - per_head // 3
    sh = oracle.AttnShape(s=s, b=1, a=a, h=a * d, t=t, rank=rank, p=0.1, seed=1234, offset=offset)
    lo = offset + first
    assert lo < (1 << 32) < lo + A * per_head
    print("masks 530B shard", flush=True)
    _compare(sh, "fwd")
    _compare(sh, "dv")
    _compare(sh, "dq")
    _compare(sh, "dv", two_pass=True)
    _compare(sh, "dq", two_pass=True)


def test_fused_kernel_masks_175B_shard_pipelined_column_pass():
    """The 175B shard (s = 2048, 12 heads of 128), where the library picks the software-pipelined column pass: its mask and the
    mask inside the dS tiles it stores, every head, low counter word overflowing inside head 5."""
    s, a, t, rank, d = 2048, 96, 8, 6, 128
    A = a // t
    first = (rank * A) * s * s // 8
    per_head = s * s // 8
    offset = (1 << 32) - first - 5 * per_head - per_head // 7
    sh = oracle.AttnShape(s=s, b=1, a=a, h=a * d, t=t, rank=rank, p=0.1, seed=4321, offset=offset)
    print("masks 175B shard", flush=True)
    _compare(sh, "dv")
    _compare(sh, "dq")
