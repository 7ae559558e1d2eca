"""Pins for the oracle's INT32 pooling and per-branch dyadic concatenation (Appendix E: the Inception module)."""
import itertools

import numpy as np
import pytest

import oracle
import workloads as wl
from helpers import rq_exact, dyadic_from_real


def test_window_sum_vs_library_average_pool():
    """count-include-pad average pool of the float64 library, times the window size, is the window sum exactly."""
    import torch
    import torch.nn.functional as F
    g = np.random.default_rng(3)
    for (N, H, W, C, R, stride, pad) in ((2, 8, 9, 5, 3, 1, 1), (1, 7, 7, 4, 3, 2, 1), (1, 6, 6, 3, 2, 2, 0), (1, 9, 9, 2, 5, 1, 2)):
        x = g.integers(-(1 << 20), 1 << 20, size=(N, H, W, C))
        s = oracle.pool2d_sum_int(x.astype(np.int32), None, None, N=N, H=H, W=W, C=C, R=R, S=R, stride=stride, pad=pad,
                                  x_dt=oracle.S32, y_dt=oracle.S32)
        ref = F.avg_pool2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2), R, stride, pad, count_include_pad=True) * (R * R)
        assert np.array_equal(s.astype(np.int64), np.rint(ref.permute(0, 2, 3, 1).numpy()).astype(np.int64))


def test_window_sum_rescaled_is_the_rounded_average():
    """With 1/(R*S) folded into the dyadic number the result is the rounded mean (within the DN error), exact against rationals."""
    g = np.random.default_rng(5)
    N, H, W, C = 1, 6, 7, 6
    x = g.integers(0, 128, size=(N, H, W, C))
    b1, c1 = dyadic_from_real(1.0 / 9.0)
    b = np.full(C, b1, np.int32); c = np.full(C, c1, np.uint8)
    b[2] = 2 * b1                                # per-channel multipliers are honoured
    y = oracle.pool2d_sum_int(x.astype(np.uint8), b, c, N=N, H=H, W=W, C=C, R=3, S=3, stride=1, pad=1, x_dt=oracle.U8, y_dt=oracle.U8,
                              y_lo=0, y_hi=255)
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    for p, q, k in itertools.product(range(H), range(W), range(C)):
        s = int(xp[0, p:p + 3, q:q + 3, k].sum())
        assert int(y[0, p, q, k]) == min(max(rq_exact(s, b[k], c[k]), 0), 255)
        if k != 2:
            assert abs(int(y[0, p, q, k]) - s / 9.0) <= 0.51
    # packed 4-bit input gives what its values give
    x4 = g.integers(0, 16, size=(N, H, W, C))
    a = oracle.pool2d_sum_int(wl.pack_nibbles(x4), None, None, N=N, H=H, W=W, C=C, R=3, S=3, stride=1, pad=1, x_dt=oracle.U4, y_dt=oracle.S32)
    a8 = oracle.pool2d_sum_int(x4.astype(np.uint8), None, None, N=N, H=H, W=W, C=C, R=3, S=3, stride=1, pad=1, x_dt=oracle.U8, y_dt=oracle.S32)
    assert np.array_equal(a, a8)


def test_concat_every_branch_has_its_own_dyadic_number():
    g = np.random.default_rng(9)
    P = 23
    Ks = (6, 4, 10, 2)
    dts = (oracle.S32, oracle.U8, oracle.S8, oracle.S32)
    qs, bs, cs = [], [], []
    for K, dt in zip(Ks, dts):
        if dt == oracle.S32:
            q = g.integers(-(1 << 24), 1 << 24, size=(P, K)); c = g.integers(18, 22, size=K)
        elif dt == oracle.U8:
            q = g.integers(0, 128, size=(P, K)); c = g.integers(14, 16, size=K)
        else:
            q = g.integers(-128, 128, size=(P, K)); c = g.integers(14, 16, size=K)
        qs.append(q); bs.append(g.integers(1 << 14, 1 << 15, size=K)); cs.append(c)
    stored = [q.astype({oracle.S32: np.int32, oracle.U8: np.uint8, oracle.S8: np.int8}[dt]) for q, dt in zip(qs, dts)]
    y = oracle.concat_dyadic(list(zip(stored, dts, bs, cs)), n_pixels=P, y_dt=oracle.S8, y_lo=-128, y_hi=127)
    assert y.shape == (P, sum(Ks))
    off = 0
    seen = set()
    for q, b, c, K in zip(qs, bs, cs, Ks):
        for p, k in itertools.product(range(P), range(K)):
            v = min(max(rq_exact(q[p, k], b[k], c[k]), -128), 127)
            assert int(y[p, off + k]) == v
            seen.add(v)
        off += K
    assert len(seen) > 50
    # changing one branch's multiplier changes that branch's slice only
    bs2 = [b.copy() for b in bs]; bs2[1] = bs2[1] // 2
    y2 = oracle.concat_dyadic(list(zip(stored, dts, bs2, cs)), n_pixels=P, y_dt=oracle.S8, y_lo=-128, y_hi=127)
    assert np.array_equal(np.delete(y2, np.s_[6:10], axis=1), np.delete(y, np.s_[6:10], axis=1)) and not np.array_equal(y2, y)
    # 4-bit output: packed, branch boundaries on even channels
    y4 = oracle.concat_dyadic(list(zip(stored, dts, bs, cs)), n_pixels=P, y_dt=oracle.U4, y_lo=0, y_hi=15)
    assert np.array_equal(y4, wl.pack_nibbles(np.clip(y.astype(np.int32), 0, 15)))


def test_concat_tracks_the_real_valued_module_output():
    """Appendix E's equation: integers q_i at scales S_i, each rescaled by DN(S_i / S_a); the result represents the real
    values S_i q_i at scale S_a to within half a step plus the DN error."""
    g = np.random.default_rng(12)
    P, S_a = 40, 0.05
    scales = (0.003, 0.02, 0.0007)
    branches, real = [], []
    for S_i in scales:
        K = 8
        q = g.integers(-int(3 / S_i), int(3 / S_i), size=(P, K))
        b, c = dyadic_from_real(S_i / S_a)
        branches.append((q.astype(np.int32), oracle.S32, np.full(K, b, np.int32), np.full(K, c, np.uint8)))
        real.append(q * S_i)
    y = oracle.concat_dyadic(branches, n_pixels=P, y_dt=oracle.S8, y_lo=-128, y_hi=127).astype(np.float64) * S_a
    want = np.concatenate(real, axis=1)
    assert np.abs(y - want).max() <= S_a * (0.5 + 1e-3) + 3 * 2.0 ** -15
    assert np.abs(y).max() > 2.5


def test_argument_errors():
    x = np.zeros((1, 4, 4, 3), np.int32)
    with pytest.raises(oracle.OracleError):      # raw sums are INT32
        oracle.pool2d_sum_int(x, None, None, N=1, H=4, W=4, C=3, R=3, S=3, stride=1, pad=1, x_dt=oracle.S32, y_dt=oracle.U8)
    with pytest.raises(oracle.OracleError):      # window larger than the padded image
        oracle.pool2d_sum_int(x, None, None, N=1, H=4, W=4, C=3, R=7, S=7, stride=1, pad=1, x_dt=oracle.S32, y_dt=oracle.S32)
    with pytest.raises(oracle.OracleError):      # odd branch width cannot be packed
        oracle.concat_dyadic([(np.zeros((2, 3), np.int32), oracle.S32, np.ones(3, np.int32), np.ones(3, np.uint8))], n_pixels=2,
                             y_dt=oracle.U4, y_lo=0, y_hi=15)
