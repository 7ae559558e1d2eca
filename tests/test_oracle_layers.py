"""Pins for the oracle's pooling and stand-alone residual routines and for argument checking."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as wl
from helpers import rq_exact


def test_avgpool_exact_and_close_to_mean():
    g = np.random.default_rng(4)
    N, H, W, C = 3, 7, 7, 16
    x = g.integers(0, 128, size=(N, H, W, C))
    c = np.full(C, 20, np.uint8)
    b = np.full(C, round(2 ** 20 / 49), np.int32)
    y = oracle.avgpool_int(x.astype(np.uint8), b, c, N=N, H=H, W=W, C=C, x_dt=oracle.U8, y_dt=oracle.U8, y_lo=0, y_hi=127)
    s = x.sum(axis=(1, 2))
    for n, k in itertools.product(range(N), range(C)):
        assert int(y[n, k]) == min(max(rq_exact(int(s[n, k]), b[k], 20), 0), 127)
        assert abs(int(y[n, k]) - s[n, k] / 49.0) <= 1.0
    # per-channel multipliers are honoured
    b2 = b.copy(); b2[3] *= 2
    y2 = oracle.avgpool_int(x.astype(np.uint8), b2, c, N=N, H=H, W=W, C=C, x_dt=oracle.U8, y_dt=oracle.U8, y_lo=0, y_hi=255)
    assert np.array_equal(np.delete(y2, 3, axis=1), np.delete(y, 3, axis=1))
    assert (np.abs(y2[:, 3].astype(int) - 2 * s[:, 3] / 49.0) <= 1).all()


def test_maxpool_vs_library():
    import torch
    import torch.nn.functional as F
    g = np.random.default_rng(6)
    for (N, H, W, C) in ((2, 8, 8, 4), (1, 7, 9, 6), (1, 112, 112, 2)):
        x = g.integers(0, 128, size=(N, H, W, C))
        y = oracle.maxpool_int(x.astype(np.uint8), N=N, H=H, W=W, C=C, x_dt=oracle.U8, y_dt=oracle.U8, y_lo=0, y_hi=127)
        ref = F.max_pool2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2), 3, 2, 1).permute(0, 2, 3, 1).numpy()
        assert np.array_equal(y.astype(np.int64), ref.astype(np.int64))
    # 8-bit in, packed 4-bit out (values already within 0..15)
    x = g.integers(0, 16, size=(1, 6, 6, 8))
    y4 = oracle.maxpool_int(x.astype(np.uint8), N=1, H=6, W=6, C=8, x_dt=oracle.U8, y_dt=oracle.U4, y_lo=0, y_hi=15)
    y8 = oracle.maxpool_int(x.astype(np.uint8), N=1, H=6, W=6, C=8, x_dt=oracle.U8, y_dt=oracle.U8, y_lo=0, y_hi=15)
    assert np.array_equal(y4, wl.pack_nibbles(y8.astype(np.int32)))


def test_residual_add_exact_all_types():
    g = np.random.default_rng(8)
    P, K = 37, 10
    for m_dt, lo_m, hi_m in ((oracle.S32, -(1 << 26), 1 << 26), (oracle.U8, 0, 128), (oracle.S8, -128, 128)):
        m = g.integers(lo_m, hi_m, size=(P, K))
        r = g.integers(-128, 128, size=(P, K))
        m_b = g.integers(1 << 14, 1 << 15, size=K); r_b = g.integers(1 << 14, 1 << 15, size=K)
        m_c = g.integers(30, 34, size=K) if m_dt == oracle.S32 else g.integers(14, 17, size=K)
        r_c = g.integers(14, 17, size=K)
        y = oracle.residual_add_dyadic(m, m_b, m_c, r.astype(np.int8), r_b, r_c, n_pixels=P, K=K, m_dt=m_dt, r_dt=oracle.S8,
                                       y_dt=oracle.S8, relu=0, y_lo=-128, y_hi=127)
        for p, k in itertools.product(range(P), range(K)):
            v = rq_exact(m[p, k], m_b[k], m_c[k]) + rq_exact(r[p, k], r_b[k], r_c[k])
            assert int(y[p, k]) == min(max(v, -128), 127)
        yr = oracle.residual_add_dyadic(m, m_b, m_c, r.astype(np.int8), r_b, r_c, n_pixels=P, K=K, m_dt=m_dt, r_dt=oracle.S8,
                                        y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127)
        assert np.array_equal(yr, np.clip(y.astype(int), 0, 127))


def test_argument_errors():
    x = np.zeros((1, 4, 4, 3), np.uint8); w = np.zeros((2, 3, 3, 3), np.int8); z = np.zeros(2, np.int32)
    kw = dict(N=1, H=4, W=4, C=3, K=2, R=3, S=3, stride=1, pad=1, relu=1)
    with pytest.raises(oracle.OracleError):  # clamp outside the type's range
        oracle.conv2d_int(x, w, z, z + 1, np.ones(2, np.uint8), x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8, y_lo=0, y_hi=300, **kw)
    with pytest.raises(oracle.OracleError):  # raw output must be int32
        oracle.conv2d_int(x, w, z, None, None, x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8, y_lo=0, y_hi=127, **kw)
    with pytest.raises(oracle.OracleError):  # odd channel count cannot be packed
        oracle.conv2d_int(np.zeros(24, np.uint8), np.zeros(27, np.uint8), z, z + 1, np.ones(2, np.uint8), x_dt=oracle.U4, w_dt=oracle.S4,
                          y_dt=oracle.U8, y_lo=0, y_hi=15, **kw)
