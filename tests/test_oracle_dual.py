"""Pins for the oracle's two-convolution block output (Section 3.3's residual equation with an INT32
accumulator on both branches, as Figure 2 draws a block that changes shape)."""
import itertools

import numpy as np
import pytest

import oracle
import workloads as wl
from helpers import rq_exact, conv2d_bruteforce, conv2d_f64


def _golden(golden_dir):
    vals = {}
    for line in open(str(golden_dir) + "/residual_rounding_example.txt"):
        if line.strip() and not line.startswith("#"):
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    return vals


def _case(seed, N, H, C, K, R, stride, Cs, stride_s, bits=8):
    """Main branch: R x R conv over [N,H,H,C] with `stride`; shortcut: 1x1 / stride_s over [N,Hs,Hs,Cs] giving the same
    output size."""
    g = np.random.default_rng(seed)
    pad = R // 2
    P = (H + 2 * pad - R) // stride + 1
    Hs = (P - 1) * stride_s + 1
    hi, wm = (127, 127) if bits == 8 else (15, 7)
    d = dict(N=N, K=K, H=H, W=H, C=C, R=R, S=R, stride=stride, pad=pad, Hs=Hs, Ws=Hs, Cs=Cs, Rs=1, Ss=1, stride_s=stride_s, pad_s=0)
    t = dict(x=g.integers(0, hi + 1, size=(N, H, H, C)), w=g.integers(-wm, wm + 1, size=(K, R, R, C)),
             xs=g.integers(0, hi + 1, size=(N, Hs, Hs, Cs)), ws=g.integers(-wm, wm + 1, size=(K, 1, 1, Cs)),
             bias=g.integers(-3000, 3000, size=K), bias_s=g.integers(-3000, 3000, size=K),
             b=g.integers(1 << 14, 1 << 15, size=K), b_s=g.integers(1 << 14, 1 << 15, size=K))
    kd, kds = R * R * C, Cs
    t["c"] = (14 + int(np.log2(kd * hi * wm / 8 / 40)) + g.integers(0, 2, size=K)).astype(np.uint8)
    t["c_s"] = (14 + int(np.log2(kds * hi * wm / 8 / 40)) + g.integers(0, 2, size=K)).astype(np.uint8)
    return d, t, P


def test_printed_example_each_branch_rounds_before_the_add(golden_dir):
    """Appendix G: m = 4.4 and r = 2.4 at output scale 1 give 4 + 2 = 6 on integer hardware, 7 if the real values
    were added first.  Realised with 1x1 convolutions: accumulators 22 and 12, both multiplied by 13107 / 2^16 ~ 0.2."""
    gold = _golden(golden_dir)
    one = np.ones(1, np.int32)
    kw = dict(N=1, K=1, H=1, W=1, C=1, R=1, S=1, stride=1, pad=0, Hs=1, Ws=1, Cs=1, Rs=1, Ss=1, stride_s=1, pad_s=0,
              x_dt=oracle.U8, w_dt=oracle.S8, xs_dt=oracle.U8, ws_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127)
    b, c = 13107 * one, 16 * np.ones(1, np.uint8)
    assert abs(22 * 13107 / 65536 - gold["m"]) < 1e-3 and abs(12 * 13107 / 65536 - gold["r"]) < 1e-3
    y = oracle.conv2d_dual_int(np.array([11], np.uint8), np.array([2], np.int8), 0 * one, b, c,
                               np.array([6], np.uint8), np.array([2], np.int8), 0 * one, b, c, **kw)
    assert int(y.ravel()[0]) == int(gold["integer_only_result"])
    assert round((22 + 12) * 13107 / 65536) == int(gold["fake_quant_result"])   # what joint rounding would give
    # the bias belongs to its own branch's accumulator: moving 10 units from one accumulator's inputs to its bias changes nothing
    y2 = oracle.conv2d_dual_int(np.array([6], np.uint8), np.array([2], np.int8), 10 * one, b, c,
                                np.array([1], np.uint8), np.array([2], np.int8), 10 * one, b, c, **kw)
    assert int(y2.ravel()[0]) == int(gold["integer_only_result"])


@pytest.mark.parametrize("R,stride,stride_s", [(1, 1, 1), (1, 1, 2), (3, 1, 2), (3, 1, 1)])
def test_against_bruteforce_accumulators_and_exact_rationals(R, stride, stride_s):
    d, t, P = _case(11 + R + stride_s, N=2, H=5, C=6, K=4, R=R, stride=stride, Cs=10, stride_s=stride_s)
    y = oracle.conv2d_dual_int(t["x"].astype(np.uint8), t["w"].astype(np.int8), t["bias"], t["b"], t["c"],
                               t["xs"].astype(np.uint8), t["ws"].astype(np.int8), t["bias_s"], t["b_s"], t["c_s"],
                               x_dt=oracle.U8, w_dt=oracle.S8, xs_dt=oracle.U8, ws_dt=oracle.S8, y_dt=oracle.S8,
                               relu=0, y_lo=-128, y_hi=127, **d)
    am = conv2d_bruteforce(t["x"], t["w"], (stride, stride), (R // 2, R // 2))
    as_ = conv2d_bruteforce(t["xs"], t["ws"], (stride_s, stride_s), (0, 0))
    assert am.shape == as_.shape == (2, P, P, 4)
    seen_neg = seen_pos = False
    for n, p, q, k in itertools.product(range(2), range(P), range(P), range(4)):
        v = rq_exact(am[n, p, q, k] + t["bias"][k], t["b"][k], t["c"][k]) + rq_exact(as_[n, p, q, k] + t["bias_s"][k], t["b_s"][k], t["c_s"][k])
        assert int(y[n, p, q, k]) == min(max(v, -128), 127)
        seen_neg |= -128 < v < 0
        seen_pos |= 0 < v < 127
    assert seen_neg and seen_pos


def test_equals_composition_of_pinned_routines_and_packed_operands():
    """Raw INT32 outputs of the single-convolution routine fed to the stand-alone residual addition give the same block
    output; 4-bit packed operands give what their unpacked values give."""
    d, t, P = _case(5, N=2, H=8, C=16, K=8, R=1, stride=1, Cs=32, stride_s=2, bits=4)
    args = dict(x_dt=oracle.U4, w_dt=oracle.S4, xs_dt=oracle.U4, ws_dt=oracle.S4, y_dt=oracle.U4, relu=1, y_lo=0, y_hi=15)
    y = oracle.conv2d_dual_int(wl.pack_nibbles(t["x"]), wl.pack_nibbles(t["w"]), t["bias"], t["b"], t["c"],
                               wl.pack_nibbles(t["xs"]), wl.pack_nibbles(t["ws"]), t["bias_s"], t["b_s"], t["c_s"], **d, **args)
    full = (1 << 31) - 1
    m = oracle.conv2d_int(wl.pack_nibbles(t["x"]), wl.pack_nibbles(t["w"]), t["bias"], None, None, N=2, H=8, W=8, C=16, K=8, R=1, S=1,
                          stride=1, pad=0, x_dt=oracle.U4, w_dt=oracle.S4, y_dt=oracle.S32, relu=0, y_lo=-full - 1, y_hi=full)
    r = oracle.conv2d_int(wl.pack_nibbles(t["xs"]), wl.pack_nibbles(t["ws"]), t["bias_s"], None, None, N=2, H=d["Hs"], W=d["Hs"], C=32, K=8,
                          R=1, S=1, stride=2, pad=0, x_dt=oracle.U4, w_dt=oracle.S4, y_dt=oracle.S32, relu=0, y_lo=-full - 1, y_hi=full)
    assert np.array_equal(m.astype(np.int64), conv2d_f64(t["x"], t["w"], (1, 1), (0, 0)) + t["bias"])
    ref = oracle.residual_add_dyadic(m, t["b"], t["c"], r, t["b_s"], t["c_s"], n_pixels=2 * P * P, K=8, m_dt=oracle.S32, r_dt=oracle.S32,
                                     y_dt=oracle.U4, relu=1, y_lo=0, y_hi=15)
    assert np.array_equal(y.reshape(-1), ref.reshape(-1))
    y8 = oracle.conv2d_dual_int(t["x"].astype(np.uint8), t["w"].astype(np.int8), t["bias"], t["b"], t["c"],
                                t["xs"].astype(np.uint8), t["ws"].astype(np.int8), t["bias_s"], t["b_s"], t["c_s"], **d,
                                x_dt=oracle.U8, w_dt=oracle.S8, xs_dt=oracle.U8, ws_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=15)
    assert np.array_equal(y, wl.pack_nibbles(y8.astype(np.int32)))
    assert 0 < np.count_nonzero(y8) and (y8 < 15).any()


def test_shape_mismatch_is_an_error():
    d, t, P = _case(3, N=1, H=6, C=4, K=2, R=1, stride=1, Cs=4, stride_s=1)
    d["Hs"] += 1
    with pytest.raises((oracle.OracleError, AssertionError)):
        oracle.conv2d_dual_int(t["x"].astype(np.uint8), t["w"].astype(np.int8), t["bias"], t["b"], t["c"],
                               np.zeros((1, d["Hs"], d["Ws"], 4), np.uint8), t["ws"].astype(np.int8), t["bias_s"], t["b_s"], t["c_s"],
                               x_dt=oracle.U8, w_dt=oracle.S8, xs_dt=oracle.U8, ws_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127, **d)
