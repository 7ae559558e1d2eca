"""Pins for the oracle's quantised convolution / GEMM layer (Section 3.1, Appendix D)."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as wl
from helpers import (rq_exact, dyadic_from_real, quantize_symmetric_per_channel, conv2d_bruteforce, conv2d_f64)


def _raw_acc(case, stride, pad):
    """Accumulator + bias through the oracle (INT32 output, no requantisation)."""
    return oracle.conv2d_int(case["x"], case["w"], case["bias"], None, None, N=case["N"], H=case["H"], W=case["W"],
                             C=case["C"], K=case["K"], R=case["R"], S=case["S"], stride=stride, pad=pad,
                             x_dt=oracle.U8 if case["bits"] == 8 else oracle.U4,
                             w_dt=oracle.S8 if case["bits"] == 8 else oracle.S4,
                             y_dt=oracle.S32, relu=0, y_lo=-(1 << 31), y_hi=(1 << 31) - 1)


@pytest.mark.parametrize("R,S", [(1, 1), (3, 3), (2, 3)])
@pytest.mark.parametrize("stride", [(1, 1), (2, 2), (2, 1)])
@pytest.mark.parametrize("pad", [(0, 0), (1, 1), (1, 2)])
def test_accumulator_vs_python_bruteforce(R, S, stride, pad):
    case = wl.conv_case(seed=100 + R * 7 + S, N=2, H=6, W=5, C=4, K=3, R=R, S=S, stride=1, pad=0, bits=8)
    got = _raw_acc(case, stride, pad)
    want = conv2d_bruteforce(case["x_vals"], case["w_vals"], stride, pad) + case["bias"].astype(np.int64)
    assert np.array_equal(got.astype(np.int64), want)


@pytest.mark.parametrize("shape", [(2, 9, 11, 16, 8, 3, 3, (1, 1), (1, 1)), (1, 14, 14, 32, 24, 1, 1, (2, 2), (0, 0)),
                                   (3, 8, 8, 6, 10, 5, 5, (2, 2), (2, 2)), (1, 17, 13, 3, 8, 7, 7, (2, 2), (3, 3))])
def test_accumulator_vs_float64_library_conv(shape):
    N, H, W, C, K, R, S, stride, pad = shape
    case = wl.conv_case(seed=7, N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=1, pad=0, bits=8)
    got = _raw_acc(case, stride, pad)
    want = conv2d_f64(case["x_vals"], case["w_vals"], stride, pad) + case["bias"].astype(np.int64)
    assert np.array_equal(got.astype(np.int64), want)


def test_full_layer_vs_exact_rationals():
    """conv + bias + dyadic + residual (rounded separately) + ReLU + clamp, all in Python ints."""
    case = wl.conv_case(seed=21, N=1, H=5, W=5, C=8, K=6, R=3, S=3, stride=1, pad=1, bits=8, with_residual=True,
                        c_range=(24, 27))
    y = oracle.conv2d_int(case["x"], case["w"], case["bias"], case["b"], case["c"], N=1, H=5, W=5, C=8, K=6, R=3, S=3,
                          stride=1, pad=1, x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127,
                          residual=case["residual"], res_b=case["res_b"], res_c=case["res_c"], res_dt=oracle.U8)
    acc = conv2d_bruteforce(case["x_vals"], case["w_vals"], (1, 1), (1, 1))
    seen_mid = 0
    for p, q, k in itertools.product(range(5), range(5), range(6)):
        t = int(acc[0, p, q, k]) + int(case["bias"][k])
        v = rq_exact(t, case["b"][k], case["c"][k]) + rq_exact(case["res_vals"][0, p, q, k], case["res_b"][k], case["res_c"][k])
        v = min(max(v, 0), 127)
        seen_mid += 0 < v < 127
        assert int(y[0, p, q, k]) == v
    assert seen_mid > 20  # the case is not saturated


def test_signed_output_no_relu_and_signed_residual():
    case = wl.conv_case(seed=22, N=1, H=4, W=4, C=8, K=4, R=1, S=1, stride=1, pad=0, bits=8, with_residual=True,
                        res_signed=True, c_range=(22, 24))
    y = oracle.conv2d_int(case["x"], case["w"], case["bias"], case["b"], case["c"], N=1, H=4, W=4, C=8, K=4, R=1, S=1,
                          stride=1, pad=0, x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.S8, relu=0, y_lo=-128, y_hi=127,
                          residual=case["residual"], res_b=case["res_b"], res_c=case["res_c"], res_dt=oracle.S8)
    acc = conv2d_bruteforce(case["x_vals"], case["w_vals"], (1, 1), (0, 0))
    neg = 0
    for p, q, k in itertools.product(range(4), range(4), range(4)):
        t = int(acc[0, p, q, k]) + int(case["bias"][k])
        v = rq_exact(t, case["b"][k], case["c"][k]) + rq_exact(case["res_vals"][0, p, q, k], case["res_b"][k], case["res_c"][k])
        v = min(max(v, -128), 127)
        neg += v < 0
        assert int(y[0, p, q, k]) == v
    assert neg > 0


def test_gemm_vs_numpy_int64_matmul():
    g = np.random.default_rng(9)
    M, N, K = 13, 10, 40
    x = g.integers(0, 128, size=(M, K))
    w = g.integers(-127, 128, size=(N, K))
    bias = g.integers(-1000, 1000, size=N)
    y = oracle.gemm_int(x.astype(np.uint8), w.astype(np.int8), bias, None, None, M=M, N=N, K=K,
                        x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.S32)
    assert np.array_equal(y.astype(np.int64), x.astype(np.int64) @ w.astype(np.int64).T + bias)


def test_int4_encoding_invariant_and_roundtrip():
    """A packed 4-bit layer equals the 8-bit layer on the same logical values."""
    case = wl.conv_case(seed=33, N=2, H=7, W=7, C=16, K=8, R=3, S=3, stride=1, pad=1, bits=4, with_residual=True,
                        c_range=(19, 21), bias_mag=256)
    assert np.array_equal(oracle.unpack(case["x"], oracle.U4), case["x_vals"].ravel())
    assert np.array_equal(oracle.unpack(case["w"], oracle.S4), case["w_vals"].ravel())
    # nibble order: even element in the low nibble
    assert int(case["x"].ravel()[0]) == int(case["x_vals"].ravel()[0]) | (int(case["x_vals"].ravel()[1]) << 4)
    kw = dict(N=2, H=7, W=7, C=16, K=8, R=3, S=3, stride=1, pad=1, relu=1, y_lo=0, y_hi=15,
              res_b=case["res_b"], res_c=case["res_c"])
    y4 = oracle.conv2d_int(case["x"], case["w"], case["bias"], case["b"], case["c"], x_dt=oracle.U4, w_dt=oracle.S4,
                           y_dt=oracle.U4, residual=case["residual"], res_dt=oracle.U4, **kw)
    y8 = oracle.conv2d_int(case["x_vals"].astype(np.uint8), case["w_vals"].astype(np.int8), case["bias"], case["b"],
                           case["c"], x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8,
                           residual=case["res_vals"].astype(np.uint8), res_dt=oracle.U8, **kw)
    assert y4.shape == (2, 7, 7, 4)
    assert np.array_equal(oracle.unpack(y4, oracle.U4), y8.ravel().astype(np.int32))
    assert np.array_equal(wl.pack_nibbles(y8.astype(np.int32)), y4)
    assert 0 < (y8 > 0).mean() < 1


def test_negative_int4_weights_sign_extend():
    w = np.array([[-8, -7, -1, 0, 1, 7, -3, 3]], dtype=np.int32)
    packed = wl.pack_nibbles(w)
    assert list(oracle.unpack(packed, oracle.S4)) == list(w[0])
    assert list(oracle.unpack(packed, oracle.U4)) == [8, 9, 15, 0, 1, 7, 13, 3]


def test_no_int32_overflow_bounds_and_detection():
    """Closed-form bound: R*S*C*xmax*wmax + |bias| stays below 2^31 for every layer of the workloads;
    the oracle flags an accumulator that does leave int32."""
    worst = 0
    for arch in (18, 50):
        for l in wl.resnet_layers(arch):
            xmax = 255 if l["kind"] == "stem" else 127
            worst = max(worst, l["R"] * l["S"] * l["C"] * xmax * 127 + (1 << 24))
    assert worst < (1 << 31)
    assert 4608 * 127 * 127 + (1 << 15) == 74355200
    # 2^31 / (255*128) = 65793.0..: a 1x1 conv over that many channels of extreme values overflows
    C = 65800
    x = np.full((1, 1, 1, C), 255, dtype=np.uint8)
    w = np.full((1, 1, 1, C), -128, dtype=np.int8)
    with pytest.raises(oracle.OracleError) as e:
        oracle.conv2d_int(x, w, np.zeros(1, np.int32), None, None, N=1, H=1, W=1, C=C, K=1, R=1, S=1, stride=1, pad=0,
                          x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.S32, relu=0, y_lo=-(1 << 31), y_hi=(1 << 31) - 1)
    assert e.value.code == oracle.ERR_OVERFLOW


def test_folded_batchnorm_matches_unfolded_and_integer_path_tracks_real():
    """Appendix D: CONV_BN(h) = (beta W / sigma) h + (gamma - beta mu / sigma); the bias is quantised at scale
    S_h * S_Wbar so it adds to the accumulator; Section 3.1: the dyadic requantiser reproduces Int(a / S_a)."""
    g = np.random.default_rng(17)
    N, H, Wd, C, K = 1, 6, 6, 8, 5
    h = np.abs(g.normal(0, 1, size=(N, H, Wd, C)))
    Wt = g.normal(0, 0.2, size=(K, 3, 3, C))
    beta, gamma = g.uniform(0.5, 1.5, K), g.normal(0, 0.3, K)
    mu, sigma = g.normal(0, 0.5, K), g.uniform(0.5, 2.0, K)
    import torch
    import torch.nn.functional as F
    def conv(hh, ww):
        y = F.conv2d(torch.from_numpy(hh).permute(0, 3, 1, 2), torch.from_numpy(ww).permute(0, 3, 1, 2), padding=1)
        return y.permute(0, 2, 3, 1).numpy()
    unfolded = beta * (conv(h, Wt) - mu) / sigma + gamma
    Wbar = Wt * (beta / sigma).reshape(K, 1, 1, 1)
    bbar = gamma - beta * mu / sigma
    folded = conv(h, Wbar) + bbar
    assert np.allclose(unfolded, folded, rtol=1e-9, atol=1e-12)
    # quantise: activations unsigned 8-bit range 0..127 (zero point 0 after ReLU), weights symmetric per channel
    S_h = h.max() / 127.0
    q_h = np.rint(h / S_h).astype(np.int64)
    q_w, S_w = quantize_symmetric_per_channel(Wbar, 8)
    assert np.abs(q_w).max() <= 127
    q_b = np.rint(bbar / (S_h * S_w)).astype(np.int64)         # S_bbar = S_h * S_Wbar
    real_out = np.maximum(folded, 0)
    S_a = real_out.max() / 127.0
    bc = [dyadic_from_real(S_h * s / S_a) for s in S_w]
    b = np.array([v[0] for v in bc], dtype=np.int32)
    c = np.array([v[1] for v in bc], dtype=np.uint8)
    y = oracle.conv2d_int(q_h.astype(np.uint8), q_w.astype(np.int8), q_b.astype(np.int32), b, c, N=N, H=H, W=Wd, C=C, K=K,
                          R=3, S=3, stride=1, pad=1, x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127)
    # (i) against Int(a/S_a) of the real-valued fake-quantised layer: at most one step apart (DN error 2^-15)
    a = conv(q_h * S_h, q_w * S_w.reshape(K, 1, 1, 1)) + q_b * S_h * S_w
    fake = np.clip(np.floor(a / S_a + 0.5), 0, 127)
    assert np.abs(y.astype(np.int64) - fake.astype(np.int64)).max() <= 1
    assert (y.astype(np.int64) == fake.astype(np.int64)).mean() > 0.98
    # (ii) against the un-quantised layer: within the accumulated quantisation error
    #      |h - S_h q_h| <= S_h/2, |W - S_w q_w| <= S_w/2, |bbar - S_b q_b| <= S_h S_w / 2, 72 taps per output,
    #      plus half a step for the final rounding and one step for the dyadic approximation
    err_in = 0.5 * S_h * np.abs(Wbar).reshape(K, -1).sum(1) + 0.5 * S_w * 72 * (h.max() + 0.5 * S_h) + 0.5 * S_h * S_w
    bound = err_in / S_a + 1.5
    assert (np.abs(y * S_a - real_out) / S_a <= bound + 1e-9).all()
    assert 0.1 < (y > 0).mean() and y.max() >= 100
