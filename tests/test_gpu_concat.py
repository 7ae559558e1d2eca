"""GPU parity: hawq_pool2d_sum_int and hawq_concat_dyadic (Appendix E: the pooling branch carried in INT32 and the
concatenation with one dyadic number per branch) vs the CPU oracle, bit-exact; and an Inception-style module assembled
from the library's calls against the same assembly of oracle routines."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

_NP = {0: np.uint8, 1: np.int8, 2: np.uint8, 3: np.uint8, 4: np.int32}


@pytest.fixture(scope="module")
def hawq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2011_10680_amd as h
    h.load_library()
    return h


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _empty(shape, dt):
    import torch
    shape = list(shape)
    if dt in (2, 3):
        shape[-1] //= 2
    tdt = {np.uint8: torch.uint8, np.int8: torch.int8, np.int32: torch.int32}[_NP[dt]]
    return torch.full(shape, 0x5A, dtype=tdt, device="cuda")


def _draw(g, shape, dt):
    if dt == oracle.S32:
        return g.integers(-(1 << 22), 1 << 22, size=shape).astype(np.int32)
    if dt == oracle.U8:
        return g.integers(0, 128, size=shape).astype(np.uint8)
    if dt == oracle.S8:
        return g.integers(-128, 128, size=shape).astype(np.int8)
    return wl.pack_nibbles(g.integers(0, 16, size=shape))


# (N, H, W, C, R, stride, pad, x_dt, y_dt): the Inception pooling branch (3x3 / 1 / 1 on INT32) and variations
_POOLS = [
    (2, 17, 17, 64, 3, 1, 1, oracle.S32, oracle.S32),
    (2, 17, 17, 64, 3, 1, 1, oracle.S32, oracle.U8),
    (3, 9, 11, 6, 3, 2, 1, oracle.S32, oracle.S8),      # odd sizes, C % 4 != 0
    (1, 8, 8, 32, 2, 2, 0, oracle.U8, oracle.U8),
    (2, 7, 7, 16, 5, 1, 2, oracle.U4, oracle.U4),
    (1, 35, 35, 192, 3, 1, 1, oracle.U8, oracle.S32),
    (2, 5, 13, 8, 3, 1, 1, oracle.U8, oracle.U4),       # the 3x3 fast path with a ragged last block of columns, packed output
    (1, 3, 3, 4, 3, 1, 1, oracle.S32, oracle.S8),
    (0, 8, 8, 4, 3, 1, 1, oracle.S32, oracle.S32),      # empty batch
]


@pytest.mark.parametrize("case", _POOLS)
def test_pool_sum(hawq, case):
    import torch
    from gpu_util import assert_same
    N, H, W, C, R, stride, pad, x_dt, y_dt = case
    g = np.random.default_rng(sum(case))
    x = _draw(g, (N, H, W, C), x_dt)
    raw = y_dt == oracle.S32
    hi_in = {oracle.S32: 1 << 22, oracle.U8: 127, oracle.S8: 128, oracle.U4: 15}[x_dt]
    lo, hi = {oracle.U8: (0, 255), oracle.S8: (-128, 127), oracle.U4: (0, 15), oracle.S32: (0, 0)}[y_dt]
    b = c = None
    if not raw:
        b = g.integers(1 << 14, 1 << 15, size=C).astype(np.int32)
        c = ((14 if x_dt == oracle.S32 else 16) + int(np.ceil(np.log2(R * R * hi_in / max(hi, 1)))) + g.integers(-1, 1, size=C)).astype(np.uint8)
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    y = _empty((max(N, 1), P, Q, C), y_dt)      # (an empty torch tensor has a null pointer, which the interface rejects)
    hawq.hawq_pool2d_sum_int(N, H, W, C, R, R, stride, stride, pad, pad, x_dt, y_dt, _dev(x) if N else _dev(np.zeros(4, np.uint8)),
                             None if raw else _dev(b), None if raw else _dev(c), lo, hi, y)
    torch.cuda.synchronize()
    if N == 0:
        assert bool((y == 0x5A).all())      # nothing was written
        return
    want = oracle.pool2d_sum_int(x, b, c, N=N, H=H, W=W, C=C, R=R, S=R, stride=stride, pad=pad, x_dt=x_dt, y_dt=y_dt,
                                 **({} if raw else dict(y_lo=lo, y_hi=hi)))
    assert_same(y.cpu().numpy(), want, "pool %r" % (case,))
    if not raw:
        v = oracle.unpack(want, y_dt)
        assert len(np.unique(v)) >= 6 and (v == hi).mean() < 0.3


# branches (K, dtype) and the output type
_CONCATS = [
    ([(64, oracle.S32), (96, oracle.S32), (32, oracle.S32), (64, oracle.S32)], oracle.U8),     # four INT32 branches
    ([(64, oracle.S32), (48, oracle.U8), (16, oracle.S8), (32, oracle.U4)], oracle.U8),
    ([(6, oracle.S32), (10, oracle.U8), (2, oracle.S32)], oracle.S8),                           # no 4-channel alignment
    ([(8, oracle.S32), (6, oracle.U8), (4, oracle.S32)], oracle.U4),                            # packed output, offsets 8 and 14
    ([(5, oracle.S32), (3, oracle.S8)], oracle.U8),                                              # odd widths
    ([(128, oracle.S32)], oracle.U4),                                                            # a single branch: plain requantisation
]


@pytest.mark.parametrize("case", _CONCATS)
def test_concat(hawq, case):
    import torch
    from gpu_util import assert_same
    spec, y_dt = case
    P = 777
    g = np.random.default_rng(len(spec) * 31 + y_dt)
    lo, hi = {oracle.U8: (0, 127), oracle.S8: (-128, 127), oracle.U4: (0, 15)}[y_dt]
    br_o, br_d = [], []
    for K, dt in spec:
        q = _draw(g, (P, K), dt)
        mag = {oracle.S32: 1 << 22, oracle.U8: 127, oracle.S8: 128, oracle.U4: 15}[dt]
        b = g.integers(1 << 14, 1 << 15, size=K).astype(np.int32)
        c = (14 + int(np.ceil(np.log2(mag / (hi + 1)))) + g.integers(0, 2, size=K)).astype(np.uint8)
        br_o.append((q, dt, b, c))
        br_d.append((_dev(q), dt, _dev(b), _dev(c)))
    Kt = sum(K for K, _ in spec)
    y = _empty((P, Kt), y_dt)
    hawq.hawq_concat_dyadic(P, br_d, y_dt, lo, hi, y)
    torch.cuda.synchronize()
    want = oracle.concat_dyadic(br_o, n_pixels=P, y_dt=y_dt, y_lo=lo, y_hi=hi)
    assert_same(y.cpu().numpy(), want, "concat %r" % (case,))
    assert len(np.unique(oracle.unpack(want, y_dt))) >= 6


def test_inception_style_module(hawq):
    """The module of Appendix E's figure: the input feature map is INT32; it is requantised to 4 bits for three
    convolutional branches (1x1; 1x1 -> 3x3; 1x1 -> 3x3 -> 3x3), the pooling branch sums 3x3 windows of the INT32 map
    itself, and the four INT32 results are concatenated with one dyadic number each (the pool's carries the 1/9)."""
    import torch
    from gpu_util import assert_same
    g = np.random.default_rng(2011)
    N, H, C = 4, 17, 64
    P = N * H * H
    h = g.integers(0, 1 << 20, size=(N, H, H, C)).astype(np.int32)
    ones = lambda K, v: np.full(K, v, np.int32)
    sh = lambda K, v: np.full(K, v, np.uint8)

    def conv_params(K, Rr, Cc, m2=75.0):
        w = g.integers(-7, 8, size=(K, Rr, Rr, Cc))
        sig = np.sqrt(Rr * Rr * Cc * m2 * 18.7)      # accumulator spread: taps x E[x^2] x E[w^2]
        return dict(w=wl.pack_nibbles(w), bias=np.rint(sig * g.uniform(-0.3, 0.7, size=K)).astype(np.int32),
                    b=g.integers(1 << 14, 1 << 15, size=K).astype(np.int32),
                    c=(int(np.floor(np.log2(1.5 * (1 << 14) * sig / 5.0))) + g.integers(0, 2, size=K)).astype(np.uint8), K=K, R=Rr, C=Cc)

    L = dict(b1=conv_params(64, 1, C), b2a=conv_params(48, 1, C), b2b=conv_params(64, 3, 48, 25.0),
             b3a=conv_params(64, 1, C), b3b=conv_params(96, 3, 64, 25.0), b3c=conv_params(96, 3, 96, 25.0))
    rq_in = (ones(C, 1 << 14), sh(C, 30))                 # INT32 map -> 4-bit: 2^20 * 2^-16 = 16 levels
    out_dn = {k: (g.integers(1 << 14, 1 << 15, size=n).astype(np.int32), sh(n, v)) for k, n, v in
              (("b1", 64, 18), ("b2", 64, 19), ("b3", 96, 20))}
    pool_dn = (np.rint((1 << 15) / 9.0 * g.uniform(0.9, 1.1, size=C)).astype(np.int32), sh(C, 28))

    # ---- oracle assembly ----
    def o_conv(p, x, raw):
        return oracle.conv2d_int(x, p["w"], p["bias"], None if raw else p["b"], None if raw else p["c"], N=N, H=H, W=H, C=p["C"], K=p["K"],
                                 R=p["R"], S=p["R"], stride=1, pad=p["R"] // 2, x_dt=oracle.U4, w_dt=oracle.S4,
                                 y_dt=oracle.S32 if raw else oracle.U4, relu=0 if raw else 1,
                                 y_lo=-(1 << 31) if raw else 0, y_hi=(1 << 31) - 1 if raw else 15)
    h4 = oracle.concat_dyadic([(h.reshape(P, C), oracle.S32, *rq_in)], n_pixels=P, y_dt=oracle.U4, y_lo=0, y_hi=15)
    o1 = o_conv(L["b1"], h4, True)
    o2 = o_conv(L["b2b"], o_conv(L["b2a"], h4, False), True)
    o3 = o_conv(L["b3c"], o_conv(L["b3b"], o_conv(L["b3a"], h4, False), False), True)
    op = oracle.pool2d_sum_int(h, None, None, N=N, H=H, W=H, C=C, R=3, S=3, stride=1, pad=1, x_dt=oracle.S32, y_dt=oracle.S32)
    want = oracle.concat_dyadic([(o1.reshape(P, -1), oracle.S32, *out_dn["b1"]), (o2.reshape(P, -1), oracle.S32, *out_dn["b2"]),
                                 (o3.reshape(P, -1), oracle.S32, *out_dn["b3"]), (op.reshape(P, -1), oracle.S32, *pool_dn)],
                                n_pixels=P, y_dt=oracle.U8, y_lo=0, y_hi=127)

    # ---- the same assembly through the C interface ----
    def d_conv(p, x, raw):
        d = hawq.ConvDesc(N=N, H=H, W=H, C=p["C"], K=p["K"], R=p["R"], S=p["R"], stride_h=1, stride_w=1, pad_h=p["R"] // 2, pad_w=p["R"] // 2,
                          x_dtype=hawq.U4, w_dtype=hawq.S4, y_dtype=hawq.S32 if raw else hawq.U4, res_dtype=hawq.U8,
                          relu=0 if raw else 1, y_lo=-(1 << 31) if raw else 0, y_hi=(1 << 31) - 1 if raw else 15, x_hi=0)
        y = _empty((N, H, H, p["K"]), hawq.S32 if raw else hawq.U4)
        hawq.hawq_conv2d_int(d, x, _dev(p["w"]), _dev(p["bias"]), None if raw else _dev(p["b"]), None if raw else _dev(p["c"]),
                             None, None, None, y)
        return y
    hd = _dev(h)
    h4d = _empty((P, C), hawq.U4)
    hawq.hawq_concat_dyadic(P, [(hd, hawq.S32, _dev(rq_in[0]), _dev(rq_in[1]))], hawq.U4, 0, 15, h4d)
    g1 = d_conv(L["b1"], h4d, True)
    g2 = d_conv(L["b2b"], d_conv(L["b2a"], h4d, False), True)
    g3 = d_conv(L["b3c"], d_conv(L["b3b"], d_conv(L["b3a"], h4d, False), False), True)
    gp = _empty((N, H, H, C), hawq.S32)
    hawq.hawq_pool2d_sum_int(N, H, H, C, 3, 3, 1, 1, 1, 1, hawq.S32, hawq.S32, hd, None, None, 0, 0, gp)
    y = _empty((P, 64 + 64 + 96 + C), hawq.U8)
    dn = lambda k: (_dev(out_dn[k][0]), _dev(out_dn[k][1]))
    hawq.hawq_concat_dyadic(P, [(g1, hawq.S32, *dn("b1")), (g2, hawq.S32, *dn("b2")), (g3, hawq.S32, *dn("b3")),
                                (gp, hawq.S32, _dev(pool_dn[0]), _dev(pool_dn[1]))], hawq.U8, 0, 127, y)
    torch.cuda.synchronize()
    assert_same(h4d.cpu().numpy(), h4, "4-bit input of the convolutional branches")
    assert_same(gp.cpu().numpy(), op, "INT32 pooling branch")
    assert_same(y.cpu().numpy(), want, "module output")
    for lo_, hi_ in ((0, 64), (64, 128), (128, 224), (224, 288)):     # every branch contributes a spread of values
        v = want[:, lo_:hi_]
        assert len(np.unique(v)) > 20 and (v == 127).mean() < 0.3 and (v == 0).mean() < 0.7, (lo_, hi_)
