"""GPU parity of the resident-pixel 3x3 kernel and the fused bottleneck tail (3x3 -> 1x1 + shortcut in one launch):
hawq_conv_fragment_weights, hawq_conv2d_int with hawq_conv_desc::w_fragments, hawq_bottleneck_tail_int -- each against
the oracle (the fused launch against the oracle's two layers one after the other), bit for bit."""
import math

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hawq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2011_10680_amd as h
    h.load_library()
    return h


def _centre(case, x_hi=127, out_hi=127, seed=0):
    """Shift chosen from the accumulator spread so that outputs cover the clamp range (b per channel as drawn, c jittered)."""
    kdim = case["R"] * case["S"] * case["C"]
    sigma = math.sqrt(kdim * (x_hi * x_hi / 3.0) * (127 * 128 / 3.0)) + 1
    c0 = int(math.floor(math.log2(1.5 * (1 << 14) / ((out_hi / 3.0) / sigma))))
    g = np.random.default_rng(case["K"] + kdim + seed)
    case["c"] = (c0 + g.integers(0, 2, size=case["K"])).astype(np.uint8)
    case["bias"] = np.rint(sigma * g.uniform(-0.5, 0.5, size=case["K"])).astype(np.int32)
    return case


def _frag(hawq, d, w_dev):
    import torch
    nb = hawq.hawq_conv_fragment_weights_bytes(d)
    assert nb == ((d.K + 31) // 32) * 32 * d.R * d.S * d.C
    wf = torch.full((nb,), 0x5A, dtype=torch.uint8, device="cuda")
    hawq.hawq_conv_fragment_weights(d, w_dev, wf)
    return wf


def _frag_definition(w, K, row):
    """[ceil(K/32)][row/64][2][64][16]: lane = khalf*32 + rho holds bytes (kk*2 + khalf)*16.. of step t of channel
    32 g + ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3)."""
    G, steps = (K + 31) // 32, row // 64
    full = np.zeros((G * 32, row), dtype=np.uint8)
    full[:K] = w.reshape(K, row).view(np.uint8)
    out = np.zeros((G, steps, 2, 64, 16), dtype=np.uint8)
    for lane in range(64):
        rho, khalf = lane & 31, lane >> 5
        ch = ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3)
        for kk in range(2):
            src = full.reshape(G, 32, steps, 64)[:, ch, :, (kk * 2 + khalf) * 16:(kk * 2 + khalf) * 16 + 16]
            out[:, :, kk, lane, :] = src
    return out


@pytest.mark.parametrize("K,R,C", [(256, 3, 256), (100, 1, 128), (32, 3, 64)])
def test_fragment_weights_copy_is_the_documented_order(hawq, K, R, C):
    import torch
    from gpu_util import to_dev
    g = np.random.default_rng(K + C)
    w = g.integers(-127, 128, size=(K, R, R, C)).astype(np.int8)
    d = hawq.ConvDesc(N=1, H=8, W=8, C=C, K=K, R=R, S=R, stride_h=1, stride_w=1, pad_h=R // 2, pad_w=R // 2, x_dtype=hawq.U8,
                      w_dtype=hawq.S8, y_dtype=hawq.U8, res_dtype=hawq.U8, relu=1, y_lo=0, y_hi=127, x_hi=127)
    wf = _frag(hawq, d, to_dev(w))
    torch.cuda.synchronize()
    assert np.array_equal(wf.cpu().numpy().reshape(-1), _frag_definition(w, K, R * R * C).reshape(-1))


# N, H, W, C, K, residual (None / "u8" / "s8"), wide parameters
PLAIN = [(3, 14, 14, 256, 256, None, False), (2, 28, 28, 128, 128, None, False), (1, 13, 11, 256, 512, "u8", False),
         (2, 9, 28, 128, 256, "s8", False), (1, 5, 3, 128, 128, "u8", True), (5, 7, 7, 256, 256, None, True),
         (1, 1, 1, 128, 128, None, False), (1, 2, 300, 128, 128, None, False),   # last: wider than the kernel's patch -> other kernel
         (9, 7, 7, 512, 512, None, False), (3, 7, 7, 512, 512, "u8", False), (2, 5, 14, 512, 256, "s8", True),
         # 128 channels reach this kernel from forty 256-pixel tiles on (fewer: the tiled kernel, as the small cases above)
         (14, 28, 28, 128, 128, None, False), (14, 28, 28, 128, 256, "s8", False), (15, 27, 26, 128, 128, "u8", True)]


@pytest.mark.parametrize("N,H,W,C,K,res,wide", PLAIN)
def test_conv3x3_with_fragment_weights(hawq, N, H, W, C, K, res, wide):
    import torch
    from gpu_util import to_dev, assert_same
    case = _centre(wl.conv_case(seed=N + H + W + C + K, N=N, H=H, W=W, C=C, K=K, R=3, S=3, stride=1, pad=1, bits=8,
                                with_residual=res is not None, res_signed=res == "s8"))
    if wide:   # multiplier and shift scaled together: same dyadic number, outside the narrow evaluation's range
        case["b"] = (case["b"].astype(np.int64) << 13).astype(np.int32)
        case["c"] = (case["c"].astype(np.int32) + 13).astype(np.uint8)
    res_dt = hawq.S8 if res == "s8" else hawq.U8
    d = hawq.ConvDesc(N=N, H=H, W=W, C=C, K=K, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, x_dtype=hawq.U8, w_dtype=hawq.S8,
                      y_dtype=hawq.U8, res_dtype=res_dt, relu=1, y_lo=0, y_hi=127, x_hi=127)
    w = to_dev(case["w"])
    wf = _frag(hawq, d, w)
    d.w_fragments = wf.data_ptr()
    y = torch.full((N, H, W, K), 0x5A, dtype=torch.uint8, device="cuda")
    r = case["residual"]
    hawq.hawq_conv2d_int(d, to_dev(case["x"]), w, to_dev(case["bias"]), to_dev(case["b"]), to_dev(case["c"]),
                         to_dev(r), to_dev(case["res_b"]) if r is not None else None, to_dev(case["res_c"]) if r is not None else None, y)
    torch.cuda.synchronize()
    want = oracle.conv2d_int(case["x"], case["w"], case["bias"], case["b"], case["c"], N=N, H=H, W=W, C=C, K=K, R=3, S=3, stride=1,
                             pad=1, x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127, residual=r,
                             res_b=case["res_b"], res_c=case["res_c"], res_dt=res_dt)
    assert_same(y.cpu().numpy(), want)
    assert 0.05 < np.mean(want > 0) and np.mean(want == 127) < 0.5


# N, H, W, C, K, output type, wide parameters: packed 4-bit operands on the same kernel
PACKED = [(3, 14, 14, 256, 256, "u4", False), (2, 28, 28, 128, 128, "u4", False), (1, 13, 11, 256, 512, "u8", False),
          (9, 7, 7, 512, 512, "u4", False), (2, 9, 5, 128, 256, "u4", True), (40, 28, 28, 128, 128, "u4", False)]


@pytest.mark.parametrize("N,H,W,C,K,ydt,wide", PACKED)
def test_conv3x3_packed_4bit_with_fragment_weights(hawq, N, H, W, C, K, ydt, wide):
    import torch
    from gpu_util import to_dev, assert_same
    case = wl.conv_case(seed=3 * N + H + W + C + K, N=N, H=H, W=W, C=C, K=K, R=3, S=3, stride=1, pad=1, bits=4)
    kdim = 9 * C
    sigma = math.sqrt(kdim * (15 * 15 / 3.0) * (7 * 8 / 3.0)) + 1
    hi = 15 if ydt == "u4" else 127
    c0 = int(math.floor(math.log2(1.5 * (1 << 14) / ((hi / 3.0) / sigma))))
    g = np.random.default_rng(K + kdim)
    case["c"] = (c0 + g.integers(0, 2, size=K)).astype(np.uint8)
    case["bias"] = np.rint(sigma * g.uniform(-0.5, 0.5, size=K)).astype(np.int32)
    case["x"][0, 0, 0, :8] = 0xFF          # nibble extremes: activations 15, weights -1 / -8 / 7 in both halves of a byte
    case["w"][0, 0, 0, :8] = [0xFF, 0x88, 0x77, 0x8F, 0xF8, 0x78, 0x87, 0x00]
    case["w_vals"][0, 0, 0, :16] = [-1, -1, -8, -8, 7, 7, -1, -8, -8, -1, -8, 7, 7, -8, 0, 0]
    if wide:
        case["b"] = (case["b"].astype(np.int64) << 13).astype(np.int32)
        case["c"] = (case["c"].astype(np.int32) + 13).astype(np.uint8)
    y_dt = hawq.U4 if ydt == "u4" else hawq.U8
    d = hawq.ConvDesc(N=N, H=H, W=W, C=C, K=K, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, x_dtype=hawq.U4, w_dtype=hawq.S4,
                      y_dtype=y_dt, res_dtype=hawq.U8, relu=1, y_lo=0, y_hi=hi, x_hi=0)
    w = to_dev(case["w"])
    nb = hawq.hawq_conv_fragment_weights_bytes(d)
    assert nb == ((K + 31) // 32) * 32 * 9 * C        # 4-bit weights are expanded to bytes in the copy
    wf = torch.full((nb,), 0x5A, dtype=torch.uint8, device="cuda")
    hawq.hawq_conv_fragment_weights(d, w, wf)
    torch.cuda.synchronize()
    # the copy's definition: signed bytes, of every 32 elements the 16 even ones first, then the 16 odd ones
    wv = case["w_vals"].reshape(K, 9 * C // 32, 16, 2).transpose(0, 1, 3, 2).reshape(K, 9 * C).astype(np.int8)
    assert np.array_equal(wf.cpu().numpy().reshape(-1), _frag_definition(wv, K, 9 * C).reshape(-1))
    d.w_fragments = wf.data_ptr()
    y = torch.full((N, H, W, K // 2 if ydt == "u4" else K), 0x5A, dtype=torch.uint8, device="cuda")
    hawq.hawq_conv2d_int(d, to_dev(case["x"]), w, to_dev(case["bias"]), to_dev(case["b"]), to_dev(case["c"]), None, None, None, y)
    torch.cuda.synchronize()
    want = oracle.conv2d_int(case["x"], case["w"], case["bias"], case["b"], case["c"], N=N, H=H, W=W, C=C, K=K, R=3, S=3, stride=1,
                             pad=1, x_dt=oracle.U4, w_dt=oracle.S4, y_dt=oracle.U4 if ydt == "u4" else oracle.U8, relu=1, y_lo=0, y_hi=hi)
    assert_same(y.cpu().numpy(), want)
    vals = oracle.unpack(want, oracle.U4) if ydt == "u4" else want.reshape(-1)
    assert 0.05 < np.mean(vals > 0) and np.mean(vals == hi) < 0.5


# N, H, W, C, K2, shortcut type, intermediate clamp, wide parameters
TAIL = [(3, 14, 14, 256, 1024, "u8", 127, False), (2, 28, 28, 128, 512, "u8", 127, False), (1, 9, 11, 128, 256, "s8", 127, False),
        (2, 7, 13, 256, 512, "u8", 15, False), (1, 5, 5, 128, 128, "u8", 127, True), (4, 14, 14, 256, 256, "s8", 127, True),
        (1, 1, 1, 256, 1024, "u8", 127, False)]


@pytest.mark.parametrize("N,H,W,C,K2,res,mid_hi,wide", TAIL)
def test_bottleneck_tail_equals_the_two_layers(hawq, N, H, W, C, K2, res, mid_hi, wide):
    import torch
    from gpu_util import to_dev, assert_same
    c2 = _centre(wl.conv_case(seed=7 * N + H + W + C, N=N, H=H, W=W, C=C, K=C, R=3, S=3, stride=1, pad=1, bits=8), out_hi=mid_hi)
    c3 = _centre(wl.conv_case(seed=K2 + H + W, N=N, H=H, W=W, C=C, K=K2, R=1, S=1, stride=1, pad=0, bits=8, with_residual=True,
                              res_signed=res == "s8"), x_hi=mid_hi // 2 + 1, seed=1)
    if wide:
        c3["b"] = (c3["b"].astype(np.int64) << 12).astype(np.int32)
        c3["c"] = (c3["c"].astype(np.int32) + 12).astype(np.uint8)
    res_dt = hawq.S8 if res == "s8" else hawq.U8
    h = oracle.conv2d_int(c2["x"], c2["w"], c2["bias"], c2["b"], c2["c"], N=N, H=H, W=W, C=C, K=C, R=3, S=3, stride=1, pad=1,
                          x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=mid_hi)
    want = oracle.conv2d_int(h, c3["w"], c3["bias"], c3["b"], c3["c"], N=N, H=H, W=W, C=C, K=K2, R=1, S=1, stride=1, pad=0,
                             x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127, residual=c3["residual"],
                             res_b=c3["res_b"], res_c=c3["res_c"], res_dt=res_dt)
    d2 = hawq.ConvDesc(N=N, H=H, W=W, C=C, K=C, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, x_dtype=hawq.U8, w_dtype=hawq.S8,
                       y_dtype=hawq.U8, res_dtype=hawq.U8, relu=1, y_lo=0, y_hi=mid_hi, x_hi=127)
    d3 = hawq.ConvDesc(N=N, H=H, W=W, C=C, K=K2, R=1, S=1, stride_h=1, stride_w=1, pad_h=0, pad_w=0, x_dtype=hawq.U8, w_dtype=hawq.S8,
                       y_dtype=hawq.U8, res_dtype=res_dt, relu=1, y_lo=0, y_hi=127, x_hi=0)
    w2f, w3f = _frag(hawq, d2, to_dev(c2["w"])), _frag(hawq, d3, to_dev(c3["w"]))
    y = torch.full((N, H, W, K2), 0x5A, dtype=torch.uint8, device="cuda")
    hawq.hawq_bottleneck_tail_int(d2, to_dev(c2["x"]), w2f, to_dev(c2["bias"]), to_dev(c2["b"]), to_dev(c2["c"]),
                                  d3, w3f, to_dev(c3["bias"]), to_dev(c3["b"]), to_dev(c3["c"]),
                                  to_dev(c3["residual"]), to_dev(c3["res_b"]), to_dev(c3["res_c"]), y)
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), want)
    assert 0.05 < np.mean(h > 0) and 0.05 < np.mean(want > 0) and np.mean(want == 127) < 0.5


def test_bottleneck_tail_refuses_other_shapes(hawq):
    """Valid requests outside the fused kernel's shapes are refused (nothing is launched), invalid ones are errors."""
    import torch
    t = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    ti = torch.zeros(1 << 12, dtype=torch.int32, device="cuda")
    def desc(C, K, R, x_hi=127, **kw):
        d = dict(N=1, H=4, W=4, C=C, K=K, R=R, S=R, stride_h=1, stride_w=1, pad_h=R // 2, pad_w=R // 2, x_dtype=hawq.U8,
                 w_dtype=hawq.S8, y_dtype=hawq.U8, res_dtype=hawq.U8, relu=1, y_lo=0, y_hi=127, x_hi=x_hi)
        d.update(kw)
        return hawq.ConvDesc(**d)
    def call(d2, d3):
        hawq.hawq_bottleneck_tail_int(d2, t, t, ti, ti, t, d3, t, ti, ti, t, t, ti, t, t)
    for d2, d3, status in [(desc(64, 64, 3), desc(64, 256, 1), 6),                 # 64 channels: not served
                           (desc(128, 128, 3, x_hi=0), desc(128, 512, 1), 6),     # unsigned bytes above 127
                           (desc(128, 128, 3), desc(128, 500, 1), 6),             # K not a multiple of 128
                           (desc(128, 128, 3, stride_h=2), desc(128, 512, 1), 6),
                           (desc(128, 128, 3, y_hi=300), desc(128, 512, 1), 4),   # clamp outside the type
                           (desc(128, 128, 3), desc(128, 512, 1, w_dtype=hawq.S4), 3)]:
        with pytest.raises(hawq.HawqError) as e:
            call(d2, d3)
        assert e.value.status == status, (e.value.status, status)
