"""GPU parity of the resident-pixel 1x1 kernel: hawq_conv2d_int on 1x1 layers with hawq_conv_desc::w_fragments (one
convolution, with and without a shortcut tensor, one and several passes of 256 output channels per workgroup) against the
oracle, bit for bit.  The kernel's two-convolution form needs the network plan's 16-bit guarantee and is covered by the
network tests (test_gpu_dual.py, test_gpu_resnet.py)."""
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


def _centre(case, C, K, x_hi=127, out_hi=127):
    sigma = math.sqrt(C * (x_hi * x_hi / 3.0) * (127 * 128 / 3.0)) + 1
    c0 = int(math.floor(math.log2(1.5 * (1 << 14) / ((out_hi / 3.0) / sigma))))
    g = np.random.default_rng(K + C)
    case["c"] = (c0 + g.integers(0, 2, size=K)).astype(np.uint8)
    case["bias"] = np.rint(sigma * g.uniform(-0.5, 0.5, size=K)).astype(np.int32)
    return case


# N, H, W, C, K, residual (None / "u8" / "s8"), wide parameters.  Tiles are 128 pixels (C = 512, 1024) or 64 (C = 2048); a
# workgroup takes several groups of 256 channels once tiles x groups fill the chip: 41 tiles x 2048 channels -> 2 passes,
# 161 tiles x 1024 channels -> 4 passes.
CASES = [(4, 7, 7, 512, 2048, "u8", False), (3, 7, 7, 512, 1024, "s8", False), (2, 5, 3, 512, 256, None, True),
         (8, 14, 14, 1024, 256, None, False), (1, 3, 5, 1024, 512, "u8", True), (6, 7, 7, 2048, 512, None, False),
         (1, 1, 1, 2048, 256, None, False), (3, 7, 7, 2048, 1024, "s8", False),
         (105, 7, 7, 512, 2048, "u8", False), (105, 14, 14, 512, 1024, "s8", False), (105, 14, 14, 512, 1024, None, True),
         (2, 7, 7, 512, 1000, None, False), (2, 7, 7, 768, 256, None, False)]   # last two: shapes the kernel leaves to others


@pytest.mark.parametrize("N,H,W,C,K,res,wide", CASES)
def test_conv1x1_with_fragment_weights(hawq, N, H, W, C, K, res, wide):
    import torch
    from gpu_util import to_dev, assert_same
    case = _centre(wl.conv_case(seed=N + H + W + C + K, N=N, H=H, W=W, C=C, K=K, R=1, S=1, stride=1, pad=0, bits=8,
                                with_residual=res is not None, res_signed=res == "s8"), C, K)
    if wide:   # multiplier and shift scaled together: same dyadic number, outside the narrow evaluation's range
        case["b"] = (case["b"].astype(np.int64) << 13).astype(np.int32)
        case["c"] = (case["c"].astype(np.int32) + 13).astype(np.uint8)
    res_dt = hawq.S8 if res == "s8" else hawq.U8
    d = hawq.ConvDesc(N=N, H=H, W=W, C=C, K=K, R=1, S=1, stride_h=1, stride_w=1, pad_h=0, pad_w=0, x_dtype=hawq.U8, w_dtype=hawq.S8,
                      y_dtype=hawq.U8, res_dtype=res_dt, relu=1, y_lo=0, y_hi=127, x_hi=127)
    w = to_dev(case["w"])
    nb = hawq.hawq_conv_fragment_weights_bytes(d)
    assert nb == ((K + 31) // 32) * 32 * C
    wf = torch.full((nb,), 0x5A, dtype=torch.uint8, device="cuda")
    hawq.hawq_conv_fragment_weights(d, w, wf)
    d.w_fragments = wf.data_ptr()
    y = torch.full((N, H, W, K), 0x5A, dtype=torch.uint8, device="cuda")
    r = case["residual"]
    hawq.hawq_conv2d_int(d, to_dev(case["x"]), w, to_dev(case["bias"]), to_dev(case["b"]), to_dev(case["c"]),
                         to_dev(r), to_dev(case["res_b"]) if r is not None else None, to_dev(case["res_c"]) if r is not None else None, y)
    torch.cuda.synchronize()
    want = oracle.conv2d_int(case["x"], case["w"], case["bias"], case["b"], case["c"], N=N, H=H, W=W, C=C, K=K, R=1, S=1, stride=1,
                             pad=0, x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127, residual=r,
                             res_b=case["res_b"], res_c=case["res_c"], res_dt=res_dt)
    assert_same(y.cpu().numpy(), want)
    assert 0.05 < np.mean(want > 0) and np.mean(want == 127) < 0.5


def test_conv1x1_signed_output_and_clamp_window(hawq):
    """Signed 8-bit output without ReLU (the tensor a transition layer stores) and a clamp window inside the type's range."""
    import torch
    from gpu_util import to_dev, assert_same
    N, H, W, C, K = 5, 7, 7, 1024, 512
    case = _centre(wl.conv_case(seed=77, N=N, H=H, W=W, C=C, K=K, R=1, S=1, stride=1, pad=0, bits=8), C, K)
    for y_dt, o_dt, relu, lo, hi in ((hawq.S8, oracle.S8, 0, -128, 127), (hawq.S8, oracle.S8, 0, -100, 90), (hawq.U8, oracle.U8, 1, 3, 200)):
        d = hawq.ConvDesc(N=N, H=H, W=W, C=C, K=K, R=1, S=1, stride_h=1, stride_w=1, pad_h=0, pad_w=0, x_dtype=hawq.U8, w_dtype=hawq.S8,
                          y_dtype=y_dt, res_dtype=hawq.U8, relu=relu, y_lo=lo, y_hi=hi, x_hi=127)
        w = to_dev(case["w"])
        wf = torch.zeros((hawq.hawq_conv_fragment_weights_bytes(d),), dtype=torch.uint8, device="cuda")
        hawq.hawq_conv_fragment_weights(d, w, wf)
        d.w_fragments = wf.data_ptr()
        y = torch.full((N, H, W, K), 0x5A, dtype=torch.uint8, device="cuda")
        hawq.hawq_conv2d_int(d, to_dev(case["x"]), w, to_dev(case["bias"]), to_dev(case["b"]), to_dev(case["c"]), None, None, None, y)
        torch.cuda.synchronize()
        want = oracle.conv2d_int(case["x"], case["w"], case["bias"], case["b"], case["c"], N=N, H=H, W=W, C=C, K=K, R=1, S=1, stride=1,
                                 pad=0, x_dt=oracle.U8, w_dt=oracle.S8, y_dt=o_dt, relu=relu, y_lo=lo, y_hi=hi)
        got = y.cpu().numpy()
        assert_same(got.view(np.int8) if y_dt == hawq.S8 else got, want)
