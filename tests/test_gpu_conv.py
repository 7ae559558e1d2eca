"""GPU parity: hawq_conv2d_int / hawq_gemm_int through the C interface vs the CPU oracle, bit-exact."""
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


def _scale_c(case, bits):
    """Replace the literal shift distribution by one centred on the accumulator spread so outputs
    are spread over the clamp range (keeps b per channel, c per channel jittered by 0/1)."""
    import math
    kdim = case["R"] * case["S"] * case["C"]
    hi, wm = (127, 127) if bits == 8 else (15, 7)
    sigma = math.sqrt(kdim * (hi * hi / 3.0) * (wm * (wm + 1) / 3.0)) + 1
    c0 = int(math.floor(math.log2(1.5 * (1 << 14) / ((hi / 3.0) / sigma))))
    g = np.random.default_rng(case["K"] + kdim)
    case["c"] = (c0 + g.integers(0, 2, size=case["K"])).astype(np.uint8)
    case["bias"] = np.rint(sigma * g.uniform(-0.5, 0.5, size=case["K"])).astype(np.int32)
    return case


def test_config0_single_conv_literal(hawq):
    """The single-layer configuration exactly as specified (56x56x64 -> 64, 3x3, literal b/c/bias draws)."""
    from gpu_util import run_conv_gpu, assert_same
    case = wl.conv_case(seed=1000, N=1, H=56, W=56, C=64, K=64, R=3, S=3, stride=1, pad=1, bits=8)
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.U8, x_hi=127)
    assert_same(got, want, "config 0")


# (N, H, W, C, K, R, S, stride, pad): several tiles plus ragged pixel and channel tails
_SHAPES8 = [
    (1, 56, 56, 64, 64, 3, 3, 1, 1),
    (3, 13, 13, 64, 64, 3, 3, 1, 1),      # 507 pixels: ragged last pixel tile
    (2, 13, 11, 128, 192, 3, 3, 2, 1),    # K not a multiple of 128
    (2, 15, 15, 64, 80, 1, 1, 1, 0),      # K % 64 != 0, K % 16 == 0
    (2, 9, 9, 64, 72, 1, 1, 1, 0),        # K % 16 != 0: element-wise epilogue
    (5, 14, 14, 256, 64, 1, 1, 2, 0),     # strided 1x1
    (1, 10, 12, 192, 96, 5, 3, 1, 2),     # non-square window, pad 2
    (8, 64, 64, 64, 256, 1, 1, 1, 0),     # 512 tiles of 128x128: the large-tile kernel
    (16, 64, 64, 64, 64, 3, 3, 1, 1),     # 512 tiles of 64x128: the K=64 kernel
    (1, 7, 7, 512, 512, 3, 3, 1, 1),      # small M, deep K
]


@pytest.mark.parametrize("shape", _SHAPES8)
def test_int8_conv_shapes(hawq, shape):
    from gpu_util import run_conv_gpu, assert_same
    N, H, W, C, K, R, S, stride, pad = shape
    case = _scale_c(wl.conv_case(seed=sum(shape), N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, bits=8), 8)
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.U8, x_hi=127)
    assert_same(got, want, str(shape))
    assert 0.05 < (want > 0).mean() and (want == 127).mean() < 0.5


# 1x1 convolutions with C = 64 / 128 and many pixels: the persistent streaming kernel
_SHAPES_PW = [
    (3, 57, 59, 64, 80, 1, 1, 1, 0, 8, False),     # ragged pixel tail, K % 32 != 0
    (4, 56, 56, 128, 512, 1, 1, 1, 0, 8, True),    # expanding 1x1 with shortcut
    (4, 112, 112, 64, 128, 1, 1, 2, 0, 8, False),  # strided
    (4, 56, 56, 64, 256, 1, 1, 1, 0, 4, True),     # packed 4-bit, 4-bit shortcut
    (3, 60, 60, 128, 64, 1, 1, 2, 0, 4, False),    # packed 4-bit, strided, ragged
    (9, 33, 31, 64, 64, 1, 1, 1, 0, 8, True),
    (11, 56, 56, 256, 128, 1, 1, 2, 0, 8, False),  # C = 256, strided
    (3, 59, 59, 256, 96, 1, 1, 1, 0, 8, True),     # C = 256, ragged, shortcut
    (5, 56, 56, 256, 64, 1, 1, 1, 0, 4, False),    # C = 256, packed 4-bit
]


@pytest.mark.parametrize("shape", _SHAPES_PW)
def test_pointwise_streaming_shapes(hawq, shape):
    from gpu_util import run_conv_gpu, assert_same
    N, H, W, C, K, R, S, stride, pad, bits, res = shape
    case = _scale_c(wl.conv_case(seed=sum(shape[:9]), N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, bits=bits,
                                 with_residual=res), bits)
    if bits == 8:
        got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.U8, res_dt=hawq.U8, x_hi=127)
    else:
        got, want = run_conv_gpu(case, hawq.U4, hawq.S4, hawq.U4, res_dt=hawq.U4, y_hi=15)
    assert_same(got, want, str(shape))
    v = want.astype(np.int32) if bits == 8 else oracle.unpack(want, oracle.U4)
    assert 0.05 < (v > 0).mean() < 0.999


def test_pointwise_streaming_signed_shortcut_and_wide_parameters(hawq):
    """Signed 8-bit shortcut (a transition output), and multipliers outside the narrow path's range
    (c > 31, b >= 2^c) which must take the exact 64-bit path."""
    from gpu_util import run_conv_gpu, assert_same
    case = _scale_c(wl.conv_case(seed=123, N=4, H=56, W=56, C=64, K=256, R=1, S=1, stride=1, pad=0, bits=8,
                                 with_residual=True, res_signed=True), 8)
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.U8, res_dt=hawq.S8, x_hi=127)
    assert_same(got, want, "signed shortcut")
    wide = dict(case)
    wide["b"] = (case["b"].astype(np.int64) << 14).astype(np.int32)      # b up to 2^29
    wide["c"] = (case["c"].astype(np.int32) + 14).astype(np.uint8)       # same scale, c around 39
    got, want2 = run_conv_gpu(wide, hawq.U8, hawq.S8, hawq.U8, res_dt=hawq.S8, x_hi=127)
    assert_same(got, want2, "wide parameters")
    assert np.array_equal(want, want2)   # scaling numerator and shift together leaves the result unchanged
    huge = dict(case)
    huge["c"] = np.full_like(case["c"], 3)                               # b / 2^c ~ 3000: saturates, needs 64 bits
    got, want3 = run_conv_gpu(huge, hawq.U8, hawq.S8, hawq.S8, res_dt=hawq.S8, relu=0, y_lo=-128, y_hi=127, x_hi=127)
    assert_same(got, want3, "saturating parameters")


@pytest.mark.parametrize("C,K,spread", [(64, 256, "aligned"), (64, 256, "none"), (256, 1024, "aligned"), (256, 1024, "none"), (128, 96, "edge")])
def test_pointwise_register_form_shortcut_shift_alignment(hawq, C, K, spread):
    """The register-resident epilogue brings every channel's shortcut shift to one wave-uniform value: per-channel shifts
    that just admit one ("aligned": the window of valid values has width 1), that admit none ("none": the staged form
    must take over), zero and tiny multipliers, full-range unsigned shortcut bytes (0..255)."""
    from gpu_util import run_conv_gpu, assert_same
    case = _scale_c(wl.conv_case(seed=C + K + len(spread), N=3, H=56, W=56, C=C, K=K, R=1, S=1, stride=1, pad=0, bits=8,
                                 with_residual=True), 8)
    g = np.random.default_rng(K)
    case["residual"] = g.integers(0, 256, size=case["residual"].shape).astype(np.uint8)
    if spread == "aligned":      # 15-bit multipliers: valid T in [max rc, min rc + 7] = [17, 17]
        case["res_c"] = g.integers(10, 18, size=K).astype(np.uint8)
        case["res_c"][:2] = (10, 17)
    elif spread == "none":
        case["res_c"] = g.integers(5, 21, size=K).astype(np.uint8)
        case["res_c"][:2] = (5, 20)
    else:
        case["res_c"] = g.integers(14, 17, size=K).astype(np.uint8)
        case["res_b"] = case["res_b"].copy()
        case["res_b"][0] = 0
        case["res_b"][1] = 1
        case["res_b"][2] = (1 << 22) - 1       # the largest multiplier the form takes ...
        case["res_c"][2] = 22
        case["res_b"][5] = 3
        case["res_c"][5] = 1                    # ... next to a shift of 1
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.U8, res_dt=hawq.U8, x_hi=127)
    assert_same(got, want, "%d -> %d, %s" % (C, K, spread))
    assert 0.05 < (want > 0).mean() and len(np.unique(want)) > 50


# few tiles and a long reduction: the tiled kernel's eight-buffer operand ring
@pytest.mark.parametrize("shape", [
    (8, 14, 14, 256, 256, 3, 3, 1, 1, False),     # 36 K-steps
    (9, 13, 11, 192, 384, 3, 3, 1, 1, True),      # 27 K-steps (padded to 32), ragged tiles, shortcut
    (6, 14, 14, 1024, 128, 1, 1, 1, 0, False),    # 16 K-steps, pointwise
    (24, 14, 14, 512, 256, 3, 3, 2, 1, False),    # strided, 72 K-steps
    (128, 7, 7, 512, 512, 3, 3, 1, 1, False),     # the 7x7 layer of ResNet50 at batch 128: 196 tiles
])
def test_tiled_kernel_deep_ring(hawq, shape):
    from gpu_util import run_conv_gpu, assert_same
    N, H, W, C, K, R, S, stride, pad, res = shape
    case = _scale_c(wl.conv_case(seed=sum(shape[:9]), N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, bits=8,
                                 with_residual=res), 8)
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.U8, res_dt=hawq.U8, x_hi=127)
    assert_same(got, want, str(shape))
    assert 0.05 < (want > 0).mean() and (want == 127).mean() < 0.5


# 1x1 with C = 256 and K >= 256 (a multiple of 128), many pixels: the streaming kernel whose four waves share a stage
@pytest.mark.parametrize("N,H,W,K,stride,res,res_signed,y_dt,y_hi", [
    (11, 28, 28, 1024, 1, True, False, 0, 127),     # the expanding 1x1 of ResNet50 stage 3
    (3, 57, 55, 384, 1, False, False, 0, 127),      # ragged pixel tail, three workgroups per pixel group
    (11, 56, 56, 512, 2, False, False, 1, 127),     # strided transition, signed output
    (12, 27, 29, 256, 1, True, True, 2, 15),        # signed shortcut, packed 4-bit output
])
def test_pointwise_shared_stage_shapes(hawq, N, H, W, K, stride, res, res_signed, y_dt, y_hi):
    from gpu_util import run_conv_gpu, assert_same
    case = _scale_c(wl.conv_case(seed=N + H + K, N=N, H=H, W=W, C=256, K=K, R=1, S=1, stride=stride, pad=0, bits=8,
                                 with_residual=res, res_signed=res_signed), 8)
    if y_hi == 15:
        case["c"] = (case["c"] + 3).astype(np.uint8)
    signed_out = y_dt == 1
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, y_dt, res_dt=hawq.S8 if res_signed else hawq.U8,
                             relu=0 if signed_out else 1, y_lo=-128 if signed_out else 0, y_hi=y_hi, x_hi=127)
    assert_same(got, want, str((N, H, W, K)))
    v = oracle.unpack(want, oracle.U4) if y_dt == 2 else want.astype(np.int32)
    assert 0.05 < (v != 0).mean() and (v == y_hi).mean() < 0.5


def test_pointwise_shared_stage_wide_parameters(hawq):
    from gpu_util import run_conv_gpu, assert_same
    case = _scale_c(wl.conv_case(seed=91, N=11, H=28, W=28, C=256, K=512, R=1, S=1, stride=1, pad=0, bits=8,
                                 with_residual=True), 8)
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.U8, res_dt=hawq.U8, x_hi=127)
    assert_same(got, want, "narrow")
    wide = dict(case)
    wide["b"] = (case["b"].astype(np.int64) << 14).astype(np.int32)
    wide["c"] = (case["c"].astype(np.int32) + 14).astype(np.uint8)
    got, want2 = run_conv_gpu(wide, hawq.U8, hawq.S8, hawq.U8, res_dt=hawq.U8, x_hi=127)
    assert_same(got, want2, "wide parameters")
    assert np.array_equal(want, want2)


# 3x3 / stride 1 / pad 1 with 64 -> 64 channels and many pixels: the persistent kernel with resident weights
@pytest.mark.parametrize("N,H,W,res,res_signed,y_dt,y_hi", [
    (11, 56, 56, False, False, 0, 127),     # ResNet50 stage-1 shape
    (11, 56, 56, True, False, 0, 127),      # ResNet18 stage-1 shape: shortcut added
    (13, 53, 51, True, True, 0, 127),       # ragged tile tail, odd image size, signed shortcut
    (40, 30, 29, False, False, 2, 15),      # narrow images (several image rows per tile), packed 4-bit output
    (70, 22, 23, True, False, 1, 127),      # many small images: tiles straddle images; signed output
])
def test_conv3x3_64_channels_resident_weights(hawq, N, H, W, res, res_signed, y_dt, y_hi):
    from gpu_util import run_conv_gpu, assert_same
    case = _scale_c(wl.conv_case(seed=N + H + W, N=N, H=H, W=W, C=64, K=64, R=3, S=3, stride=1, pad=1, bits=8,
                                 with_residual=res, res_signed=res_signed), 8)
    if y_hi == 15:
        case["c"] = (case["c"] + 3).astype(np.uint8)     # 4-bit output range: eight times coarser
    signed_out = y_dt == 1
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, y_dt, res_dt=hawq.S8 if res_signed else hawq.U8,
                             relu=0 if signed_out else 1, y_lo=-128 if signed_out else 0, y_hi=y_hi, x_hi=127)
    assert_same(got, want, str((N, H, W)))
    v = oracle.unpack(want, oracle.U4) if y_dt == 2 else want.astype(np.int32)
    assert 0.05 < (v != 0).mean() and (v == y_hi).mean() < 0.5


@pytest.mark.parametrize("N,H,W,res", [(11, 56, 56, False), (12, 55, 53, True), (40, 30, 29, True)])
def test_conv3x3_64_channels_packed_int4(hawq, N, H, W, res):
    """Packed 4-bit activations, weights, shortcut and output through the persistent 3x3 kernel."""
    from gpu_util import run_conv_gpu, assert_same
    case = _scale_c(wl.conv_case(seed=N + H + W + 4, N=N, H=H, W=W, C=64, K=64, R=3, S=3, stride=1, pad=1, bits=4,
                                 with_residual=res), 4)
    got, want = run_conv_gpu(case, hawq.U4, hawq.S4, hawq.U4, res_dt=hawq.U4, y_hi=15)
    assert_same(got, want, str((N, H, W)))
    v = oracle.unpack(want, oracle.U4)
    assert 0.05 < (v > 0).mean() < 0.999


def test_conv3x3_64_channels_wide_parameters(hawq):
    """Multipliers outside the narrow epilogue's range take the exact 64-bit path inside the persistent kernel."""
    from gpu_util import run_conv_gpu, assert_same
    case = _scale_c(wl.conv_case(seed=31, N=11, H=56, W=56, C=64, K=64, R=3, S=3, stride=1, pad=1, bits=8,
                                 with_residual=True), 8)
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.U8, res_dt=hawq.U8, x_hi=127)
    assert_same(got, want, "narrow")
    wide = dict(case)
    wide["b"] = (case["b"].astype(np.int64) << 14).astype(np.int32)
    wide["c"] = (case["c"].astype(np.int32) + 14).astype(np.uint8)
    got, want2 = run_conv_gpu(wide, hawq.U8, hawq.S8, hawq.U8, res_dt=hawq.U8, x_hi=127)
    assert_same(got, want2, "wide parameters")
    assert np.array_equal(want, want2)


@pytest.mark.parametrize("res_signed,y_dt,relu,lo,hi", [(False, 0, 1, 0, 127), (True, 0, 1, 0, 127), (True, 1, 0, -128, 127),
                                                         (False, 4, 0, -100000, 100000), (False, 2, 1, 0, 15)])
def test_int8_conv_residual_and_output_types(hawq, res_signed, y_dt, relu, lo, hi):
    from gpu_util import run_conv_gpu, assert_same
    case = _scale_c(wl.conv_case(seed=77, N=2, H=14, W=14, C=128, K=256, R=1, S=1, stride=1, pad=0, bits=8,
                                 with_residual=True, res_signed=res_signed), 8)
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, y_dt, res_dt=hawq.S8 if res_signed else hawq.U8, relu=relu,
                             y_lo=lo, y_hi=hi, x_hi=127)
    assert_same(got, want)


def test_raw_int32_accumulator_output(hawq):
    from gpu_util import run_conv_gpu, assert_same
    case = wl.conv_case(seed=5, N=2, H=8, W=8, C=64, K=48, R=3, S=3, stride=1, pad=1, bits=8)
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.S32, raw=True, y_lo=0, y_hi=0, x_hi=127)
    assert_same(got, want)


_SHAPES4 = [(n, N, H, W, C, K, R, S, st, pd) for (n, N, H, W, C, K, R, S, st, pd) in wl.int4_sweep_shapes(batch=2)]


@pytest.mark.parametrize("shape", _SHAPES4, ids=[s[0] for s in _SHAPES4])
def test_int4_sweep_shapes_small_batch(hawq, shape):
    """ResNet18-shaped INT4 sweep (packed operands, packed output) at batch 2, centred scales."""
    from gpu_util import run_conv_gpu, assert_same
    name, N, H, W, C, K, R, S, stride, pad = shape
    case = _scale_c(wl.conv_case(seed=len(name), N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, bits=4), 4)
    got, want = run_conv_gpu(case, hawq.U4, hawq.S4, hawq.U4, y_hi=15)
    assert_same(got, want, name)
    v = oracle.unpack(want, oracle.U4)
    assert 0.05 < (v > 0).mean() and (v == 15).mean() < 0.5


@pytest.mark.parametrize("shape", [s for s in wl.int4_sweep_shapes(batch=8)], ids=[s[0] for s in wl.int4_sweep_shapes(batch=8)])
def test_config1_int4_sweep_literal(hawq, shape):
    """The INT4 sweep configuration as specified: batch 8, literal (b, c, bias) draws, clamp 0..15."""
    from gpu_util import run_conv_gpu, assert_same
    name, N, H, W, C, K, R, S, stride, pad = shape
    case = wl.conv_case(seed=1001, N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, bits=4)
    got, want = run_conv_gpu(case, hawq.U4, hawq.S4, hawq.U4, y_hi=15)
    assert_same(got, want, name)


def test_int4_conv_residual_u4_and_8bit_output(hawq):
    from gpu_util import run_conv_gpu, assert_same
    case = _scale_c(wl.conv_case(seed=9, N=2, H=14, W=14, C=64, K=128, R=3, S=3, stride=1, pad=1, bits=4, with_residual=True), 4)
    got, want = run_conv_gpu(case, hawq.U4, hawq.S4, hawq.U4, res_dt=hawq.U4, y_hi=15)
    assert_same(got, want)
    # 4-bit layer feeding an 8-bit consumer
    case["c"] = (case["c"].astype(np.int32) - 3).astype(np.uint8)
    got, want = run_conv_gpu(case, hawq.U4, hawq.S4, hawq.U8, res_dt=hawq.U4, y_hi=127)
    assert_same(got, want)


# 4-bit layers whose channel count is a multiple of 128: the packed operands go to LDS as they are and are split into
# nibbles at the matrix instruction.  Ragged pixel and channel tails, padding, stride, every tile shape, a shortcut,
# both output widths, the weight extremes -8 and 7 next to activation 15, and a reduction of 4608.
_SHAPES_PK = [
    (3, 13, 11, 128, 128, 3, 3, 1, 1, False, 4),    # few pixels: 64x64 tile
    (9, 29, 27, 128, 80, 3, 3, 1, 1, True, 4),      # K < 128, ragged channel tail, shortcut
    (5, 28, 28, 256, 160, 3, 3, 2, 1, False, 4),    # strided, ragged channel tile
    (12, 28, 28, 128, 128, 3, 3, 1, 1, True, 8),    # 128x128 tiles, 8-bit output
    (16, 7, 7, 512, 512, 3, 3, 1, 1, False, 4),     # 36 K-steps of 128 channels
    (7, 15, 15, 384, 64, 1, 1, 1, 0, False, 4),     # 1x1, three K-steps
    (2, 9, 9, 128, 32, 5, 5, 1, 2, False, 4),       # 5x5 taps
]


@pytest.mark.parametrize("shape", _SHAPES_PK)
def test_int4_packed_lds_form(hawq, shape):
    from gpu_util import run_conv_gpu, assert_same
    N, H, W, C, K, R, S, stride, pad, res, ybits = shape
    case = _scale_c(wl.conv_case(seed=sum(shape[:9]) + 77, N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, bits=4,
                                 with_residual=res), 4)
    # plant the extremes: a pixel of all 15s against a filter of all -8s and one of all 7s
    xu = oracle.unpack(case["x"], oracle.U4).reshape(N, H, W, C)
    wu = oracle.unpack(case["w"], oracle.S4).reshape(K, R, S, C)
    xu[0, H // 2, W // 2, :] = 15
    wu[0] = -8
    wu[K - 1] = 7
    case["x"] = wl.pack_nibbles(xu).reshape(case["x"].shape)
    case["w"] = wl.pack_nibbles(wu).reshape(case["w"].shape)
    if ybits == 8:
        case["c"] = (case["c"].astype(np.int32) - 3).astype(np.uint8)
        got, want = run_conv_gpu(case, hawq.U4, hawq.S4, hawq.U8, res_dt=hawq.U4, y_hi=127)
        v = want.astype(np.int32)
    else:
        got, want = run_conv_gpu(case, hawq.U4, hawq.S4, hawq.U4, res_dt=hawq.U4, y_hi=15)
        v = oracle.unpack(want, oracle.U4)
    assert_same(got, want, str(shape))
    assert 0.03 < (v > 0).mean() < 0.999


@pytest.mark.parametrize("shape", [(2, 20, 20, 3, 64, 7, 7, 2, 3), (1, 9, 9, 24, 10, 3, 3, 1, 1), (2, 6, 6, 64, 32, 1, 1, 1, 0)])
def test_direct_kernel_shapes_and_full_range_u8(hawq, shape):
    """Shapes the matrix-core kernel does not take: C not a multiple of 64, and unsigned inputs up to 255."""
    from gpu_util import run_conv_gpu, assert_same
    N, H, W, C, K, R, S, stride, pad = shape
    case = _scale_c(wl.conv_case(seed=3, N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, bits=8), 8)
    g = np.random.default_rng(1)
    case["x"] = g.integers(0, 256, size=case["x"].shape, dtype=np.uint8)   # full unsigned range
    got, want = run_conv_gpu(case, hawq.U8, hawq.S8, hawq.U8, x_hi=0)
    assert_same(got, want, str(shape))


def test_empty_batch_and_errors(hawq):
    import torch
    d = hawq.ConvDesc(N=0, H=8, W=8, C=64, K=64, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, x_dtype=hawq.U8,
                      w_dtype=hawq.S8, y_dtype=hawq.U8, res_dtype=hawq.U8, relu=1, y_lo=0, y_hi=127, x_hi=127)
    z8 = torch.zeros(64, dtype=torch.uint8, device="cuda")
    z32 = torch.zeros(64, dtype=torch.int32, device="cuda")
    hawq.hawq_conv2d_int(d, z8, z8, z32, z32, z8, None, None, None, z8)   # N = 0: nothing to do
    torch.cuda.synchronize()


def test_gemm_fc_shape(hawq):
    """The last layer: [N,2048] x [1000,2048]^T -> raw INT32 logits (1000 is not a multiple of 16)."""
    import torch
    from gpu_util import to_dev, assert_same
    g = np.random.default_rng(12)
    M, N, K = 37, 1000, 2048
    x = g.integers(0, 128, size=(M, K), dtype=np.uint8)
    w = g.integers(-127, 128, size=(N, K)).astype(np.int8)
    bias = g.integers(-(1 << 15), 1 << 15, size=N).astype(np.int32)
    y = torch.empty((M, N), dtype=torch.int32, device="cuda")
    hawq.hawq_gemm_int(M, N, K, hawq.U8, hawq.S8, hawq.S32, to_dev(x), to_dev(w), to_dev(bias), None, None, 0, 0, 0, y)
    torch.cuda.synchronize()
    want = oracle.gemm_int(x, w, bias, None, None, M=M, N=N, K=K, x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.S32)
    assert_same(y.cpu().numpy(), want)
    assert np.array_equal(want.astype(np.int64), x.astype(np.int64) @ w.astype(np.int64).T + bias)


@pytest.mark.parametrize("M,N,K,requant", [(37, 1000, 2048, False), (130, 96, 512, True), (5, 64, 64, True), (300, 72, 1024, True),
                                           (512, 40, 1536, False), (513, 64, 512, False)])
def test_gemm_unsigned_bytes_over_the_whole_range(hawq, M, N, K, requant):
    """HAWQ_U8 rows holding every byte value 0..255 (the matrix instruction reads signed bytes: values above 127 must not
    be read as negative), raw INT32 and requantised outputs; and the same 0..127 data passed as HAWQ_S8 and as HAWQ_U8."""
    import torch
    from gpu_util import to_dev, assert_same
    g = np.random.default_rng(M + N + K)
    x = g.integers(0, 256, size=(M, K), dtype=np.uint8)
    n = min(256, K)
    x[0, :n] = np.arange(256 - n, 256, dtype=np.uint8)
    x[-1] = 255
    w = g.integers(-127, 128, size=(N, K)).astype(np.int8)
    bias = g.integers(-(1 << 15), 1 << 15, size=N).astype(np.int32)
    b = g.integers(1 << 14, 1 << 15, size=N).astype(np.int32)
    c = np.full(N, 15 + int(np.ceil(np.log2(K * 40.0))), dtype=np.uint8)
    for x_np, x_dt in ((x, hawq.U8), ((x >> 1), hawq.U8), ((x >> 1), hawq.S8)):
        if requant:
            y = torch.full((M, N), 0x5A, dtype=torch.uint8, device="cuda")
            hawq.hawq_gemm_int(M, N, K, x_dt, hawq.S8, hawq.U8, to_dev(x_np), to_dev(w), to_dev(bias), to_dev(b), to_dev(c), 1, 0, 127, y)
            want = oracle.gemm_int(x_np.view(np.int8) if x_dt == hawq.S8 else x_np, w, bias, b, c, M=M, N=N, K=K, x_dt=x_dt,
                                   w_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127)
        else:
            y = torch.full((M, N), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
            hawq.hawq_gemm_int(M, N, K, x_dt, hawq.S8, hawq.S32, to_dev(x_np), to_dev(w), to_dev(bias), None, None, 0, 0, 0, y)
            want = oracle.gemm_int(x_np.view(np.int8) if x_dt == hawq.S8 else x_np, w, bias, None, None, M=M, N=N, K=K, x_dt=x_dt,
                                   w_dt=oracle.S8, y_dt=oracle.S32)
            assert np.array_equal(want.astype(np.int64), x_np.astype(np.int64) @ w.astype(np.int64).T + bias)
        torch.cuda.synchronize()
        assert_same(y.cpu().numpy(), want, "x_dt %d" % x_dt)
    if requant:
        assert 0.02 < np.mean(want > 0) and np.mean(want == 127) < 0.5


@pytest.mark.parametrize("shape", [(3, 14, 14, 256, 200, 3, 3, 1, 1, 8), (2, 28, 28, 128, 128, 3, 3, 2, 1, 8), (5, 9, 9, 1024, 96, 1, 1, 1, 0, 8),
                                   (12, 28, 28, 128, 128, 3, 3, 1, 1, 4), (4, 14, 14, 256, 72, 3, 3, 1, 1, 4)])
def test_blocked_weight_copy_gives_the_same_bits(hawq, shape):
    """hawq_conv_block_weights + hawq_conv_desc::w_blocked: the implicit-GEMM kernel reads the blocked copy (ragged channel
    tiles: rows past K are zero blocks), every other kernel ignores it.  Same output as without, and as the oracle."""
    import torch
    from gpu_util import run_conv_gpu, assert_same, to_dev
    N, H, W, C, K, R, S, stride, pad, bits = shape
    case = _scale_c(wl.conv_case(seed=sum(shape), N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, bits=bits), bits)
    x_dt, w_dt = (hawq.U8, hawq.S8) if bits == 8 else (hawq.U4, hawq.S4)
    y_hi = 127 if bits == 8 else 15
    ref, want = run_conv_gpu(case, x_dt, w_dt, x_dt, y_hi=y_hi, x_hi=127 if bits == 8 else 0)
    assert_same(ref, want, "plain weights %r" % (shape,))
    d = hawq.ConvDesc(N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride_h=stride, stride_w=stride, pad_h=pad, pad_w=pad, x_dtype=x_dt,
                      w_dtype=w_dt, y_dtype=x_dt, res_dtype=hawq.U8, relu=1, y_lo=0, y_hi=y_hi, x_hi=127 if bits == 8 else 0)
    nb = hawq.hawq_conv_blocked_weights_bytes(d)
    row = R * S * C * bits // 8
    assert nb == ((K + 63) // 64) * 64 * row
    w = to_dev(case["w"])
    wb = torch.full((nb,), 0x5A, dtype=torch.uint8, device="cuda")
    hawq.hawq_conv_block_weights(d, w, wb)
    torch.cuda.synchronize()
    # the copy against its definition: block (k / 64, step) holds 64 rows x 64 bytes
    wh = case["w"].reshape(K, row).view(np.uint8) if case["w"].dtype != np.uint8 else case["w"].reshape(K, row)
    blk = wb.cpu().numpy().reshape((K + 63) // 64, row // 64, 64, 64)
    full = np.zeros((((K + 63) // 64) * 64, row), dtype=np.uint8)
    full[:K] = wh
    assert np.array_equal(blk, full.reshape(-1, 64, row // 64, 64).transpose(0, 2, 1, 3))
    d.w_blocked = wb.data_ptr()
    P, Q = case["P"], case["Q"]
    y = torch.full((N, P, Q, K if bits == 8 else K // 2), 0x5A, dtype=torch.uint8, device="cuda")
    hawq.hawq_conv2d_int(d, to_dev(case["x"]), w, to_dev(case["bias"]), to_dev(case["b"]), to_dev(case["c"]), None, None, None, y)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().reshape(-1), np.asarray(want).reshape(-1).view(np.uint8))
