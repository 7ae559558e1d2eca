"""Seeded random tensors for the benchmark configurations.

Everything here is drawn from ``numpy.random.Generator(PCG64(seed))``; the draw
order inside every function is fixed and documented so that a case can be
re-created from its seed alone.

Value ranges (from the benchmark definition):
  * 8-bit activations  : unsigned, 0..127   (network image input: 0..255)
  * 4-bit activations  : unsigned, 0..15
  * 8-bit weights      : signed, -127..127  (symmetric, per output channel)
  * 4-bit weights      : signed, -7..7
  * bias               : int32
  * dyadic multiplier  : b in [2^14, 2^15), shift c an integer
4-bit tensors are packed two per byte along the innermost (channel) axis,
even element in the low nibble.
"""
import math

import numpy as np

from .layers import resnet_layers, resnet_group_names

ACT_HI = {8: 127, 4: 15}
W_MAX = {8: 127, 4: 7}


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def pack_nibbles(a):
    """Pack integers (each fitting 4 bits, signed or unsigned) two per byte
    along the last axis: element 2i -> bits 0..3, element 2i+1 -> bits 4..7."""
    a = np.asarray(a)
    if a.shape[-1] % 2:
        raise ValueError("last axis must be even to pack nibbles")
    u = (a.astype(np.int16) & 0xF).astype(np.uint8)
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


def _store_act(vals, bits):
    return pack_nibbles(vals) if bits == 4 else vals.astype(np.uint8)


def _store_w(vals, bits):
    return pack_nibbles(vals) if bits == 4 else vals.astype(np.int8)


def conv_case(seed, N, H, W, C, K, R, S, stride, pad, bits=8, with_residual=False,
              res_signed=False, c_range=(20, 30), bias_mag=1 << 15):
    """One integer conv layer with the literal distributions of the single-layer
    configurations.  Draw order: x, w, bias, b, c, [residual, res_b, res_c].

    Returns a dict with the logical (unpacked) integer arrays under ``*_vals``
    and the byte-format arrays under ``x``, ``w``, ``residual``.
    """
    g = _rng(seed)
    hi, wm = ACT_HI[bits], W_MAX[bits]
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    x = g.integers(0, hi + 1, size=(N, H, W, C), dtype=np.int32)
    w = g.integers(-wm, wm + 1, size=(K, R, S, C), dtype=np.int32)
    bias = g.integers(-bias_mag, bias_mag + 1, size=K, dtype=np.int32)
    b = g.integers(1 << 14, 1 << 15, size=K, dtype=np.int32)
    c = g.integers(c_range[0], c_range[1] + 1, size=K, dtype=np.int32).astype(np.uint8)
    case = dict(N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, P=P, Q=Q, bits=bits,
                x_vals=x, w_vals=w, x=_store_act(x, bits), w=_store_w(w, bits),
                bias=bias, b=b, c=c, relu=1, y_lo=0, y_hi=hi,
                residual=None, res_b=None, res_c=None, res_signed=res_signed)
    if with_residual:
        if res_signed:
            r = g.integers(-128, 128, size=(N, P, Q, K), dtype=np.int32)
            case["residual"] = r.astype(np.int8)
        else:
            r = g.integers(0, hi + 1, size=(N, P, Q, K), dtype=np.int32)
            case["residual"] = _store_act(r, bits)
        case["res_vals"] = r
        case["res_b"] = g.integers(1 << 14, 1 << 15, size=K, dtype=np.int32)
        case["res_c"] = g.integers(13, 17, size=K, dtype=np.int32).astype(np.uint8)
    return case


def int4_sweep_shapes(batch=8):
    """(name, N, H, W, C, K, R, S, stride, pad) for the ResNet18-shaped sweep."""
    out = []
    for hw, ch in ((56, 64), (28, 128), (14, 256), (7, 512)):
        out.append(("3x3s1_%dx%dx%d" % (hw, hw, ch), batch, hw, hw, ch, ch, 3, 3, 1, 1))
    for hw, ch in ((56, 64), (28, 128), (14, 256)):
        out.append(("3x3s2_%dx%dx%d_%d" % (hw, hw, ch, 2 * ch), batch, hw, hw, ch, 2 * ch, 3, 3, 2, 1))
    for hw, ch in ((56, 64), (28, 128), (14, 256)):
        out.append(("1x1s2_%dx%dx%d_%d" % (hw, hw, ch, 2 * ch), batch, hw, hw, ch, 2 * ch, 1, 1, 2, 0))
    return out


def make_image_batch(seed, N, image_hw=224):
    """uint8 NHWC image batch, uniform in 0..255."""
    return _rng(seed).integers(0, 256, size=(N, image_hw, image_hw, 3), dtype=np.uint8)


def draw_bits(arch, seed, p_int4=0.5):
    """Seeded per-group bit widths: one Bernoulli(p_int4) draw per group in
    canonical order; conv1 and fc always 8 (their draws are still consumed)."""
    g = _rng(seed)
    bits = {}
    for name in resnet_group_names(arch):
        four = g.random() < p_int4
        bits[name] = 4 if (four and name not in ("conv1", "fc")) else 8
    return bits


# Second-moment estimates E[x^2] / hi^2 of the tensor a conv reads, used only to
# centre the synthetic requantisation scale so activations neither die nor
# saturate (a trained network gets this from calibration; we have no data).
_M2_POST_RELU = 0.075
_M2_POST_POOL = 0.28
_M2_BLOCK_OUT = 0.10
_M2_IMAGE = 255.0 * 511.0 / 6.0


def _shift_for(scale):
    """Shift c0 such that 1.5*2^14 / 2^c0 is about `scale`."""
    return int(math.floor(math.log2(1.5 * (1 << 14) / scale)))


def make_resnet(arch, seed, bits=None, image_hw=224, num_classes=1000, int32_shortcut=False):
    """Random integer parameters for a whole integer-only ResNet.

    int32_shortcut: every block with a transition convolution adds that convolution's INT32 accumulator
    directly (both branches rescaled from INT32); the same draws are made, and the transition layer's shift
    is then raised by the shortcut shift of the block's last convolution minus 15, so that its multiplier
    maps the accumulator to the block's output scale instead of to a stored signed 8-bit tensor.

    `bits` maps group name -> 4 | 8 (default: all 8).  Per layer the draw order
    is w, bias, b, c, [res_b, res_c]; after the last layer: pool_b, pool_c.

    Returns dict(arch, image_hw, layers=[...], pool_b, pool_c, bits) where each
    layer dict carries the shape entries of ``resnet_layers`` plus
      bits, w (int8 KRSC or packed nibbles), w_vals (int32 logical),
      bias, b, c, res_b, res_c (None unless has_residual),
      in_hi (largest input activation), relu, y_lo, y_hi, y_bits.
    Storage rule: a tensor is stored at the bit width of the conv that consumes
    it; a transition (ds) output is always signed 8-bit; the tensor entering
    the average pool, the pooled vector and the fc input are 8-bit.
    """
    g = _rng(seed)
    shapes = resnet_layers(arch, image_hw, num_classes)
    groups = resnet_group_names(arch)
    if bits is None:
        bits = {n: 8 for n in groups}
    for l in shapes:
        if l["group"] not in bits:
            raise ValueError("bits lacks group " + l["group"])
    if bits["conv1"] != 8 or bits["fc"] != 8:
        raise ValueError("first and last layer stay 8-bit")

    # bit width of the consumer of every conv's output
    def consumer_bits(i):
        l = shapes[i]
        if l["kind"] in ("ds",):
            return 8
        if l["kind"] == "fc":
            return 32
        # next non-ds layer in canonical order consumes the output (for the
        # block's last conv: the next block's c1, or the pool/fc: 8-bit)
        if l["has_residual"] or l["kind"] == "stem":
            j = i + 1
            while j < len(shapes) and shapes[j]["kind"] == "ds":
                j += 1
            nxt = shapes[j]
            return 8 if nxt["kind"] == "fc" else bits[nxt["group"]]
        return bits[shapes[i + 1]["group"]]

    layers = []
    block_in_bits = None
    for i, l in enumerate(shapes):
        lb = bits[l["group"]]
        d = dict(l)
        d["bits"] = lb
        wm = W_MAX[lb]
        kdim = l["R"] * l["S"] * l["C"]
        if l["kind"] == "stem":
            m2 = _M2_IMAGE
            in_hi = 255
        else:
            in_hi = ACT_HI[lb]
            if l["kind"] in ("c1", "ds"):
                first = (l["stage"] == 1 and l["block"] == 0)
                m2 = (_M2_POST_POOL if first else _M2_BLOCK_OUT) * in_hi * in_hi
            elif l["kind"] == "fc":
                m2 = 0.05 * in_hi * in_hi
            else:
                m2 = _M2_POST_RELU * in_hi * in_hi
        var_w = wm * (wm + 1) / 3.0
        sigma = math.sqrt(kdim * m2 * var_w)
        w = g.integers(-wm, wm + 1, size=(l["K"], l["R"], l["S"], l["C"]), dtype=np.int32)
        d["w_vals"] = w
        d["w"] = _store_w(w, lb)
        d["in_hi"] = in_hi
        K = l["K"]
        if l["kind"] == "fc":
            d["bias"] = g.integers(-(1 << 15), (1 << 15) + 1, size=K, dtype=np.int32)
            d["b"] = g.integers(1 << 14, 1 << 15, size=K, dtype=np.int32)  # unused: raw int32 logits
            d["c"] = np.full(K, 20, dtype=np.uint8)
            d["res_b"] = d["res_c"] = None
            d.update(relu=0, y_lo=-(1 << 31), y_hi=(1 << 31) - 1, y_bits=32)
            layers.append(d)
            continue
        yb = consumer_bits(i)
        hi = ACT_HI[yb]
        if l["kind"] == "ds":
            bias_lo, bias_hi, target = -0.5, 0.5, 40.0
            d.update(relu=0, y_lo=-128, y_hi=127, y_bits=8)
        elif l["has_residual"]:
            bias_lo, bias_hi, target = -0.25, 0.75, hi / 4.0
            d.update(relu=1, y_lo=0, y_hi=hi, y_bits=yb)
        else:
            bias_lo, bias_hi, target = -0.1, 0.9, hi / 3.0
            d.update(relu=1, y_lo=0, y_hi=hi, y_bits=yb)
        d["bias"] = np.rint(sigma * g.uniform(bias_lo, bias_hi, size=K)).astype(np.int32)
        c0 = _shift_for(target / (1.04 * sigma))
        d["b"] = g.integers(1 << 14, 1 << 15, size=K, dtype=np.int32)
        d["c"] = (c0 + g.integers(0, 2, size=K)).astype(np.uint8)
        if l["kind"] == "c1":
            block_in_bits = lb
        if l["has_residual"]:
            # shortcut: the block input stored at block_in_bits, or the ds output (signed 8-bit);
            # ds comes after this layer in canonical order, so look ahead
            has_ds = i + 1 < len(shapes) and shapes[i + 1]["kind"] == "ds"
            res_hi = 127 if (has_ds or block_in_bits == 8) else 15
            shift = 16 + int(round(math.log2((res_hi + 1) / (hi + 1))))
            d["res_b"] = g.integers(1 << 14, 1 << 15, size=K, dtype=np.int32)
            d["res_c"] = np.full(K, shift, dtype=np.uint8)
            d["res_bits"] = 8 if has_ds else block_in_bits
            d["res_signed"] = bool(has_ds)
        else:
            d["res_b"] = d["res_c"] = None
        layers.append(d)

    for i, d in enumerate(layers):
        d["int32_shortcut"] = False
        if int32_shortcut and d["kind"] == "ds":
            last = layers[i - 1]
            assert last["has_residual"]
            d["c"] = (d["c"].astype(np.int32) + last["res_c"].astype(np.int32) - 15).astype(np.uint8)
            d["int32_shortcut"] = True
            last["int32_shortcut"] = True

    c_last = shapes[-1]["C"]
    hw_pool = shapes[-2]["P"] * shapes[-2]["Q"]
    pc = 14 + max(1, int(math.ceil(math.log2(hw_pool))))
    pool_b = np.rint((1 << pc) / hw_pool * g.uniform(0.9, 1.1, size=c_last)).astype(np.int32)
    pool_c = np.full(c_last, pc, dtype=np.uint8)
    return dict(arch=arch, image_hw=image_hw, num_classes=num_classes, layers=layers,
                pool_b=pool_b, pool_c=pool_c, bits=dict(bits))
