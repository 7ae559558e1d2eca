"""Offline converter: floating-point convolution + batch-norm parameters and static activation scales
-> the integer parameters the hot path consumes (folded INT8 / packed INT4 weights, INT32 bias, dyadic
multipliers).  Runs once, on the host, before any inference; nothing here is on the timed path.

Notation follows the paper.  A real tensor r is represented as r = S * q with an integer q and a real
scale S (Section 3.1; zero point 0: activations are post-ReLU, weights symmetric).  For one layer

    q_out = Int( (S_h * S_w / S_out) * (q_w * q_h + q_bias) )           (Section 3.1, requantisation)

the real multiplier S_h S_w / S_out is replaced by a dyadic number b / 2^c (Section 3.1, DN), the
batch norm is folded into the convolution first (Appendix D), the bias is quantised at scale
S_h * S_w so that it adds directly to the INT32 accumulator (Appendix D), and the shortcut of a
residual block is rescaled by its own dyadic number S_res / S_out before the integer add (Section 3.3).
"""
import numpy as np

from .binding import hawq_net_layer_info, hawq_net_num_layers

ACT_HI = {8: 127, 4: 15}       # largest activation integer per bit width (unsigned, post-ReLU)
W_MAX = {8: 127, 4: 7}         # largest weight magnitude per bit width (symmetric)


def fold_bn(W, beta, gamma, mean, var, eps=1e-5):
    """Appendix D: CONV_BN(h) = beta * (W h - mean) / sigma + gamma = Wbar h + bbar with
    Wbar = beta * W / sigma and bbar = gamma - beta * mean / sigma (beta is the batch norm's scale,
    gamma its shift, sigma = sqrt(var + eps) the running standard deviation).  W is [K, R, S, C]."""
    W = np.asarray(W, dtype=np.float64)
    sigma = np.sqrt(np.asarray(var, dtype=np.float64) + eps)
    g = np.asarray(beta, dtype=np.float64) / sigma
    Wbar = W * g.reshape(-1, 1, 1, 1)
    bbar = np.asarray(gamma, dtype=np.float64) - g * np.asarray(mean, dtype=np.float64)
    return Wbar, bbar


def quantize_weights(Wbar, bits):
    """Symmetric quantisation per output channel (Section 3.1; appendix on the quantisation method):
    S_w = 2 max|w| / (2^bits - 1), q_w = Int(w / S_w) with round-to-nearest, Z = 0; the one value that rounds to
    2^(bits-1) is clipped to the symmetric range.  Returns (q_w int32 [K,R,S,C], S_w float64 [K])."""
    Wbar = np.asarray(Wbar, dtype=np.float64)
    wm = W_MAX[bits]
    amax = np.abs(Wbar).reshape(Wbar.shape[0], -1).max(axis=1)
    S_w = np.where(amax > 0, 2.0 * amax / ((1 << bits) - 1), 1.0)
    q = np.clip(np.rint(Wbar / S_w.reshape(-1, 1, 1, 1)), -wm, wm).astype(np.int32)
    return q, S_w


def dyadic(s, width=15):
    """DN of Section 3.1: a positive real s as b / 2^c with a `width`-bit integer numerator,
    b in [2^(width-1), 2^width): relative error at most 2^-width.  Arrays in, (int32 b, uint8 c) out."""
    s = np.atleast_1d(np.asarray(s, dtype=np.float64))
    if np.any(s <= 0) or not np.all(np.isfinite(s)):
        raise ValueError("dyadic: scales must be positive and finite")
    m, e = np.frexp(s)                       # s = m * 2^e, m in [0.5, 1)
    b = np.rint(m * (1 << width)).astype(np.int64)
    c = width - e.astype(np.int64)
    carry = b == (1 << width)                # rounding reached 2^width: renormalise
    b = np.where(carry, b >> 1, b)
    c = np.where(carry, c - 1, c)
    if np.any(c < 1) or np.any(c > 62):
        raise ValueError("dyadic: scale out of the representable range (shift would be %s)" % (c.min() if np.any(c < 1) else c.max()))
    return b.astype(np.int32), c.astype(np.uint8)


def pack_int4(q):
    """Two 4-bit values per byte along the innermost (channel) axis, even element in the low nibble."""
    q = np.asarray(q)
    if q.shape[-1] % 2:
        raise ValueError("packed 4-bit tensors need an even innermost dimension")
    u = (q.astype(np.int32) & 0xF).astype(np.uint8)
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


def convert_conv(W, beta, gamma, mean, var, S_in, S_out, bits, S_res=None, eps=1e-5):
    """One convolution + batch norm -> integer parameters.  S_in: scale of the input activation tensor,
    S_out: scale of the tensor this layer produces (after the residual add, if any), S_res: scale of the
    shortcut tensor (None: no shortcut).  Returns dict(w, w_vals, bias, b, c, res_b, res_c, bits, S_w)."""
    Wbar, bbar = fold_bn(W, beta, gamma, mean, var, eps)
    q_w, S_w = quantize_weights(Wbar, bits)
    acc_scale = S_in * S_w                                   # scale of the INT32 accumulator, per channel
    bias = np.rint(bbar / acc_scale)
    if np.any(np.abs(bias) >= 2.0 ** 31):
        raise ValueError("bias does not fit INT32 at scale S_h * S_w")
    b, c = dyadic(acc_scale / S_out)
    out = dict(w_vals=q_w, w=pack_int4(q_w) if bits == 4 else q_w.astype(np.int8), bias=bias.astype(np.int32), b=b, c=c,
               res_b=None, res_c=None, bits=bits, S_w=S_w)
    if S_res is not None:
        rb, rc = dyadic(np.full(q_w.shape[0], S_res / S_out))
        out["res_b"], out["res_c"] = rb, rc
    return out


def _shape(info):
    return {k: info[k] for k in ("name", "C", "K", "R", "S", "stride", "pad", "H", "W", "P", "Q", "has_residual")}


def convert_resnet(arch, params, scales, bits=None, image_hw=224, num_classes=1000, eps=1e-5):
    """Whole ResNet18 / ResNet50.

    params[name] for every layer name of the canonical order ("conv1", "layer1.0.c1", ..., "fc"):
        dict(W=[K,R,S,C] float, beta, gamma, mean, var)      convolution + batch norm
        dict(W=[K,1,1,C] float, bias=[K])                    fc
    scales: dict of real scales (real = scale * integer):
        "image": input image; name -> scale of the tensor that layer produces (for the last convolution of a
        block: the block output, i.e. after the shortcut add and ReLU; for a transition convolution "…ds": its
        signed 8-bit output); "pool": the pooled vector.  The fc output stays INT32 at scale S_pool * S_w.
    bits: dict name -> 4 | 8 (default 8 everywhere); a transition convolution takes its block's c1 width;
        conv1 and fc are 8-bit.  The scale of a tensor must have been calibrated for the integer range of the
        layer that consumes it (0..15 for a 4-bit consumer).
    Returns dict(arch, image_hw, num_classes, layers=[...], pool_b, pool_c, fc_scale) with `layers` in the
    form HawqNet takes.
    """
    n = hawq_net_num_layers(arch)
    infos = [hawq_net_layer_info(arch, image_hw, num_classes, i) for i in range(n)]
    bits = dict(bits or {})
    layers = []
    block_in = None        # scale of the current block's input tensor
    prev_out = None        # scale of the tensor the previous main-branch layer produced
    fc_scale = None
    for info in infos:
        name = info["name"]
        p = params[name]
        kind = name.split(".")[-1] if "." in name else name
        lb = bits.get(name, 8)
        if kind == "ds":
            lb = bits.get(name[:-2] + "c1", 8)
        if kind == "conv1":
            S_in = scales["image"]
        elif kind == "fc":
            S_in = scales["pool"]
        elif kind in ("c1", "ds"):
            if kind == "c1":
                block_in = prev_out
            S_in = block_in
        else:
            S_in = prev_out
        if kind == "fc":
            q_w, S_w = quantize_weights(p["W"], 8)
            bias = np.rint(np.asarray(p["bias"], dtype=np.float64) / (S_in * S_w))
            K = q_w.shape[0]
            layers.append(dict(_shape(info), w_vals=q_w, w=q_w.astype(np.int8), bias=bias.astype(np.int32),
                               b=np.full(K, 1 << 14, dtype=np.int32), c=np.full(K, 15, dtype=np.uint8),   # unused: raw logits
                               res_b=None, res_c=None, bits=8, S_w=S_w))
            fc_scale = S_in * S_w
            continue
        S_res = None
        if info["has_residual"]:
            # the shortcut is the block input, or the transition convolution's output when the block has one
            # (it follows this layer in the canonical order)
            ds_name = name.rsplit(".", 1)[0] + ".ds"
            S_res = scales[ds_name] if ds_name in params else block_in
        d = convert_conv(p["W"], p["beta"], p["gamma"], p["mean"], p["var"], S_in, scales[name], lb, S_res, eps)
        d.update(_shape(info))
        layers.append(d)
        if kind != "ds":
            prev_out = scales[name]
    last = [f for f in infos if f["name"] != "fc" and not f["name"].endswith(".ds")][-1]   # its output enters the average pool
    HW = last["P"] * last["Q"]
    C_last = last["K"]
    pool_b, pool_c = dyadic(np.full(C_last, prev_out / (HW * scales["pool"])))   # Appendix E: 1/(H*W) folded in
    return dict(arch=arch, image_hw=image_hw, num_classes=num_classes, layers=layers, pool_b=pool_b, pool_c=pool_c,
                fc_scale=fc_scale)
