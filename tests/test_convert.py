"""Offline converter (float conv + batch norm + static scales -> integer parameters): pins of its steps against
independent test-side definitions (tests/helpers.py, float64 library convolution), the integer network it produces
against a real-valued simulation, and -- on the GPU -- that the product path runs the converted network bit-exactly
like the oracle."""
import numpy as np
import pytest

import oracle
from oracle import resnet as onet
import workloads as wl
from helpers import dyadic_from_real, quantize_symmetric_per_channel

import paper_2011_10680_amd.convert as cv


def _conv_f64(x, w, stride, pad):
    import torch
    import torch.nn.functional as F
    xt = torch.from_numpy(np.asarray(x, dtype=np.float64)).permute(0, 3, 1, 2).contiguous()
    wt = torch.from_numpy(np.asarray(w, dtype=np.float64)).permute(0, 3, 1, 2).contiguous()
    return F.conv2d(xt, wt, stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()


def test_fold_bn_is_the_identity_of_appendix_d():
    g = np.random.default_rng(1)
    W = g.normal(size=(6, 3, 3, 5))
    beta, gamma = g.uniform(0.5, 1.5, 6), g.normal(size=6)
    mean, var = g.normal(size=6), g.uniform(0.2, 2.0, 6)
    h = g.normal(size=(2, 7, 7, 5))
    conv = _conv_f64(h, W, 1, 1)
    bn = beta * (conv - mean) / np.sqrt(var + 1e-5) + gamma
    Wbar, bbar = cv.fold_bn(W, beta, gamma, mean, var, 1e-5)
    assert np.allclose(_conv_f64(h, Wbar, 1, 1) + bbar, bn, rtol=1e-10, atol=1e-10)


@pytest.mark.parametrize("bits", [8, 4])
def test_weight_quantisation_matches_the_independent_helper(bits):
    g = np.random.default_rng(bits)
    W = g.normal(size=(9, 3, 3, 8)) * g.uniform(0.01, 10, size=(9, 1, 1, 1))
    q, S = cv.quantize_weights(W, bits)
    q2, S2 = quantize_symmetric_per_channel(W, bits)
    assert np.array_equal(q, q2) and np.allclose(S, S2, rtol=1e-15)
    wm = (1 << (bits - 1)) - 1
    assert q.min() >= -wm and q.max() <= wm
    assert np.all(np.abs(q).reshape(9, -1).max(axis=1) == wm)                 # every channel uses its full range
    assert np.all(np.abs(W - S.reshape(-1, 1, 1, 1) * q) <= S.reshape(-1, 1, 1, 1) * 0.5 + 1e-12)


def test_dyadic_numbers_match_the_helper_and_the_error_bound():
    g = np.random.default_rng(3)
    s = np.concatenate([2.0 ** g.uniform(-20, 3, 500), [0.5, 1.0, 2.0 ** -7, (1 << 15) / 2.0 ** 15 - 2.0 ** -17]])
    b, c = cv.dyadic(s)
    for si, bi, ci in zip(s, b, c):
        assert (bi, ci) == tuple(int(v) for v in dyadic_from_real(si))
    assert b.min() >= 1 << 14 and b.max() < 1 << 15
    assert np.all(np.abs(b / 2.0 ** c.astype(np.float64) - s) <= s * 2.0 ** -15)
    with pytest.raises(ValueError):
        cv.dyadic([0.0])
    with pytest.raises(ValueError):
        cv.dyadic([2.0 ** 20])


def test_pack_int4_is_the_oracle_encoding():
    g = np.random.default_rng(4)
    q = g.integers(-7, 8, size=(5, 3, 3, 8))
    assert np.array_equal(np.asarray(oracle.unpack(cv.pack_int4(q), oracle.S4)).ravel(), q.ravel())


def test_one_converted_layer_tracks_the_real_valued_layer():
    """Integer layer (oracle) on quantised inputs vs the real-valued conv + BN + ReLU: the difference is bounded by
    the weight / bias / output rounding steps (Section 3.1: the integer pipeline computes Int(S_h S_w / S_out (...)))."""
    g = np.random.default_rng(5)
    N, H, C, K = 2, 9, 16, 12
    W = g.normal(size=(K, 3, 3, C)) / np.sqrt(9 * C)
    beta, gamma = g.uniform(0.8, 1.2, K), g.normal(size=K) * 0.1
    mean, var = g.normal(size=K) * 0.1, g.uniform(0.5, 1.5, K)
    q_h = g.integers(0, 128, size=(N, H, H, C)).astype(np.uint8)
    S_h = 1.0 / 64
    real_in = S_h * q_h
    real_out = np.maximum(beta * (_conv_f64(real_in, W, 1, 1) - mean) / np.sqrt(var + 1e-5) + gamma, 0)
    S_out = real_out.max() / 127
    d = cv.convert_conv(W, beta, gamma, mean, var, S_h, S_out, 8)
    q_out = oracle.conv2d_int(q_h, d["w"], d["bias"], d["b"], d["c"], N=N, H=H, W=H, C=C, K=K, R=3, S=3, stride=(1, 1),
                              pad=(1, 1), x_dt=oracle.U8, w_dt=oracle.S8, y_dt=oracle.U8, relu=1, y_lo=0, y_hi=127)
    # error budget in real units: weights off by <= S_w/2 each (sum over 9C taps of |h|), bias by S_h S_w / 2,
    # the dyadic multiplier by 2^-15 relative, the output by S_out / 2
    w_err = 0.5 * d["S_w"] * _conv_f64(np.abs(real_in), np.ones((1, 3, 3, C)), 1, 1).max()
    bound = w_err + 0.5 * S_h * d["S_w"] + 2.0 ** -15 * real_out.max() + 0.5 * S_out + 1e-9
    err = np.abs(S_out * q_out.astype(np.float64) - real_out)
    assert np.all(err <= bound.reshape(1, 1, 1, K)), (err.max(), bound.max())
    assert err.mean() < 0.6 * S_out          # in practice: about one output rounding step


def _float_resnet(arch, image_hw, num_classes, seed):
    """Random float ResNet in the converter's input format, plus a float64 forward that records every tensor's range."""
    import paper_2011_10680_amd as hawq
    g = np.random.default_rng(seed)
    infos = [hawq.hawq_net_layer_info(arch, image_hw, num_classes, i) for i in range(hawq.hawq_net_num_layers(arch))]
    params = {}
    for f in infos:
        K, R, S, C = f["K"], f["R"], f["S"], f["C"]
        W = g.normal(size=(K, R, S, C)) * np.sqrt(2.0 / (R * S * C))
        if f["name"] == "fc":
            params[f["name"]] = dict(W=W, bias=g.normal(size=K) * 0.05)
        else:
            last = f["has_residual"]
            params[f["name"]] = dict(W=W, beta=g.uniform(0.3, 0.6, K) if last else g.uniform(0.8, 1.2, K),
                                     gamma=g.normal(size=K) * 0.1, mean=g.normal(size=K) * 0.05, var=g.uniform(0.8, 1.2, K))
    return infos, params


def _float_forward(infos, params, x_real, arch):
    """float64 forward; returns logits and the max of every tensor the converter needs a scale for."""
    import torch
    import torch.nn.functional as F
    info = {f["name"]: f for f in infos}
    rng = {}

    def conv_bn(name, h, relu):
        f, p = info[name], params[name]
        y = _conv_f64(h, p["W"], f["stride"], f["pad"])
        y = p["beta"] * (y - p["mean"]) / np.sqrt(p["var"] + 1e-5) + p["gamma"]
        return np.maximum(y, 0) if relu else y

    h = conv_bn("conv1", x_real, True)
    rng["conv1"] = h.max()
    h = F.max_pool2d(torch.from_numpy(h).permute(0, 3, 1, 2), 3, 2, 1).permute(0, 2, 3, 1).numpy()
    names = [f["name"] for f in infos]
    blocks = sorted({n.rsplit(".", 1)[0] for n in names if n.startswith("layer")}, key=lambda s: [int(v) for v in s[5:].split(".")])
    for blk in blocks:
        x_in = h
        t = conv_bn(blk + ".c1", x_in, True)
        rng[blk + ".c1"] = t.max()
        if arch == 50:
            t = conv_bn(blk + ".c2", t, True)
            rng[blk + ".c2"] = t.max()
            lastn = blk + ".c3"
        else:
            lastn = blk + ".c2"
        main = conv_bn(lastn, t, False)
        if blk + ".ds" in info:
            sc = conv_bn(blk + ".ds", x_in, False)
            rng[blk + ".ds"] = np.abs(sc).max()
        else:
            sc = x_in
        h = np.maximum(main + sc, 0)
        rng[lastn] = h.max()
    pooled = h.mean(axis=(1, 2))
    rng["pool"] = pooled.max()
    p = params["fc"]
    logits = pooled @ p["W"].reshape(p["W"].shape[0], -1).T + p["bias"]
    return logits, rng


def _converted_net(arch=18, image_hw=64, num_classes=40, seed=11, batch=4):
    infos, params = _float_resnet(arch, image_hw, num_classes, seed)
    x = wl.make_image_batch(seed, batch, image_hw=image_hw)
    S_img = 1.0 / 255
    logits, rng = _float_forward(infos, params, S_img * x.astype(np.float64), arch)
    scales = {"image": S_img}
    for k, v in rng.items():
        scales[k] = 1.1 * v / (128 if k.endswith(".ds") else 127)      # 10 % head room over the calibration batch
    net = cv.convert_resnet(arch, params, scales, image_hw=image_hw, num_classes=num_classes)
    return net, x, logits


def test_converted_resnet18_tracks_the_float_network():
    net, x, logits = _converted_net()
    q = onet.forward(net, x)
    approx = q.astype(np.float64) * net["fc_scale"].reshape(1, -1)
    # 8-bit everywhere: the integer network reproduces the float logits closely
    cos = np.sum(approx * logits, axis=1) / (np.linalg.norm(approx, axis=1) * np.linalg.norm(logits, axis=1))
    assert np.all(cos > 0.98), cos
    assert np.abs(approx - logits).max() < 0.25 * np.abs(logits).max()
    assert len(np.unique(q)) > 50


@pytest.mark.gpu
def test_converted_resnet18_runs_bit_exactly_on_the_gpu():
    import torch
    import paper_2011_10680_amd as hawq
    net, x, _ = _converted_net()
    want = onet.forward(net, x)
    hn = hawq.HawqNet(net["arch"], net["layers"], net["pool_b"], net["pool_c"], image_hw=net["image_hw"],
                      num_classes=net["num_classes"])
    N = x.shape[0]
    ws = torch.empty(hn.workspace_bytes(N), dtype=torch.uint8, device="cuda")
    out = torch.empty((N, net["num_classes"]), dtype=torch.int32, device="cuda")
    hn.hawq_forward_resnet(torch.from_numpy(x).cuda(), N, out, ws)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)
    hn.close()
