"""Pins for the oracle's network walk: topology totals from Table 1, an independent float64
library composition end to end, non-degeneracy of the synthetic networks."""
import numpy as np
import pytest

import oracle
from oracle import resnet as onet
import workloads as wl
from conftest import read_golden


def _macs(layers):
    # layers: (name, C, K, R, stride, pad, H_in, P_out)
    return {n: P * P * K * R * R * C for (n, C, K, R, s, p, H, P) in layers}


@pytest.mark.parametrize("arch", [18, 50])
def test_topology_reproduces_table1_bops_and_size(arch, golden_dir):
    gold = read_golden(golden_dir + "/table1_bops_size.txt")
    topo = onet.topology(arch)
    macs = _macs(topo)
    total = sum(macs.values())
    weights = sum(K * R * R * C for (n, C, K, R, s, p, H, P) in topo)
    pre = "resnet%d_" % arch
    assert round(total * 32 * 32 / 1e9) == gold[pre + "w32a32_gbops"]
    assert round(total * 8 * 8 / 1e9) == gold[pre + "w8a8_gbops"]
    w4a4 = ((macs["conv1"] + macs["fc"]) * 64 + (total - macs["conv1"] - macs["fc"]) * 16) / 1e9
    assert int(w4a4) == gold[pre + "w4a4_gbops"]          # the table truncates: 34.7 -> 34, 67.5 -> 67
    assert abs(weights / 2 ** 20 - gold[pre + "w8_size_mb"]) / gold[pre + "w8_size_mb"] < 0.012
    # the stride-on-3x3 variant of ResNet50 would give 262 GBOPS at W8A8, not 247
    if arch == 50:
        assert abs(total / 1e9 - 3.858) < 1e-3
    # the generator's shape table and the oracle's topology agree
    shapes = wl.resnet_layers(arch)
    assert [(l["name"], l["C"], l["K"], l["R"], l["stride"], l["pad"], l["H"], l["P"]) for l in shapes] == topo


def _torch_forward(net, x):
    """Independent composition with float64 library ops (exact below 2^53)."""
    import torch
    import torch.nn.functional as F
    L = {l["name"]: l for l in net["layers"]}
    order = [l["name"] for l in net["layers"]]

    def vals(l):
        return torch.from_numpy(l["w_vals"].astype(np.float64)).permute(0, 3, 1, 2).contiguous()

    def requant(t, b, c):  # t: [N,K,H,W] float64 holding integers
        ti = t.numpy().astype(np.int64)
        bb = b.astype(np.int64).reshape(1, -1, 1, 1)
        cc = c.astype(np.int64).reshape(1, -1, 1, 1)
        return (ti * bb + (np.int64(1) << (cc - 1))) // (np.int64(1) << cc)

    def acc(l, inp):
        return F.conv2d(inp, vals(l), stride=l["stride"], padding=l["pad"]) + torch.from_numpy(l["bias"].astype(np.float64)).reshape(1, -1, 1, 1)

    def conv(l, inp, res=None, sc_acc=None):
        t = acc(l, inp)
        y = requant(t, l["b"], l["c"])
        if sc_acc is not None:          # the shortcut convolution's INT32 accumulator, rescaled by that layer's own (b, c)
            y = y + requant(sc_acc[1], sc_acc[0]["b"], sc_acc[0]["c"])
        elif res is not None:
            y = y + requant(res, l["res_b"], l["res_c"])
        if l["relu"]:
            y = np.maximum(y, 0)
        return torch.from_numpy(np.clip(y, l["y_lo"], l["y_hi"]).astype(np.float64))

    t = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    t = conv(L["conv1"], t)
    t = F.max_pool2d(t, 3, 2, 1)
    blocks = []
    for n in order:
        pre = n.rsplit(".", 1)[0]
        if n.startswith("layer") and pre not in blocks:
            blocks.append(pre)
    for pre in blocks:
        inp = t
        ds = L.get(pre + ".ds")
        sc_acc = (ds, acc(ds, inp)) if (ds is not None and ds["int32_shortcut"]) else None
        sc = None if sc_acc is not None else (conv(ds, inp) if ds is not None else inp)
        u = conv(L[pre + ".c1"], inp)
        if (pre + ".c3") in L:
            u = conv(L[pre + ".c2"], u)
            t = conv(L[pre + ".c3"], u, res=sc, sc_acc=sc_acc)
        else:
            t = conv(L[pre + ".c2"], u, res=sc, sc_acc=sc_acc)
    s = t.sum(dim=(2, 3)).numpy().astype(np.int64)
    pb, pc = net["pool_b"].astype(np.int64), net["pool_c"].astype(np.int64)
    pooled = np.clip((s * pb + (1 << (pc - 1))) // (1 << pc), 0, 127)
    fc = L["fc"]
    return pooled @ fc["w_vals"].reshape(fc["K"], -1).astype(np.int64).T + fc["bias"].astype(np.int64)


@pytest.mark.parametrize("arch,mixed,int32_sc", [(18, False, False), (50, False, False), (18, True, False), (50, True, False),
                                                 (18, False, True), (50, True, True)])
def test_forward_equals_independent_float64_composition(arch, mixed, int32_sc):
    bits = wl.draw_bits(arch, 77 + arch) if mixed else None
    net = wl.make_resnet(arch, seed=500 + arch, bits=bits, image_hw=64, num_classes=40, int32_shortcut=int32_sc)
    assert sum(l["int32_shortcut"] and l["kind"] == "ds" for l in net["layers"]) == ((3 if arch == 18 else 4) if int32_sc else 0)
    if mixed:
        assert 0 < sum(l["bits"] == 4 for l in net["layers"]) < len(net["layers"])
    x = wl.make_image_batch(3, 2, image_hw=64)
    got = onet.forward(net, x)
    want = _torch_forward(net, x)
    assert got.dtype == np.int32 and got.shape == (2, 40)
    assert np.array_equal(got.astype(np.int64), want)
    assert np.abs(got[0] - got[1]).max() > 0


@pytest.mark.parametrize("arch,mixed,int32_sc", [(18, False, False), (50, True, False), (50, False, True)])
def test_synthetic_network_is_not_degenerate(arch, mixed, int32_sc):
    """Random weights with arbitrary scales would saturate within a few layers and make bit-exactness
    vacuous; the generator centres every layer's scale analytically.  Check it worked."""
    bits = wl.draw_bits(arch, 4000 + arch) if mixed else None
    net = wl.make_resnet(arch, seed=1000 + arch, bits=bits, int32_shortcut=int32_sc)
    x = wl.make_image_batch(7, 1)
    keep = {}
    logits = onet.forward(net, x, keep)
    L = {l["name"]: l for l in net["layers"]}
    first_bits = net["layers"][1]["bits"]
    for name, t in keep.items():
        if name == "fc":
            continue
        if name in L and L[name]["kind"] == "ds":
            v = t.astype(np.int32).ravel()
            assert (v == -128).mean() < 0.15 and (v == 127).mean() < 0.15 and v.std() > 10
            continue
        yb = L[name]["y_bits"] if name in L else (first_bits if name == "pool" else 8)
        v = oracle.unpack(t, oracle.U4) if (yb == 4 and name != "conv1") else t.astype(np.int32).ravel()
        hi = 15 if yb == 4 else 127
        assert (v == 0).mean() < 0.60, name
        assert (v >= hi).mean() < 0.20, name
        assert v.max() <= hi
    assert len(np.unique(logits)) > 500
