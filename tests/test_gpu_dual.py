"""GPU parity: hawq_conv2d_dual_int (a block output with a convolution on both branches, both INT32 accumulators rescaled
and added) and the network forward with INT32 shortcuts, vs the CPU oracle, bit-exact."""
import numpy as np
import pytest

import oracle
from oracle import resnet as onet
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hawq():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2011_10680_amd as h
    h.load_library()
    return h


def _case(seed, N, H, C, K, R, Cs, stride_s, bits=8, bits_s=None, wide=False):
    """Seeded operands: main R x R / stride 1 convolution over [N,H,H,C], 1x1 / stride_s shortcut over [N,Hs,Hs,Cs]; shifts
    centred on the accumulator spread so that outputs cover the clamp range."""
    bits_s = bits_s or bits
    g = np.random.default_rng(seed)
    pad = R // 2
    P = H
    Hs = (P - 1) * stride_s + 1 + (stride_s - 1) * int(g.integers(0, 2))   # with or without an unused last row / column
    hi, wm = (127, 127) if bits == 8 else (15, 7)
    his, wms = (127, 127) if bits_s == 8 else (15, 7)
    t = dict(N=N, K=K, H=H, C=C, R=R, pad=pad, P=P, Hs=Hs, Cs=Cs, stride_s=stride_s, bits=bits, bits_s=bits_s)
    t["x"] = g.integers(0, hi + 1, size=(N, H, H, C), dtype=np.int32)
    t["w"] = g.integers(-wm, wm + 1, size=(K, R, R, C), dtype=np.int32)
    t["xs"] = g.integers(0, his + 1, size=(N, Hs, Hs, Cs), dtype=np.int32)
    t["ws"] = g.integers(-wms, wms + 1, size=(K, 1, 1, Cs), dtype=np.int32)
    sig = np.sqrt(R * R * C * (hi * hi / 3.0) * (wm * (wm + 1) / 3.0)) + 1
    sigs = np.sqrt(Cs * (his * his / 3.0) * (wms * (wms + 1) / 3.0)) + 1
    t["bias"] = np.rint(sig * g.uniform(-0.5, 0.5, size=K)).astype(np.int32)
    t["bias_s"] = np.rint(sigs * g.uniform(-0.5, 0.5, size=K)).astype(np.int32)
    t["b"] = g.integers(1 << 14, 1 << 15, size=K, dtype=np.int32)
    t["b_s"] = g.integers(1 << 14, 1 << 15, size=K, dtype=np.int32)
    t["c"] = (int(np.floor(np.log2(1.5 * (1 << 14) * sig / 30.0))) + g.integers(0, 2, size=K)).astype(np.uint8)
    t["c_s"] = (int(np.floor(np.log2(1.5 * (1 << 14) * sigs / 30.0))) + g.integers(0, 2, size=K)).astype(np.uint8)
    if wide:   # numerators beyond the narrow evaluation's range on a few channels: same values, other code path
        for nb, nc in (("b", "c"), ("b_s", "c_s")):
            sel = g.random(K) < 0.1
            sel[0] = True
            t[nb] = np.where(sel, t[nb].astype(np.int64) << 15, t[nb]).astype(np.int32)
            t[nc] = np.where(sel, t[nc].astype(np.int32) + 15, t[nc]).astype(np.uint8)
    return t


def _store(v, bits, signed):
    if bits == 4:
        return wl.pack_nibbles(v)
    return v.astype(np.int8 if signed else np.uint8)


def _run(hawq, t, y_dt, relu, y_lo, y_hi):
    import torch
    from gpu_util import to_dev, out_shape
    N, K, H, C, R, P, Hs, Cs, ss = (t[k] for k in ("N", "K", "H", "C", "R", "P", "Hs", "Cs", "stride_s"))
    x_dt, w_dt = (hawq.U8, hawq.S8) if t["bits"] == 8 else (hawq.U4, hawq.S4)
    xs_dt, ws_dt = (hawq.U8, hawq.S8) if t["bits_s"] == 8 else (hawq.U4, hawq.S4)
    x, w = _store(t["x"], t["bits"], False), _store(t["w"], t["bits"], True)
    xs, ws = _store(t["xs"], t["bits_s"], False), _store(t["ws"], t["bits_s"], True)
    d = hawq.ConvDesc(N=N, H=H, W=H, C=C, K=K, R=R, S=R, stride_h=1, stride_w=1, pad_h=t["pad"], pad_w=t["pad"], x_dtype=x_dt,
                      w_dtype=w_dt, y_dtype=y_dt, res_dtype=hawq.U8, relu=relu, y_lo=y_lo, y_hi=y_hi, x_hi=127 if t["bits"] == 8 else 0)
    dsc = hawq.ConvDesc(N=N, H=Hs, W=Hs, C=Cs, K=K, R=1, S=1, stride_h=ss, stride_w=ss, pad_h=0, pad_w=0, x_dtype=xs_dt,
                        w_dtype=ws_dt, y_dtype=y_dt, res_dtype=hawq.U8, relu=0, y_lo=y_lo, y_hi=y_hi, x_hi=127 if t["bits_s"] == 8 else 0)
    y = torch.full(out_shape((N, P, P, K), y_dt), 0x5A, dtype=torch.int8 if y_dt == hawq.S8 else torch.uint8, device="cuda")
    hawq.hawq_conv2d_dual_int(d, to_dev(x), to_dev(w), to_dev(t["bias"]), to_dev(t["b"]), to_dev(t["c"]),
                              dsc, to_dev(xs), to_dev(ws), to_dev(t["bias_s"]), to_dev(t["b_s"]), to_dev(t["c_s"]), y)
    torch.cuda.synchronize()
    want = oracle.conv2d_dual_int(x, w, t["bias"], t["b"], t["c"], xs, ws, t["bias_s"], t["b_s"], t["c_s"],
                                  N=N, K=K, H=H, W=H, C=C, R=R, S=R, stride=1, pad=t["pad"], x_dt=x_dt, w_dt=w_dt,
                                  Hs=Hs, Ws=Hs, Cs=Cs, Rs=1, Ss=1, stride_s=ss, pad_s=0, xs_dt=xs_dt, ws_dt=ws_dt,
                                  y_dt=y_dt, relu=relu, y_lo=y_lo, y_hi=y_hi)
    return y.cpu().numpy(), want


# (N, H, C, K, R, Cs, stride_s): the transition blocks of ResNet50 / ResNet18 in miniature, ragged pixel and channel tiles
_SHAPES = [
    (2, 28, 64, 256, 1, 64, 1),       # stage 1 of ResNet50: one K-step per branch, 12.25 pixel tiles
    (3, 14, 128, 512, 1, 256, 2),     # stage 2: strided shortcut
    (2, 7, 512, 2048, 1, 1024, 2),    # stage 4: a single partial pixel tile, 8 + 16 K-steps, 16 channel tiles
    (2, 14, 128, 128, 3, 64, 2),      # ResNet18: 3x3 main branch (zero padding) + strided 1x1 shortcut
    (1, 9, 64, 192, 1, 128, 1),       # K not a multiple of the channel tile
    (5, 16, 256, 144, 3, 192, 1),     # ragged everything
    (3, 7, 512, 512, 3, 256, 2),      # stage 4 of ResNet18: few tiles, 72 + 4 K-steps -> the quarter-size tiles
    (2, 7, 512, 600, 3, 320, 2),      # the same with a ragged channel tile and five shortcut K-steps
]


@pytest.mark.parametrize("shape", _SHAPES)
def test_matrix_core_form(hawq, shape):
    from gpu_util import assert_same
    N, H, C, K, R, Cs, ss = shape
    t = _case(sum(shape), N, H, C, K, R, Cs, ss)
    got, want = _run(hawq, t, hawq.U8, 1, 0, 127)
    assert_same(got, want, "dual conv %r" % (shape,))
    assert 0.02 < (want == 0).mean() < 0.9 and (want == 127).mean() < 0.2    # the case exercises the arithmetic
    got, want = _run(hawq, t, hawq.S8, 0, -128, 127)
    assert_same(got, want, "dual conv, signed output %r" % (shape,))
    assert (want < 0).any() and (want > 0).any()


def test_wide_multipliers_and_4bit_output(hawq):
    from gpu_util import assert_same
    t = _case(99, 3, 14, 128, 256, 1, 256, 2)
    ref, _ = _run(hawq, t, hawq.U8, 1, 0, 127)
    tw = _case(99, 3, 14, 128, 256, 1, 256, 2, wide=True)
    got, want = _run(hawq, tw, hawq.U8, 1, 0, 127)
    assert_same(got, want, "wide multipliers")
    assert_same(got, ref, "scaling numerator and shift together changes nothing")
    got, want = _run(hawq, t, hawq.U4, 1, 0, 15)
    assert_same(got, want, "packed 4-bit output")
    got, want = _run(hawq, tw, hawq.U4, 1, 0, 15)
    assert_same(got, want, "packed 4-bit output, wide multipliers")


@pytest.mark.parametrize("kw", [dict(C=48, Cs=64), dict(C=64, Cs=40), dict(K=72), dict(bits=4), dict(bits_s=4), dict(bits=4, bits_s=4)])
def test_other_shapes_and_widths_take_the_exact_general_kernel(hawq, kw):
    from gpu_util import assert_same
    a = dict(N=2, H=6, C=64, K=64, R=1, Cs=64, stride_s=2, bits=8, bits_s=None)
    a.update(kw)
    t = _case(7 + len(kw), **a)
    hi = 127
    got, want = _run(hawq, t, hawq.U8, 1, 0, hi)
    assert_same(got, want, "general dual conv %r" % (kw,))
    assert (want > 0).any()


def _forward_gpu(hawq, net, x, keep):
    import torch
    N = x.shape[0]
    hn = hawq.HawqNet(net["arch"], net["layers"], net["pool_b"], net["pool_c"], image_hw=net["image_hw"],
                      num_classes=net["num_classes"], keep_activations=keep)
    ws = torch.empty(hn.workspace_bytes(N), dtype=torch.uint8, device="cuda")
    logits = torch.empty((N, net["num_classes"]), dtype=torch.int32, device="cuda")
    hn.hawq_forward_resnet(torch.from_numpy(x).cuda(), N, logits, ws)
    torch.cuda.synchronize()
    acts, names = {}, []
    wsh = ws.cpu().numpy() if keep else None
    for s in range(hn.num_steps()):
        o = hn.step_output(N, s)
        names.append(o["name"])
        if keep and o["bytes"]:
            acts[o["name"]] = wsh[o["offset"]:o["offset"] + o["bytes"]]
    out = logits.cpu().numpy()
    hn.close()
    return out, acts, names


@pytest.mark.parametrize("arch,mixed,N", [(18, False, 2), (50, False, 2), (50, True, 2)])
def test_network_with_int32_shortcuts(hawq, arch, mixed, N):
    """Transition blocks in the two-accumulator form: all-8-bit networks run them as one launch each (no transition
    tensor is stored); with 4-bit layers in a transition block the raw accumulators pass through the workspace."""
    bits = wl.draw_bits(arch, 4000 + arch) if mixed else None
    net = wl.make_resnet(arch, seed=1000 + arch, bits=bits, int32_shortcut=True)
    plain = wl.make_resnet(arch, seed=1000 + arch, bits=bits)
    x = wl.make_image_batch(7, N)
    keep = {}
    want = onet.forward(net, x, keep)
    assert not np.array_equal(want, onet.forward(plain, x))     # the option changes the arithmetic
    got, acts, names = _forward_gpu(hawq, net, x, True)
    assert not any(n in keep for n in names if n.endswith(".ds"))
    if not mixed:
        assert not any(n.endswith(".ds") for n in names)          # one launch per transition block
    for name, w in keep.items():
        if name == "fc":
            continue
        wv = np.ascontiguousarray(w).view(np.uint8).ravel()
        assert name in acts and np.array_equal(acts[name], wv), name
    assert np.array_equal(got, want)
    got2, _, _ = _forward_gpu(hawq, net, x, False)
    assert np.array_equal(got2, want)


# shapes the persistent streaming form serves (many pixels; (C, Cs) = (64, 64) or (128, 256); K a multiple of 128)
@pytest.mark.parametrize("shape", [(3, 56, 64, 256, 1, 64, 1), (11, 28, 128, 512, 1, 256, 2), (5, 47, 64, 384, 1, 64, 2)])
def test_streaming_form(hawq, shape):
    from gpu_util import assert_same
    N, H, C, K, R, Cs, ss = shape
    t = _case(sum(shape), N, H, C, K, R, Cs, ss)
    got, want = _run(hawq, t, hawq.U8, 1, 0, 127)
    assert_same(got, want, "streaming dual conv %r" % (shape,))
    assert 0.02 < (want == 0).mean() < 0.9 and (want == 127).mean() < 0.2
    tw = _case(sum(shape), N, H, C, K, R, Cs, ss, wide=True)
    got, want2 = _run(hawq, tw, hawq.U8, 1, 0, 127)
    assert_same(got, want2, "streaming dual conv, wide multipliers %r" % (shape,))
    assert_same(want2, want, "oracle: scaling numerator and shift together changes nothing")
    got, want = _run(hawq, t, hawq.U4, 1, 0, 15)
    assert_same(got, want, "streaming dual conv, packed 4-bit output %r" % (shape,))


@pytest.mark.parametrize("int32_sc", [False, True])
def test_network_batch_that_pairs_transition_and_last_convolution(hawq, int32_sc):
    """ResNet50 at a batch where stages 1 and 2 have enough pixels for the one-launch form of (transition, last convolution).
    With stored shortcuts the pair must give the bits of the two separate launches (the network that keeps its activations
    never pairs them) and of the oracle; wide multipliers on the paired layers take the exact path with the same result."""
    N = 11
    net = wl.make_resnet(50, seed=2024, int32_shortcut=int32_sc)
    x = wl.make_image_batch(5, N)
    want = onet.forward(net, x)
    got, _, names = _forward_gpu(hawq, net, x, False)
    assert np.array_equal(got, want)
    got_keep, _, _ = _forward_gpu(hawq, net, x, True)
    assert np.array_equal(got_keep, want)
    L = {l["name"]: l for l in net["layers"]}
    for name, keys in (("layer1.0.ds", ("b", "c")), ("layer2.0.c3", ("b", "c")), ("layer1.0.c3", ("res_b", "res_c"))):
        if int32_sc and keys[0] == "res_b":
            continue
        l = L[name]
        l[keys[0]] = (l[keys[0]].astype(np.int64) << 15).astype(np.int32)
        l[keys[1]] = (l[keys[1]].astype(np.int32) + 15).astype(np.uint8)
    assert np.array_equal(onet.forward(net, x[:2]), want[:2])
    got, _, _ = _forward_gpu(hawq, net, x, False)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("arch,int32_sc", [(18, True), (50, True), (50, False)])
def test_network_int32_shortcuts_when_the_16_bit_form_does_not_apply(hawq, arch, int32_sc):
    """All-8-bit networks normally run a transition block's two-accumulator launch in the eight-wave form that keeps the
    main branch's rescaled term in 16 bits; the plan allows that only when a bound computed from the weights shows
    the term fits.  A bias of 2^30 on a few channels of each block's last convolution breaks the bound (those outputs
    saturate): the plan must fall back to the form with two full accumulator sets, same bits as the oracle."""
    net = wl.make_resnet(arch, seed=2000 + arch, image_hw=64, int32_shortcut=int32_sc)   # (False: the stored-shortcut pairs)
    for l in net["layers"]:
        if l["name"].endswith(".0.c2" if arch == 18 else ".0.c3"):
            l["bias"] = l["bias"].copy()
            l["bias"][0] = 1 << 30
            l["bias"][5] = -(1 << 30)
    x = wl.make_image_batch(11, 3, image_hw=64)
    want = onet.forward(net, x)
    import torch
    hn = hawq.HawqNet(arch, net["layers"], net["pool_b"], net["pool_c"], image_hw=64)
    ws = torch.empty(hn.workspace_bytes(3), dtype=torch.uint8, device="cuda")
    logits = torch.empty((3, 1000), dtype=torch.int32, device="cuda")
    hn.hawq_forward_resnet(torch.from_numpy(x).cuda(), 3, logits, ws)
    torch.cuda.synchronize()
    hn.close()
    assert np.array_equal(logits.cpu().numpy(), want)
