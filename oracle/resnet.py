"""Oracle walk of an integer-only ResNet18 / ResNet50 (test infrastructure only).

The network is the composition of the individually pinned layer routines of
``hawq_oracle.c``, in the order a standard ResNet prescribes:

    conv1 7x7/2 (+ReLU) -> max pool 3x3/2 -> residual blocks -> global average
    pool -> fully connected layer -> INT32 logits

BasicBlock (ResNet18):   c1 3x3/s ReLU -> c2 3x3 + shortcut -> ReLU
Bottleneck (ResNet50):   c1 1x1/s ReLU -> c2 3x3 ReLU -> c3 1x1 + shortcut -> ReLU
with the stride on c1 of the first block of stages 2-4 (the arrangement whose
operation count reproduces Table 1's BOPS).  The shortcut is the block input, or a
1x1/s transition convolution (no ReLU, signed output) when the shape changes.
The residual addition rescales both branches with their own dyadic numbers
(Section 3.3); a block with a transition layer feeds the same stored block input to
both 1x1 convolutions (Figure 2).  A transition layer flagged ``int32_shortcut``
is not stored at all: the block's output is formed from the two INT32 accumulators,
each rescaled by its own dyadic number (the transition layer's (b, c) then map its
accumulator to the block's output scale).

Mixed precision (Section 3.4: weights and activations of a layer share one bit
width): a tensor is stored at the width of the convolution that reads it, the
producer's clamp enforcing the range 0..127 (8-bit) or 0..15 (4-bit); the
transition output is signed 8-bit; conv1, the pooled vector and fc are 8-bit
(Appendix H keeps the first and last layer at 8 bits).

This module has its own copy of the topology; the parameter list it is handed
is checked against it layer by layer.
"""
import numpy as np

from . import (U8, S8, U4, S4, S32, conv2d_int, conv2d_dual_int, gemm_int, avgpool_int, maxpool_int)

_WIDTHS = (64, 128, 256, 512)
_DEPTHS = {18: (2, 2, 2, 2), 50: (3, 4, 6, 3)}
_ACT_HI = {8: 127, 4: 15}


def _act_dt(bits):
    return U8 if bits == 8 else U4


def _w_dt(bits):
    return S8 if bits == 8 else S4


def _conv_out(h, r, s, p):
    return (h + 2 * p - r) // s + 1


class _Cursor:
    def __init__(self, layers):
        self.layers = layers
        self.i = 0

    def peek(self, k=0):
        return self.layers[self.i + k] if self.i + k < len(self.layers) else None

    def take(self, name, C, K, R, stride, pad):
        l = self.layers[self.i]
        self.i += 1
        got = (l["name"], l["C"], l["K"], l["R"], l["S"], l["stride"], l["pad"])
        want = (name, C, K, R, R, stride, pad)
        if got != want:
            raise ValueError("layer %d: expected %r, got %r" % (self.i - 1, want, got))
        return l


def topology(arch, image_hw=224, num_classes=1000):
    """The oracle's own layer list: (name, C, K, R, stride, pad, H_in, P_out)."""
    out = [("conv1", 3, 64, 7, 2, 3, image_hw, _conv_out(image_hw, 7, 2, 3))]
    h = _conv_out(out[0][7], 3, 2, 1)
    cin = 64
    for si, (wd, nb) in enumerate(zip(_WIDTHS, _DEPTHS[arch])):
        for bi in range(nb):
            s = 2 if (si > 0 and bi == 0) else 1
            cout = wd * (4 if arch == 50 else 1)
            ho = _conv_out(h, 1, s, 0)
            pre = "layer%d.%d" % (si + 1, bi)
            if arch == 50:
                out.append((pre + ".c1", cin, wd, 1, s, 0, h, ho))
                out.append((pre + ".c2", wd, wd, 3, 1, 1, ho, ho))
                out.append((pre + ".c3", wd, cout, 1, 1, 0, ho, ho))
            else:
                out.append((pre + ".c1", cin, wd, 3, s, 1, h, ho))
                out.append((pre + ".c2", wd, cout, 3, 1, 1, ho, ho))
            if s != 1 or cin != cout:
                out.append((pre + ".ds", cin, cout, 1, s, 0, h, ho))
            cin, h = cout, ho
    out.append(("fc", cin, num_classes, 1, 1, 0, 1, 1))
    return out


def forward(net, x, keep=None):
    """INT32 logits [N, classes] for a uint8 NHWC image batch.

    ``net`` is the parameter dict made by ``workloads.make_resnet``.  If ``keep``
    is a dict, every stored tensor is recorded in it under its producer's name
    ('conv1', 'pool', 'layer1.0.c1', ..., 'avgpool', 'fc').
    """
    arch = net["arch"]
    x = np.ascontiguousarray(x, dtype=np.uint8)
    N, H, W, C0 = x.shape
    assert C0 == 3 and H == W == net["image_hw"]
    cur = _Cursor(net["layers"])

    def note(name, t):
        if keep is not None:
            keep[name] = t

    def run_conv(l, inp, n_h, in_dt, out_bits, relu, signed_out=False, res=None, res_dt=U8):
        bits = l["bits"]
        if signed_out:
            y_dt, lo, hi = S8, -128, 127
        else:
            y_dt, lo, hi = _act_dt(out_bits), 0, _ACT_HI[out_bits]
        return conv2d_int(inp, l["w"], l["bias"], l["b"], l["c"], N=N, H=n_h, W=n_h, C=l["C"], K=l["K"],
                          R=l["R"], S=l["S"], stride=l["stride"], pad=l["pad"],
                          x_dt=in_dt, w_dt=_w_dt(bits), y_dt=y_dt, relu=relu, y_lo=lo, y_hi=hi,
                          residual=res, res_b=l["res_b"] if res is not None else None,
                          res_c=l["res_c"] if res is not None else None, res_dt=res_dt)

    # bit width of the conv that will read the next stored tensor
    def next_reader_bits(k=0):
        j = k
        while cur.peek(j) is not None and cur.peek(j)["name"].endswith(".ds"):
            j += 1
        nxt = cur.peek(j)
        return 8 if (nxt is None or nxt["name"] == "fc") else nxt["bits"]

    l = cur.take("conv1", 3, 64, 7, 2, 3)
    assert l["bits"] == 8
    stage_in_bits = next_reader_bits()
    # conv1 output stays in an 8-bit container (the pool reads it), already clamped to the range
    # of the tensor the pool will store
    t = conv2d_int(x, l["w"], l["bias"], l["b"], l["c"], N=N, H=H, W=W, C=3, K=64, R=7, S=7, stride=2, pad=3,
                   x_dt=U8, w_dt=S8, y_dt=U8, relu=1, y_lo=0, y_hi=_ACT_HI[stage_in_bits])
    note("conv1", t)
    h = _conv_out(H, 7, 2, 3)
    t = maxpool_int(t, N=N, H=h, W=h, C=64, x_dt=U8, y_dt=_act_dt(stage_in_bits), y_lo=0, y_hi=_ACT_HI[stage_in_bits])
    note("pool", t)
    h = _conv_out(h, 3, 2, 1)
    cin, in_bits = 64, stage_in_bits

    for si, (wd, nb) in enumerate(zip(_WIDTHS, _DEPTHS[arch])):
        for bi in range(nb):
            s = 2 if (si > 0 and bi == 0) else 1
            cout = wd * (4 if arch == 50 else 1)
            ho = _conv_out(h, 1, s, 0)
            pre = "layer%d.%d" % (si + 1, bi)
            block_in, block_in_dt = t, _act_dt(in_bits)
            has_ds = s != 1 or cin != cout
            if arch == 50:
                l1 = cur.take(pre + ".c1", cin, wd, 1, s, 0)
                l2 = cur.take(pre + ".c2", wd, wd, 3, 1, 1)
                l3 = cur.take(pre + ".c3", wd, cout, 1, 1, 0)
                mids = [l1, l2]
                last = l3
            else:
                l1 = cur.take(pre + ".c1", cin, wd, 3, s, 1)
                l2 = cur.take(pre + ".c2", wd, cout, 3, 1, 1)
                mids = [l1]
                last = l2
            lds = cur.take(pre + ".ds", cin, cout, 1, s, 0) if has_ds else None
            assert l1["bits"] == in_bits, "block input is stored at c1's width"
            if lds is not None:
                assert lds["bits"] == l1["bits"], "transition conv shares c1's width"
            out_bits = next_reader_bits()
            # main branch
            u, u_dt, u_h = block_in, block_in_dt, h
            chain = mids + [last]
            for j, lj in enumerate(mids):
                ob = chain[j + 1]["bits"]
                u = run_conv(lj, u, u_h, u_dt, ob, relu=1)
                note(lj["name"], u)
                u_dt, u_h = _act_dt(ob), _conv_out(u_h, lj["R"], lj["stride"], lj["pad"])
            # shortcut
            if lds is not None and lds.get("int32_shortcut"):
                t = conv2d_dual_int(u, last["w"], last["bias"], last["b"], last["c"],
                                    block_in, lds["w"], lds["bias"], lds["b"], lds["c"],
                                    N=N, K=cout, H=u_h, W=u_h, C=last["C"], R=last["R"], S=last["S"], stride=last["stride"],
                                    pad=last["pad"], x_dt=u_dt, w_dt=_w_dt(last["bits"]),
                                    Hs=h, Ws=h, Cs=cin, Rs=1, Ss=1, stride_s=s, pad_s=0, xs_dt=block_in_dt, ws_dt=_w_dt(lds["bits"]),
                                    y_dt=_act_dt(out_bits), relu=1, y_lo=0, y_hi=_ACT_HI[out_bits])
                note(last["name"], t)
                cin, h, in_bits = cout, ho, out_bits
                continue
            if lds is not None:
                sc = run_conv(lds, block_in, h, block_in_dt, 8, relu=0, signed_out=True)
                note(lds["name"], sc)
                sc_dt = S8
            else:
                sc, sc_dt = block_in, block_in_dt
            t = run_conv(last, u, u_h, u_dt, out_bits, relu=1, res=sc, res_dt=sc_dt)
            note(last["name"], t)
            cin, h, in_bits = cout, ho, out_bits

    assert in_bits == 8
    t = avgpool_int(t, net["pool_b"], net["pool_c"], N=N, H=h, W=h, C=cin, x_dt=U8, y_dt=U8, y_lo=0, y_hi=127)
    note("avgpool", t)
    l = cur.take("fc", cin, net["num_classes"], 1, 1, 0)
    assert l["bits"] == 8
    logits = gemm_int(t, l["w"], l["bias"], None, None, M=N, N=l["K"], K=cin, x_dt=U8, w_dt=S8, y_dt=S32)
    note("fc", logits)
    assert cur.i == len(net["layers"])
    return logits
