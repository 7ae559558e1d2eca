"""Layer shapes of the paper's ResNet workloads, as plain data.

ResNet18 uses two 3x3 convolutions per block; ResNet50 uses 1x1 / 3x3 / 1x1
bottlenecks with the stride-2 on the first 1x1 of a transition block (the
original "v1" arrangement -- the only one whose multiply-accumulate total
reproduces the BOPS column of Table 1).  The canonical layer order is

    conv1, then for every stage and block: c1, c2, [c3], [ds], and finally fc

and every consumer of these inputs (oracle, HIP library) walks its own copy of
the topology and checks the shapes it is handed against it.
"""

_STAGE_WIDTH = (64, 128, 256, 512)
_BLOCKS = {18: (2, 2, 2, 2), 50: (3, 4, 6, 3)}


def _out(h, r, stride, pad):
    return (h + 2 * pad - r) // stride + 1


def resnet_layers(arch, image_hw=224, num_classes=1000):
    """List of dicts, one per conv / fc layer, in canonical order.

    Keys: name, kind ('stem' | 'c1' | 'c2' | 'c3' | 'ds' | 'fc'), stage, block,
    C, K, R, S, stride, pad, H, W (input size), P, Q (output size),
    has_residual (the layer's epilogue adds the block's shortcut),
    group (layers that must share a bit width carry the same group name).
    """
    if arch not in _BLOCKS:
        raise ValueError("arch must be 18 or 50")
    bottleneck = arch == 50
    expansion = 4 if bottleneck else 1
    out = []
    h = image_hw
    p = _out(h, 7, 2, 3)
    out.append(dict(name="conv1", kind="stem", stage=0, block=0, C=3, K=64, R=7, S=7,
                    stride=2, pad=3, H=h, W=h, P=p, Q=p, has_residual=False, group="conv1"))
    h = _out(p, 3, 2, 1)  # max pool 3x3 / 2, pad 1
    c_in = 64
    for si, (width, nblocks) in enumerate(zip(_STAGE_WIDTH, _BLOCKS[arch])):
        for bi in range(nblocks):
            stride = 2 if (bi == 0 and si > 0) else 1
            c_out = width * expansion
            need_ds = (stride != 1) or (c_in != c_out)
            pre = "layer%d.%d" % (si + 1, bi)
            h_out = _out(h, 1, stride, 0)
            if bottleneck:
                out.append(dict(name=pre + ".c1", kind="c1", stage=si + 1, block=bi, C=c_in, K=width,
                                R=1, S=1, stride=stride, pad=0, H=h, W=h, P=h_out, Q=h_out,
                                has_residual=False, group=pre + ".in"))
                out.append(dict(name=pre + ".c2", kind="c2", stage=si + 1, block=bi, C=width, K=width,
                                R=3, S=3, stride=1, pad=1, H=h_out, W=h_out, P=h_out, Q=h_out,
                                has_residual=False, group=pre + ".c2"))
                out.append(dict(name=pre + ".c3", kind="c3", stage=si + 1, block=bi, C=width, K=c_out,
                                R=1, S=1, stride=1, pad=0, H=h_out, W=h_out, P=h_out, Q=h_out,
                                has_residual=True, group=pre + ".c3"))
            else:
                out.append(dict(name=pre + ".c1", kind="c1", stage=si + 1, block=bi, C=c_in, K=width,
                                R=3, S=3, stride=stride, pad=1, H=h, W=h, P=h_out, Q=h_out,
                                has_residual=False, group=pre + ".in"))
                out.append(dict(name=pre + ".c2", kind="c2", stage=si + 1, block=bi, C=width, K=c_out,
                                R=3, S=3, stride=1, pad=1, H=h_out, W=h_out, P=h_out, Q=h_out,
                                has_residual=True, group=pre + ".c2"))
            if need_ds:
                out.append(dict(name=pre + ".ds", kind="ds", stage=si + 1, block=bi, C=c_in, K=c_out,
                                R=1, S=1, stride=stride, pad=0, H=h, W=h, P=h_out, Q=h_out,
                                has_residual=False, group=pre + ".in"))
            c_in = c_out
            h = h_out
    out.append(dict(name="fc", kind="fc", stage=5, block=0, C=c_in, K=num_classes, R=1, S=1,
                    stride=1, pad=0, H=1, W=1, P=1, Q=1, has_residual=False, group="fc"))
    return out


def resnet_group_names(arch):
    """Bit-width groups in first-appearance order (conv1 and fc included)."""
    seen = []
    for l in resnet_layers(arch):
        if l["group"] not in seen:
            seen.append(l["group"])
    return seen
