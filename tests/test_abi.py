"""CPU-side checks of the C interface: the library loads without a GPU, exports every symbol the header
declares, and rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "hawq.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2011_10680_amd as hawq
    from paper_2011_10680_amd import build
    if build.is_stale():
        build.build()
    return hawq.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hawq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"hawq_conv2d_int", "hawq_gemm_int", "hawq_residual_add_dyadic", "hawq_avgpool_int",
            "hawq_forward_resnet"} <= set(names)
    for n in names:
        assert hasattr(lib, n), "libhawq.so does not export " + n


def test_topology_queries_match_the_paper_workloads(lib):
    import paper_2011_10680_amd as hawq
    import workloads as wl
    for arch in (18, 50):
        shapes = wl.resnet_layers(arch)
        assert hawq.hawq_net_num_layers(arch) == len(shapes)
        macs = 0
        for i, s in enumerate(shapes):
            info = hawq.hawq_net_layer_info(arch, 224, 1000, i)
            for k in ("name", "C", "K", "R", "S", "stride", "pad", "H", "W", "P", "Q"):
                assert info[k] == s[k], (arch, i, k)
            assert bool(info["has_residual"]) == s["has_residual"]
            assert bool(info["is_ds"]) == (s["kind"] == "ds")
            macs += info["P"] * info["Q"] * info["K"] * info["R"] * info["S"] * info["C"]
        # Table 1 BOPS at W8A8: 116 G (ResNet18), 247 G (ResNet50)
        assert round(macs * 64 / 1e9) == {18: 116, 50: 247}[arch]
    assert hawq.hawq_net_num_layers(34) == 0


def _desc(**kw):
    import paper_2011_10680_amd as hawq
    d = dict(N=1, H=8, W=8, C=64, K=64, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, x_dtype=hawq.U8,
             w_dtype=hawq.S8, y_dtype=hawq.U8, res_dtype=hawq.U8, relu=1, y_lo=0, y_hi=127, x_hi=127)
    d.update(kw)
    return hawq.ConvDesc(**d)


def test_conv_argument_validation_on_host(lib):
    """Pointers are never dereferenced on the host, so small fake non-null addresses are enough to reach
    the later checks; every case must fail before a launch."""
    import paper_2011_10680_amd as hawq
    P = ctypes.c_void_p(4096)
    call = lambda d, x=P, w=P, bias=P, b=P, c=P, res=None, rb=None, rc=None, y=P: lib.hawq_conv2d_int(
        ctypes.byref(d), x, w, bias, b, c, res, rb, rc, y, None)
    assert call(_desc(), x=None) == 1                                  # HAWQ_ERR_NULL
    assert call(_desc(), b=None) == 1                                  # b without c
    assert call(_desc(), res=P) == 1                                   # residual without its multipliers
    assert call(_desc(H=0)) == 2                                       # HAWQ_ERR_SHAPE
    assert call(_desc(R=11, S=11, pad_h=0, pad_w=0)) == 2              # window larger than the image
    assert call(_desc(x_dtype=hawq.U4, w_dtype=hawq.S4, C=63)) == 2    # odd packed channel count
    assert call(_desc(y_dtype=hawq.U4, y_hi=15, K=63)) == 2
    assert call(_desc(w_dtype=hawq.S4)) == 3                           # HAWQ_ERR_DTYPE: widths differ
    assert call(_desc(x_dtype=hawq.S32)) == 3
    assert call(_desc(y_dtype=hawq.U8), b=None, c=None) == 3           # raw output must be INT32
    assert call(_desc(y_hi=300)) == 4                                  # HAWQ_ERR_RANGE
    assert call(_desc(y_lo=5, y_hi=4)) == 4
    assert call(_desc(x_hi=300)) == 4
    assert call(_desc(C=65536 * 2, R=1, S=1, pad_h=0, pad_w=0, x_hi=255)) == 5   # HAWQ_ERR_OVERFLOW: 2^17*255*128 >= 2^31
    assert call(_desc(N=1 << 20, H=64, W=64)) == 6                     # HAWQ_ERR_UNSUPPORTED: tensor >= 2 GiB
    assert call(_desc(N=0)) == 0                                       # empty batch: nothing to do
    assert lib.hawq_status_string(5).decode().lower().startswith("int32")


def test_blocked_weight_copy_size_and_validation_on_host(lib):
    """Size of the blocked copy (whole 64-channel blocks of 64-byte pieces) and the cases with none; the copy call fails
    before any launch on null pointers, layers without a blocked form and misaligned pointers."""
    import paper_2011_10680_amd as hawq
    size = lambda **kw: lib.hawq_conv_blocked_weights_bytes(ctypes.byref(_desc(**kw)))
    assert size(C=64, K=100) == 128 * 9 * 64
    assert size(C=256, K=64, R=1, S=1, pad_h=0, pad_w=0) == 64 * 256
    assert size(C=96) == 0 and size(C=64, x_dtype=hawq.U4, w_dtype=hawq.S4) == 0
    assert size(C=128, K=65, x_dtype=hawq.U4, w_dtype=hawq.S4) == 128 * 9 * 64
    assert lib.hawq_conv_blocked_weights_bytes(None) == 0
    P = ctypes.c_void_p(4096)
    d = _desc()
    assert lib.hawq_conv_block_weights(ctypes.byref(d), None, P, None) == 1
    assert lib.hawq_conv_block_weights(ctypes.byref(d), P, None, None) == 1
    assert lib.hawq_conv_block_weights(None, P, P, None) == 1
    assert lib.hawq_conv_block_weights(ctypes.byref(_desc(C=96)), P, P, None) == 6
    assert lib.hawq_conv_block_weights(ctypes.byref(d), ctypes.c_void_p(4100), P, None) == 6


def test_fragment_weight_copy_and_fused_tail_validate_on_host(lib):
    """Size of the fragment-ordered copy (whole groups of 32 channels, bytes also for 4-bit weights) and the cases with
    none; the copy call and the fused bottleneck tail fail before any launch on null pointers, misaligned pointers and
    layer pairs the kernel does not take."""
    import paper_2011_10680_amd as hawq
    size = lambda **kw: lib.hawq_conv_fragment_weights_bytes(ctypes.byref(_desc(**kw)))
    assert size(C=128, K=128) == 128 * 9 * 128
    assert size(C=256, K=100, R=1, S=1, pad_h=0, pad_w=0) == 128 * 256
    assert size(C=128, K=33, x_dtype=hawq.U4, w_dtype=hawq.S4) == 64 * 9 * 128     # expanded to one byte per weight
    assert size(C=96) == 0 and size(C=128, w_dtype=hawq.U8) == 0
    assert lib.hawq_conv_fragment_weights_bytes(None) == 0
    P = ctypes.c_void_p(4096)
    d = _desc(C=128, K=128)
    assert lib.hawq_conv_fragment_weights(ctypes.byref(d), None, P, None) == 1
    assert lib.hawq_conv_fragment_weights(ctypes.byref(d), P, None, None) == 1
    assert lib.hawq_conv_fragment_weights(None, P, P, None) == 1
    assert lib.hawq_conv_fragment_weights(ctypes.byref(_desc(C=96)), P, P, None) == 6
    assert lib.hawq_conv_fragment_weights(ctypes.byref(d), P, ctypes.c_void_p(4104), None) == 6
    d2 = _desc(N=2, H=14, W=14, C=256, K=256)
    d3 = _desc(N=2, H=14, W=14, C=256, K=1024, R=1, S=1, pad_h=0, pad_w=0)
    tail = lambda a, b, x=P, w2=P, b2=P, w3=P, b3=P, res=P, y=P: lib.hawq_bottleneck_tail_int(
        ctypes.byref(a), x, w2, P, b2, P, ctypes.byref(b), w3, P, b3, P, res, P, P, y, None)
    assert tail(d2, d3, w2=None) == 1 and tail(d2, d3, w3=None) == 1 and tail(d2, d3, res=None) == 1 and tail(d2, d3, b3=None) == 1
    assert tail(d2, d3, x=None) == 1 and tail(d2, d3, y=None) == 1
    assert tail(_desc(N=2, H=14, W=14, C=256, K=256, y_lo=5, y_hi=3), d3) == 4
    assert tail(d2, _desc(N=2, H=14, W=14, C=256, K=1024, R=1, S=1, pad_h=0, pad_w=0, y_dtype=9)) == 3
    for bad2, bad3 in ((_desc(N=2, H=14, W=14, C=256, K=256, stride_h=2, stride_w=2), d3),          # strided 3x3
                       (_desc(N=2, H=14, W=14, C=192, K=192), _desc(N=2, H=14, W=14, C=192, K=768, R=1, S=1, pad_h=0, pad_w=0)),
                       (d2, _desc(N=2, H=14, W=14, C=128, K=1024, R=1, S=1, pad_h=0, pad_w=0)),         # channel counts do not chain
                       (d2, _desc(N=2, H=7, W=7, C=256, K=1024, R=1, S=1, pad_h=0, pad_w=0)),           # other image
                       (d2, _desc(N=2, H=14, W=14, C=256, K=1024, R=1, S=1, pad_h=0, pad_w=0, y_dtype=hawq.U4, y_hi=15)),
                       (_desc(N=2, H=14, W=14, C=256, K=256, x_dtype=hawq.U4, w_dtype=hawq.S4, x_hi=0), d3)):
        assert tail(bad2, bad3) == 6
    assert tail(d2, d3, w2=ctypes.c_void_p(4100)) == 6
    assert lib.hawq_noalloc_workspace_limit() == 64 << 20
    assert lib.hawq_forward_resnet_noalloc(None, P, 1, P, None) == 1


def test_dual_conv_argument_validation_on_host(lib):
    import paper_2011_10680_amd as hawq
    P = ctypes.c_void_p(4096)
    main = dict(N=2, H=8, W=8, C=64, K=128, R=3, S=3)
    short = dict(N=2, H=15, W=15, C=128, K=128, R=1, S=1, stride_h=2, stride_w=2, pad_h=0, pad_w=0)

    def call(dm, dsc, **ptrs):
        a = dict(x=P, w=P, bias=P, b=P, c=P, xs=P, ws=P, bias_s=P, b_s=P, c_s=P, y=P)
        a.update(ptrs)
        return lib.hawq_conv2d_dual_int(ctypes.byref(dm), a["x"], a["w"], a["bias"], a["b"], a["c"], ctypes.byref(dsc), a["xs"],
                                        a["ws"], a["bias_s"], a["b_s"], a["c_s"], a["y"], None)
    assert call(_desc(**main), _desc(**short), xs=None) == 1                      # HAWQ_ERR_NULL
    assert call(_desc(**main), _desc(**short), b_s=None) == 1                     # both branches are requantised
    assert call(_desc(**main), _desc(**dict(short, H=17, W=17))) == 2             # output sizes differ -> HAWQ_ERR_SHAPE
    assert call(_desc(**main), _desc(**dict(short, K=64))) == 2
    assert call(_desc(**main), _desc(**dict(short, R=3, S=3, H=17, W=17))) == 2   # shortcut must be 1x1
    assert call(_desc(**main), _desc(**dict(short, w_dtype=hawq.S4))) == 3        # operand widths of one branch must agree
    assert call(_desc(**dict(main, y_dtype=hawq.S32, y_lo=-5, y_hi=5)), _desc(**short)) == 3
    assert call(_desc(**dict(main, y_hi=300)), _desc(**short)) == 4
    assert call(_desc(**main), _desc(**dict(short, C=65536 * 2, x_hi=255))) == 5   # the shortcut's own overflow bound
    assert call(_desc(**dict(main, N=0)), _desc(**dict(short, N=0))) == 0


def test_other_entry_points_validate_on_host(lib):
    P = ctypes.c_void_p(4096)
    assert lib.hawq_gemm_int(4, 0, 64, 0, 1, 4, P, P, P, None, None, 0, 0, 0, P, None) == 2
    assert lib.hawq_gemm_int(4, 8, 64, 0, 1, 0, P, P, P, None, None, 0, 0, 127, P, None) == 3
    assert lib.hawq_gemm_int(0, 8, 64, 0, 1, 4, P, P, P, None, None, 0, 0, 0, P, None) == 0
    assert lib.hawq_residual_add_dyadic(10, 8, 4, 0, 0, P, P, P, None, P, P, 1, 0, 127, P, None) == 1
    assert lib.hawq_residual_add_dyadic(10, 7, 2, 0, 0, P, P, P, P, P, P, 1, 0, 127, P, None) == 2
    assert lib.hawq_residual_add_dyadic(10, 8, 4, 0, 0, P, P, P, P, P, P, 1, 0, 256, P, None) == 4
    assert lib.hawq_avgpool_int(1, 7, 7, 64, 4, 0, P, P, P, 0, 127, P, None) == 3
    assert lib.hawq_avgpool_int(1, 7, 7, 64, 0, 0, P, None, P, 0, 127, P, None) == 1
    assert lib.hawq_maxpool_int(1, 8, 8, 63, 0, 2, P, 0, 15, P, None) == 2
    assert lib.hawq_forward_resnet(None, P, 1, P, P, 0, None) == 1
    assert lib.hawq_probe_mfma_peak(100, None) == 1
    t = ctypes.c_double(0)
    assert lib.hawq_probe_mfma_peak(0, ctypes.byref(t)) == 4 and lib.hawq_probe_mfma_peak(2000000, ctypes.byref(t)) == 4
    assert lib.hawq_net_split_first(None, 128) == 0
    pool = lambda *a: lib.hawq_pool2d_sum_int(*a, None)
    assert pool(1, 8, 8, 4, 3, 3, 1, 1, 1, 1, 4, 4, None, None, None, 0, 0, P) == 1
    assert pool(1, 8, 8, 4, 3, 3, 1, 1, 1, 1, 4, 4, P, P, None, 0, 0, P) == 1          # b without c
    assert pool(1, 8, 8, 4, 3, 3, 0, 1, 1, 1, 4, 4, P, None, None, 0, 0, P) == 2        # stride 0
    assert pool(1, 2, 2, 4, 5, 5, 1, 1, 1, 1, 4, 4, P, None, None, 0, 0, P) == 2        # window larger than the padded image
    assert pool(1, 8, 8, 4, 3, 3, 1, 1, 1, 1, 4, 0, P, None, None, 0, 127, P) == 3      # raw sums must be INT32
    assert pool(1, 8, 8, 4, 3, 3, 1, 1, 1, 1, 4, 0, P, P, P, 0, 300, P) == 4
    assert pool(1, 8, 8, 3, 3, 3, 1, 1, 1, 1, 2, 0, P, P, P, 0, 127, P) == 2            # odd packed channel count
    assert pool(0, 8, 8, 4, 3, 3, 1, 1, 1, 1, 4, 4, P, None, None, 0, 0, P) == 0
    from paper_2011_10680_amd.binding import ConcatBranch
    br = (ConcatBranch * 2)()
    for i, (K, dt) in enumerate(((6, 4), (4, 0))):
        br[i].q, br[i].b, br[i].c, br[i].K, br[i].dtype = 4096, 4096, 4096, K, dt
    assert lib.hawq_concat_dyadic(10, 2, None, 0, 0, 127, P, None) == 1
    assert lib.hawq_concat_dyadic(10, 0, br, 0, 0, 127, P, None) == 2
    assert lib.hawq_concat_dyadic(0, 2, br, 0, 0, 127, P, None) == 0                     # no pixels: nothing to do
    assert lib.hawq_concat_dyadic(10, 2, br, 0, 0, 300, P, None) == 4
    br[1].K = 3
    assert lib.hawq_concat_dyadic(10, 2, br, 2, 0, 15, P, None) == 2                     # odd branch width, packed output
    br[1].K = 4; br[1].dtype = 9
    assert lib.hawq_concat_dyadic(10, 2, br, 0, 0, 127, P, None) == 3
    br[1].dtype = 0; br[0].b = None
    assert lib.hawq_concat_dyadic(10, 2, br, 0, 0, 127, P, None) == 1


def test_net_create_rejects_bad_parameters_before_touching_the_gpu(lib):
    import numpy as np
    import paper_2011_10680_amd as hawq
    import workloads as wl
    net = wl.make_resnet(18, seed=1, image_hw=64, num_classes=10)
    bad = [dict(l) for l in net["layers"]]
    bad[3]["c"] = bad[3]["c"].copy(); bad[3]["c"][0] = 0          # shift of 0 is outside 1..62
    with pytest.raises(hawq.HawqError) as e:
        hawq.HawqNet(18, bad, net["pool_b"], net["pool_c"], image_hw=64, num_classes=10)
    assert e.value.status == 4
    bad = [dict(l) for l in net["layers"]]
    bad[0]["bits"] = 4                                            # first layer must stay 8-bit
    with pytest.raises(hawq.HawqError) as e:
        hawq.HawqNet(18, bad, net["pool_b"], net["pool_c"], image_hw=64, num_classes=10)
    assert e.value.status == 3
    arr_flag = [dict(l) for l in net["layers"]]
    idx = {l["name"]: i for i, l in enumerate(arr_flag)}
    arr_flag[idx["layer2.0.ds"]]["int32_shortcut"] = True
    arr_flag[idx["layer2.0.c2"]]["res_b"] = arr_flag[idx["layer2.0.c2"]]["res_c"] = None   # unused in that form: may be absent ...
    arr_flag[idx["layer2.1.c2"]]["res_b"] = None                  # ... but not on a block with an identity shortcut
    with pytest.raises(hawq.HawqError) as e:
        hawq.HawqNet(18, arr_flag, net["pool_b"], net["pool_c"], image_hw=64, num_classes=10)
    assert e.value.status == 1
    with pytest.raises(hawq.HawqError) as e:                      # wrong layer count
        hawq.HawqNet(18, net["layers"][:-1], net["pool_b"], net["pool_c"], image_hw=64, num_classes=10)
    assert e.value.status == 2
