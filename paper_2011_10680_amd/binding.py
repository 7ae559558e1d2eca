"""ctypes binding with the same names as the C entry points.  Argument marshalling only.

Tensors are ``torch`` CUDA (HIP) tensors; the binding passes ``data_ptr()`` and the current
stream handle.  The library is loaded from ``libhawq.so`` next to this file; if it is missing
the import of any entry point fails loudly (there is no fallback path)."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhawq.so")

U8, S8, U4, S4, S32 = 0, 1, 2, 3, 4
_STATUS_NAMES = {0: "HAWQ_OK", 1: "HAWQ_ERR_NULL", 2: "HAWQ_ERR_SHAPE", 3: "HAWQ_ERR_DTYPE", 4: "HAWQ_ERR_RANGE",
                 5: "HAWQ_ERR_OVERFLOW", 6: "HAWQ_ERR_UNSUPPORTED", 7: "HAWQ_ERR_DEVICE", 8: "HAWQ_ERR_WORKSPACE"}


class HawqError(RuntimeError):
    def __init__(self, status, what):
        super().__init__("%s: %s (%s)" % (what, _STATUS_NAMES.get(status, status), status_string(status)))
        self.status = status


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w",
                 "x_dtype", "w_dtype", "y_dtype", "res_dtype", "relu", "y_lo", "y_hi", "x_hi")] + [("w_blocked", ctypes.c_void_p), ("w_fragments", ctypes.c_void_p)]


class LayerParams(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("bias", ctypes.c_void_p), ("b", ctypes.c_void_p), ("c", ctypes.c_void_p),
                ("res_b", ctypes.c_void_p), ("res_c", ctypes.c_void_p), ("bits", ctypes.c_int32), ("flags", ctypes.c_int32)]


LAYER_INT32_SHORTCUT = 1


class ConcatBranch(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("b", ctypes.c_void_p), ("c", ctypes.c_void_p), ("K", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class LayerInfo(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 24)] + [(n, ctypes.c_int32) for n in
                ("C", "K", "R", "S", "stride", "pad", "H", "W", "P", "Q", "has_residual", "is_ds")]


_lib = None


def load_library():
    """Load libhawq.so (built by ``paper_2011_10680_amd.build``); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libhawq.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback for the HIP path)")
    lib = ctypes.CDLL(_LIB_PATH)
    i32, i64, vp, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    lib.hawq_conv2d_int.restype = ctypes.c_int
    lib.hawq_conv2d_int.argtypes = [ctypes.POINTER(ConvDesc)] + [vp] * 10
    lib.hawq_conv2d_dual_int.restype = ctypes.c_int
    lib.hawq_conv2d_dual_int.argtypes = [ctypes.POINTER(ConvDesc)] + [vp] * 5 + [ctypes.POINTER(ConvDesc)] + [vp] * 7
    lib.hawq_gemm_int.restype = ctypes.c_int
    lib.hawq_gemm_int.argtypes = [i32] * 6 + [vp] * 5 + [i32] * 3 + [vp, vp]
    lib.hawq_residual_add_dyadic.restype = ctypes.c_int
    lib.hawq_residual_add_dyadic.argtypes = [i64, i32, i32, i32, i32] + [vp] * 6 + [i32] * 3 + [vp, vp]
    lib.hawq_avgpool_int.restype = ctypes.c_int
    lib.hawq_avgpool_int.argtypes = [i32] * 6 + [vp] * 3 + [i32, i32, vp, vp]
    lib.hawq_maxpool_int.restype = ctypes.c_int
    lib.hawq_maxpool_int.argtypes = [i32] * 6 + [vp, i32, i32, vp, vp]
    lib.hawq_pool2d_sum_int.restype = ctypes.c_int
    lib.hawq_pool2d_sum_int.argtypes = [i32] * 12 + [vp] * 3 + [i32, i32, vp, vp]
    lib.hawq_concat_dyadic.restype = ctypes.c_int
    lib.hawq_concat_dyadic.argtypes = [i64, i32, ctypes.POINTER(ConcatBranch), i32, i32, i32, vp, vp]
    lib.hawq_net_num_layers.restype = i32
    lib.hawq_net_num_layers.argtypes = [i32]
    lib.hawq_net_layer_info.restype = ctypes.c_int
    lib.hawq_net_layer_info.argtypes = [i32, i32, i32, i32, ctypes.POINTER(LayerInfo)]
    lib.hawq_net_create.restype = ctypes.c_int
    lib.hawq_net_create.argtypes = [i32, i32, i32, ctypes.POINTER(LayerParams), i32, vp, vp, i32, ctypes.POINTER(vp)]
    lib.hawq_net_destroy.restype = None
    lib.hawq_net_destroy.argtypes = [vp]
    lib.hawq_net_workspace_bytes.restype = sz
    lib.hawq_net_workspace_bytes.argtypes = [vp, i32]
    lib.hawq_net_num_steps.restype = i32
    lib.hawq_net_num_steps.argtypes = [vp]
    lib.hawq_net_step_output.restype = ctypes.c_int
    lib.hawq_net_step_output.argtypes = [vp, i32, i32, ctypes.c_char_p, ctypes.POINTER(sz), ctypes.POINTER(sz),
                                         ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.hawq_net_step_cost.restype = ctypes.c_int
    lib.hawq_net_step_cost.argtypes = [vp, i32, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.hawq_forward_resnet.restype = ctypes.c_int
    lib.hawq_forward_resnet.argtypes = [vp, vp, i32, vp, vp, sz, vp]
    lib.hawq_forward_resnet_noalloc.restype = ctypes.c_int
    lib.hawq_forward_resnet_noalloc.argtypes = [vp, vp, i32, vp, vp]
    lib.hawq_noalloc_workspace_limit.restype = sz
    lib.hawq_noalloc_workspace_limit.argtypes = []
    lib.hawq_forward_resnet_timed.restype = ctypes.c_int
    lib.hawq_forward_resnet_timed.argtypes = [vp, vp, i32, vp, vp, sz, vp, ctypes.POINTER(ctypes.c_float)]
    lib.hawq_tune_set_tile.restype = None
    lib.hawq_tune_set_tile.argtypes = [i32]
    lib.hawq_net_split_first.restype = i32
    lib.hawq_net_split_first.argtypes = [vp, i32]
    lib.hawq_conv_blocked_weights_bytes.restype = ctypes.c_size_t
    lib.hawq_conv_blocked_weights_bytes.argtypes = [ctypes.POINTER(ConvDesc)]
    lib.hawq_conv_block_weights.restype = ctypes.c_int
    lib.hawq_conv_block_weights.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp]
    lib.hawq_conv_fragment_weights_bytes.restype = ctypes.c_size_t
    lib.hawq_conv_fragment_weights_bytes.argtypes = [ctypes.POINTER(ConvDesc)]
    lib.hawq_conv_fragment_weights.restype = ctypes.c_int
    lib.hawq_conv_fragment_weights.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp]
    lib.hawq_bottleneck_tail_int.restype = ctypes.c_int
    lib.hawq_bottleneck_tail_int.argtypes = [ctypes.POINTER(ConvDesc)] + [vp] * 5 + [ctypes.POINTER(ConvDesc)] + [vp] * 9
    lib.hawq_probe_mfma_peak.restype = ctypes.c_int
    lib.hawq_probe_mfma_peak.argtypes = [i32, ctypes.POINTER(ctypes.c_double)]
    lib.hawq_tune_set_split.restype = None
    lib.hawq_tune_set_split.argtypes = [i32]
    lib.hawq_tune_set_fusion.restype = None
    lib.hawq_tune_set_fusion.argtypes = [i32]
    lib.hawq_status_string.restype = ctypes.c_char_p
    lib.hawq_status_string.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def status_string(status):
    try:
        return load_library().hawq_status_string(int(status)).decode()
    except Exception:  # library missing: still give a usable message
        return "?"


def _check(st, what):
    if st != 0:
        raise HawqError(st, what)


def _p(t):
    """Device pointer of a torch tensor (or None)."""
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(stream)
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def hawq_conv2d_int(desc, x, w, bias, b, c, residual, res_b, res_c, y, stream=None):
    _check(load_library().hawq_conv2d_int(ctypes.byref(desc), _p(x), _p(w), _p(bias), _p(b), _p(c), _p(residual),
                                           _p(res_b), _p(res_c), _p(y), _stream(stream)), "hawq_conv2d_int")


def hawq_conv2d_dual_int(desc, x, w, bias, b, c, desc_s, xs, ws, bias_s, b_s, c_s, y, stream=None):
    _check(load_library().hawq_conv2d_dual_int(ctypes.byref(desc), _p(x), _p(w), _p(bias), _p(b), _p(c), ctypes.byref(desc_s),
                                                _p(xs), _p(ws), _p(bias_s), _p(b_s), _p(c_s), _p(y), _stream(stream)),
           "hawq_conv2d_dual_int")


def hawq_gemm_int(M, N, Kdim, x_dt, w_dt, y_dt, x, w, bias, b, c, relu, y_lo, y_hi, y, stream=None):
    _check(load_library().hawq_gemm_int(M, N, Kdim, x_dt, w_dt, y_dt, _p(x), _p(w), _p(bias), _p(b), _p(c), relu, y_lo,
                                         y_hi, _p(y), _stream(stream)), "hawq_gemm_int")


def hawq_residual_add_dyadic(n_pixels, K, m_dt, r_dt, y_dt, m, m_b, m_c, r, r_b, r_c, relu, y_lo, y_hi, y, stream=None):
    _check(load_library().hawq_residual_add_dyadic(n_pixels, K, m_dt, r_dt, y_dt, _p(m), _p(m_b), _p(m_c), _p(r), _p(r_b),
                                                    _p(r_c), relu, y_lo, y_hi, _p(y), _stream(stream)),
           "hawq_residual_add_dyadic")


def hawq_avgpool_int(N, H, W, C, x_dt, y_dt, x, b, c, y_lo, y_hi, y, stream=None):
    _check(load_library().hawq_avgpool_int(N, H, W, C, x_dt, y_dt, _p(x), _p(b), _p(c), y_lo, y_hi, _p(y), _stream(stream)),
           "hawq_avgpool_int")


def hawq_maxpool_int(N, H, W, C, x_dt, y_dt, x, y_lo, y_hi, y, stream=None):
    _check(load_library().hawq_maxpool_int(N, H, W, C, x_dt, y_dt, _p(x), y_lo, y_hi, _p(y), _stream(stream)),
           "hawq_maxpool_int")


def hawq_pool2d_sum_int(N, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w, x_dt, y_dt, x, b, c, y_lo, y_hi, y, stream=None):
    _check(load_library().hawq_pool2d_sum_int(N, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w, x_dt, y_dt, _p(x), _p(b), _p(c),
                                               y_lo, y_hi, _p(y), _stream(stream)), "hawq_pool2d_sum_int")


def hawq_concat_dyadic(n_pixels, branches, y_dt, y_lo, y_hi, y, stream=None):
    """branches: list of (q, dtype, b, c) device tensors; K is taken from b."""
    arr = (ConcatBranch * len(branches))()
    for i, (q, dt, b, c) in enumerate(branches):
        arr[i].q, arr[i].b, arr[i].c = q.data_ptr(), b.data_ptr(), c.data_ptr()
        arr[i].K, arr[i].dtype = b.numel(), dt
    _check(load_library().hawq_concat_dyadic(n_pixels, len(branches), arr, y_dt, y_lo, y_hi, _p(y), _stream(stream)),
           "hawq_concat_dyadic")


def hawq_tune_set_tile(tile):
    load_library().hawq_tune_set_tile(int(tile))


def hawq_conv_blocked_weights_bytes(desc):
    return int(load_library().hawq_conv_blocked_weights_bytes(ctypes.byref(desc)))


def hawq_conv_block_weights(desc, w, w_blocked, stream=None):
    _check(load_library().hawq_conv_block_weights(ctypes.byref(desc), _p(w), _p(w_blocked), _stream(stream)),
           "hawq_conv_block_weights")


def hawq_conv_fragment_weights_bytes(desc):
    return int(load_library().hawq_conv_fragment_weights_bytes(ctypes.byref(desc)))


def hawq_conv_fragment_weights(desc, w, w_fragments, stream=None):
    _check(load_library().hawq_conv_fragment_weights(ctypes.byref(desc), _p(w), _p(w_fragments), _stream(stream)),
           "hawq_conv_fragment_weights")


def hawq_bottleneck_tail_int(desc2, x, w2_fragments, bias2, b2, c2, desc3, w3_fragments, bias3, b3, c3, residual, res_b, res_c, y,
                             stream=None):
    _check(load_library().hawq_bottleneck_tail_int(ctypes.byref(desc2), _p(x), _p(w2_fragments), _p(bias2), _p(b2), _p(c2),
                                                    ctypes.byref(desc3), _p(w3_fragments), _p(bias3), _p(b3), _p(c3), _p(residual),
                                                    _p(res_b), _p(res_c), _p(y), _stream(stream)), "hawq_bottleneck_tail_int")


def hawq_probe_mfma_peak(iters=4000):
    """TOP/s of a register-only INT8 MFMA loop on the current device (see the header)."""
    tops = ctypes.c_double(0.0)
    _check(load_library().hawq_probe_mfma_peak(int(iters), ctypes.byref(tops)), "hawq_probe_mfma_peak")
    return tops.value


def hawq_tune_set_split(n_first):
    """Measurement hook: 0 = the library's batch-split rule, -1 = never split, n = first part of n images."""
    load_library().hawq_tune_set_split(int(n_first))


def hawq_noalloc_workspace_limit():
    return int(load_library().hawq_noalloc_workspace_limit())


def hawq_tune_set_fusion(mode):
    """Measurement hook: 1 = later networks fuse bottleneck tails wherever the kernel applies, 2 = only at 256 input
    channels, 0 = the plan's rule."""
    load_library().hawq_tune_set_fusion(int(mode))


def hawq_net_num_layers(arch):
    return load_library().hawq_net_num_layers(arch)


def hawq_net_layer_info(arch, image_hw, num_classes, index):
    info = LayerInfo()
    _check(load_library().hawq_net_layer_info(arch, image_hw, num_classes, index, ctypes.byref(info)), "hawq_net_layer_info")
    d = {n: getattr(info, n) for n, _ in LayerInfo._fields_ if n != "name"}
    d["name"] = info.name.decode()
    return d


class HawqNet:
    """Owner of a ``hawq_net*``.  ``layers`` is the list of per-layer dicts of host numpy arrays in
    canonical order (keys w, bias, b, c, res_b, res_c, bits and optionally int32_shortcut on a transition layer),
    as made by the workload generator or the converter."""

    def __init__(self, arch, layers, pool_b, pool_c, image_hw=224, num_classes=1000, keep_activations=False):
        import numpy as np
        lib = load_library()
        self._keepalive = []

        def hp(a, dt):
            if a is None:
                return None
            a = np.ascontiguousarray(a, dtype=dt)
            self._keepalive.append(a)
            return a.ctypes.data

        arr = (LayerParams * len(layers))()
        for i, l in enumerate(layers):
            arr[i].w = hp(l["w"], np.uint8 if l["bits"] == 4 else np.int8)
            arr[i].bias = hp(l["bias"], np.int32)
            arr[i].b = hp(l["b"], np.int32)
            arr[i].c = hp(l["c"], np.uint8)
            arr[i].res_b = hp(l.get("res_b"), np.int32)
            arr[i].res_c = hp(l.get("res_c"), np.uint8)
            arr[i].bits = int(l["bits"])
            arr[i].flags = LAYER_INT32_SHORTCUT if (l.get("int32_shortcut") and l["name"].endswith(".ds")) else 0
        handle = ctypes.c_void_p()
        _check(lib.hawq_net_create(arch, image_hw, num_classes, arr, len(layers), hp(pool_b, np.int32), hp(pool_c, np.uint8),
                                   1 if keep_activations else 0, ctypes.byref(handle)), "hawq_net_create")
        self._h = handle
        self._keepalive = []
        self.arch, self.image_hw, self.num_classes = arch, image_hw, num_classes

    def close(self):
        if getattr(self, "_h", None):
            load_library().hawq_net_destroy(self._h)
            self._h = None

    __del__ = close

    def workspace_bytes(self, N):
        return load_library().hawq_net_workspace_bytes(self._h, N)

    def num_steps(self):
        return load_library().hawq_net_num_steps(self._h)

    def step_output(self, N, step):
        name = ctypes.create_string_buffer(24)
        off, nbytes = ctypes.c_size_t(), ctypes.c_size_t()
        dt = ctypes.c_int32()
        dims = (ctypes.c_int32 * 4)()
        _check(load_library().hawq_net_step_output(self._h, N, step, name, ctypes.byref(off), ctypes.byref(nbytes),
                                                   ctypes.byref(dt), dims), "hawq_net_step_output")
        return dict(name=name.value.decode(), offset=off.value, bytes=nbytes.value, dtype=dt.value, dims=tuple(dims))

    def step_cost(self, N, step):
        macs, nbytes = ctypes.c_double(), ctypes.c_double()
        _check(load_library().hawq_net_step_cost(self._h, N, step, ctypes.byref(macs), ctypes.byref(nbytes)), "hawq_net_step_cost")
        return macs.value, nbytes.value

    def split_first(self, N):
        return int(load_library().hawq_net_split_first(self._h, int(N)))

    def hawq_forward_resnet(self, x, N, logits, workspace, stream=None):
        _check(load_library().hawq_forward_resnet(self._h, _p(x), N, _p(logits), _p(workspace),
                                                  workspace.numel() * workspace.element_size(), _stream(stream)),
               "hawq_forward_resnet")

    def hawq_forward_resnet_noalloc(self, x, N, logits, stream=None):
        _check(load_library().hawq_forward_resnet_noalloc(self._h, _p(x), N, _p(logits), _stream(stream)),
               "hawq_forward_resnet_noalloc")

    def hawq_forward_resnet_timed(self, x, N, logits, workspace, stream=None):
        ms = (ctypes.c_float * self.num_steps())()
        _check(load_library().hawq_forward_resnet_timed(self._h, _p(x), N, _p(logits), _p(workspace),
                                                        workspace.numel() * workspace.element_size(), _stream(stream), ms),
               "hawq_forward_resnet_timed")
        return list(ms)
