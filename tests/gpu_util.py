"""Shared plumbing of the GPU parity tests: run one case through the C interface (via the thin
binding) and through the CPU oracle on the same seeded inputs."""
import numpy as np

import oracle
import paper_2011_10680_amd as hawq

_NP_OF = {hawq.U8: np.uint8, hawq.S8: np.int8, hawq.U4: np.uint8, hawq.S4: np.uint8, hawq.S32: np.int32}


def to_dev(a):
    import torch
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def out_shape(shape, dt):
    shape = list(shape)
    if dt in (hawq.U4, hawq.S4):
        shape[-1] //= 2
    return shape


def run_conv_gpu(case, x_dt, w_dt, y_dt, res_dt=hawq.U8, relu=1, y_lo=0, y_hi=127, x_hi=0, raw=False, stride=None, pad=None):
    """Returns (gpu_result, oracle_result) as numpy arrays in storage format."""
    import torch
    sh, sw = stride if stride is not None else (case["stride"], case["stride"])
    ph, pw = pad if pad is not None else (case["pad"], case["pad"])
    N, H, W, C, K, R, S = (case[k] for k in "NHWCKRS")
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    d = hawq.ConvDesc(N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride_h=sh, stride_w=sw, pad_h=ph, pad_w=pw,
                      x_dtype=x_dt, w_dtype=w_dt, y_dtype=y_dt, res_dtype=res_dt, relu=relu, y_lo=y_lo, y_hi=y_hi, x_hi=x_hi)
    res = case.get("residual")
    y = torch.full(out_shape((N, P, Q, K), y_dt), 0x5A if y_dt != hawq.S32 else 0x5A5A5A5A,
                   dtype={np.uint8: torch.uint8, np.int8: torch.int8, np.int32: torch.int32}[_NP_OF[y_dt]], device="cuda")
    b = None if raw else to_dev(case["b"])
    c = None if raw else to_dev(case["c"])
    hawq.hawq_conv2d_int(d, to_dev(case["x"]), to_dev(case["w"]), to_dev(case["bias"]), b, c,
                         to_dev(res), to_dev(case.get("res_b")) if res is not None else None,
                         to_dev(case.get("res_c")) if res is not None else None, y)
    torch.cuda.synchronize()
    want = oracle.conv2d_int(case["x"], case["w"], case["bias"], None if raw else case["b"], None if raw else case["c"],
                             N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=(sh, sw), pad=(ph, pw), x_dt=x_dt, w_dt=w_dt,
                             y_dt=y_dt, relu=relu, y_lo=y_lo, y_hi=y_hi, residual=res,
                             res_b=case.get("res_b") if res is not None else None,
                             res_c=case.get("res_c") if res is not None else None, res_dt=res_dt)
    return y.cpu().numpy(), want


def assert_same(got, want, what=""):
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError("%s: %d of %d elements differ; first at %s: gpu=%s oracle=%s" % (
            what, len(bad), got.size, tuple(bad[0]), got[tuple(bad[0])], want[tuple(bad[0])]))
