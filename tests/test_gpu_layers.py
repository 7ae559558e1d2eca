"""GPU parity: stand-alone residual add, average pool and max pool vs the CPU oracle, bit-exact."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hawq():
    import torch
    assert torch.cuda.is_available()
    import paper_2011_10680_amd as h
    h.load_library()
    return h


@pytest.mark.parametrize("m_dt,r_dt,y_dt,K,relu,lo,hi", [
    (4, 1, 0, 256, 1, 0, 127),     # INT32 main branch (the accumulator) + signed shortcut -> u8
    (0, 0, 0, 64, 1, 0, 127),
    (1, 0, 1, 10, 0, -128, 127),   # K % 4 != 0
    (2, 2, 2, 64, 1, 0, 15),       # packed 4-bit everywhere
    (0, 2, 4, 6, 0, -1000, 1000),
])
def test_residual_add(hawq, m_dt, r_dt, y_dt, K, relu, lo, hi):
    import torch
    from gpu_util import to_dev, out_shape, assert_same
    g = np.random.default_rng(K + m_dt)
    P = 1000 + 37

    def draw(dt):
        if dt == 4:
            return g.integers(-(1 << 20), 1 << 20, size=(P, K)).astype(np.int32)
        if dt == 0:
            return g.integers(0, 128, size=(P, K)).astype(np.uint8)
        if dt == 1:
            return g.integers(-128, 128, size=(P, K)).astype(np.int8)
        return wl.pack_nibbles(g.integers(0, 16, size=(P, K)))
    m, r = draw(m_dt), draw(r_dt)
    m_b = g.integers(1 << 14, 1 << 15, size=K).astype(np.int32)
    r_b = g.integers(1 << 14, 1 << 15, size=K).astype(np.int32)
    m_c = (g.integers(27, 30, size=K) if m_dt == 4 else g.integers(14, 17, size=K)).astype(np.uint8)
    r_c = g.integers(14, 17, size=K).astype(np.uint8)
    tdt = {0: torch.uint8, 1: torch.int8, 2: torch.uint8, 3: torch.uint8, 4: torch.int32}[y_dt]
    y = torch.zeros(out_shape((P, K), y_dt), dtype=tdt, device="cuda")
    hawq.hawq_residual_add_dyadic(P, K, m_dt, r_dt, y_dt, to_dev(m), to_dev(m_b), to_dev(m_c), to_dev(r), to_dev(r_b),
                                  to_dev(r_c), relu, lo, hi, y)
    torch.cuda.synchronize()
    want = oracle.residual_add_dyadic(m, m_b, m_c, r, r_b, r_c, n_pixels=P, K=K, m_dt=m_dt, r_dt=r_dt, y_dt=y_dt,
                                      relu=relu, y_lo=lo, y_hi=hi)
    assert_same(y.cpu().numpy(), want)


@pytest.mark.parametrize("N,H,W,C,x_dt,y_dt", [(5, 7, 7, 2048, 0, 0), (3, 7, 7, 512, 0, 0), (2, 3, 5, 10, 1, 1), (2, 4, 4, 64, 2, 0)])
def test_avgpool(hawq, N, H, W, C, x_dt, y_dt):
    import torch
    from gpu_util import to_dev, assert_same
    g = np.random.default_rng(C)
    if x_dt == 0:
        x = g.integers(0, 128, size=(N, H, W, C)).astype(np.uint8)
    elif x_dt == 1:
        x = g.integers(-128, 128, size=(N, H, W, C)).astype(np.int8)
    else:
        x = wl.pack_nibbles(g.integers(0, 16, size=(N, H, W, C)))
    b = np.rint((1 << 20) / (H * W) * g.uniform(0.9, 1.1, size=C)).astype(np.int32)
    c = np.full(C, 20, np.uint8)
    lo, hi = (-128, 127) if y_dt == 1 else (0, 127)
    y = torch.zeros((N, C), dtype=torch.int8 if y_dt == 1 else torch.uint8, device="cuda")
    hawq.hawq_avgpool_int(N, H, W, C, x_dt, y_dt, to_dev(x), to_dev(b), to_dev(c), lo, hi, y)
    torch.cuda.synchronize()
    want = oracle.avgpool_int(x, b, c, N=N, H=H, W=W, C=C, x_dt=x_dt, y_dt=y_dt, y_lo=lo, y_hi=hi)
    assert_same(y.cpu().numpy(), want)


@pytest.mark.parametrize("N,H,W,C,x_dt,y_dt,hi", [(3, 112, 112, 64, 0, 0, 127), (2, 112, 112, 64, 0, 2, 15), (2, 9, 7, 10, 0, 0, 127),
                                                   (1, 8, 8, 6, 1, 1, 127), (1, 10, 10, 8, 2, 2, 15),
                                                   # 4-bit input, 8-bit output: a thread owns two channels and stores both
                                                   (1, 10, 10, 8, 2, 0, 127), (2, 7, 9, 6, 3, 1, 127), (1, 9, 9, 10, 3, 3, 7)])
def test_maxpool(hawq, N, H, W, C, x_dt, y_dt, hi):
    import torch
    from gpu_util import to_dev, out_shape, assert_same
    g = np.random.default_rng(H + C)
    if x_dt == 0:
        x = g.integers(0, hi + 1, size=(N, H, W, C)).astype(np.uint8)
    elif x_dt == 1:
        x = g.integers(-128, 128, size=(N, H, W, C)).astype(np.int8)
    else:
        x = wl.pack_nibbles(g.integers(0, 16, size=(N, H, W, C)))
    lo = {1: -128, 3: -8}.get(y_dt, 0)
    P, Q = (H - 1) // 2 + 1, (W - 1) // 2 + 1
    y = torch.zeros(out_shape((N, P, Q, C), y_dt), dtype=torch.int8 if y_dt == 1 else torch.uint8, device="cuda")
    hawq.hawq_maxpool_int(N, H, W, C, x_dt, y_dt, to_dev(x), lo, hi, y)
    torch.cuda.synchronize()
    want = oracle.maxpool_int(x, N=N, H=H, W=W, C=C, x_dt=x_dt, y_dt=y_dt, y_lo=lo, y_hi=hi)
    assert_same(y.cpu().numpy(), want)


def test_mfma_loop_probe_reports_a_plausible_rate(hawq):
    """The register-only INT8 MFMA loop: between a fifth of and the whole datasheet peak (5.03 POP/s).  (No stability
    check: the first call after an idle spell runs at lower clocks than the next.)"""
    for _ in range(3):
        t = hawq.hawq_probe_mfma_peak(2000)
        assert 1000.0 < t < 5100.0
