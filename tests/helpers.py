"""Test-side helpers: things the paper defines around the hot path (quantiser,
DN, batch-norm folding) written independently of both the oracle and the HIP
library, in exact Python integers / Fractions / float64."""
import math
from fractions import Fraction

import numpy as np


def rq_exact(t, b, c):
    """round-to-nearest, ties toward +inf, of t*b/2^c in exact rationals."""
    return math.floor(Fraction(int(t) * int(b), 2 ** int(c)) + Fraction(1, 2))


def dyadic_from_real(s):
    """DN(s): (b, c) with b in [2^14, 2^15) and b/2^c within 2^-15 relative of s."""
    m, e = math.frexp(s)  # s = m * 2^e, m in [0.5, 1)
    b = int(round(m * (1 << 15)))
    c = 15 - e
    if b == (1 << 15):
        b >>= 1
        c -= 1
    return b, c


def quantize_symmetric_per_channel(w, bits):
    """S = 2 max|w| / (2^bits - 1) per output channel (axis 0), q = round(w / S)."""
    flat = np.abs(w.reshape(w.shape[0], -1)).max(axis=1)
    S = 2.0 * flat / (2 ** bits - 1)
    q = np.rint(w / S.reshape((-1,) + (1,) * (w.ndim - 1))).astype(np.int64)
    lim = 2 ** (bits - 1) - 1  # max|w|/S = (2^bits - 1)/2 sits half a step above the last level: truncate
    return np.clip(q, -lim, lim), S


def conv2d_bruteforce(x, w, stride, pad):
    """7-loop cross-correlation on Python ints. x [N,H,W,C], w [K,R,S,C] -> [N,P,Q,K]."""
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    sh, sw = stride
    ph, pw = pad
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    out = [[[[0] * K for _ in range(Q)] for _ in range(P)] for _ in range(N)]
    xl, wl = x.tolist(), w.tolist()
    for n in range(N):
        for p in range(P):
            for q in range(Q):
                for k in range(K):
                    acc = 0
                    for r in range(R):
                        ih = p * sh - ph + r
                        if not 0 <= ih < H:
                            continue
                        for s in range(S):
                            iw = q * sw - pw + s
                            if not 0 <= iw < W:
                                continue
                            xr, wr = xl[n][ih][iw], wl[k][r][s]
                            for c in range(C):
                                acc += xr[c] * wr[c]
                    out[n][p][q][k] = acc
    return np.array(out, dtype=np.int64).reshape(N, P, Q, K)


def conv2d_f64(x, w, stride, pad):
    """Library routine: torch float64 conv2d (exact for |values| < 2^53)."""
    import torch
    import torch.nn.functional as F
    xt = torch.from_numpy(np.asarray(x, dtype=np.float64)).permute(0, 3, 1, 2).contiguous()
    wt = torch.from_numpy(np.asarray(w, dtype=np.float64)).permute(0, 3, 1, 2).contiguous()
    y = F.conv2d(xt, wt, stride=stride, padding=pad)
    return np.rint(y.permute(0, 2, 3, 1).numpy()).astype(np.int64)
