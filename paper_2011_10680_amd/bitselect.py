"""Hardware-aware mixed-precision selection (Section 3.4): choose a bit width per layer group by an integer linear
programme that minimises the summed sensitivity subject to limits on model size, bit operations and latency --
with the latency table measured on this GPU by the library's own kernels.

    minimise    sum_i Omega_i^(b_i)
    subject to  sum_i M_i^(b_i) <= size limit,  sum_i G_i^(b_i) <= BOPS limit,  sum_i Q_i^(b_i) <= latency limit

M_i is the size of layer i at b_i bits, G_i = b_w b_a MAC_i its bit operations (weights and activations of a layer share
one width), Q_i its measured latency.  Any subset of the limits may be given.  The sensitivities Omega are an input:
the paper takes a Hessian-based perturbation measured on training data, which this repository does not have;
`quantization_perturbation` gives the data-free part of that metric (the squared weight perturbation) as a stand-in.
On MI355X there is no INT4 matrix instruction, so 4 bits buy bytes and not multiply-accumulates: the measured Q_i
differ from the BOPS model layer by layer, which is exactly what the latency constraint is for.
"""
import numpy as np

from .binding import hawq_net_layer_info, hawq_net_num_layers


def group_of(name):
    """Layers that must share a bit width form a group: a transition convolution goes with its block's first one."""
    return name[:-2] + "c1" if name.endswith(".ds") else name


def layer_costs(arch, image_hw=224, num_classes=1000, choices=(4, 8)):
    """Per group: weight bytes M and bit operations G for every bit choice (conv1 and fc are fixed at 8 bits and
    appear with identical entries).  Returns (group names in network order, M [G, B] bytes, G [G, B] bit operations)."""
    names, M, Gb = [], {}, {}
    for i in range(hawq_net_num_layers(arch)):
        f = hawq_net_layer_info(arch, image_hw, num_classes, i)
        g = group_of(f["name"])
        if g not in M:
            names.append(g)
            M[g] = np.zeros(len(choices))
            Gb[g] = np.zeros(len(choices))
        params = f["K"] * f["R"] * f["S"] * f["C"]
        macs = params * f["P"] * f["Q"]
        for j, b in enumerate(choices):
            bb = 8 if f["name"] in ("conv1", "fc") else b
            M[g][j] += params * bb / 8.0
            Gb[g][j] += float(bb) * bb * macs
    return names, np.array([M[g] for g in names]), np.array([Gb[g] for g in names])


def quantization_perturbation(W, bits):
    """|| Q(W) - W ||^2 with the converter's per-channel symmetric quantiser: the data-free factor of the
    second-order sensitivity metric (stand-in when no Hessian information is available)."""
    from .convert import quantize_weights
    q, S = quantize_weights(W, bits)
    return float(np.sum((np.asarray(W, dtype=np.float64) - q * S.reshape(-1, 1, 1, 1)) ** 2))


def solve(omega, size=None, bops=None, latency=None, size_limit=None, bops_limit=None, latency_limit=None, fixed=None):
    """Exact solution of the selection problem.  omega, size, bops, latency: [L, B] arrays (row = layer group, column =
    bit choice); a limit of None drops that constraint.  fixed: {row: column} choices imposed beforehand.
    Returns (choice [L] column indices, objective) or raises ValueError if the limits cannot be met."""
    from scipy.optimize import Bounds, LinearConstraint, milp
    omega = np.asarray(omega, dtype=np.float64)
    L, B = omega.shape
    A, lo, hi = [], [], []
    for i in range(L):                                   # exactly one choice per group
        row = np.zeros(L * B)
        row[i * B:(i + 1) * B] = 1
        A.append(row); lo.append(1); hi.append(1)
    for tab, lim in ((size, size_limit), (bops, bops_limit), (latency, latency_limit)):
        if lim is None:
            continue
        if tab is None:
            raise ValueError("a limit needs its cost table")
        A.append(np.asarray(tab, dtype=np.float64).reshape(-1)); lo.append(-np.inf); hi.append(float(lim))
    ub = np.ones(L * B)
    lb = np.zeros(L * B)
    for i, j in (fixed or {}).items():
        lb[i * B + j] = 1
    res = milp(c=omega.reshape(-1), integrality=np.ones(L * B), bounds=Bounds(lb, ub),
               constraints=LinearConstraint(np.array(A), np.array(lo), np.array(hi)))
    if not res.success:
        raise ValueError("bit selection infeasible under the given limits: " + str(res.message))
    x = np.rint(res.x).reshape(L, B)
    choice = x.argmax(axis=1)
    return choice, float(omega[np.arange(L), choice].sum())


def measure_group_latencies(net_by_choice, batch, image, repeats=5):
    """Measured latency table Q [G, B] in milliseconds for one batch size: net_by_choice maps a bit choice to a
    HawqNet in which every selectable group runs at that width; the per-launch device times of the library's timed
    forward are summed per group (a transition convolution into its block's first group; conv1 carries the fused max
    pool).  Returns (group names, Q)."""
    import torch
    names = None
    cols = []
    for b in sorted(net_by_choice):
        hn = net_by_choice[b]
        ws = torch.empty(hn.workspace_bytes(batch), dtype=torch.uint8, device="cuda")
        logits = torch.empty((batch, hn.num_classes), dtype=torch.int32, device="cuda")
        for _ in range(2):
            hn.hawq_forward_resnet(image, batch, logits, ws)
        per = np.median(np.array([hn.hawq_forward_resnet_timed(image, batch, logits, ws) for _ in range(repeats)]), axis=0)
        acc, order = {}, []
        for s in range(hn.num_steps()):
            nm = hn.step_output(batch, s)["name"]
            g = "conv1" if nm == "pool" else ("fc" if nm == "avgpool" else group_of(nm))
            if g not in acc:
                acc[g] = 0.0
                order.append(g)
            acc[g] += float(per[s])
        if names is None:
            names = order
        cols.append([acc[g] for g in names])
    return names, np.array(cols).T
