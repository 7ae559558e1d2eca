"""Hardware-aware bit selection on this GPU, end to end (Section 3.4; the analogue of Table 2's latency-constrained rows).

    python -m paper_2011_10680_amd.bitselect_report [--arch 50] [--batch 128] [--out DIR]

1. Latency table: the integer-only network is built twice with synthetic seeded parameters -- every selectable layer
   group at 8 bits, then at 4 bits (conv1 and fc stay 8-bit, Appendix H) -- and the per-launch device times of the
   library's timed forward are summed per group: Q[g][b] in microseconds, measured with the library's own kernels.
2. Sensitivities: the paper's second-order metric needs training data; the data-free factor || Q_b(W) - W ||^2 on
   seeded Gaussian weights of the layer's shape (He scaling) stands in for it, so the objective still prefers to keep
   8 bits where 4-bit rounding perturbs most.
3. The selection ILP (minimise summed sensitivity subject to a latency limit) is solved exactly at three limits between
   the all-INT4 and all-INT8 latencies ("high", "medium", "low" budget), and every selected network is built and its
   forward timed as a whole (HIP events on the launch stream, as bench.py does).
Writes <out>/bitselect.json (tables, selections, timings) and prints a Markdown summary; the selections are also
written as <out>/bits_<name>.json for `bench.py --bits-json`.
"""
import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def synthetic_sensitivity(arch, names, seed=7):
    """Omega [G, 2] for the choices (4, 8): summed squared quantisation perturbation of seeded Gaussian weights."""
    import paper_2011_10680_amd as hawq
    from . import bitselect as bs
    g = np.random.Generator(np.random.PCG64(seed))
    omega = {n: np.zeros(2) for n in names}
    for i in range(hawq.hawq_net_num_layers(arch)):
        f = hawq.hawq_net_layer_info(arch, 224, 1000, i)
        W = g.normal(0.0, np.sqrt(2.0 / (f["R"] * f["S"] * f["C"])), size=(f["K"], f["R"], f["S"], f["C"]))
        for j, b in enumerate((4, 8)):
            omega[bs.group_of(f["name"])][j] += bs.quantization_perturbation(W, b)
    return np.array([omega[n] for n in names])


def time_forward(hn, x, batch, steps=100, warmup=20):
    import torch
    ws = torch.empty(hn.workspace_bytes(batch), dtype=torch.uint8, device="cuda")
    logits = torch.empty((batch, hn.num_classes), dtype=torch.int32, device="cuda")
    for _ in range(warmup):
        hn.hawq_forward_resnet(x, batch, logits, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        hn.hawq_forward_resnet(x, batch, logits, ws)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--arch", type=int, default=50)
    ap.add_argument("--batch", type=int, default=128)
    ap.add_argument("--out", default=os.path.join(ROOT, "bitselect_out"))
    args = ap.parse_args()
    import torch
    import paper_2011_10680_amd as hawq
    from . import bitselect as bs
    import workloads as wl
    hawq.load_library()
    os.makedirs(args.out, exist_ok=True)
    arch, N = args.arch, args.batch
    groups = wl.resnet_group_names(arch)
    x = torch.from_numpy(wl.make_image_batch(11, N)).cuda()

    def build(bits):
        p = wl.make_resnet(arch, seed=1003, bits=bits)
        return hawq.HawqNet(arch, p["layers"], p["pool_b"], p["pool_c"])

    uniform = {b: {g: (8 if g in ("conv1", "fc") else b) for g in groups} for b in (4, 8)}
    nets = {b: build(uniform[b]) for b in (4, 8)}
    names, Q = bs.measure_group_latencies(nets, N, x, repeats=7)       # [G, 2] milliseconds, columns (4, 8)
    t_uniform = {b: time_forward(nets[b], x, N) for b in (4, 8)}
    for hn in nets.values():
        hn.close()
    cost_names, M, G = bs.layer_costs(arch)
    # (the workload generator calls the group of a block's first convolution and its transition layer "<block>.in")
    wl_name = lambda n: n[:-2] + "in" if n.endswith(".c1") else n
    assert names == cost_names and [wl_name(n) for n in names] == groups
    omega = synthetic_sensitivity(arch, names)
    fixed = {0: 1, len(names) - 1: 1}                                   # conv1 and fc stay at 8 bits
    q4, q8 = Q[:, 0].sum(), Q[:, 1].sum()
    lo, hi = min(q4, q8), max(q4, q8)
    floor = Q.min(axis=1).sum()                                        # the fastest any assignment can be, by the table
    out = dict(arch=arch, batch=N, groups=names, latency_ms=Q.tolist(), omega=omega.tolist(), size_bytes=M.tolist(), bops=G.tolist(),
               sum_latency_int4_ms=q4, sum_latency_int8_ms=q8, sum_latency_fastest_ms=floor,
               forward_ms_all_int4=t_uniform[4], forward_ms_all_int8=t_uniform[8], selections=[])
    for label, frac in (("high", 0.75), ("medium", 0.5), ("low", 0.1)):
        limit = floor + frac * (hi - floor)
        choice, obj = bs.solve(omega, latency=Q, latency_limit=limit, fixed=fixed)
        bits = {wl_name(n): (4, 8)[c] for n, c in zip(names, choice)}
        hn = build(bits)
        t = time_forward(hn, x, N)
        hn.close()
        with open(os.path.join(args.out, "bits_%s.json" % label), "w") as f:
            json.dump(bits, f, indent=1)
        out["selections"].append(dict(budget=label, latency_limit_ms=limit, table_latency_ms=float(Q[np.arange(len(names)), choice].sum()),
                                      objective=obj, groups_int4=int(sum(b == 4 for b in bits.values())), forward_ms=t,
                                      images_per_s=N / t * 1e3, size_mb=float(M[np.arange(len(names)), choice].sum() / 1e6),
                                      bits=bits))
    with open(os.path.join(args.out, "bitselect.json"), "w") as f:
        json.dump(out, f, indent=1)
    print("| budget | latency limit (table, ms) | selected (table, ms) | groups at 4 bits | weight MB | sensitivity | forward ms | images/s |")
    print("|---|---|---|---|---|---|---|---|")
    print("| all INT8 | - | %.3f | 0 | %.1f | %.3g | %.3f | %.0f |" % (q8, M[:, 1].sum() / 1e6, omega[:, 1].sum(), t_uniform[8], N / t_uniform[8] * 1e3))
    for s in out["selections"]:
        print("| %s | %.3f | %.3f | %d of %d | %.1f | %.3g | %.3f | %.0f |" % (s["budget"], s["latency_limit_ms"], s["table_latency_ms"],
              s["groups_int4"], len(names), s["size_mb"], s["objective"], s["forward_ms"], s["images_per_s"]))
    print("| all INT4 | - | %.3f | %d | %.1f | %.3g | %.3f | %.0f |" % (q4, len(names) - 2, M[:, 0].sum() / 1e6, omega[:, 0].sum(), t_uniform[4], N / t_uniform[4] * 1e3))


if __name__ == "__main__":
    main()
