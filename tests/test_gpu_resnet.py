"""GPU parity: hawq_forward_resnet vs the oracle's network walk, every stored tensor and the INT32 logits."""
import numpy as np
import pytest

import oracle
from oracle import resnet as onet
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hawq():
    import torch
    assert torch.cuda.is_available()
    import paper_2011_10680_amd as h
    h.load_library()
    return h


def _forward_gpu(hawq, net, x, keep):
    import torch
    N = x.shape[0]
    hn = hawq.HawqNet(net["arch"], net["layers"], net["pool_b"], net["pool_c"], image_hw=net["image_hw"],
                      num_classes=net["num_classes"], keep_activations=keep)
    ws = torch.empty(hn.workspace_bytes(N), dtype=torch.uint8, device="cuda")
    logits = torch.empty((N, net["num_classes"]), dtype=torch.int32, device="cuda")
    xd = torch.from_numpy(x).cuda()
    hn.hawq_forward_resnet(xd, N, logits, ws)
    torch.cuda.synchronize()
    acts = {}
    if keep:
        wsh = ws.cpu().numpy()
        for s in range(hn.num_steps()):
            o = hn.step_output(N, s)
            if o["bytes"]:
                acts[o["name"]] = (wsh[o["offset"]:o["offset"] + o["bytes"]], o["dtype"], o["dims"])
    out = logits.cpu().numpy()
    hn.close()
    return out, acts


@pytest.mark.parametrize("arch,mixed,N", [(18, False, 2), (50, False, 2), (18, True, 2), (50, True, 3)])
def test_layerwise_and_logits(hawq, arch, mixed, N):
    """Every layer's stored activation (as the paper's deployment check compares layer by layer) and
    the final INT32 logits are identical to the oracle's."""
    bits = wl.draw_bits(arch, 4000 + arch) if mixed else None
    net = wl.make_resnet(arch, seed=1000 + arch, bits=bits)
    x = wl.make_image_batch(7, N)
    keep = {}
    want = onet.forward(net, x, keep)
    got, acts = _forward_gpu(hawq, net, x, True)
    assert set(acts) == set(keep) - {"fc"}
    for name, (raw, dt, dims) in acts.items():
        w = np.ascontiguousarray(keep[name]).view(np.uint8).ravel()
        assert raw.size == w.size, (name, raw.size, w.size, dims)
        if not np.array_equal(raw, w):
            bad = np.flatnonzero(raw != w)
            raise AssertionError("%s: %d of %d bytes differ, first at %d (gpu %d, oracle %d)" % (
                name, bad.size, w.size, bad[0], raw[bad[0]], w[bad[0]]))
    assert np.array_equal(got, want)
    # reusing workspace slots must not change anything
    got2, _ = _forward_gpu(hawq, net, x, False)
    assert np.array_equal(got2, want)


@pytest.mark.parametrize("image_hw,N", [(64, 3), (100, 2), (224, 1)])
def test_fused_stem_with_wide_parameters_and_odd_sizes(hawq, image_hw, N):
    """conv1 fused with the max pool (no kept activations): multipliers of conv1 outside the narrow epilogue's range
    take the exact 64-bit path inside the fused kernel; image sizes whose pooled size is not a multiple of the
    pooled tile (7 x 8) exercise the ragged tiles.  Scaling numerator and shift together must not change a bit."""
    net = wl.make_resnet(18, seed=77, image_hw=image_hw)
    x = wl.make_image_batch(9, N, image_hw=image_hw)
    want = onet.forward(net, x)
    got, _ = _forward_gpu(hawq, net, x, False)
    assert np.array_equal(got, want)
    conv1 = net["layers"][0]
    conv1["b"] = (conv1["b"].astype(np.int64) << 14).astype(np.int32)
    conv1["c"] = (conv1["c"].astype(np.int32) + 14).astype(np.uint8)
    assert np.array_equal(onet.forward(net, x), want)
    got, _ = _forward_gpu(hawq, net, x, False)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("image_hw,N,ties", [(64, 2, True), (36, 3, True), (64, 2, False)])
def test_fused_stem_pools_before_it_requantises(hawq, image_hw, N, ties):
    """The fused conv1 + max pool kernel takes the window maximum of the INT32 accumulators and requantises once (the
    requantisation never decreases in the accumulator).  Cases where that order could show: channels with multiplier 0
    (every output is rq(., 0, c) = 0), channels whose accumulators are all far below zero (ReLU clamps the maximum), channels
    with the largest admissible multiplier and shift 1, and a bias that puts the maxima right at rounding boundaries."""
    net = wl.make_resnet(18, seed=78, image_hw=image_hw)
    x = wl.make_image_batch(10, N, image_hw=image_hw)
    conv1 = net["layers"][0]
    conv1["b"] = conv1["b"].copy(); conv1["c"] = conv1["c"].copy(); conv1["bias"] = conv1["bias"].copy()
    conv1["b"][0:8] = 0
    conv1["bias"][8:16] = -(1 << 28)
    conv1["bias"][16:24] = (1 << 28)
    conv1["b"][24:28] = (1 << 30) - 1; conv1["c"][24:28] = 31         # just below one half per accumulator step
    if ties:   # one half per accumulator step: every odd value is a tie (outside the narrow evaluation: the exact 64-bit form)
        conv1["b"][28:32] = 1; conv1["c"][28:32] = 1
    want = onet.forward(net, x)
    got, _ = _forward_gpu(hawq, net, x, False)
    assert np.array_equal(got, want)
    # the same through the unfused kernels (kept activations): conv1's tensor, the pooled tensor, logits
    got_keep, _ = _forward_gpu(hawq, net, x, True)
    assert np.array_equal(got_keep, want)


@pytest.mark.parametrize("arch,batch,mixed,seed,int32_sc", [(18, 64, False, 1002, True), (50, 128, False, 1003, True), (50, 256, True, 1004, False),
                                                            (18, 64, False, 1002, False), (50, 128, False, 1003, False)])
def test_full_size_configs_whole_batch_against_oracle(hawq, arch, batch, mixed, seed, int32_sc):
    """The network configurations at their full batch, in the launch configuration the benchmark times
    (reused workspace slots, the batch as two parts on two streams where the library's rule says so).  The oracle
    computes every image of the batch (in chunks, to bound its memory) and all batch x 1000 INT32 logits must be
    equal.  On top of that: run-to-run identical bits, and the same image gives the same logits wherever it sits
    in the batch."""
    import torch
    bits = wl.draw_bits(arch, 4000 + arch) if mixed else None
    net = wl.make_resnet(arch, seed=seed, bits=bits, int32_shortcut=int32_sc)   # the benchmark's workloads: both transition forms
    x = wl.make_image_batch(seed + 1, batch)
    x[batch - 1] = x[0]                      # duplicate image at the other end of the batch
    hn = hawq.HawqNet(arch, net["layers"], net["pool_b"], net["pool_c"])
    ws = torch.empty(hn.workspace_bytes(batch), dtype=torch.uint8, device="cuda")
    logits = torch.empty((batch, 1000), dtype=torch.int32, device="cuda")
    xd = torch.from_numpy(x).cuda()
    hn.hawq_forward_resnet(xd, batch, logits, ws)
    torch.cuda.synchronize()
    got = logits.cpu().numpy()
    ws.fill_(0x5A)
    logits.zero_()
    hn.hawq_forward_resnet(xd, batch, logits, ws)
    torch.cuda.synchronize()
    assert np.array_equal(logits.cpu().numpy(), got), "two runs differ"
    assert np.array_equal(got[0], got[batch - 1]), "same image, different logits at another batch position"
    hn.close()
    chunk = 32
    for i0 in range(0, batch, chunk):
        want = onet.forward(net, x[i0:i0 + chunk])
        if not np.array_equal(got[i0:i0 + chunk], want):
            bad = np.argwhere(got[i0:i0 + chunk] != want)
            raise AssertionError("image %d of the full batch differs from the oracle (%d logits in images %d..%d differ)" % (
                i0 + bad[0][0], len(bad), i0, i0 + chunk - 1))
        print("images %d..%d of %d equal the oracle" % (i0, min(batch, i0 + chunk) - 1, batch), flush=True)
    assert len({got[i].tobytes() for i in range(batch - 1)}) == batch - 1   # distinct images, distinct logits


@pytest.mark.parametrize("arch,N,first,hw", [(18, 13, 5, 64), (50, 6, 4, 64), (18, 9, 8, 64),
                                             (18, 100, 0, 64),    # first = 0: the library's rule, 56 + 44
                                             (18, 100, 0, 34),    # the same at another image size
                                             (18, 100, 0, 33)])   # odd image side: the second part would start misaligned -> one part
def test_batch_split_over_two_streams_same_bits(hawq, arch, N, first, hw):
    """A large batch runs as two parts on two streams.  Forced here at small sizes (odd parts, the second part's image,
    logits and workspace offsets): same bits as the unsplit forward and as the oracle; called on a side stream right
    behind the copy that delivers the images, twice in a row with different images (the second call must not
    overtake the first on the library's own stream), and once more after the hook is reset."""
    import torch
    net = wl.make_resnet(arch, seed=31 + N, image_hw=hw, int32_shortcut=(arch == 50))
    xa = wl.make_image_batch(3, N, image_hw=hw)
    xb = wl.make_image_batch(4, N, image_hw=hw)
    want_a, want_b = onet.forward(net, xa), onet.forward(net, xb)
    hn = hawq.HawqNet(arch, net["layers"], net["pool_b"], net["pool_c"], image_hw=hw)
    try:
        hawq.hawq_tune_set_split(first)
        assert hn.split_first(N) == (first if first else (0 if hw % 2 else 56))
        ws = torch.empty(hn.workspace_bytes(N), dtype=torch.uint8, device="cuda")
        ws.fill_(0xA5)
        side = torch.cuda.Stream()
        pinned_a, pinned_b = torch.from_numpy(xa).pin_memory(), torch.from_numpy(xb).pin_memory()
        xd = torch.empty(xa.shape, dtype=torch.uint8, device="cuda")
        la = torch.zeros((N, 1000), dtype=torch.int32, device="cuda")
        lb = torch.zeros((N, 1000), dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            xd.copy_(pinned_a, non_blocking=True)
            hn.hawq_forward_resnet(xd, N, la, ws, side.cuda_stream)
            xd.copy_(pinned_b, non_blocking=True)          # overwrites the images: must wait for both parts of the first call
            hn.hawq_forward_resnet(xd, N, lb, ws, side.cuda_stream)
        side.synchronize()
        assert np.array_equal(la.cpu().numpy(), want_a)
        assert np.array_equal(lb.cpu().numpy(), want_b)
        hawq.hawq_tune_set_split(-1)
        lc = torch.zeros((N, 1000), dtype=torch.int32, device="cuda")
        hn.hawq_forward_resnet(xd, N, lc, ws)
        torch.cuda.synchronize()
        assert np.array_equal(lc.cpu().numpy(), want_b)
    finally:
        hawq.hawq_tune_set_split(0)
        hn.close()


def test_forward_captured_in_a_graph_replays_like_eager(hawq):
    """The forward (here split over the caller's stream and the library's second stream) recorded into a HIP graph:
    every replay, with new images and eager work in between, gives the eager bits."""
    import torch
    N = 12
    net = wl.make_resnet(18, seed=5, image_hw=64)
    hn = hawq.HawqNet(18, net["layers"], net["pool_b"], net["pool_c"], image_hw=64)
    try:
        hawq.hawq_tune_set_split(8)
        assert hn.split_first(N) == 8
        ws = torch.empty(hn.workspace_bytes(N), dtype=torch.uint8, device="cuda")
        x = torch.from_numpy(wl.make_image_batch(1, N, image_hw=64)).cuda()
        logits = torch.zeros((N, 1000), dtype=torch.int32, device="cuda")
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            hn.hawq_forward_resnet(x, N, logits, ws, s.cuda_stream)
            s.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s):
                hn.hawq_forward_resnet(x, N, logits, ws, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        for i in range(3):
            xi = wl.make_image_batch(20 + i, N, image_hw=64)
            x.copy_(torch.from_numpy(xi).cuda())
            logits.zero_()
            ws.fill_(i)
            g.replay()
            torch.cuda.synchronize()
            got = logits.cpu().numpy()
            logits.zero_()
            hn.hawq_forward_resnet(x, N, logits, ws)      # eager, between the replays
            torch.cuda.synchronize()
            assert np.array_equal(got, logits.cpu().numpy()), "replay %d" % i
            assert np.array_equal(got, onet.forward(net, xi)), "replay %d against the oracle" % i
    finally:
        hawq.hawq_tune_set_split(0)
        hn.close()


@pytest.mark.parametrize("N,hw,int32_sc", [(5, 224, True), (9, 112, False), (3, 64, True)])
def test_fused_bottleneck_tails_in_the_network(hawq, N, hw, int32_sc):
    """ResNet50 with the 3x3 -> 1x1 + shortcut tails of its identity blocks run as one launch each (the plan's rule keeps
    them as two launches; the hook forces the fused form): fewer launches that do work, same logits as the oracle and as
    the unfused plan."""
    import torch
    net = wl.make_resnet(50, seed=61, image_hw=hw, int32_shortcut=int32_sc)
    x = wl.make_image_batch(62, N, image_hw=hw)
    want = onet.forward(net, x)
    outs, working = [], []
    try:
        for mode in (0, 1):
            hawq.hawq_tune_set_fusion(mode)
            hn = hawq.HawqNet(50, net["layers"], net["pool_b"], net["pool_c"], image_hw=hw)
            ws = torch.full((hn.workspace_bytes(N),), 0x77, dtype=torch.uint8, device="cuda")
            logits = torch.zeros((N, 1000), dtype=torch.int32, device="cuda")
            hn.hawq_forward_resnet(torch.from_numpy(x).cuda(), N, logits, ws)
            torch.cuda.synchronize()
            outs.append(logits.cpu().numpy())
            working.append(sum(hn.step_cost(N, s)[0] > 0 for s in range(hn.num_steps())))
            hn.close()
    finally:
        hawq.hawq_tune_set_fusion(0)
    assert np.array_equal(outs[0], want) and np.array_equal(outs[1], want)
    # stage 2 (image side / 8 <= 28) and stage 3 (<= 14) identity blocks: 3 + 5 launches fewer at these image sizes
    assert working[0] - working[1] == 8, working
