"""GPU test of the entry point that allocates nothing: hawq_forward_resnet_noalloc (its workspace is a fixed array in
the library's device code) against hawq_forward_resnet (caller's workspace) and the oracle, two calls in a row, the
second with a smaller batch; requests beyond the array's size are refused."""
import numpy as np
import pytest

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


@pytest.mark.parametrize("arch,hw,N1,N2", [(50, 64, 7, 3), (18, 96, 12, 5)])
def test_noalloc_forward_equals_the_workspace_forward(hawq, arch, hw, N1, N2):
    import torch
    net = wl.make_resnet(arch, seed=200 + arch, image_hw=hw, int32_shortcut=(arch == 50))
    hn = hawq.HawqNet(arch, net["layers"], net["pool_b"], net["pool_c"], image_hw=hw)
    try:
        limit = hawq.hawq_noalloc_workspace_limit()
        assert limit == 64 << 20
        for call, N in enumerate((N1, N2)):          # the second call is smaller and finds the first call's leftovers
            x = wl.make_image_batch(300 + call, N, image_hw=hw)
            xd = torch.from_numpy(x).cuda()
            assert hn.workspace_bytes(N) <= limit
            ws = torch.full((hn.workspace_bytes(N),), 0x33, dtype=torch.uint8, device="cuda")
            ref = torch.zeros((N, 1000), dtype=torch.int32, device="cuda")
            hn.hawq_forward_resnet(xd, N, ref, ws)
            got = torch.full((N, 1000), -1, dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            free_before = torch.cuda.mem_get_info()[0]      # device memory not allocated by anyone (hipMemGetInfo)
            hn.hawq_forward_resnet_noalloc(xd, N, got)
            torch.cuda.synchronize()
            assert torch.cuda.mem_get_info()[0] >= free_before, "the call allocated device memory"
            assert np.array_equal(got.cpu().numpy(), ref.cpu().numpy()), "call %d (batch %d)" % (call, N)
            assert np.array_equal(got.cpu().numpy(), onet.forward(net, x)), "call %d against the oracle" % call
    finally:
        hn.close()


def test_noalloc_forward_refuses_what_does_not_fit(hawq):
    import torch
    net = wl.make_resnet(18, seed=11, image_hw=64)
    hn = hawq.HawqNet(18, net["layers"], net["pool_b"], net["pool_c"], image_hw=64)
    try:
        limit = hawq.hawq_noalloc_workspace_limit()
        N = 1
        while hn.workspace_bytes(N) <= limit:
            N *= 2
        x = torch.zeros((N, 64, 64, 3), dtype=torch.uint8, device="cuda")
        logits = torch.full((N, 1000), 7, dtype=torch.int32, device="cuda")
        with pytest.raises(hawq.HawqError) as e:
            hn.hawq_forward_resnet_noalloc(x, N, logits)
        assert e.value.status == 8          # HAWQ_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert int((logits != 7).sum()) == 0   # nothing was launched
        with pytest.raises(hawq.HawqError) as e:
            hn.hawq_forward_resnet_noalloc(x, 0, logits)
        assert e.value.status == 2
    finally:
        hn.close()
