"""The allocation-free entry point gives ffps_exact's results bit for bit: called
through the C ABI twice in a row, the second time on a smaller input (the
device-resident scratch array keeps the first call's contents in between), and
it allocates no device memory while doing so."""
import numpy as np
import pytest

from paper_2604_17720_amd import inputs

pytestmark = pytest.mark.gpu

GRID = 2


@pytest.fixture(scope="module")
def fb():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2604_17720_amd.binding as b
    b.lib()
    return b


def _both(fb, x, M, start, variant):
    """(index, distance bits) of ffps_exact and of ffps_exact_noalloc on the same cloud."""
    import torch
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    B = xd.shape[0]
    ws = fb.make_workspace(B, xd.shape[1], M)
    idx, md = fb.ffps_exact(xd, M, start, variant, return_maxdist=True, workspace=ws)
    assert fb.ffps_last_status(ws) == 0
    out = torch.full((B, M), -1, dtype=torch.int32, device="cuda")
    omd = torch.zeros((B, M), dtype=torch.float32, device="cuda")
    st = torch.full((2,), 77, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    fb.ffps_exact_noalloc(xd, M, out, start, variant, out_maxdist=omd, out_status=st)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    assert after == before                      # no allocation through torch either
    assert fb.ffps_last_status(st) == 0
    assert fb.ffps_last_rounds(st) == fb.ffps_last_rounds(ws)
    return (idx.cpu().numpy(), md.cpu().numpy().view(np.uint32),
            out.cpu().numpy(), omd.cpu().numpy().view(np.uint32))


@pytest.mark.parametrize("variant", [0, GRID])
def test_two_calls_in_a_row_second_one_smaller(fb, oracle, variant):
    big = inputs.make_config(4, N=60000)                 # all CUs, one cloud
    small = np.stack([inputs.planes_and_clusters(9000, 8100 + i) for i in range(3)])  # three clusters
    for x, M, start in ((big, 900, 0), (small, 300, 8999)):
        print(f"no-alloc N={x.shape[1]} B={x.shape[0]} M={M} variant={variant}", flush=True)
        i0, d0, i1, d1 = _both(fb, x, M, start, variant)
        assert np.array_equal(i0, i1)
        assert np.array_equal(d0, d1)
        assert np.array_equal(i1, oracle.fps_exact(x, M, start))


def test_small_clouds_and_limits(fb, oracle):
    import torch
    x = inputs.make_config(2, B=5)                       # one workgroup per cloud
    i0, d0, i1, d1 = _both(fb, x, 512, 0, 0)
    assert np.array_equal(i0, i1) and np.array_equal(d0, d1)
    xd = torch.from_numpy(x).cuda()
    out = torch.empty((5, 512), dtype=torch.int32, device="cuda")
    with pytest.raises(fb.FlashFPSError) as e:           # streaming needs a distance array
        fb.ffps_exact_noalloc(xd, 512, out, 0, fb.FFPS_VARIANT_STREAM)
    assert e.value.code == fb.FFPS_ERR_UNSUPPORTED_SIZE
