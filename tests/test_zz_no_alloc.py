"""The selection entry point that allocates nothing, against the allocating one (and the oracle)."""
import numpy as np
import pytest

from paper_2110_10548_amd import workloads


@pytest.fixture(scope="module")
def B():
    from paper_2110_10548_amd import binding
    binding.lib()
    return binding


def _inputs(seed, n, torch):
    rng = workloads.SplitMix64(seed)
    cost = np.array([rng.below(997) / 8.0 for _ in range(n)], dtype=np.float64)          # many ties
    index = np.array([rng.next_u64() >> 16 for _ in range(n)], dtype=np.uint64)
    return cost, index, torch.from_numpy(cost).cuda(), torch.from_numpy(index.view(np.int64)).cuda()


@pytest.mark.gpu
def test_topk_without_allocation_matches_the_allocating_call(B, oracle):
    import torch
    nan = torch.zeros(1, dtype=torch.int32, device="cuda")
    # two calls in a row on the same fixed scratch, the second smaller (fewer stage-1 lists, shorter lists)
    for seed, n, k in ((11, 300_007, 64), (12, 4_099, 10), (13, 50, 64)):
        cost, index, dc, di = _inputs(seed, n, torch)
        kk = min(k, n)
        ref = torch.full((kk,), -7, dtype=torch.int64, device="cuda")
        got = torch.full((kk,), -7, dtype=torch.int64, device="cuda")
        B.p2_topk_device(dc.data_ptr(), 1, di.data_ptr(), n, k, ref.data_ptr())
        free_before = torch.cuda.mem_get_info()[0]
        B.p2_topk_device_noalloc(dc.data_ptr(), 1, di.data_ptr(), n, k, got.data_ptr(), nan.data_ptr())
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before
        assert got.cpu().tolist() == ref.cpu().tolist() == oracle.topk(cost, index, k).tolist()
        assert int(nan.item()) == 0
    # a NaN is flagged on the device and left out of the list
    cost, index, dc, di = _inputs(14, 1000, torch)
    dc[17] = float("nan")
    got = torch.full((5,), -7, dtype=torch.int64, device="cuda")
    B.p2_topk_device_noalloc(dc.data_ptr(), 1, di.data_ptr(), 1000, 5, got.data_ptr(), nan.data_ptr())
    torch.cuda.synchronize()
    cost[17] = np.inf
    assert int(nan.item()) == 1 and got.cpu().tolist() == oracle.topk(cost, index, 5).tolist()
    # strided costs, no flag word
    cost, index, dc, di = _inputs(15, 2048, torch)
    wide = torch.zeros((2048, 3), dtype=torch.float64, device="cuda")
    wide[:, 1] = dc
    got = torch.full((8,), -7, dtype=torch.int64, device="cuda")
    B.p2_topk_device_noalloc(wide.data_ptr() + 8, 3, di.data_ptr(), 2048, 8, got.data_ptr())
    torch.cuda.synchronize()
    assert got.cpu().tolist() == oracle.topk(cost, index, 8).tolist()
    with pytest.raises(B.P2Error) as e:
        B.p2_topk_device_noalloc(dc.data_ptr(), 1, di.data_ptr(), 2048, 65, got.data_ptr())
    assert e.value.code == B.P2_EUNSUPPORTED
