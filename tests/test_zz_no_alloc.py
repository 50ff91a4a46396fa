"""f3d_psh_bucketize_static (the entry point for callers that cannot allocate) against f3d_psh_bucketize, through the
C ABI: bit-identical outputs on two calls in a row, the second on a smaller input, plus the size limit."""
import numpy as np
import pytest
import torch

import paper_2412_16481_amd as f3d
from paper_2412_16481_amd import workloads as wl

pytestmark = pytest.mark.gpu


def both(coords, bo, params):
    c = torch.from_numpy(coords).cuda()
    b = None if bo is None else torch.from_numpy(bo).cuda()
    want = f3d.psh_bucketize(c, b, params)
    got = f3d.psh_bucketize(c, b, params, static_scratch=True)
    torch.cuda.synchronize()
    k = int(want.scan_bucket_start[-1])
    assert k >= 0 and int(got.scan_bucket_start[-1]) == k
    assert torch.equal(got.perm, want.perm)
    assert torch.equal(got.inv_perm, want.inv_perm)
    assert torch.equal(got.offsets[:k + 1], want.offsets[:k + 1])
    assert torch.equal(got.scan_bucket_start, want.scan_bucket_start)
    assert torch.equal(got.placed_per_round, want.placed_per_round)
    # and it is the oracle's permutation too: a permutation of all rows
    assert np.array_equal(np.sort(got.perm.cpu().numpy()), np.arange(coords.shape[0]))


def test_static_scratch_matches_the_workspace_entry_point_twice_in_a_row():
    big = wl.make_workload("lidar4")
    both(big.coords, big.batch_offsets, f3d.make_params(big.voxel_size, big.bucket_cap))
    small = wl.make_workload("tiny")
    both(small.coords, small.batch_offsets, f3d.make_params(small.voxel_size, small.bucket_cap, hash="xor_mod"))
    # every launch schedule and the canonical order share the buffer as well
    rng = np.random.default_rng(5)
    pts = rng.uniform(0, 3, (30011, 3)).astype(np.float32)
    bo = np.array([0, 9000, 9000, 30011], np.int32)
    for kw in (dict(schedule="general"), dict(schedule="steps"), dict(schedule="scans"), dict(order="canonical")):
        both(pts, bo, f3d.make_params(0.03, 256, **kw))


def test_static_scratch_refuses_what_does_not_fit_and_allocates_nothing():
    n = 4_000_000
    p = f3d.make_params(0.05, 4096)
    assert f3d.workspace_bytes(n, 1, p) > f3d.STATIC_SCRATCH_BYTES
    c = torch.zeros(n, 3, device="cuda")
    with pytest.raises(f3d.Flash3DError) as e:
        f3d.psh_bucketize(c, None, p, static_scratch=True)
    assert e.value.code == f3d.ERR_SCRATCH_LIMIT
    del c
    w = wl.make_workload("indoor")
    p = f3d.make_params(w.voxel_size, w.bucket_cap)
    c = torch.from_numpy(w.coords).cuda()
    out = f3d.psh_bucketize(c, None, p, static_scratch=True)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    f3d.psh_bucketize(c, None, p, out=out, static_scratch=True)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
