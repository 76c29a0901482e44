"""The allocation-free entry point (ivfpq_search_noalloc: workspace in a static device array
inside the library) against ivfpq_search with a caller workspace, through the C ABI: ids and
distance bits must be equal, on calls in a row that share the static array (a large batch,
then a smaller one, then one that splits its probes over several workgroups), and sizes
beyond the array are refused without touching the outputs."""
import numpy as np
import pytest
import torch

from paper_2312_01712_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_search_noalloc_matches_search_on_consecutive_calls():
    from paper_2312_01712_amd import binding as b
    b.load_library()
    assert torch.cuda.is_available()
    # 64-subspace shape (the specialised kernel), 96 lists, ragged sizes
    w = wl.Workload("noalloc", 60_000, 128, 96, 64, 3000, 12, 100, "sift", 96, 20.0)
    idx, centres = wl.train_index(w)
    q_all = wl.queries(w, centres).cuda()
    gi = b.IvfPqIndex.from_index(idx)
    radii = wl.calibrate_radii(w, idx, centres, 0.25)
    inf = np.full(idx.M, np.inf, np.float32)
    # second call smaller than the first; then a tiny batch (probes split over workgroups + merge
    # kernel, partial lists in the scratch); then the large one again
    for Q, nprobe, k, r in ((3000, 12, 100, radii), (700, 7, 10, inf), (3, 12, 100, radii), (3000, 12, 128, inf)):
        print(f"  noalloc case Q={Q} nprobe={nprobe} k={k}", flush=True)
        q = q_all[:Q].contiguous()
        ref_ids, ref_dist = gi.search(q, nprobe, k, r)
        out = (torch.full((Q, k), -5, dtype=torch.int64, device="cuda"),
               torch.full((Q, k), -5.0, dtype=torch.float32, device="cuda"))
        ids, dist = gi.search_noalloc(q, nprobe, k, r, out)
        torch.cuda.synchronize()
        assert torch.equal(ids, ref_ids), (Q, nprobe, k)
        assert torch.equal(dist.view(torch.int32), ref_dist.view(torch.int32)), (Q, nprobe, k)
    # an empty batch is a no-op
    e = (torch.empty((0, 5), dtype=torch.int64, device="cuda"), torch.empty((0, 5), dtype=torch.float32, device="cuda"))
    gi.search_noalloc(q_all[:0].contiguous(), 4, 5, radii, e)
    gi.close()


def test_search_noalloc_refuses_sizes_beyond_its_scratch():
    from paper_2312_01712_amd import binding as b
    b.load_library()
    # 40 000 lists: 128 queries x 40 000 floats of proposals fit, 9 000 000 (query, probe) pairs do not
    rng = np.random.default_rng(3)
    nlist, D, M, N = 40_000, 8, 4, 5000
    labels = np.sort(rng.integers(0, nlist, N))
    offs = np.zeros(nlist + 1, np.int64)
    offs[1:] = np.cumsum(np.bincount(labels, minlength=nlist))
    idx = wl.Index(N=N, D=D, nlist=nlist, M=M, centroids=rng.standard_normal((nlist, D)).astype(np.float32),
                   codebooks=rng.standard_normal((M, 256, D // M)).astype(np.float32), list_offsets=offs,
                   codes=rng.integers(0, 256, (N, M)).astype(np.uint8), ids=np.arange(N, dtype=np.int64))
    gi = b.IvfPqIndex.from_index(idx)
    radii = np.full(M, np.inf, np.float32)
    Q, nprobe, k = 9000, 1000, 5
    q = torch.from_numpy(rng.standard_normal((Q, D)).astype(np.float32)).cuda()
    out = (torch.full((Q, k), -5, dtype=torch.int64, device="cuda"), torch.full((Q, k), -5.0, dtype=torch.float32, device="cuda"))
    with pytest.raises(b.IvfpqError) as e:
        gi.search_noalloc(q, nprobe, k, radii, out)
    assert e.value.status == b.ERR_WORKSPACE and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out[0] == -5).all()) and bool((out[1] == -5.0).all())
    # the same index with a batch that fits: equal to the workspace call
    Q2 = 200
    ref = gi.search(q[:Q2].contiguous(), 16, k, radii)
    got = gi.search_noalloc(q[:Q2].contiguous(), 16, k, radii, (out[0][:Q2].contiguous(), out[1][:Q2].contiguous()))
    torch.cuda.synchronize()
    assert torch.equal(got[0], ref[0]) and torch.equal(got[1].view(torch.int32), ref[1].view(torch.int32))
    gi.close()
