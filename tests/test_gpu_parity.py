"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by
element on the same seeded inputs.

Bar: probe lists, keep masks, candidate sets and top-k ids are bit-exact; table
values and distances are compared bit for bit as well, because both sides use
the same fp32 operation order (the stated tolerance of 1e-4 relative is the
fallback reported in the assertion message if a bit differs).
"""

import numpy as np
import pytest
import torch

import oracle
from paper_2312_01712_amd import workloads as wl

from helpers import per_query_radii  # noqa: E402

pytestmark = pytest.mark.gpu

ORACLE_THREADS = 16   # the GPU machine gives a job 16 host cores

REL_TOL = 1e-4


def _binding():
    from paper_2312_01712_amd import binding
    return binding


def _cuda(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def say(*a):
    print(*a, flush=True)


def assert_same_float(gpu, ref, what):
    gpu, ref = np.asarray(gpu), np.asarray(ref)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    same = gpu.view(np.uint32) == ref.view(np.uint32)
    if not same.all():
        bad = np.argwhere(~same)
        rel = np.abs(gpu.astype(np.float64) - ref) / np.maximum(np.abs(ref), 1e-30)
        raise AssertionError(f"{what}: {bad.shape[0]} of {gpu.size} values differ in bits; "
                             f"max relative difference {np.nanmax(rel[~same]):.3e} "
                             f"(tolerance {REL_TOL}); first at {bad[0].tolist()}")


def cand_offsets(idx, probes):
    sizes = np.diff(idx.list_offsets)[probes].sum(1)
    offs = np.zeros(probes.shape[0] + 1, dtype=np.int64)
    offs[1:] = np.cumsum(sizes)
    return offs


def full_check(w, idx, q, radii, nprobe=None, k=None, stages=True, metric=0, mode=0):
    """All entry points against the oracle for one (index, queries, radii)."""
    b = _binding()
    nprobe = w.nprobe if nprobe is None else nprobe
    k = w.k if k is None else k
    say(f"  case {w.name}: N={idx.N} D={idx.D} nlist={idx.nlist} M={idx.M} Q={q.shape[0]} nprobe={nprobe} k={k}"
        + (f" metric={metric} mode={mode}" if metric or mode else ""))
    gi = b.IvfPqIndex.from_index(idx, metric=metric)
    dq = _cuda(q)
    okw = dict(mode=mode, metric=metric)
    o_pid, o_pd = oracle.coarse(q, idx.centroids, nprobe, metric=metric)
    if stages:
        pid, pd = gi.coarse(dq, nprobe)
        torch.cuda.synchronize()
        assert np.array_equal(pid.cpu().numpy(), o_pid), "probe lists differ"
        assert_same_float(pd.cpu().numpy(), o_pd, "probe distances")
        lut, mask = gi.build_lut(dq, _cuda(o_pid), radii, mode=mode)
        o_lut, o_mask = oracle.build_lut(q, idx.centroids, idx.codebooks, o_pid, radii, **okw)
        torch.cuda.synchronize()
        assert np.array_equal(mask.cpu().numpy().view(np.uint64), o_mask), "keep masks differ"
        assert_same_float(lut.cpu().numpy(), o_lut, "table values")
        o_offs, o_cd, o_ci = oracle.scan_all(q, idx, o_pid, radii, **okw)
        assert np.array_equal(o_offs, cand_offsets(idx, o_pid))
        cd, ci, err = gi.scan_all(dq, _cuda(o_pid), radii, _cuda(o_offs), mode=mode)
        torch.cuda.synchronize()
        assert int(err.item()) == 0
        assert np.array_equal(ci.cpu().numpy(), o_ci), "candidate sets differ"
        assert_same_float(cd.cpu().numpy(), o_cd, "candidate distances")
        ids2, dist2 = gi.scan_topk(dq, _cuda(o_pid), k, radii, mode=mode)
    ids, dist = gi.search(dq, nprobe, k, radii, mode=mode)
    torch.cuda.synchronize()
    o_ids, o_dist = oracle.search(q, idx, nprobe, k, radii, threads=8, **okw)
    assert np.array_equal(ids.cpu().numpy(), o_ids), "top-k ids differ"
    assert_same_float(dist.cpu().numpy(), o_dist, "top-k distances")
    # both ways of loading code blocks (whole, or first half with the rest on demand) must
    # give the same bits as the adaptive default
    for variant in (1, 2, 3):
        b.set_option("scan_loads", variant)
        try:
            ids_v, dist_v = gi.search(dq, nprobe, k, radii, mode=mode)
            torch.cuda.synchronize()
        finally:
            b.set_option("scan_loads", 0)
        assert np.array_equal(ids_v.cpu().numpy(), o_ids), f"top-k ids differ (scan_loads {variant})"
        assert_same_float(dist_v.cpu().numpy(), o_dist, f"top-k distances (scan_loads {variant})")
    if stages:
        assert np.array_equal(ids2.cpu().numpy(), o_ids) and np.array_equal(dist2.cpu().numpy(), dist.cpu().numpy())
    gi.close()
    return o_ids


@pytest.fixture(scope="module")
def lib():
    b = _binding()
    b.load_library()
    assert torch.cuda.is_available()
    return b


@pytest.mark.parametrize("name", ["T_gauss", "T_sift", "T_deep", "T_tti"])
@pytest.mark.parametrize("frac", [0.25, 1.0])
def test_tiny_workloads(lib, name, frac):
    w = wl.WORKLOADS[name]
    idx, centres = wl.train_index(w)
    q = wl.queries(w, centres).numpy()
    radii = wl.calibrate_radii(w, idx, centres, frac)
    full_check(w, idx, q, radii)
    # every list probed, and a single probe
    full_check(w, idx, q[:7], radii, nprobe=idx.nlist, k=w.k)
    full_check(w, idx, q[:7], radii, nprobe=1, k=w.k)


def _random_index(rng, N, D, nlist, M, sizes=None):
    """Untrained random index with a chosen list-size profile."""
    if sizes is None:
        sizes = rng.multinomial(N, np.ones(nlist) / nlist)
    sizes = np.asarray(sizes, dtype=np.int64)
    N = int(sizes.sum())
    offs = np.zeros(nlist + 1, dtype=np.int64)
    offs[1:] = np.cumsum(sizes)
    return wl.Index(N=N, D=D, nlist=nlist, M=M,
                    centroids=rng.normal(size=(nlist, D)).astype(np.float32),
                    codebooks=(0.5 * rng.normal(size=(M, 256, D // M))).astype(np.float32),
                    list_offsets=offs, codes=rng.integers(0, 256, size=(N, M), dtype=np.uint8),
                    ids=rng.permutation(N).astype(np.int64) * 3 + 1)


@pytest.mark.parametrize("M,D", [(64, 128), (48, 96), (100, 200), (16, 64), (12, 12), (5, 15), (128, 128), (7, 21)])
def test_shapes_ragged_and_empty_lists(lib, M, D):
    """Specialised (64/48/100/16 subspaces) and run-time-M kernels; lists that are
    empty, shorter than a block, exactly a block, and several blocks plus a tail."""
    rng = np.random.default_rng(M * 1000 + D)
    sizes = [0, 1, 63, 64, 65, 0, 130, 700, 5, 1500, 64 * 9, 0, 333, 2, 127, 129]
    idx = _random_index(rng, 0, D, len(sizes), M, sizes)
    q = rng.normal(size=(33, D)).astype(np.float32)
    w = wl.Workload(f"rand_M{M}", idx.N, D, idx.nlist, M, 33, 6, 100, "gauss", 1, 1.0)
    r = np.full(M, 0.9 * np.sqrt(D / M), dtype=np.float32)
    full_check(w, idx, q, r)
    full_check(w, idx, q[:5], np.full(M, np.inf, np.float32), nprobe=idx.nlist, k=128)
    full_check(w, idx, q[:3], r, nprobe=2, k=1)


@pytest.mark.parametrize("seed", range(12))
def test_random_odd_shapes(lib, seed):
    """Small random indexes in shapes no workload has: dsub 1-8, M from 1, a single list,
    empty lists, k above the number of candidates, infinite radii; both metrics, every stage."""
    rng = np.random.default_rng(2000 + seed)
    dsub = int(rng.choice([1, 2, 3, 4, 5, 8]))
    M = int(rng.choice([1, 2, 3, 7, 16]))
    D = M * dsub
    nlist = int(rng.choice([1, 2, 5, 9]))
    sizes = rng.integers(0, 200, size=nlist)
    if seed % 3 == 0 and nlist > 1:
        sizes[rng.integers(0, nlist)] = 0
    sizes[0] = max(sizes[0], 1)
    idx = _random_index(rng, 0, D, nlist, M, sizes)
    nprobe = int(rng.integers(1, nlist + 1))
    k = int(rng.choice([1, 3, 10, 100]))
    q = rng.normal(size=(9, D)).astype(np.float32)
    radii = (0.5 * np.sqrt(dsub) * rng.uniform(0.4, 1.6, size=M)).astype(np.float32)
    if seed % 4 == 1:
        radii[:] = np.inf
    w = wl.Workload(f"odd_{seed}", idx.N, D, nlist, M, 9, nprobe, k, "gauss", 1, 1.0)
    for metric in (0, 1):
        full_check(w, idx, q, radii, nprobe=nprobe, k=k, metric=metric)


@pytest.mark.parametrize("M,D", [(16, 64), (8, 16)])
def test_maximum_nprobe(lib, M, D):
    """nprobe at its limit of 1024: sixteen metadata chunks per query in one workgroup (large
    batch) and probes split over 64 workgroups (small batch); both metrics."""
    rng = np.random.default_rng(4 * M + 1)
    nlist = 1030
    sizes = rng.integers(0, 20, size=nlist)
    sizes[::50] = 0
    idx = _random_index(rng, 0, D, nlist, M, sizes)
    w = wl.Workload(f"maxprobe_M{M}", idx.N, D, nlist, M, 0, 1024, 100, "gauss", 1, 1.0)
    r = np.full(M, 0.8 * np.sqrt(D / M), dtype=np.float32)
    q = rng.normal(size=(2100, D)).astype(np.float32)
    full_check(w, idx, q[:3], r, nprobe=1024, k=100)
    full_check(w, idx, q, r, nprobe=1024, k=10, stages=False)
    full_check(w, idx, q[:3], r, nprobe=1024, k=100, metric=1)
    b = _binding()
    gi = b.IvfPqIndex.from_index(idx)
    with pytest.raises(b.IvfpqError) as e:
        gi.search(_cuda(q[:3]), 1025, 10, r)
    assert e.value.status == b.ERR_UNSUPPORTED
    gi.close()


@pytest.mark.parametrize("M,D", [(64, 128), (5, 15)])
def test_index_without_points(lib, M, D):
    """N = 0 is a valid index: every search returns k times (-1, +inf)."""
    rng = np.random.default_rng(77)
    idx = _random_index(rng, 0, D, 3, M, [0, 0, 0])
    assert idx.N == 0
    q = rng.normal(size=(5, D)).astype(np.float32)
    w = wl.Workload(f"empty_M{M}", 0, D, 3, M, 5, 2, 10, "gauss", 1, 1.0)
    for metric in (0, 1):
        o_ids = full_check(w, idx, q, np.full(M, 0.5, np.float32), nprobe=2, k=10, metric=metric)
        assert np.all(o_ids == -1)


@pytest.mark.parametrize("M,D", [(64, 128), (16, 64), (6, 12)])
def test_many_probes(lib, M, D):
    """More probed lists than the kernel stages metadata for at once (64), with and
    without the probes of a query being split over several workgroups."""
    rng = np.random.default_rng(5 + M)
    nlist = 300
    sizes = rng.integers(0, 90, size=nlist)
    sizes[::37] = 0
    idx = _random_index(rng, 0, D, nlist, M, sizes)
    w = wl.Workload(f"probes_M{M}", idx.N, D, nlist, M, 0, 150, 100, "gauss", 1, 1.0)
    r = np.full(M, 0.8 * np.sqrt(D / M), dtype=np.float32)
    q = rng.normal(size=(3000, D)).astype(np.float32)
    full_check(w, idx, q[:9], r, nprobe=150, k=100)              # few queries: probes split over workgroups
    full_check(w, idx, q[:5], r, nprobe=300, k=128)
    full_check(w, idx, q, r, nprobe=130, k=20, stages=False)     # many queries: one workgroup per query


@pytest.mark.parametrize("M,D", [(64, 128), (16, 64), (6, 12)])
def test_more_than_128_neighbours(lib, M, D):
    """k above what one pass of the kernel keeps per query (128): results come from
    several passes and must still be the oracle's, including ties that straddle a
    pass boundary, fewer candidates than k, and hit-count scores."""
    b = _binding()
    rng = np.random.default_rng(77 + M)
    nlist = 24
    sizes = rng.integers(40, 400, size=nlist)
    sizes[3] = 0
    idx = _random_index(rng, 0, D, nlist, M, sizes)
    w = wl.Workload(f"bigk_M{M}", idx.N, D, nlist, M, 0, 8, 1000, "gauss", 1, 1.0)
    r = np.full(M, 0.8 * np.sqrt(D / M), dtype=np.float32)
    q = rng.normal(size=(2100, D)).astype(np.float32)
    for k in (129, 256, 1000, 1024):
        full_check(w, idx, q[:7], r, nprobe=8, k=k, stages=(k == 1000))   # probes split over workgroups
    full_check(w, idx, q, r, nprobe=6, k=300, stages=False)               # one workgroup per query
    full_check(w, idx, q[:5], np.zeros(M, np.float32), nprobe=8, k=700, stages=False)  # every candidate ties at 0
    o_ids = full_check(w, idx, q[:9], r, nprobe=1, k=1000, stages=False)               # one list: < k candidates
    assert (o_ids == -1).any()
    # candidates end inside the first pass, and exactly at its end
    for n_first in (100, 128):
        idx2 = _random_index(rng, 0, D, 4, M, [n_first, 0, 0, 0])
        idx2.centroids[0] = 0.0
        idx2.centroids[1:] = 50.0
        w2 = wl.Workload("bigk_short", idx2.N, D, 4, M, 0, 1, 400, "gauss", 1, 1.0)
        o_ids = full_check(w2, idx2, (0.01 * q[:4]).astype(np.float32), r, nprobe=1, k=400, stages=False)
        assert (o_ids[:, :n_first] >= 0).all() and (o_ids[:, n_first:] == -1).all()
    # hit-count scores: a few distinct values, ties everywhere
    gi = b.IvfPqIndex.from_index(idx)
    for Q in (6, 2100):
        o_ids, o_dist = oracle.search(q[:Q], idx, 8, 500, r, threads=8, mode=1)
        ids, dist = gi.search(_cuda(q[:Q]), 8, 500, r, mode=1)
        assert np.array_equal(ids.cpu().numpy(), o_ids), Q
        assert_same_float(dist.cpu().numpy(), o_dist, f"hit counts, k=500, Q={Q}")
    gi.close()


@pytest.mark.parametrize("M,D", [(64, 128), (16, 64), (6, 12)])
def test_wide_selection_paths(lib, M, D):
    """k above 128 in one pass of the query-major scan (every key within the workgroup's bound
    kept in per-query slots, then sorted): the default slot count, few slots (the bound-driven
    compaction between lists runs, and queries that still overflow fall back to the pass-by-pass
    path), many slots (the batch goes through the slot arrays in chunks), and the pass-by-pass
    path alone when the caller's workspace has no room for slots.  All against the oracle."""
    b = _binding()
    rng = np.random.default_rng(177 + M)
    nlist = 20
    sizes = rng.integers(200, 1500, size=nlist)
    sizes[5] = 0
    sizes[7] = 3000          # one long list: more keys than the small slot counts hold
    idx = _random_index(rng, 0, D, nlist, M, sizes)
    r = np.full(M, 0.8 * np.sqrt(D / M), dtype=np.float32)
    q = rng.normal(size=(2100, D)).astype(np.float32)
    gi = b.IvfPqIndex.from_index(idx)
    assert gi.workspace(600, 8, 1000).numel() > gi.workspace(600, 8, 128).numel(), "no slots planned for k = 1000"
    cases = [(600, 8, 1000, 8192), (600, 8, 1000, 1024), (600, 8, 600, 2048), (300, 12, 1024, 4096),
             (2100, 6, 300, 65536), (40, 8, 129, 8192), (300, 8, 1000, 0)]
    try:
        for Q, nprobe, k, cap in cases:
            say(f"  wide selection: M={M} Q={Q} nprobe={nprobe} k={k} slots={cap}")
            if cap:
                b.set_option("wide_cap", cap)
            dq = _cuda(q[:Q])
            o_ids, o_dist = oracle.search(q[:Q], idx, nprobe, k, r, threads=ORACLE_THREADS)
            # cap 0: a workspace sized for k = 128 has no room for the slots
            ws = gi.workspace(Q, nprobe, k if cap else 128)
            ids, dist = gi.search(dq, nprobe, k, r, workspace=ws)
            torch.cuda.synchronize()
            assert np.array_equal(ids.cpu().numpy(), o_ids), (Q, nprobe, k, cap)
            assert_same_float(dist.cpu().numpy(), o_dist, f"wide selection k={k} slots={cap}")
        # every candidate at distance 0: more equal keys within the bound than the sort takes
        dq = _cuda(q[:50])
        zero = np.zeros(M, np.float32)
        b.set_option("wide_cap", 8192)
        o_ids, o_dist = oracle.search(q[:50], idx, 8, 700, zero, threads=ORACLE_THREADS)
        ids, dist = gi.search(dq, 8, 700, zero)
        assert np.array_equal(ids.cpu().numpy(), o_ids)
        assert_same_float(dist.cpu().numpy(), o_dist, "wide selection, all keys equal")
    finally:
        b.set_option("wide_cap", 8192)
        gi.close()


@pytest.mark.parametrize("metric", [0, 1])
def test_filtering_stage_many_lists(lib, metric):
    """Indexes with thousands of lists: the matrix product keeps, per query and group of 64
    lists, its six smallest values instead of writing rows, and the selection works on those.
    Random centroids (the usual case: no query flagged), a list count that is no multiple of the
    tile, and centroids sorted along a line, where a query's nearest lists are neighbours in list
    order, so that groups fill up and the flagged queries take the reference-order path."""
    b = _binding()
    rng = np.random.default_rng(4100 + metric)
    D, M = 32, 4
    cases = [("random", 9000, 16, 700), ("ragged tile", 16384 + 77, 64, 300), ("sorted line", 8192, 20, 200),
             ("zero centroids", 7000, 12, 50), ("60 000 lists", 60000, 32, 100)]
    for name, nlist, nprobe, Q in cases:
        sizes = np.zeros(nlist, dtype=np.int64)
        sizes[rng.integers(0, nlist, size=50)] = 3
        idx = _random_index(rng, 0, D, nlist, M, sizes)
        q = rng.normal(size=(Q, D)).astype(np.float32)
        if name == "sorted line":
            idx.centroids[:] = 0.0
            idx.centroids[:, 0] = np.arange(nlist, dtype=np.float32) * 0.01
            q[:, 0] = rng.uniform(5.0, 70.0, size=Q).astype(np.float32)
            q[:, 1:] *= 0.01
        if name == "zero centroids":     # proposal values of exactly 0 and equal values everywhere
            idx.centroids[: nlist // 2] = 0.0
            q[:10] = 0.0
        say(f"  filtering, many lists ({name}): nlist={nlist} nprobe={nprobe} Q={Q} metric={metric}")
        gi = b.IvfPqIndex.from_index(idx, metric=metric)
        b.coarse_fallbacks(reset=True)
        pid, pd = gi.coarse(_cuda(q), nprobe)
        torch.cuda.synchronize()
        fb = b.coarse_fallbacks()
        o_pid, o_pd = oracle.coarse(q, idx.centroids, nprobe, metric=metric)
        assert np.array_equal(pid.cpu().numpy(), o_pid), f"probe lists differ ({name})"
        assert_same_float(pd.cpu().numpy(), o_pd, f"probe distances ({name})")
        if name == "random":
            assert fb <= Q // 50, f"{fb} of {Q} queries took the reference-order path"
        if name == "sorted line" and metric == 0:
            assert fb >= Q // 2, f"only {fb} of {Q} queries took the reference-order path"
        gi.close()


def test_list_level_bound_on_odd_codebooks(lib):
    """The list-level bound uses, per two-dimensional subspace, a grid of nearest-entry distances
    over the bounding rectangle of the entries.  Codebooks that strain it: a subspace whose
    entries all coincide, one whose entries lie on a line, one with a huge offset and a tiny
    spread, one with a huge spread; queries on entries, on centroids, far outside every
    rectangle; radii small enough and k small enough for the bound to rule lists out.  With the
    grid forced on and forced off (option bound_grid), query-major and list-major: the oracle's answer."""
    b = _binding()
    rng = np.random.default_rng(2024)
    M, D, nlist = 16, 32, 40
    sizes = rng.integers(100, 600, size=nlist)
    idx = _random_index(rng, 0, D, nlist, M, sizes)
    cb = idx.codebooks                                   # [M][256][2]
    cb[0] = 0.25                                         # all entries equal
    cb[1, :, 1] = 0.0                                    # on a line
    cb[2] = 1.0e6 + 1.0e-2 * rng.normal(size=(256, 2))   # huge offset, tiny spread
    cb[3] = 1.0e4 * rng.normal(size=(256, 2))            # huge spread
    cb[4, :, 0] = cb[4, 0, 0]                            # a vertical line
    q = np.concatenate([idx.centroids[:8],                                         # residual 0
                        idx.centroids[8:16] + np.tile(cb[:, 7, :].reshape(-1), (8, 1)),   # on an entry of every subspace
                        1.0e3 * rng.normal(size=(8, D)),                          # far outside
                        rng.normal(size=(400, D))]).astype(np.float32)
    gi = b.IvfPqIndex.from_index(idx)
    try:
        for r in (np.full(M, 0.5, np.float32), np.full(M, 3.0, np.float32), np.full(M, np.inf, np.float32)):
            for nprobe, k in ((12, 5), (40, 100)):
                o_ids, o_dist = oracle.search(q, idx, nprobe, k, r, threads=ORACLE_THREADS)
                for grid in (1, 2):
                    for strategy in (b.SCAN_QUERY_MAJOR, b.SCAN_LIST_MAJOR):
                        b.set_option("bound_grid", grid)
                        ids, dist = gi.search(_cuda(q), nprobe, k, r, strategy=strategy)
                        torch.cuda.synchronize()
                        assert np.array_equal(ids.cpu().numpy(), o_ids), (float(r[0]), nprobe, k, grid, strategy)
                        assert_same_float(dist.cpu().numpy(), o_dist, f"odd codebooks r={r[0]} grid={grid}")
    finally:
        b.set_option("bound_grid", 0)
        gi.close()


def test_fewer_candidates_than_k_and_empty_probes(lib):
    rng = np.random.default_rng(11)
    sizes = [0, 3, 0, 0, 40, 0, 0, 2]
    idx = _random_index(rng, 0, 32, len(sizes), 8, sizes)
    q = np.concatenate([idx.centroids[[0, 2, 3, 5, 6]] + 0.01, rng.normal(size=(20, 32)).astype(np.float32)]).astype(np.float32)
    w = wl.Workload("sparse", idx.N, 32, idx.nlist, 8, q.shape[0], 2, 50, "gauss", 1, 1.0)
    o_ids = full_check(w, idx, q, np.full(8, np.inf, np.float32))
    assert (o_ids == -1).any()
    full_check(w, idx, q, np.full(8, 0.5, np.float32), nprobe=1, k=10)


def test_empty_index_and_single_point(lib):
    """N = 0 (every list empty) and N = 1."""
    rng = np.random.default_rng(13)
    for sizes in ([0, 0, 0, 0], [0, 0, 1, 0]):
        for M, D in ((64, 128), (5, 10)):
            idx = _random_index(rng, 0, D, len(sizes), M, sizes)
            q = rng.normal(size=(6, D)).astype(np.float32)
            w = wl.Workload("empty", idx.N, D, idx.nlist, M, 6, 3, 10, "gauss", 1, 1.0)
            o_ids = full_check(w, idx, q, np.full(M, 1.0, np.float32))
            assert (o_ids[:, 1:] == -1).all()


def test_saturated_ties_resolved_by_id(lib):
    """Radius 0 clamps every entry to 0, so every candidate ties at distance 0 and
    the k smallest ids must win; small radii saturate most candidates at sum r_m^2."""
    rng = np.random.default_rng(12)
    idx = _random_index(rng, 5000, 32, 8, 16)
    q = rng.normal(size=(9, 32)).astype(np.float32)
    w = wl.Workload("ties", idx.N, 32, 8, 16, 9, 4, 100, "gauss", 1, 1.0)
    full_check(w, idx, q, np.zeros(16, np.float32))
    full_check(w, idx, q, np.full(16, 0.05, np.float32))
    full_check(w, idx, q, np.full(16, 0.3, np.float32), nprobe=8, k=128)


def test_identity_codebook_exact_knn(lib):
    """The oracle's brute-force pin, run through the HIP path: lossless codes and
    all lists probed give the exact k nearest neighbours."""
    from helpers import identity_index, brute_knn_int
    rng = np.random.default_rng(0)
    base, idx = identity_index(rng)
    queries = rng.integers(0, 128, size=(20, idx.D)).astype(np.int64)
    b = _binding()
    gi = b.IvfPqIndex.from_index(idx)
    ids, dist = gi.search(_cuda(queries.astype(np.float32)), idx.nlist, 15, np.full(idx.M, np.inf, np.float32))
    ref_ids, ref_dist = brute_knn_int(base, queries, 15)
    assert np.array_equal(ids.cpu().numpy(), ref_ids)
    assert np.array_equal(dist.cpu().numpy().astype(np.int64), ref_dist)


@pytest.mark.parametrize("name", ["T_gauss", "T_sift", "T_tti"])
def test_hit_count_scoring_and_per_query_radii(lib, name):
    """The *_ex entry points: hit-count (mode 1) and reward/penalty (mode 2) scoring, and
    radii given per query on the device, each against the oracle, every stage."""
    b = _binding()
    w = wl.WORKLOADS[name]
    idx, centres = wl.train_index(w)
    q = wl.queries(w, centres).numpy()
    shared = wl.calibrate_radii(w, idx, centres, 0.25)
    rq = per_query_radii(w, idx, centres, q, 0.25)
    gi = b.IvfPqIndex.from_index(idx)
    dq = _cuda(q)
    o_pid, _ = oracle.coarse(q, idx.centroids, w.nprobe)
    offs = cand_offsets(idx, o_pid)
    for mode in (0, 1, 2):
        for radii, d_rq in ((shared, None), (rq, _cuda(rq))):
            kw = dict(mode=mode, query_radii=d_rq)
            host_r = shared if d_rq is None else None
            lut, mask = gi.build_lut(dq, _cuda(o_pid), host_r, **kw)
            o_lut, o_mask = oracle.build_lut(q, idx.centroids, idx.codebooks, o_pid, radii, mode=mode)
            assert np.array_equal(mask.cpu().numpy().view(np.uint64), o_mask), (mode, d_rq is not None)
            assert_same_float(lut.cpu().numpy(), o_lut, f"table values mode {mode}")
            cd, ci, err = gi.scan_all(dq, _cuda(o_pid), host_r, _cuda(offs), **kw)
            _, o_cd, o_ci = oracle.scan_all(q, idx, o_pid, radii, mode=mode)
            assert int(err.item()) == 0 and np.array_equal(ci.cpu().numpy(), o_ci)
            assert_same_float(cd.cpu().numpy(), o_cd, f"candidate scores mode {mode}")
            o_ids, o_dist = oracle.search(q, idx, w.nprobe, w.k, radii, mode=mode)
            for ids, dist in (gi.search(dq, w.nprobe, w.k, host_r, **kw),
                              gi.scan_topk(dq, _cuda(o_pid), w.k, host_r, **kw)):
                assert np.array_equal(ids.cpu().numpy(), o_ids), (mode, d_rq is not None)
                assert_same_float(dist.cpu().numpy(), o_dist, f"top-k mode {mode}")
    with pytest.raises(b.IvfpqError) as e:
        gi.search(dq, w.nprobe, w.k, shared, mode=3)
    assert e.value.status == b.ERR_INVALID_ARGUMENT
    gi.close()


def _model_arrays(md):
    return md["lo"], md["cells_per_unit"], md["map"], md["coef"], md["fallback"]


@pytest.mark.parametrize("name", ["T_sift", "T_deep", "T_tti", "C2"])
def test_dynamic_thresholds(lib, name):
    """ivfpq_query_radii against the oracle, bit for bit: fitted model (100 x 100 maps),
    several scales, queries far outside the map, and the search that consumes the radii."""
    b = _binding()
    w = wl.WORKLOADS[name]
    big = name == "C2"
    idx, centres = wl.train_index(w, device="cuda" if big else "cpu")
    q = wl.queries(w, centres).cpu().numpy()
    md = wl.fit_radius_model(w, idx, centres, 0.25)
    gi = b.IvfPqIndex.from_index(idx)
    rm = b.RadiusModel(gi, *_model_arrays(md))
    # a third of the queries pushed away from the data: projections leave the map on every side
    rng = np.random.default_rng(9)
    q = q.copy()
    far = rng.choice(q.shape[0], q.shape[0] // 3, replace=False)
    q[far] += rng.normal(0, 4 * np.abs(q).mean(), size=(far.size, q.shape[1])).astype(np.float32)
    dq = _cuda(q)
    pid, _ = gi.coarse(dq, w.nprobe)
    o_pid, _ = oracle.coarse(q, idx.centroids, 1)
    assert np.array_equal(pid.cpu().numpy()[:, 0], o_pid[:, 0])
    for scale in (1.0, 0.5, 1.7):
        say(f"[{name}] query radii, scale {scale}")
        r = gi.query_radii(rm, dq, pid, scale)
        o_r = oracle.query_radii(q, idx.centroids, o_pid[:, 0], *_model_arrays(md), scale)
        assert_same_float(r.cpu().numpy(), o_r, f"{name} radii scale {scale}")
    assert np.all(o_r > 0) and len(np.unique(o_r)) > 10
    # the radii feed the search: same result as the oracle's search with the oracle's radii
    r = gi.query_radii(rm, dq, pid, 1.0)
    o_r = oracle.query_radii(q, idx.centroids, o_pid[:, 0], *_model_arrays(md), 1.0)
    sample = np.arange(q.shape[0]) if not big else rng.choice(q.shape[0], 32, replace=False)
    ids, dist = gi.search(dq, w.nprobe, w.k, None, query_radii=r)
    o_ids, o_dist = oracle.search(q[sample], idx, w.nprobe, w.k, o_r[sample], threads=8)
    assert np.array_equal(ids.cpu().numpy()[sample], o_ids)
    assert_same_float(dist.cpu().numpy()[sample], o_dist, f"{name} search with dynamic radii")
    rm.close()
    gi.close()


def test_dynamic_threshold_model_edge_cases(lib):
    """Hand-made models: 1 x 1 grid, degree 0 and degree 8, polynomial values that are
    negative, zero, infinite (fallback), a first probe id outside the index (fallback),
    Q = 0, and the argument errors."""
    b = _binding()
    rng = np.random.default_rng(3)
    M, nlist, N, Q = 5, 7, 300, 257
    cent = rng.normal(size=(nlist, 2 * M)).astype(np.float32)
    cb = rng.normal(size=(M, 256, 2)).astype(np.float32)
    offs = np.linspace(0, N, nlist + 1).astype(np.int64)
    codes = rng.integers(0, 256, size=(N, M)).astype(np.uint8)
    gi = b.IvfPqIndex(cent, cb, offs, codes)
    q = rng.normal(size=(Q, 2 * M)).astype(np.float32) * 2
    near = rng.integers(0, nlist, size=(Q, 3)).astype(np.int32)
    for G, degree in ((1, 0), (4, 8), (37, 3), (1024, 1)):
        lo = rng.uniform(-3, -1, size=(M, 2)).astype(np.float32)
        cpu = (G / rng.uniform(2, 6, size=(M, 2))).astype(np.float32)
        fmap = rng.uniform(0, 2, size=(M, G, G)).astype(np.float32)
        coef = rng.normal(size=(M, degree + 1)).astype(np.float32)   # about half the values come out negative
        if degree == 3:
            coef[0, 3] = 3e38                                         # overflows to inf: fallback
            coef[1, :] = 0.0                                          # exactly zero: fallback
        fb = rng.uniform(0.5, 1.5, size=M).astype(np.float32)
        rm = b.RadiusModel(gi, lo, cpu, fmap, coef, fb)
        r = gi.query_radii(rm, _cuda(q), _cuda(near), 0.75)
        o_r = oracle.query_radii(q, cent, near[:, 0], lo, cpu, fmap, coef, fb, 0.75)
        assert_same_float(r.cpu().numpy(), o_r, f"grid {G} degree {degree}")
        if degree == 3:
            assert np.array_equal(o_r[:, 1], np.full(Q, fb[1] * np.float32(0.75)))
        # a first probe id outside [0, nlist): that query gets the fallback
        bad = near.copy()
        bad[5, 0], bad[6, 0] = -1, nlist
        r = gi.query_radii(rm, _cuda(q), _cuda(bad), 2.0).cpu().numpy()
        assert np.array_equal(r[5], fb * np.float32(2.0)) and np.array_equal(r[6], fb * np.float32(2.0))
        assert gi.query_radii(rm, _cuda(q[:0]), _cuda(near[:0]), 1.0).shape == (0, M)
        for scale in (-1.0, float("nan"), float("inf")):
            with pytest.raises(b.IvfpqError) as e:
                gi.query_radii(rm, _cuda(q), _cuda(near), scale)
            assert e.value.status == b.ERR_INVALID_ARGUMENT
        rm.close()
    # descriptions the library must refuse
    lo = np.zeros((M, 2), np.float32)
    cpu = np.ones((M, 2), np.float32)
    fb = np.ones(M, np.float32)
    good = dict(lo=lo, cells_per_unit=cpu, fmap=np.zeros((M, 3, 3), np.float32), coef=np.ones((M, 2), np.float32),
                fallback=fb)
    b.RadiusModel(gi, **good).close()
    bad_cases = [
        dict(good, cells_per_unit=np.zeros((M, 2), np.float32)),               # cell width infinite
        dict(good, lo=np.full((M, 2), np.nan, np.float32)),
        dict(good, fallback=-fb),
        dict(good, coef=np.ones((M, 10), np.float32)),                          # degree 9
        dict(good, fmap=np.zeros((M, 1025, 1025), np.float32)),                 # grid above the limit
    ]
    for kw in bad_cases:
        with pytest.raises(b.IvfpqError) as e:
            b.RadiusModel(gi, **kw)
        assert e.value.status == b.ERR_INVALID_ARGUMENT
    other_m = dict(lo=np.zeros((M + 1, 2), np.float32), cells_per_unit=np.ones((M + 1, 2), np.float32),
                   fmap=np.zeros((M + 1, 3, 3), np.float32), coef=np.ones((M + 1, 2), np.float32),
                   fallback=np.ones(M + 1, np.float32))
    with pytest.raises(b.IvfpqError) as e:
        b.RadiusModel(gi, **other_m)                                            # M differs from the index's
    assert e.value.status == b.ERR_INVALID_ARGUMENT
    gi.close()
    # an index whose subspaces are not two-dimensional has no density map
    gi4 = b.IvfPqIndex(rng.normal(size=(nlist, 4 * M)).astype(np.float32),
                       rng.normal(size=(M, 256, 4)).astype(np.float32), offs, codes)
    with pytest.raises(b.IvfpqError) as e:
        b.RadiusModel(gi4, **good)
    assert e.value.status == b.ERR_UNSUPPORTED
    gi4.close()


def test_hit_count_scoring_1m(lib):
    """Hit-count scoring on the 1M x 128 configuration (specialised kernel, ties en masse)."""
    b = _binding()
    w = wl.WORKLOADS["C2"]
    idx, centres = wl.train_index(w, device="cuda")
    q = wl.queries(w, centres).cpu().numpy()
    radii = wl.calibrate_radii(w, idx, centres, 0.25)
    rq = per_query_radii(w, idx, centres, q, 0.25)
    gi = b.IvfPqIndex.from_index(idx)
    sample = np.sort(np.random.default_rng(2).choice(w.Q, 256, replace=False))
    for mode, r, d_rq in ((1, radii, None), (2, radii, None), (0, rq, _cuda(rq)), (2, rq, _cuda(rq))):
        ids, dist = gi.search(_cuda(q), w.nprobe, w.k, radii if d_rq is None else None, mode=mode, query_radii=d_rq)
        rs = r if d_rq is None else r[sample]
        o_ids, o_dist = oracle.search(q[sample], idx, w.nprobe, w.k, rs, threads=ORACLE_THREADS, mode=mode)
        assert np.array_equal(ids.cpu().numpy()[sample], o_ids), (mode, d_rq is not None)
        assert_same_float(dist.cpu().numpy()[sample], o_dist, f"C2 mode {mode}")
        if mode:   # the byte table (default) and the float table give the same scores; so does the list-major scan
            try:
                b.set_option("scan_ablate", 128)
                ids_f, dist_f = gi.search(_cuda(q), w.nprobe, w.k, radii if d_rq is None else None, mode=mode, query_radii=d_rq)
            finally:
                b.set_option("scan_ablate", 0)
            ids_l, dist_l = gi.search(_cuda(q), w.nprobe, w.k, radii if d_rq is None else None, mode=mode,
                                      query_radii=d_rq, strategy=b.SCAN_LIST_MAJOR)
            for other_ids, other_dist in ((ids_f, dist_f), (ids_l, dist_l)):
                assert torch.equal(other_ids, ids) and torch.equal(other_dist.view(torch.int32), dist.view(torch.int32)), mode
    gi.close()


def _ip_radii(idx, q, frac):
    """Per-subspace radii that keep about `frac` of the entries under the inner-product keep
    rule (|q_m - e|^2 - |e|^2 <= r_m^2); input recipe only."""
    qm = q.astype(np.float64).reshape(q.shape[0], idx.M, 1, idx.dsub)
    ent = idx.codebooks.astype(np.float64)[None]
    g = ((qm - ent) ** 2).sum(-1) - (ent ** 2).sum(-1)
    r2 = np.quantile(g.transpose(1, 0, 2).reshape(idx.M, -1), frac, axis=1)
    return np.sqrt(np.maximum(r2, 0.0)).astype(np.float32)


@pytest.mark.parametrize("name", ["T_gauss", "T_sift", "T_deep", "T_tti"])
def test_inner_product_tiny_workloads(lib, name):
    """Inner-product metric, every stage and every scoring mode against the oracle."""
    w = wl.WORKLOADS[name]
    idx, centres = wl.train_index(w)
    q = wl.queries(w, centres).numpy()
    for frac in (0.3, 1.0):
        radii = _ip_radii(idx, q, frac) if frac < 1.0 else np.full(idx.M, np.inf, np.float32)
        for mode in (0, 1, 2):
            full_check(w, idx, q, radii, metric=1, mode=mode)
    radii = _ip_radii(idx, q, 0.3)
    full_check(w, idx, q[:7], radii, nprobe=idx.nlist, metric=1)
    full_check(w, idx, q[:7], radii, nprobe=1, metric=1)
    # radii per query, on the device
    b = _binding()
    rq = np.stack([_ip_radii(idx, q[i:i + 1], 0.3) for i in range(q.shape[0])])
    gi = b.IvfPqIndex.from_index(idx, metric=b.METRIC_IP)
    assert gi.info()["metric"] == 1
    for mode in (0, 2):
        o_ids, o_dist = oracle.search(q, idx, w.nprobe, w.k, rq, mode=mode, metric=1)
        ids, dist = gi.search(_cuda(q), w.nprobe, w.k, None, mode=mode, query_radii=_cuda(rq))
        assert np.array_equal(ids.cpu().numpy(), o_ids), mode
        assert_same_float(dist.cpu().numpy(), o_dist, f"per-query radii, inner product, mode {mode}")
    gi.close()


@pytest.mark.parametrize("M,D", [(64, 128), (48, 96), (100, 200), (16, 64), (12, 12), (5, 15), (128, 128)])
def test_inner_product_shapes(lib, M, D):
    """Specialised and run-time-M kernels under the inner-product metric; ragged and empty
    lists; more probes than one metadata chunk; k above one pass; negative and positive scores."""
    rng = np.random.default_rng(M * 77 + D)
    sizes = [0, 1, 63, 64, 65, 0, 130, 700, 5, 1500, 64 * 9, 0, 333, 2, 127, 129]
    idx = _random_index(rng, 0, D, len(sizes), M, sizes)
    q = rng.normal(size=(33, D)).astype(np.float32)
    q[0] = 0.0                                                     # every score is zero: ties by id
    w = wl.Workload(f"ip_M{M}", idx.N, D, idx.nlist, M, 33, 6, 100, "gauss", 1, 1.0)
    r = _ip_radii(idx, q, 0.4)
    full_check(w, idx, q, r, metric=1)
    full_check(w, idx, q[:5], np.full(M, np.inf, np.float32), nprobe=idx.nlist, k=128, metric=1)
    full_check(w, idx, q[:5], r, nprobe=idx.nlist, k=700, metric=1, stages=False)
    full_check(w, idx, q[:3], np.zeros(M, np.float32), nprobe=2, k=1, metric=1)
    qs = rng.normal(size=(2100, D)).astype(np.float32)
    full_check(w, idx, qs, r, nprobe=5, k=150, metric=1, stages=False)   # one workgroup per query, two passes
    nlist = 200
    idx2 = _random_index(rng, 0, D, nlist, M, rng.integers(0, 90, size=nlist))
    w2 = wl.Workload(f"ip_probes_M{M}", idx2.N, D, nlist, M, 0, 150, 100, "gauss", 1, 1.0)
    full_check(w2, idx2, qs[:9], _ip_radii(idx2, qs[:9], 0.4), nprobe=150, k=100, metric=1)


def test_inner_product_identity_codebook_exact_mips(lib):
    """Lossless codes, all lists probed, nothing thresholded: exact maximum inner product search."""
    from helpers import identity_index
    rng = np.random.default_rng(3)
    base, idx = identity_index(rng)
    queries = rng.integers(-64, 64, size=(20, idx.D)).astype(np.int64)
    b = _binding()
    gi = b.IvfPqIndex.from_index(idx, metric=b.METRIC_IP)
    ids, dist = gi.search(_cuda(queries.astype(np.float32)), idx.nlist, 15, np.full(idx.M, np.inf, np.float32))
    ip = queries @ base.T
    for i in range(queries.shape[0]):
        o = np.lexsort((np.arange(base.shape[0]), -ip[i]))[:15]
        assert np.array_equal(ids[i].cpu().numpy(), o)
        assert np.array_equal(dist[i].cpu().numpy().astype(np.int64), -ip[i][o])
    gi.close()


def test_inner_product_coarse_degenerate(lib):
    """Coarse stage under the inner-product metric with identical and nearly identical
    centroids (exact fallback, ties by list id) and with many lists."""
    rng = np.random.default_rng(22)
    b = _binding()
    D, M = 16, 4
    for name, cent in [
        ("all equal", np.tile(rng.normal(size=(1, D)).astype(np.float32), (5000, 1))),
        ("tiny jitter", (rng.normal(size=(1, D)) + 1e-7 * rng.normal(size=(3000, D))).astype(np.float32)),
        ("ordinary", rng.normal(size=(20000, D)).astype(np.float32)),
        ("zero", np.zeros((700, D), dtype=np.float32)),
    ]:
        nlist = cent.shape[0]
        idx = _random_index(rng, 0, D, nlist, M, np.full(nlist, 1, dtype=np.int64))
        idx.centroids = np.ascontiguousarray(cent)
        q = rng.normal(size=(20, D)).astype(np.float32)
        gi = b.IvfPqIndex.from_index(idx, metric=b.METRIC_IP)
        for nprobe in (1, 10, 200, 1000):
            nprobe = min(nprobe, nlist)
            o_pid, o_pd = oracle.coarse(q, idx.centroids, nprobe, metric=1)
            pid, pd = gi.coarse(_cuda(q), nprobe)
            torch.cuda.synchronize()
            assert np.array_equal(pid.cpu().numpy(), o_pid), (name, nprobe)
            assert_same_float(pd.cpu().numpy(), o_pd, f"{name} nprobe={nprobe}")
        gi.close()
        say(f"  coarse (inner product), {name}: ok")


def test_coarse_degenerate_centroids(lib):
    """Thousands of identical or nearly identical centroids: the proposal's slack window
    cannot separate them, so the exact fallback and the (distance, list id) tie order
    decide; and duplicated centroids among ordinary ones."""
    rng = np.random.default_rng(21)
    b = _binding()
    D, M = 16, 4
    for name, cent in [
        ("all equal", np.tile(rng.normal(size=(1, D)).astype(np.float32), (5000, 1))),
        ("two values", np.repeat(rng.normal(size=(2, D)).astype(np.float32), 2500, axis=0)),
        ("tiny jitter", (rng.normal(size=(1, D)) + 1e-7 * rng.normal(size=(3000, D))).astype(np.float32)),
        ("duplicates", np.concatenate([rng.normal(size=(300, D)), rng.normal(size=(300, D))[rng.integers(0, 300, 700)]]).astype(np.float32)),
    ]:
        nlist = cent.shape[0]
        sizes = np.full(nlist, 2, dtype=np.int64)
        idx = _random_index(rng, 0, D, nlist, M, sizes)
        idx.centroids = np.ascontiguousarray(cent)
        q = rng.normal(size=(20, D)).astype(np.float32)
        gi = b.IvfPqIndex.from_index(idx)
        for nprobe in (1, 10, 200, 1000):
            nprobe = min(nprobe, nlist)
            o_pid, o_pd = oracle.coarse(q, idx.centroids, nprobe)
            pid, pd = gi.coarse(_cuda(q), nprobe)
            torch.cuda.synchronize()
            assert np.array_equal(pid.cpu().numpy(), o_pid), (name, nprobe)
            assert_same_float(pd.cpu().numpy(), o_pd, f"{name} nprobe={nprobe}")
        gi.close()
        say(f"  coarse, {name}: ok")


def test_query_chunks_large_nlist(lib):
    """So many lists that the coarse scores of all queries exceed the 1 GiB the planner allows
    at once: the queries go through coarse quantisation in several chunks."""
    rng = np.random.default_rng(31)
    D, M, nlist, Q = 8, 4, 70001, 4200     # 3712 queries fit the first chunk
    sizes = np.zeros(nlist, dtype=np.int64)
    sizes[rng.permutation(nlist)[:40000]] = 1
    idx = _random_index(rng, 0, D, nlist, M, sizes)
    q = rng.normal(size=(Q, D)).astype(np.float32)
    b = _binding()
    gi = b.IvfPqIndex.from_index(idx)
    assert gi.workspace_bytes(Q, 7, 5) < (1 << 30) + 16 * Q * 7 + 4096
    from concurrent.futures import ThreadPoolExecutor
    cuts = np.linspace(0, Q, 9).astype(int)
    with ThreadPoolExecutor(8) as ex:   # the oracle routine is single-threaded; ctypes releases the GIL
        parts = list(ex.map(lambda i: oracle.coarse(q[cuts[i]:cuts[i + 1]], idx.centroids, 7), range(8)))
    o_pid, o_pd = np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])
    pid, pd = gi.coarse(_cuda(q), 7)
    torch.cuda.synchronize()
    assert np.array_equal(pid.cpu().numpy(), o_pid)
    assert_same_float(pd.cpu().numpy(), o_pd, "probe distances, chunked queries")
    r = np.full(M, 1.0, np.float32)
    o_ids, o_dist = oracle.search(q, idx, 7, 5, r, threads=8)
    ids, dist = gi.search(_cuda(q), 7, 5, r)
    assert np.array_equal(ids.cpu().numpy(), o_ids)
    assert_same_float(dist.cpu().numpy(), o_dist, "top-k, chunked queries")
    gi.close()


@pytest.mark.parametrize("shape", [("sift", 128, 64, 20.0), ("deep", 96, 48, 0.1), ("tti", 200, 100, 0.25),
                                   ("gauss", 64, 16, 0.15)])
def test_pruning_switches_do_not_change_results(lib, shape):
    """The early exit, the per-query switch to plain scanning and the block loading modes are
    optimisations only: with each of them forced off (or on) the answers stay the oracle's.
    Shapes of the specialised kernels; data on which pruning works (sift, tti) and on which the
    switch to plain scanning triggers (deep)."""
    b = _binding()
    family, D, M, sigma = shape
    w = wl.Workload(f"sw_{family}", 30_000, D, 32, M, 24, 12, 50, family, 64, sigma)
    idx, centres = wl.train_index(w)
    q = wl.queries(w, centres).numpy()
    nprobe = w.nprobe                                 # more lists than the switch looks at
    for radii in (wl.calibrate_radii(w, idx, centres, 0.25), np.full(idx.M, np.inf, np.float32)):
        o_ids, o_dist = oracle.search(q, idx, nprobe, w.k, radii, threads=8)
        gi = b.IvfPqIndex.from_index(idx)
        try:
            for ablate in (0, 8, 16, 32, 64, 104, 88):
                for loads in (0, 1, 2, 3):
                    b.set_option("scan_ablate", ablate)
                    b.set_option("scan_loads", loads)
                    ids, dist = gi.search(_cuda(q), nprobe, w.k, radii)
                    assert np.array_equal(ids.cpu().numpy(), o_ids), (ablate, loads)
                    assert_same_float(dist.cpu().numpy(), o_dist, f"ablate {ablate} loads {loads}")
            b.set_option("scan_ablate", 0)
            b.set_option("scan_loads", 0)
            for grid in (1, 2):       # the list-level bound with and without the nearest-entry grid
                for strategy in (b.SCAN_QUERY_MAJOR, b.SCAN_LIST_MAJOR):
                    b.set_option("bound_grid", grid)
                    ids, dist = gi.search(_cuda(q), nprobe, w.k, radii, strategy=strategy)
                    assert np.array_equal(ids.cpu().numpy(), o_ids), ("grid", grid, strategy)
                    assert_same_float(dist.cpu().numpy(), o_dist, f"bound_grid {grid}")
        finally:
            b.set_option("scan_ablate", 0)
            b.set_option("scan_loads", 0)
            b.set_option("bound_grid", 0)
            gi.close()
    # the inner-product kernel has its own early exit, list skip and list-level bound
    radii = _ip_radii(idx, q, 0.25)
    o_ids, o_dist = oracle.search(q, idx, nprobe, w.k, radii, threads=8, metric=1)
    gi = b.IvfPqIndex.from_index(idx, metric=b.METRIC_IP)
    try:
        for ablate in (0, 8, 64):
            for loads in (0, 1):
                b.set_option("scan_ablate", ablate)
                b.set_option("scan_loads", loads)
                ids, dist = gi.search(_cuda(q), nprobe, w.k, radii)
                assert np.array_equal(ids.cpu().numpy(), o_ids), ("ip", ablate, loads)
                assert_same_float(dist.cpu().numpy(), o_dist, f"ip ablate {ablate} loads {loads}")
    finally:
        b.set_option("scan_ablate", 0)
        b.set_option("scan_loads", 0)
        gi.close()


def test_batch_sizes_and_probe_groups(lib):
    """Q = 1, 2, 100, 3000: small batches split the probes of a query over several
    workgroups and merge; results must not depend on that."""
    w = wl.WORKLOADS["T_sift"]
    idx, centres = wl.train_index(w)
    radii = wl.calibrate_radii(w, idx, centres, 0.25)
    b = _binding()
    gi = b.IvfPqIndex.from_index(idx)
    q_all = wl.queries(w, centres, 3000).numpy()
    o_ids, o_dist = oracle.search(q_all, idx, 12, 20, radii, threads=8)
    for Q in (1, 2, 100, 3000):
        ids, dist = gi.search(_cuda(q_all[:Q]), 12, 20, radii)
        assert np.array_equal(ids.cpu().numpy(), o_ids[:Q]), Q
        assert_same_float(dist.cpu().numpy(), o_dist[:Q], f"Q={Q}")
    ids, dist = gi.search(_cuda(q_all[:0]), 12, 20, radii)
    assert ids.shape == (0, 20)
    for nw in (4, 8, 16, 0):
        b.set_option("scan_waves", nw)
        ids, dist = gi.search(_cuda(q_all[:300]), 12, 20, radii)
        assert np.array_equal(ids.cpu().numpy(), o_ids[:300]), nw
    # run twice: bitwise identical
    a1 = gi.search(_cuda(q_all), 12, 20, radii)
    a2 = gi.search(_cuda(q_all), 12, 20, radii)
    assert torch.equal(a1[0], a2[0]) and torch.equal(a1[1], a2[1])


def test_argument_errors(lib):
    b = lib
    w = wl.WORKLOADS["T_gauss"]
    idx, centres = wl.train_index(w)
    gi = b.IvfPqIndex.from_index(idx)
    q = _cuda(wl.queries(w, centres).numpy())
    ok = np.full(idx.M, 1.0, np.float32)
    sentinel = torch.full((q.shape[0], 5), -7, dtype=torch.int64, device="cuda")
    sd = torch.full((q.shape[0], 5), -7.0, dtype=torch.float32, device="cuda")
    for kwargs, status in [
        (dict(nprobe=0, k=5, radii=ok), b.ERR_INVALID_ARGUMENT),
        (dict(nprobe=idx.nlist + 1, k=5, radii=ok), b.ERR_INVALID_ARGUMENT),
        (dict(nprobe=2, k=0, radii=ok), b.ERR_INVALID_ARGUMENT),
        (dict(nprobe=2, k=1025, radii=ok), b.ERR_UNSUPPORTED),
        (dict(nprobe=2, k=5, radii=np.full(idx.M, -1.0, np.float32)), b.ERR_INVALID_ARGUMENT),
        (dict(nprobe=2, k=5, radii=np.full(idx.M, np.nan, np.float32)), b.ERR_INVALID_ARGUMENT),
        (dict(nprobe=2, k=5, radii=ok, workspace=torch.empty(256, dtype=torch.uint8, device="cuda")), b.ERR_WORKSPACE),
    ]:
        with pytest.raises(b.IvfpqError) as e:
            kw = dict(kwargs)
            kk = kw.pop("k")
            if kk == 5:
                kw["out"] = (sentinel, sd)
            gi.search(q, kw.pop("nprobe"), kk, kw.pop("radii"), **kw)
        assert e.value.status == status, (kwargs, e.value)
        assert b.last_error() != ""
    torch.cuda.synchronize()
    assert bool((sentinel == -7).all()) and bool((sd == -7.0).all())   # outputs untouched
    # scan_all refuses offsets that do not match the probed lists
    pid, _ = gi.coarse(q, 2)
    bad = torch.zeros(q.shape[0] + 1, dtype=torch.int64, device="cuda")
    _, _, err = gi.scan_all(q, pid, ok, bad)
    torch.cuda.synchronize()
    assert int(err.item()) > 0


def test_c1_full(lib):
    """The 100k-point configuration end to end, every query, every stage."""
    w = wl.WORKLOADS["C1"]
    idx, centres = wl.train_index(w, device="cuda")
    q = wl.queries(w, centres).cpu().numpy()
    radii = wl.calibrate_radii(w, idx, centres, w.keep_frac)
    full_check(w, idx, q[:64], radii)
    full_check(w, idx, q, radii, stages=False)


def _lm_options(b, first=1, cap=0):
    b.set_option("lm_first", first)
    b.set_option("lm_cap", cap)


@pytest.mark.parametrize("family,D,M,sigma", [("sift", 128, 64, 20.0), ("deep", 96, 48, 0.1), ("gauss", 64, 16, 0.15)])
def test_list_major_scan_matches_oracle(lib, family, D, M, sigma):
    """The list-major batched scan (queries that probe a list share one pass over its codes,
    two per interleaved table) returns the oracle's ids and distance bits: every shape it is
    built for, thresholded and unthresholded, all three scorings, shared and per-query radii,
    1 / 2 / 5 lists scanned query-major first, a candidate buffer so small that queries overflow
    and are redone query-major, probe lists with invalid ids and empty lists (scan_topk), odd and
    even numbers of queries per list, and batches down to one query."""
    b = _binding()
    w = wl.Workload(f"lm_{family}", 40_000, D, 48, M, 301, 12, 100, family, 96, sigma)
    idx, centres = wl.train_index(w)
    q = wl.queries(w, centres).numpy()
    dq = _cuda(q)
    gi = b.IvfPqIndex.from_index(idx)
    LM = b.SCAN_LIST_MAJOR
    try:
        for radii in (wl.calibrate_radii(w, idx, centres, 0.25), np.full(M, np.inf, np.float32)):
            o_ids, o_dist = oracle.search(q, idx, w.nprobe, w.k, radii, threads=8)
            for first, cap in ((1, 4096), (2, 2048), (5, 4096), (2, 64), (1, 64)):
                _lm_options(b, first, cap)
                ids, dist = gi.search(dq, w.nprobe, w.k, radii, strategy=LM)
                torch.cuda.synchronize()
                assert np.array_equal(ids.cpu().numpy(), o_ids), (family, first, cap)
                assert_same_float(dist.cpu().numpy(), o_dist, f"list-major {family} first={first} cap={cap}")
            _lm_options(b)
            # smaller batches (a single query: every task is half empty), other k
            for Q, k in ((1, 100), (2, 7), (77, 128)):
                ok_ids, ok_dist = oracle.search(q[:Q], idx, w.nprobe, k, radii, threads=8)
                ids, dist = gi.search(_cuda(q[:Q]), w.nprobe, k, radii, strategy=LM)
                assert np.array_equal(ids.cpu().numpy(), ok_ids), (family, Q, k)
                assert_same_float(dist.cpu().numpy(), ok_dist, f"list-major {family} Q={Q} k={k}")
        # hit-count scorings and per-query radii
        shared = wl.calibrate_radii(w, idx, centres, 0.25)
        rq = per_query_radii(w, idx, centres, q, 0.25)
        for mode in (1, 2, 0):
            for radii, d_rq in ((shared, None), (rq, _cuda(rq))):
                o_ids, o_dist = oracle.search(q, idx, w.nprobe, w.k, radii, threads=8, mode=mode)
                ids, dist = gi.search(dq, w.nprobe, w.k, shared if d_rq is None else None, mode=mode,
                                      query_radii=d_rq, strategy=LM)
                assert np.array_equal(ids.cpu().numpy(), o_ids), (family, mode, d_rq is not None)
                assert_same_float(dist.cpu().numpy(), o_dist, f"list-major {family} mode {mode}")
        # given probe lists: ids outside the index and empty lists count as empty probes; nprobe not above
        # the lists scanned first falls back to the query-major scan
        rng = np.random.default_rng(9)
        pid = rng.integers(0, idx.nlist, size=(q.shape[0], 9)).astype(np.int32)
        for row in pid:                       # distinct lists per row, as the filtering stage gives them
            row[:] = rng.choice(idx.nlist, 9, replace=False)
        ref = gi.scan_topk(dq, _cuda(pid), 50, shared)
        pid_bad = pid.copy()
        pid_bad[::3, 4] = -1
        pid_bad[1::3, 7] = idx.nlist + 5
        ref_bad = gi.scan_topk(dq, _cuda(pid_bad), 50, shared)
        for p_arr, r in ((pid, ref), (pid_bad, ref_bad)):
            got = gi.scan_topk(dq, _cuda(p_arr), 50, shared, strategy=LM)
            assert torch.equal(got[0], r[0]) and torch.equal(got[1].view(torch.int32), r[1].view(torch.int32))
        got = gi.scan_topk(dq, _cuda(pid[:, :2].copy()), 50, shared, strategy=LM)
        r2 = gi.scan_topk(dq, _cuda(pid[:, :2].copy()), 50, shared)
        assert torch.equal(got[0], r2[0]) and torch.equal(got[1].view(torch.int32), r2[1].view(torch.int32))
        # run twice: bitwise identical (the order in which pairs and candidates land is not fixed, the result is)
        a1 = gi.search(dq, w.nprobe, w.k, shared, strategy=LM)
        a2 = gi.search(dq, w.nprobe, w.k, shared, strategy=LM)
        assert torch.equal(a1[0], a2[0]) and torch.equal(a1[1], a2[1])
        # a workspace sized for the query-major scan is refused before anything runs
        small = gi.workspace(q.shape[0], w.nprobe, w.k)
        with pytest.raises(b.IvfpqError) as e:
            gi.search(dq, w.nprobe, w.k, shared, workspace=small, strategy=LM)
        assert e.value.status == b.ERR_WORKSPACE
    finally:
        _lm_options(b)
        gi.close()


def test_list_major_request_on_unsupported_shapes_is_served_query_major(lib):
    """Inner-product indexes, k above 128 and shapes the list-major kernel is not built for
    take the query-major path whatever the strategy says; results are the oracle's."""
    b = _binding()
    rng = np.random.default_rng(21)
    sizes = [0, 1, 63, 64, 65, 0, 130, 700, 5, 1500, 64 * 9, 0, 333, 2, 127, 129]
    for M, D, metric, k in ((100, 200, 0, 50), (12, 12, 0, 50), (64, 128, 1, 50), (64, 128, 0, 200)):
        idx = _random_index(rng, 0, D, len(sizes), M, sizes)
        q = rng.normal(size=(33, D)).astype(np.float32)
        r = np.full(M, 0.9 * np.sqrt(D / M), dtype=np.float32)
        gi = b.IvfPqIndex.from_index(idx, metric=metric)
        o_ids, o_dist = oracle.search(q, idx, 6, k, r, threads=8, metric=metric)
        ids, dist = gi.search(_cuda(q), 6, k, r, strategy=b.SCAN_LIST_MAJOR)
        assert np.array_equal(ids.cpu().numpy(), o_ids), (M, D, metric, k)
        assert_same_float(dist.cpu().numpy(), o_dist, f"M={M} metric={metric} k={k}")
        gi.close()


def test_list_major_ragged_lists(lib):
    """Hand-made list sizes (empty, one point, one block, a block and a point, long), every list
    probed, so that tasks see every block count; 64- and 48-subspace shapes."""
    b = _binding()
    for M, D in ((64, 128), (48, 96), (16, 64)):
        rng = np.random.default_rng(M)
        # 5000 points: longer than the head pass takes at 64 subspaces (those queries' nearest list is
        # ranked by the query-major kernel), within it at 48 and 16
        sizes = [0, 1, 63, 64, 65, 0, 130, 700, 5, 1500, 64 * 9, 0, 333, 2, 127, 129, 64 * 17 + 1, 5000]
        idx = _random_index(rng, 0, D, len(sizes), M, sizes)
        # the list of 700 points holds 400 copies of one code: more equal distances than the head
        # pass's selection collects, so its queries fall back too; ids decide among the copies
        lo = int(idx.list_offsets[7])
        idx.codes[lo + 100:lo + 500] = idx.codes[lo + 100]
        q = rng.normal(size=(45, D)).astype(np.float32)
        # queries sitting on centroids, so that every list is some query's nearest one
        q[:len(sizes)] = idx.centroids + 0.01 * rng.normal(size=idx.centroids.shape).astype(np.float32)
        gi = b.IvfPqIndex.from_index(idx)
        for r in (np.full(M, 0.9 * np.sqrt(D / M), dtype=np.float32), np.full(M, np.inf, np.float32)):
            for nprobe, k in ((idx.nlist, 128), (6, 100), (3, 1)):
                o_ids, o_dist = oracle.search(q, idx, nprobe, k, r, threads=8)
                ids, dist = gi.search(_cuda(q), nprobe, k, r, strategy=b.SCAN_LIST_MAJOR)
                assert np.array_equal(ids.cpu().numpy(), o_ids), (M, nprobe, k)
                assert_same_float(dist.cpu().numpy(), o_dist, f"ragged M={M} nprobe={nprobe} k={k}")
        gi.close()


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "C5_10M", "C5"])
def test_full_size_configs_sampled_queries(lib, name):
    """The full-size indexes -- the three 1M-point configurations, the 100M-point one, and a
    10M-point scale model of it -- in the batch shape the benchmark times (all Q queries in
    one call); the oracle checks a seeded sample of the outputs (512 queries; 256 on the 100M
    index, where an oracle query costs 25 M look-ups).  The 100M index is the only one whose
    code array passes 4 GiB, so its list and chunk offsets exercise the 64-bit arithmetic."""
    w = wl.WORKLOADS[name]
    idx, centres = wl.train_index(w, device="cuda", progress=say)
    q = wl.queries(w, centres).cpu().numpy()
    b = _binding()
    gi = b.IvfPqIndex.from_index(idx)
    if name == "C5":
        assert gi.info()["code_bytes"] > (1 << 32), gi.info()
    dq = _cuda(q)
    fracs = (0.10, 0.25, 0.50, 1.0) if name == "C2" else (0.25, 1.0)
    sample = np.sort(np.random.default_rng(1).choice(w.Q, 256 if name == "C5" else 512, replace=False))
    for frac in fracs:
        radii = wl.calibrate_radii(w, idx, centres, frac)
        ids, dist = gi.search(dq, w.nprobe, w.k, radii)
        torch.cuda.synchronize()
        o_ids, o_dist = oracle.search(q[sample], idx, w.nprobe, w.k, radii, threads=ORACLE_THREADS)
        assert np.array_equal(ids.cpu().numpy()[sample], o_ids), (name, frac)
        assert_same_float(dist.cpu().numpy()[sample], o_dist, f"{name} keep={frac}")
        say(f"  {name} keep={frac}: {len(sample)} sampled queries match the oracle")
        # the strategy is the library's choice above; forced either way the whole batch has the same bits
        for st in (b.SCAN_QUERY_MAJOR, b.SCAN_LIST_MAJOR):
            ids_s, dist_s = gi.search(dq, w.nprobe, w.k, radii, strategy=st)
            torch.cuda.synchronize()
            assert torch.equal(ids_s, ids) and torch.equal(dist_s.view(torch.int32), dist.view(torch.int32)), (name, frac, st)
        say(f"  {name} keep={frac}: query-major and list-major scans give the same {w.Q} x {w.k} results")
    # properties that hold for every query at full size
    ids_np, dist_np = ids.cpu().numpy(), dist.cpu().numpy()
    assert np.all(np.diff(dist_np, axis=1) >= 0) and ids_np.min() >= 0 and ids_np.max() < w.N
    assert all(len(set(r.tolist())) == w.k for r in ids_np[:500])
    gi.close()
