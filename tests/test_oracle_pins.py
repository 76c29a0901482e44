"""Pins for the CPU oracle: what the paper and the mathematics fix, computed
here by independent means (integer brute force, float64 numpy closed forms,
the paper's ray/sphere formulation), never by calling the oracle twice.

Note on one requested invariant: with the clamp r_m^2 for entries outside the
radius (reading R1 in the oracle header) a filtered entry has d2 > r_m^2 and is
replaced by the SMALLER value, so thresholded distances are <= the
unthresholded ones, not >=.  The tests below assert the direction that is
mathematically true for this clamp; the deviation from the wording of the build
target is deliberate.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2312_01712_amd import workloads as wl


# ----------------------------------------------------------------------------
# helpers (independent of the oracle)
# ----------------------------------------------------------------------------

from helpers import identity_index, brute_knn_int, per_query_radii  # noqa: E402


@pytest.fixture(scope="module")
def tiny():
    out = {}
    for name in ("T_gauss", "T_sift", "T_deep", "T_tti"):
        w = wl.WORKLOADS[name]
        idx, centres = wl.train_index(w)
        q = wl.queries(w, centres).numpy()
        out[name] = (w, idx, centres, q)
    return out


def reconstruct(idx):
    """cent[list(x)] + concat_m codebook[m][code_m], float64, in stored row order."""
    labels = np.repeat(np.arange(idx.nlist), np.diff(idx.list_offsets))
    rec = idx.centroids[labels].astype(np.float64)
    ent = idx.codebooks.astype(np.float64)[np.arange(idx.M)[None, :], idx.codes.astype(np.int64)]  # [N][M][dsub]
    return rec + ent.reshape(idx.N, idx.D), labels


def per_subspace_d2(idx, q, c):
    """float64 squared distances between the residual projections of query q
    w.r.t. list c and the entries coded by each point of list c: [n_c][M]."""
    b, e = idx.list_offsets[c], idx.list_offsets[c + 1]
    res = (q.astype(np.float32) - idx.centroids[c]).astype(np.float64).reshape(idx.M, idx.dsub)
    ent = idx.codebooks.astype(np.float64)[np.arange(idx.M)[None, :], idx.codes[b:e].astype(np.int64)]
    return ((ent - res[None]) ** 2).sum(-1)


# ----------------------------------------------------------------------------
# 1. whole path == exact kNN on identity-codebook indexes (paper Sec. 6.4:
#    probing every list is a Flat index; with lossless codes the search is exact)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 1])
def test_identity_codebook_equals_bruteforce(seed):
    rng = np.random.default_rng(seed)
    base, idx = identity_index(rng)
    Q, k = 20, 15
    queries = rng.integers(0, 128, size=(Q, idx.D)).astype(np.int64)
    radii = np.full(idx.M, np.inf, dtype=np.float32)
    ids, dist = oracle.search(queries.astype(np.float32), idx, idx.nlist, k, radii)
    ref_ids, ref_dist = brute_knn_int(base, queries, k)
    assert np.array_equal(ids, ref_ids)
    assert np.array_equal(dist.astype(np.int64), ref_dist) and np.all(dist == np.floor(dist))
    # recall is 1 by construction; the double-precision reference agrees too
    eid, edist = oracle.exact_knn(base.astype(np.float32), queries.astype(np.float32), k)
    assert np.array_equal(eid, ref_ids) and np.array_equal(edist, ref_dist.astype(np.float64))


def test_identity_codebook_partial_probe_is_subset_exact():
    """With nprobe < nlist the result is the exact kNN restricted to the probed lists."""
    rng = np.random.default_rng(7)
    base, idx = identity_index(rng, N=900, D=8, nlist=5)
    queries = rng.integers(0, 128, size=(10, idx.D)).astype(np.int64)
    nprobe, k = 2, 12
    radii = np.full(idx.M, np.inf, dtype=np.float32)
    ids, dist = oracle.search(queries.astype(np.float32), idx, nprobe, k, radii)
    cent = idx.centroids.astype(np.int64)
    labels = np.empty(idx.N, dtype=np.int64)
    labels[idx.ids] = np.repeat(np.arange(idx.nlist), np.diff(idx.list_offsets))
    for q in range(queries.shape[0]):
        dc = ((cent - queries[q]) ** 2).sum(-1)
        probes = np.lexsort((np.arange(idx.nlist), dc))[:nprobe]
        members = np.nonzero(np.isin(labels, probes))[0]
        d = ((base[members] - queries[q]) ** 2).sum(-1)
        o = np.lexsort((members, d))[:k]
        assert np.array_equal(ids[q], members[o])
        assert np.array_equal(dist[q].astype(np.int64), d[o])


# ----------------------------------------------------------------------------
# 2. coarse stage
# ----------------------------------------------------------------------------

def test_coarse_full_permutation_and_argmin(tiny):
    for name, (w, idx, _, q) in tiny.items():
        ids, dist = oracle.coarse(q, idx.centroids, idx.nlist)
        d64 = ((q.astype(np.float64)[:, None, :] - idx.centroids.astype(np.float64)[None]) ** 2).sum(-1)
        for i in range(q.shape[0]):
            assert sorted(ids[i].tolist()) == list(range(idx.nlist))          # a permutation
            assert np.all(np.diff(dist[i]) >= 0)                               # ascending
            np.testing.assert_allclose(dist[i], d64[i][ids[i]], rtol=1e-5)     # fp32 chain vs double
            ref = np.argsort(d64[i], kind="stable")
            gaps = np.diff(d64[i][ref]) > 1e-5 * d64[i][ref][1:]
            # wherever the double distances are clearly separated the order must agree
            same = ids[i] == ref
            assert np.all(same[:-1][gaps & np.r_[True, gaps[:-1]]])
        ids1, _ = oracle.coarse(q, idx.centroids, 1)
        assert np.array_equal(ids1[:, 0], ids[:, 0])
        well = np.sort(d64, 1)[:, 1] - np.sort(d64, 1)[:, 0] > 1e-5 * np.sort(d64, 1)[:, 1]
        assert np.array_equal(ids1[well, 0], d64.argmin(1)[well])
        idsp, distp = oracle.coarse(q, idx.centroids, w.nprobe)
        assert np.array_equal(idsp, ids[:, :w.nprobe]) and np.array_equal(distp, dist[:, :w.nprobe])


def test_coarse_tie_break_by_list_id():
    cent = np.array([[1.0, 0.0], [0.0, 1.0], [-1.0, 0.0], [0.0, -1.0], [3.0, 3.0]], dtype=np.float32)
    ids, dist = oracle.coarse(np.zeros((1, 2), np.float32), cent, 5)
    assert ids[0].tolist() == [0, 1, 2, 3, 4] and dist[0].tolist() == [1, 1, 1, 1, 18]


# ----------------------------------------------------------------------------
# 3. unthresholded table + ADC == ||q - reconstruct(x)||^2 (paper Sec. 2.1, B-D)
# ----------------------------------------------------------------------------

def test_adc_equals_reconstruction_distance(tiny):
    for name, (w, idx, _, q) in tiny.items():
        probes, _ = oracle.coarse(q, idx.centroids, w.nprobe)
        radii = np.full(idx.M, np.inf, dtype=np.float32)
        offs, dist, ids = oracle.scan_all(q, idx, probes, radii)
        rec, _ = reconstruct(idx)
        row_of = np.empty(idx.N, dtype=np.int64)
        row_of[idx.ids] = np.arange(idx.N)
        for i in range(q.shape[0]):
            sl = slice(offs[i], offs[i + 1])
            expect_rows = np.concatenate([np.arange(idx.list_offsets[c], idx.list_offsets[c + 1]) for c in probes[i]])
            assert np.array_equal(row_of[ids[sl]], expect_rows)                # candidate set and order
            ref = ((rec[expect_rows] - q[i].astype(np.float64)) ** 2).sum(-1)
            np.testing.assert_allclose(dist[sl], ref, rtol=1e-4, atol=1e-30)


# ----------------------------------------------------------------------------
# 4. thresholded table / ADC: closed form and invariants
# ----------------------------------------------------------------------------

def test_thresholded_adc_closed_form_and_invariants(tiny):
    for name, (w, idx, centres, q) in tiny.items():
        probes, _ = oracle.coarse(q, idx.centroids, w.nprobe)
        inf = np.full(idx.M, np.inf, dtype=np.float32)
        r25 = wl.calibrate_radii(w, idx, centres, 0.25)
        r50 = np.maximum(wl.calibrate_radii(w, idx, centres, 0.50), r25)
        offs, d_inf, ids_inf = oracle.scan_all(q, idx, probes, inf)
        _, d_25, ids_25 = oracle.scan_all(q, idx, probes, r25)
        _, d_50, _ = oracle.scan_all(q, idx, probes, r50)
        _, d_big, _ = oracle.scan_all(q, idx, probes, np.full(idx.M, 1e18, np.float32))
        _, d_zero, _ = oracle.scan_all(q, idx, probes, np.zeros(idx.M, np.float32))
        assert np.array_equal(ids_inf, ids_25)
        # (i) thresholded <= unthresholded, (iv) monotone in the radii
        assert np.all(d_25 <= d_50) and np.all(d_50 <= d_inf)
        # (iii) bounded by the saturation value sum r_m^2 (same fp32 order)
        sat = np.float32(0.0)
        for m in range(idx.M):
            sat = np.float32(sat + np.float32(r25[m] * r25[m]))
        assert np.all(d_25 <= sat)
        # (v) a huge finite radius equals +inf; radius 0 gives 0 everywhere
        assert np.array_equal(d_big, d_inf)
        assert np.all(d_zero == 0.0)
        # (ii) closed form: sum_m min(d2_m, r_m^2) in float64; equality of thr and
        # unthr exactly where every subspace was kept
        r2 = (r25.astype(np.float64)) ** 2
        n_sat = 0
        for i in range(q.shape[0]):
            pos = offs[i]
            for c in probes[i]:
                d2 = per_subspace_d2(idx, q[i], c)
                n = d2.shape[0]
                ref = np.minimum(d2, r2[None]).sum(-1)
                np.testing.assert_allclose(d_25[pos:pos + n], ref, rtol=2e-5, atol=1e-30)
                all_kept = np.all(d2 < r2[None] * (1 - 1e-5), axis=1)
                assert np.array_equal(d_25[pos:pos + n][all_kept], d_inf[pos:pos + n][all_kept])
                some_cut = np.any(d2 > r2[None] * (1 + 1e-5), axis=1)
                assert np.all(d_25[pos:pos + n][some_cut] < d_inf[pos:pos + n][some_cut])
                none_kept = np.all(d2 > r2[None] * (1 + 1e-5), axis=1)
                assert np.all(d_25[pos:pos + n][none_kept] == sat)
                n_sat += int(none_kept.sum())
                pos += n
            assert pos == offs[i + 1]


def test_lut_values_mask_and_keep_fraction(tiny):
    for name, (w, idx, centres, q) in tiny.items():
        probes, _ = oracle.coarse(q, idx.centroids, w.nprobe)
        for frac in (0.10, 0.25, 0.50):
            radii = wl.calibrate_radii(w, idx, centres, frac)
            lut, mask = oracle.build_lut(q, idx.centroids, idx.codebooks, probes, radii)
            res = (q[:, None, :] - idx.centroids[probes]).astype(np.float64)             # [Q][P][D]
            res = res.reshape(q.shape[0], w.nprobe, idx.M, 1, idx.dsub)
            d2 = ((res - idx.codebooks.astype(np.float64)[None, None]) ** 2).sum(-1)      # [Q][P][M][256]
            r2 = (radii.astype(np.float64) ** 2)[None, None, :, None]
            np.testing.assert_allclose(lut, np.minimum(d2, r2), rtol=1e-5, atol=1e-30)
            bits = ((mask[..., None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(bool)
            bits = bits.reshape(q.shape[0], w.nprobe, idx.M, 256)
            clear = np.abs(d2 - r2) > 1e-5 * r2
            assert np.array_equal(bits[clear], (d2 <= r2)[clear])
            assert abs(bits.mean() - frac) < 0.05, (name, frac, bits.mean())
        lut_inf, mask_inf = oracle.build_lut(q, idx.centroids, idx.codebooks, probes,
                                             np.full(idx.M, np.inf, np.float32))
        assert np.all(mask_inf == np.uint64(0xFFFFFFFFFFFFFFFF))


# ----------------------------------------------------------------------------
# 5. the paper's ray/sphere formulation of the keep rule (Sec. 4.2; Algorithm 2)
# ----------------------------------------------------------------------------

def _ray_sphere(R, thr_scaled, d):
    """A ray starts on the plane z = 2s at planar distance d from a sphere of
    radius R centred on the plane z = 2s+1 and travels along +z.  It meets the
    sphere after t_hit = 1 - sqrt(R^2 - d^2) (if d <= R) and is cut off at
    t_max = 1 - sqrt(R^2 - thr_scaled^2)."""
    t_max = 1.0 - math.sqrt(R * R - thr_scaled * thr_scaled)
    if d > R:
        return False, None, t_max
    t_hit = 1.0 - math.sqrt(R * R - d * d)
    return t_hit <= t_max, t_hit, t_max


def test_paper_tmax_example(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "tmax_example.txt")) if l.strip() and l[0] != "#"]
    R, thr, scale, tmax = map(float, rows[0])
    assert _ray_sphere(R, thr * scale, 0.0)[2] == pytest.approx(tmax, abs=1e-12)


def test_keep_rule_matches_ray_sphere_hits(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "tmax_example.txt")) if l.strip() and l[0] != "#"]
    R, thr, scale, tmax = map(float, rows[0])
    rng = np.random.default_rng(3)
    nlist, M, D = 3, 2, 4
    cent = rng.uniform(-0.2, 0.2, size=(nlist, D)).astype(np.float32)
    cb = rng.uniform(-0.7, 0.7, size=(M, 256, 2)).astype(np.float32)
    q = rng.uniform(-0.3, 0.3, size=(5, D)).astype(np.float32)
    probes = np.tile(np.arange(nlist, dtype=np.int32), (5, 1))
    radii = np.full(M, thr * scale, dtype=np.float32)
    lut, mask = oracle.build_lut(q, cent, cb, probes, radii)
    n_hit = 0
    for qi in range(5):
        for c in range(nlist):
            for m in range(M):
                o = (q[qi, 2 * m:2 * m + 2] - cent[c, 2 * m:2 * m + 2]).astype(np.float64)  # ray origin (x, y)
                for e in range(256):
                    d = float(np.hypot(*(cb[m, e].astype(np.float64) - o)))
                    hit, t_hit, t_max = _ray_sphere(R, thr * scale, d)
                    assert t_max == pytest.approx(tmax, abs=1e-7)
                    if abs(d - thr * scale) < 1e-5:
                        continue
                    kept = bool((int(mask[qi, c, m, e >> 6]) >> (e & 63)) & 1)
                    assert kept == hit
                    if hit:
                        n_hit += 1
                        # hit-shader distance: L2^2 = R^2 - (1 - t_hit)^2
                        assert lut[qi, c, m, e] == pytest.approx(R * R - (1.0 - t_hit) ** 2, rel=1e-4, abs=1e-9)
                    else:
                        assert lut[qi, c, m, e] == np.float32(radii[m] * radii[m])
    assert n_hit > 100


# ----------------------------------------------------------------------------
# 5b. hit-count scoring (paper Sec. 5.4) and per-query radii (Sec. 4.1)
# ----------------------------------------------------------------------------

def test_hit_count_scores_match_their_definition(tiny):
    """Mode 1: M minus the number of subspaces whose coded entry lies inside the radius.
    Mode 2: M minus the reward/penalty score (+1 inside the half-radius inner sphere,
    0 inside the outer sphere only, -1 outside both).  Both from float64 distances."""
    for name, (w, idx, centres, q) in tiny.items():
        probes, _ = oracle.coarse(q, idx.centroids, w.nprobe)
        radii = wl.calibrate_radii(w, idx, centres, 0.25)
        r = radii.astype(np.float64)[None, :]
        offs, d1, ids1 = oracle.scan_all(q, idx, probes, radii, mode=1)
        _, d2m, ids2 = oracle.scan_all(q, idx, probes, radii, mode=2)
        _, d0, ids0 = oracle.scan_all(q, idx, probes, radii, mode=0)
        assert np.array_equal(ids1, ids0) and np.array_equal(ids2, ids0)
        assert np.all(d1 == np.floor(d1)) and np.all(d2m == np.floor(d2m))
        assert np.all(d1 <= d2m) and np.all(d2m <= d1 + idx.M) and d1.max() <= idx.M and d2m.max() <= 2 * idx.M
        checked = 0
        for i in range(q.shape[0]):
            pos = offs[i]
            for c in probes[i]:
                dd = np.sqrt(per_subspace_d2(idx, q[i], c))                 # [n][M] distances
                n = dd.shape[0]
                clear = np.all((np.abs(dd - r) > 1e-5 * r) & (np.abs(dd - 0.5 * r) > 1e-5 * r), axis=1)
                hits = (dd <= r).sum(1)
                score = (dd <= 0.5 * r).sum(1) - (dd > r).sum(1)
                assert np.array_equal(d1[pos:pos + n][clear], (idx.M - hits)[clear])
                assert np.array_equal(d2m[pos:pos + n][clear], (idx.M - score)[clear])
                checked += int(clear.sum())
                pos += n
        assert checked > 1000
        # the table itself: 0/1 (and 0/1/2) values, consistent with the keep mask of the outer radius
        lut1, mask1 = oracle.build_lut(q, idx.centroids, idx.codebooks, probes, radii, mode=1)
        lut2, mask2 = oracle.build_lut(q, idx.centroids, idx.codebooks, probes, radii, mode=2)
        _, mask0 = oracle.build_lut(q, idx.centroids, idx.codebooks, probes, radii, mode=0)
        assert np.array_equal(mask1, mask0) and np.array_equal(mask2, mask0)
        bits = ((mask0[..., None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(bool).reshape(lut1.shape)
        assert np.array_equal(lut1 == 0.0, bits) and set(np.unique(lut1)) <= {0.0, 1.0}
        assert np.array_equal(lut2 == 2.0, ~bits) and set(np.unique(lut2)) <= {0.0, 1.0, 2.0}
        # ranking by the penalty is ranking by the score; ties go to the smaller id
        ids, dist = oracle.search(q, idx, w.nprobe, w.k, radii, mode=1)
        for i in range(q.shape[0]):
            sl = slice(offs[i], offs[i + 1])
            o = np.lexsort((ids1[sl], d1[sl]))[:w.k]
            assert np.array_equal(ids[i], ids1[sl][o]) and np.array_equal(dist[i], d1[sl][o])


def test_per_query_radii(tiny):
    """radii[Q][M]: each query is searched as if its own row were the shared radii."""
    for name, (w, idx, centres, q) in tiny.items():
        rq = per_query_radii(w, idx, centres, q, 0.25)
        assert rq.shape == (q.shape[0], idx.M) and np.all(rq > 0)
        for mode in (0, 1, 2):
            ids, dist = oracle.search(q, idx, w.nprobe, w.k, rq, mode=mode)
            for i in (0, 1, q.shape[0] - 1):
                ids_i, dist_i = oracle.search(q[i:i + 1], idx, w.nprobe, w.k, rq[i], mode=mode)
                assert np.array_equal(ids[i], ids_i[0]) and np.array_equal(dist[i], dist_i[0])
        # a constant per-query array equals the shared form
        shared = wl.calibrate_radii(w, idx, centres, 0.25)
        a = oracle.search(q, idx, w.nprobe, w.k, np.tile(shared[None], (q.shape[0], 1)))
        b = oracle.search(q, idx, w.nprobe, w.k, shared)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
        # closed form with per-query radii: truncated sum in float64
        probes, _ = oracle.coarse(q, idx.centroids, w.nprobe)
        offs, d, _ = oracle.scan_all(q, idx, probes, rq)
        for i in range(0, q.shape[0], 7):
            pos = offs[i]
            for c in probes[i]:
                d2 = per_subspace_d2(idx, q[i], c)
                ref = np.minimum(d2, (rq[i].astype(np.float64) ** 2)[None]).sum(-1)
                np.testing.assert_allclose(d[pos:pos + d2.shape[0]], ref, rtol=2e-5, atol=1e-30)
                pos += d2.shape[0]


# ----------------------------------------------------------------------------
# 6. top-k
# ----------------------------------------------------------------------------

def test_topk_against_sort_padding_and_ties():
    rng = np.random.default_rng(5)
    d = rng.integers(0, 50, size=4000).astype(np.float32)      # many ties
    ids = rng.permutation(4000).astype(np.int64)
    oi, od = oracle.topk(d, ids, 100)
    o = np.lexsort((ids, d))[:100]
    assert np.array_equal(oi, ids[o]) and np.array_equal(od, d[o])
    oi, od = oracle.topk(d[:7], ids[:7], 10)
    o = np.lexsort((ids[:7], d[:7]))
    assert np.array_equal(oi[:7], ids[:7][o]) and np.all(oi[7:] == -1) and np.all(np.isinf(od[7:]))
    oi, od = oracle.topk(np.full(500, 2.5, np.float32), ids[:500], 20)
    assert np.array_equal(oi, np.sort(ids[:500])[:20]) and np.all(od == 2.5)
    oi, od = oracle.topk(np.zeros(0, np.float32), np.zeros(0, np.int64), 3)
    assert np.all(oi == -1) and np.all(np.isinf(od))


# ----------------------------------------------------------------------------
# 7. the fused routine is the composition of its stages; threads do not matter
# ----------------------------------------------------------------------------

def test_search_is_composition_of_stages(tiny):
    for name, (w, idx, centres, q) in tiny.items():
        radii = wl.calibrate_radii(w, idx, centres, 0.25)
        ids, dist = oracle.search(q, idx, w.nprobe, w.k, radii)
        probes, _ = oracle.coarse(q, idx.centroids, w.nprobe)
        offs, cd, ci = oracle.scan_all(q, idx, probes, radii)
        for i in range(q.shape[0]):
            o = np.lexsort((ci[offs[i]:offs[i + 1]], cd[offs[i]:offs[i + 1]]))[:w.k]
            assert np.array_equal(ids[i], ci[offs[i]:offs[i + 1]][o])
            assert np.array_equal(dist[i], cd[offs[i]:offs[i + 1]][o])
        ids_t, dist_t = oracle.search(q, idx, w.nprobe, w.k, radii, threads=3)
        assert np.array_equal(ids, ids_t) and np.array_equal(dist, dist_t)


def test_recall_sane_and_monotone(tiny):
    """Recall on synthetic data is unpinned (the paper's numbers are for datasets
    that are absent); only its direction is checked."""
    w, idx, centres, q = tiny["T_gauss"]
    base = wl.base_vectors(w, centres).numpy()
    truth, _ = oracle.exact_knn(base, q, w.k)
    inf = np.full(idx.M, np.inf, np.float32)
    r_all = wl.recall_at_k(oracle.search(q, idx, idx.nlist, w.k, inf)[0], truth)[0]
    r_few = wl.recall_at_k(oracle.search(q, idx, 1, w.k, inf)[0], truth)[0]
    r_thr = wl.recall_at_k(oracle.search(q, idx, idx.nlist, w.k, wl.calibrate_radii(w, idx, centres, 0.10))[0], truth)[0]
    assert r_all >= r_few and r_all >= r_thr and r_all > 0.3


# ----------------------------------------------------------------------------
# 9. inner-product metric (paper Sec. 4.2 "Inner Product Similarity Support")
# ----------------------------------------------------------------------------

def _ip_radii(idx, q, frac):
    """Per-subspace radii that keep about `frac` of the entries under the inner-product
    rule (an entry is kept iff |q_m - e|^2 - |e|^2 <= r_m^2), from float64."""
    qm = q.astype(np.float64).reshape(q.shape[0], idx.M, 1, idx.dsub)
    ent = idx.codebooks.astype(np.float64)[None]
    g = ((qm - ent) ** 2).sum(-1) - (ent ** 2).sum(-1)                       # [Q][M][256]
    r2 = np.quantile(g.transpose(1, 0, 2).reshape(idx.M, -1), frac, axis=1)
    return np.sqrt(np.maximum(r2, 0.0)).astype(np.float32)


@pytest.mark.parametrize("seed", [0, 1])
def test_ip_identity_codebook_equals_bruteforce_mips(seed):
    """Lossless integer codes, every list probed, nothing thresholded: the search is exact
    maximum inner product search (all arithmetic exact in fp32)."""
    rng = np.random.default_rng(100 + seed)
    base, idx = identity_index(rng)
    Q, k = 20, 15
    queries = rng.integers(-64, 64, size=(Q, idx.D)).astype(np.int64)
    radii = np.full(idx.M, np.inf, dtype=np.float32)
    ids, dist = oracle.search(queries.astype(np.float32), idx, idx.nlist, k, radii, metric=1)
    ip = queries @ base.T                                                    # int64, exact
    for i in range(Q):
        o = np.lexsort((np.arange(base.shape[0]), -ip[i]))[:k]
        assert np.array_equal(ids[i], o)
        assert np.array_equal(dist[i].astype(np.int64), -ip[i][o])
    eid, edist = oracle.exact_knn(base.astype(np.float32), queries.astype(np.float32), k, metric=1)
    assert np.array_equal(eid, ids) and np.array_equal(edist, dist.astype(np.float64))
    # fewer probes: lists by largest q.centroid (ties to the smaller list id), exact within them
    nprobe = 2
    ids2, dist2 = oracle.search(queries.astype(np.float32), idx, nprobe, k, radii, metric=1)
    pid, pdist = oracle.coarse(queries.astype(np.float32), idx.centroids, nprobe, metric=1)
    cent = idx.centroids.astype(np.int64)
    labels = np.empty(idx.N, dtype=np.int64)
    labels[idx.ids] = np.repeat(np.arange(idx.nlist), np.diff(idx.list_offsets))
    for i in range(Q):
        sc = -(cent @ queries[i])
        probes = np.lexsort((np.arange(idx.nlist), sc))[:nprobe]
        assert np.array_equal(pid[i], probes) and np.array_equal(pdist[i].astype(np.int64), sc[probes])
        members = np.nonzero(np.isin(labels, probes))[0]
        o = np.lexsort((members, -ip[i][members]))[:k]
        assert np.array_equal(ids2[i], members[o])
        assert np.array_equal(dist2[i].astype(np.int64), -ip[i][members][o])


def test_ip_coarse_orders_lists_by_inner_product(tiny):
    for name, (w, idx, _, q) in tiny.items():
        ids, dist = oracle.coarse(q, idx.centroids, idx.nlist, metric=1)
        s64 = -(q.astype(np.float64) @ idx.centroids.astype(np.float64).T)
        scale = np.linalg.norm(q, axis=1)[:, None] * np.linalg.norm(idx.centroids, axis=1)[None, :]
        for i in range(q.shape[0]):
            assert sorted(ids[i].tolist()) == list(range(idx.nlist))
            assert np.all(np.diff(dist[i]) >= 0)
            assert np.all(np.abs(dist[i] - s64[i][ids[i]]) <= 1e-5 * scale[i][ids[i]] + 1e-30)
            ref = np.argsort(s64[i], kind="stable")
            gaps = np.diff(s64[i][ref]) > 1e-5 * scale[i].max()
            same = ids[i] == ref
            assert np.all(same[:-1][gaps & np.r_[True, gaps[:-1]]])


def test_ip_table_keep_rule_identity_and_clamp(tiny):
    """The keep rule is the paper's enlarged sphere (radius^2 = r^2 + |e|^2 around the entry,
    ray from the query's projection); kept values satisfy the paper's identity
    IP = (|e|^2 + |q|^2 - L2^2) / 2 with L2^2 taken from the (separately pinned) L2 table of
    a list whose centroid is the origin; missed entries hold the bound (r^2 - |q_m|^2) / 2."""
    for name, (w, idx, _, q) in tiny.items():
        radii = _ip_radii(idx, q, 0.3)
        probes = np.zeros((q.shape[0], 1), dtype=np.int32)
        lut, mask = oracle.build_lut(q, idx.centroids, idx.codebooks, probes, radii, metric=1)
        lut, mask = lut[:, 0], mask[:, 0]
        bits = ((mask[..., None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(bool).reshape(lut.shape)
        qm = q.astype(np.float64).reshape(q.shape[0], idx.M, 1, idx.dsub)
        ent = idx.codebooks.astype(np.float64)[None]
        e2 = (ent ** 2).sum(-1)
        l2 = ((qm - ent) ** 2).sum(-1)
        r2 = radii.astype(np.float64)[None, :, None] ** 2
        inside = l2 <= r2 + e2                                              # enlarged sphere
        scale = (qm ** 2).sum(-1) + e2 + r2
        clear = np.abs(l2 - r2 - e2) > 1e-5 * scale
        assert np.array_equal(bits[clear], inside[clear]) and clear.mean() > 0.99
        assert 0.2 < bits.mean() < 0.4
        # identity against the L2 table of a zero centroid (residual == query)
        zero_c = np.zeros((1, idx.D), dtype=np.float32)
        l2_lut, _ = oracle.build_lut(q, zero_c, idx.codebooks, probes, np.full(idx.M, np.inf, np.float32))
        ip_from_l2 = (e2 + (qm ** 2).sum(-1) - l2_lut[:, 0].astype(np.float64)) / 2
        kept = bits
        assert np.all(np.abs(-lut.astype(np.float64) - ip_from_l2)[kept] <= 2e-6 * scale[kept])
        # the clamp
        clampv = np.broadcast_to((r2 - (qm ** 2).sum(-1)) / 2, lut.shape)
        assert np.all(np.abs(lut.astype(np.float64) - clampv)[~kept] <= 2e-6 * scale[~kept])
        # the table does not depend on the list
        lut_b, _ = oracle.build_lut(q, idx.centroids, idx.codebooks, probes + (idx.nlist - 1), radii, metric=1)
        assert np.array_equal(lut_b[:, 0], lut)
        # no radius: everything kept, value = -IP
        lut_inf, mask_inf = oracle.build_lut(q, idx.centroids, idx.codebooks, probes,
                                             np.full(idx.M, np.inf, np.float32), metric=1)
        assert np.all(mask_inf == np.uint64(0xFFFFFFFFFFFFFFFF))
        ip64 = (qm * ent).sum(-1)
        assert np.all(np.abs(lut_inf[:, 0].astype(np.float64) + ip64) <= 2e-6 * scale)


def test_ip_scores_closed_forms(tiny):
    """Unthresholded: score = -<q, reconstruction>.  Thresholded: list term plus
    sum_m -max(ip_m, thr_m); hit counts = number of subspaces with ip_m < thr_m."""
    for name, (w, idx, _, q) in tiny.items():
        probes, pdist = oracle.coarse(q, idx.centroids, w.nprobe, metric=1)
        rec, labels = reconstruct(idx)
        inf = np.full(idx.M, np.inf, dtype=np.float32)
        offs, d, ids = oracle.scan_all(q, idx, probes, inf, metric=1)
        pos_of = {int(v): i for i, v in enumerate(idx.ids)}
        radii = _ip_radii(idx, q, 0.3)
        _, dt, idst = oracle.scan_all(q, idx, probes, radii, metric=1)
        _, d1, _ = oracle.scan_all(q, idx, probes, radii, mode=1, metric=1)
        _, d2m, _ = oracle.scan_all(q, idx, probes, radii, mode=2, metric=1)
        assert np.array_equal(idst, ids)
        r2 = radii.astype(np.float64) ** 2
        checked = 0
        for i in range(q.shape[0]):
            rows = np.array([pos_of[int(v)] for v in ids[offs[i]:offs[i + 1]]])
            q64 = q[i].astype(np.float64)
            want = -(rec[rows] @ q64)
            scale = np.linalg.norm(rec[rows], axis=1) * np.linalg.norm(q64) + 1e-30
            assert np.all(np.abs(d[offs[i]:offs[i + 1]] - want) <= 1e-5 * scale)
            # thresholded closed form
            qm = q64.reshape(idx.M, idx.dsub)
            ent = idx.codebooks.astype(np.float64)[np.arange(idx.M)[None, :], idx.codes[rows].astype(np.int64)]
            ipm = (ent * qm[None]).sum(-1)                                   # [n][M]
            thr = ((qm ** 2).sum(-1) - r2) / 2
            thr_in = ((qm ** 2).sum(-1) - r2 / 4) / 2
            start = -(idx.centroids[labels[rows]].astype(np.float64) @ q64)
            want_t = start - np.maximum(ipm, thr[None]).sum(1)
            assert np.all(np.abs(dt[offs[i]:offs[i + 1]] - want_t) <= 2e-5 * (scale + np.abs(thr).sum()))
            band = 1e-5 * ((qm ** 2).sum(-1)[None] + (ent ** 2).sum(-1) + r2[None])
            clear = np.all((np.abs(ipm - thr[None]) > band) & (np.abs(ipm - thr_in[None]) > band), axis=1)
            miss = (ipm < thr[None]).sum(1)
            pen = miss + (ipm < thr_in[None]).sum(1)
            assert np.array_equal(d1[offs[i]:offs[i + 1]][clear], miss[clear])
            assert np.array_equal(d2m[offs[i]:offs[i + 1]][clear], pen[clear])
            checked += int(clear.sum())
        assert checked > 1000
        # thresholding can only lower a score (the clamp is a bound no missed entry reaches)
        assert np.all(dt <= d + 1e-5 * (np.abs(d) + 1))
        # search = top-k of those scores by (score, id)
        ids_s, dist_s = oracle.search(q, idx, w.nprobe, w.k, radii, metric=1)
        for i in range(q.shape[0]):
            sl = slice(offs[i], offs[i + 1])
            o = np.lexsort((ids[sl], dt[sl]))[:w.k]
            assert np.array_equal(ids_s[i], ids[sl][o]) and np.array_equal(dist_s[i], dt[sl][o])


# ----------------------------------------------------------------------------
# dynamic threshold (paper Sec. 4.1 "Determining Proper Threshold"; Algorithm 2)
# ----------------------------------------------------------------------------

def test_density_map_counts_points_per_cell_area():
    """Density = (projections in the cell) / (cell area), by testing the cell's
    inequalities point by point -- no floor, no index arithmetic.  Coordinates are
    multiples of 1/64 and cells are 1/4 wide, so every comparison is exact."""
    rng = np.random.default_rng(5)
    n, M, G = 3000, 3, 8
    lo = np.array([[-1.0, -1.0], [0.0, -0.5], [-2.0, 1.0]], dtype=np.float32)
    width = np.array([[0.25, 0.25], [0.25, 0.125], [0.5, 0.25]], dtype=np.float32)
    cpu = (1.0 / width).astype(np.float32)
    proj = (rng.integers(-16, G * 16 + 16, size=(n, M, 2)) / 64.0).astype(np.float32) * (width * 4)[None] + lo[None]
    dens = oracle.density_map(proj, lo, cpu, G)
    assert dens.shape == (M, G, G)
    for m in range(M):
        area = float(width[m, 0]) * float(width[m, 1])
        for i0 in range(G):
            for i1 in range(G):
                inside = np.ones(n, dtype=bool)
                for axis, i in ((0, i0), (1, i1)):
                    a = float(lo[m, axis]) + i * float(width[m, axis])
                    b = a + float(width[m, axis])
                    x = proj[:, m, axis].astype(np.float64)
                    # border cells also take what lies outside the map on their side
                    inside &= ((x >= a) | (i == 0)) & ((x < b) | (i == G - 1))
                assert dens[m, i0, i1] == inside.sum() / area, (m, i0, i1)
    assert np.isclose(dens.sum(axis=(1, 2)) @ np.ones(M), sum(n / (float(w0) * float(w1)) for w0, w1 in width))


def test_query_radii_hand_example():
    """Two subspaces, a 3 x 3 grid with nine different values per subspace (a transposed
    or shifted cell shows), two lists, polynomial 0.5 + 0.25 f + 2 f^2; every number
    below is a dyadic fraction worked out by hand."""
    cent = np.array([[1.0, -1.0, 0.5, 2.0], [0.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    lo = np.array([[-1.5, 0.0], [0.0, -3.0]], dtype=np.float32)
    cpu = np.array([[1.0, 2.0], [0.5, 1.0]], dtype=np.float32)   # cell widths (1, 1/2) and (2, 1)
    fmap = np.array([[[0.0, 0.25, 0.5], [0.75, 1.0, 1.25], [1.5, 1.75, 2.0]],
                     [[2.0, 1.75, 1.5], [1.25, 1.0, 0.75], [0.5, 0.25, 0.0]]], dtype=np.float32)
    coef = np.array([[0.5, 0.25, 2.0], [1.0, 0.0, -1.0]], dtype=np.float32)
    fallback = np.array([7.0, 9.0], dtype=np.float32)
    q = np.array([[1.25, -0.25, 3.0, 0.25],     # list 0: residual (0.25, 0.75 | 2.5, -1.75)
                  [1.25, -0.25, 3.0, 0.25]],    # list 1: residual = the query itself
                 dtype=np.float32)
    near = np.array([0, 1], dtype=np.int32)
    r = oracle.query_radii(q, cent, near, lo, cpu, fmap, coef, fallback, 0.5)
    # query 0, subspace 0: t = (0.25+1.5)*1 = 1.75 -> 1 ; (0.75-0)*2 = 1.5 -> 1 ; f = 1.0
    #   p = 0.5 + 0.25 + 2 = 2.75 ; times 0.5 = 1.375
    # query 0, subspace 1: t = 2.5*0.5 = 1.25 -> 1 ; (-1.75+3)*1 = 1.25 -> 1 ; f = 1.0
    #   p = 1 - 1 = 0 -> not positive -> fallback 9 ; times 0.5 = 4.5
    # query 1, subspace 0: t = 2.75 -> 2 ; (-0.25)*2 < 0 -> 0 ; f = map[2][0] = 1.5
    #   p = 0.5 + 0.375 + 4.5 = 5.375 ; times 0.5 = 2.6875
    # query 1, subspace 1: t = 3*0.5 = 1.5 -> 1 ; (0.25+3) = 3.25 -> clamped to 2 ; f = 0.75
    #   p = 1 - 0.5625 = 0.4375 ; times 0.5 = 0.21875
    assert r.tolist() == [[1.375, 4.5], [2.6875, 0.21875]]


def test_query_radii_special_polynomials(tiny):
    """Degree 0: every radius is the constant times the scale.  Identity polynomial on a
    map that stores the cell number: the radius names the cell, which is checked against
    the cell's inequalities in float64.  Scale is a plain factor."""
    w, idx, centres, q = tiny["T_sift"]
    assert idx.dsub == 2
    M, G = idx.M, 10
    probe, _ = oracle.coarse(q, idx.centroids, 1)
    near = probe[:, 0]
    res = (q - idx.centroids[near]).reshape(-1, M, 2)
    lo = res.min(0).astype(np.float32)
    span = (res.max(0) - lo).astype(np.float32)
    cpu = (np.float32(G) / span).astype(np.float32)
    fb = np.full(M, 3.0, dtype=np.float32)
    const = np.linspace(0.5, 2.0, M).astype(np.float32)[:, None]
    r = oracle.query_radii(q, idx.centroids, near, lo, cpu, np.zeros((M, G, G), np.float32), const, fb, 1.5)
    assert np.array_equal(r, np.tile((const[:, 0] * np.float32(1.5))[None], (q.shape[0], 1)))
    cellno = np.tile(np.arange(1, G * G + 1, dtype=np.float32).reshape(1, G, G), (M, 1, 1))
    ident = np.tile(np.array([[0.0, 1.0]], dtype=np.float32), (M, 1))
    r1 = oracle.query_radii(q, idx.centroids, near, lo, cpu, cellno, ident, fb, 1.0)
    r2 = oracle.query_radii(q, idx.centroids, near, lo, cpu, cellno, ident, fb, 0.25)
    assert np.array_equal(r2, r1 * np.float32(0.25))
    cell = r1.astype(np.int64) - 1
    i0, i1 = cell // G, cell % G
    t = (res.astype(np.float64) - lo[None]) * cpu[None].astype(np.float64)   # position in cell units
    checked = 0
    for axis, i in ((0, i0), (1, i1)):
        ta = t[:, :, axis]
        clear = np.abs(ta - np.round(ta)) > 1e-4       # away from a cell border, fp32 and fp64 agree
        ok = ((ta >= i) | (i == 0)) & ((ta < i + 1) | (i == G - 1))
        assert np.all(ok[clear])
        checked += int(clear.sum())
    assert checked > 0.9 * 2 * cell.size
    # a different nearest list moves the residual: the look-up must follow it
    other = (near + 1) % idx.nlist
    r3 = oracle.query_radii(q, idx.centroids, other, lo, cpu, cellno, ident, fb, 1.0)
    assert not np.array_equal(r3, r1)


def test_fitted_radius_model_map_is_the_density_map(tiny):
    """The offline fit (input recipe) stores log(1 + density): its map must be the
    oracle's density map of the same projections, and its radii must be usable."""
    w, idx, centres, q = tiny["T_sift"]
    md = wl.fit_radius_model(w, idx, centres, 0.25, G=20, with_projections=True)
    dens = oracle.density_map(md["projections"], md["lo"], md["cells_per_unit"], 20)
    assert dens.sum() > 0
    np.testing.assert_allclose(md["map"], np.log1p(dens), rtol=1e-6, atol=1e-7)
    near, _ = oracle.coarse(q, idx.centroids, 1)
    r = oracle.query_radii(q, idx.centroids, near[:, 0], md["lo"], md["cells_per_unit"], md["map"],
                           md["coef"], md["fallback"], 1.0)
    assert np.all(r > 0) and np.all(np.isfinite(r))
    # the radii keep roughly the fraction of entries they were fitted for
    probes, _ = oracle.coarse(q, idx.centroids, 1)
    _, mask = oracle.build_lut(q, idx.centroids, idx.codebooks, probes, r)
    bits = np.unpackbits(mask.view(np.uint8)).sum() / (q.shape[0] * idx.M * 256.0)
    assert 0.1 < bits < 0.5, bits


def test_radius_model_fitted_to_true_neighbours(tiny):
    """The paper's regression target (Sec. 4.1): the radius that contains the entries of the
    query's true nearest neighbours.  Direction checks on the recipe: such radii reach most of
    the unthresholded recall, halving them (the paper's scale) costs recall, and on average
    they do contain the entries of the true neighbours of fresh queries."""
    w, idx, centres, q = tiny["T_sift"]
    md = wl.fit_radius_model(w, idx, centres, G=20, target="top", top=w.k)
    arrays = (md["lo"], md["cells_per_unit"], md["map"], md["coef"], md["fallback"])
    near, _ = oracle.coarse(q, idx.centroids, 1)
    truth = wl.exact_knn(w, centres, torch.from_numpy(q), w.k)
    rec = {}
    for scale in (1.0, 0.5):
        r = oracle.query_radii(q, idx.centroids, near[:, 0], *arrays, scale)
        ids, _ = oracle.search(q, idx, w.nprobe, w.k, r)
        rec[scale] = wl.recall_at_k(ids, truth)[0]
    ids, _ = oracle.search(q, idx, w.nprobe, w.k, np.full(idx.M, np.inf, np.float32))
    full = wl.recall_at_k(ids, truth)[0]
    assert rec[1.0] > 0.8 * full and rec[0.5] < rec[1.0]
    # containment: for fresh queries, the share of (neighbour, subspace) pairs whose entry lies
    # within the predicted radius of the query's residual w.r.t. the neighbour's list
    r = oracle.query_radii(q, idx.centroids, near[:, 0], *arrays, 1.0).astype(np.float64)
    row_of_id = np.empty(idx.N, dtype=np.int64)
    row_of_id[idx.ids] = np.arange(idx.N)
    inside = total = 0
    for i in range(q.shape[0]):
        rows = row_of_id[truth[i]]
        lists = np.searchsorted(idx.list_offsets, rows, side="right") - 1
        for row, c in zip(rows, lists):
            res = (q[i].astype(np.float64) - idx.centroids[c]).reshape(idx.M, idx.dsub)
            ent = idx.codebooks[np.arange(idx.M), idx.codes[row]].astype(np.float64)
            inside += int((np.sqrt(((res - ent) ** 2).sum(1)) <= r[i]).sum())
            total += idx.M
    assert inside / total > 0.85, inside / total


# ----------------------------------------------------------------------------
# random odd shapes against a float64 transcription of the definitions
# ----------------------------------------------------------------------------

def _definition_search(q, idx, nprobe, k, radii, metric):
    """The search path from its definitions, in float64 numpy, one query: list scores,
    nprobe best lists by (score, list), truncated table sums (L2) or negated inner
    products with the threshold bound (inner product), k best by (value, id)."""
    q = q.astype(np.float64)
    cen = idx.centroids.astype(np.float64)
    cb = idx.codebooks.astype(np.float64)
    M, dsub = idx.M, idx.dsub
    score = ((q[None] - cen) ** 2).sum(1) if metric == 0 else -(cen @ q)
    probes = np.lexsort((np.arange(idx.nlist), score))[:nprobe]
    r2 = radii.astype(np.float64) ** 2
    vals, ids = [], []
    for c in probes:
        lo, hi = idx.list_offsets[c], idx.list_offsets[c + 1]
        codes = idx.codes[lo:hi]
        ent = cb[np.arange(M)[None, :], codes]                      # [n][M][dsub]
        if metric == 0:
            res = (q - cen[c]).reshape(M, dsub)
            d2 = ((res[None] - ent) ** 2).sum(-1)
            v = np.minimum(d2, r2[None]).sum(1)
        else:
            qm = q.reshape(M, dsub)
            ip = (ent * qm[None]).sum(-1)
            thr = 0.5 * ((qm ** 2).sum(1) - r2)
            v = -(cen[c] @ q) - np.maximum(ip, thr[None]).sum(1)
        vals.append(v)
        ids.append(idx.ids[lo:hi])
    vals, ids = np.concatenate(vals), np.concatenate(ids)
    order = np.lexsort((ids, vals))[:k]
    return probes, vals[order], ids[order], np.sort(vals)


@pytest.mark.parametrize("seed", range(24))
def test_random_odd_shapes_against_definitions(seed):
    rng = np.random.default_rng(1000 + seed)
    dsub = int(rng.choice([1, 2, 3, 4, 5, 8]))
    M = int(rng.choice([1, 2, 3, 7, 16]))
    D = M * dsub
    nlist = int(rng.choice([1, 2, 5, 9]))
    sizes = rng.integers(0, 40, size=nlist)
    if seed % 3 == 0:
        sizes[rng.integers(0, nlist)] = 0                           # an empty list
    N = int(sizes.sum())
    offs = np.zeros(nlist + 1, dtype=np.int64)
    offs[1:] = np.cumsum(sizes)
    idx = wl.Index(N=N, D=D, nlist=nlist, M=M, centroids=rng.normal(size=(nlist, D)).astype(np.float32),
                   codebooks=(0.7 * rng.normal(size=(M, 256, dsub))).astype(np.float32), list_offsets=offs,
                   codes=rng.integers(0, 256, size=(N, M), dtype=np.uint8),
                   ids=(rng.permutation(N) * 2 + 5).astype(np.int64))
    nprobe = int(rng.integers(1, nlist + 1))
    k = int(rng.choice([1, 3, 10, 64]))
    q = rng.normal(size=(6, D)).astype(np.float32)
    radii = (np.sqrt(dsub) * rng.uniform(0.4, 1.6, size=M)).astype(np.float32)
    if seed % 4 == 1:
        radii[:] = np.inf
    for metric in (0, 1):
        o_ids, o_val = oracle.search(q, idx, nprobe, k, radii, metric=metric)
        o_probes, _ = oracle.coarse(q, idx.centroids, nprobe, metric=metric)
        for i in range(q.shape[0]):
            probes, vals, ids, allv = _definition_search(q[i], idx, nprobe, k, radii, metric)
            assert np.array_equal(o_probes[i], probes), (seed, metric, i)   # random scores: no near ties
            n = len(vals)
            assert np.all(o_ids[i, n:] == -1) and np.all(np.isinf(o_val[i, n:]))
            np.testing.assert_allclose(o_val[i, :n], vals, rtol=2e-5, atol=2e-5)
            # ids agree wherever the value is separated from its neighbours in the full order
            for j in range(n):
                gap = np.abs(allv - vals[j])
                if (gap < 1e-4 * (1 + abs(vals[j]))).sum() == 1:
                    assert o_ids[i, j] == ids[j], (seed, metric, i, j)


def test_recall_ground_truth_and_measure(tiny):
    """The benchmark's recall figures rest on workloads.exact_knn (streamed fp32 matrix form) and
    workloads.recall_at_k: the first must agree with the oracle's float64 brute force except
    where distances nearly tie, the second is checked on a hand-made case."""
    for name in ("T_sift", "T_tti"):
        w, idx, centres, q = tiny[name]
        base = wl.base_vectors(w, centres).numpy()
        for metric in (0, 1):
            fast = wl.exact_knn(w, centres, torch.from_numpy(q), w.k, metric=metric)
            slow, sdist = oracle.exact_knn(base, q, w.k + 1, metric=metric)
            for i in range(q.shape[0]):
                # the k-th and (k+1)-th true distances are apart: the set is well defined
                if sdist[i, w.k] - sdist[i, w.k - 1] > 1e-4 * (1 + abs(sdist[i, w.k])):
                    assert set(fast[i].tolist()) == set(slow[i, :w.k].tolist()), (name, metric, i)
            assert np.mean(fast[:, 0] == slow[:, 0]) > 0.9
    found = np.array([[1, 2, 3, -1], [9, 8, 7, 6]])
    truth = np.array([[3, 2, 5, 4], [6, 0, 1, 2]])
    rec, r1 = wl.recall_at_k(found, truth)
    assert rec == (2 + 1) / 8.0 and r1 == 1.0     # first row holds truth[0][0] = 3, second holds 6
    rec, r1 = wl.recall_at_k(np.array([[0, 1]]), np.array([[2, 0]]))
    assert rec == 0.5 and r1 == 0.0
