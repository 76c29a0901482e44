"""Input builders shared by the host and GPU tests (no search arithmetic)."""
import numpy as np

from paper_2312_01712_amd import workloads as wl


def identity_index(rng, N=1500, D=12, nlist=6):
    """Hand-built index that reconstructs every point exactly: integer data,
    integer centroids, M = D (dsub = 1), codebook[m] = {-128..127},
    code = residual + 128.  All arithmetic on it is exact in fp32."""
    base = rng.integers(0, 128, size=(N, D)).astype(np.int64)
    cent = rng.integers(0, 128, size=(nlist, D)).astype(np.int64)
    d = ((base[:, None, :] - cent[None, :, :]) ** 2).sum(-1)
    labels = d.argmin(1)
    order = np.argsort(labels, kind="stable")
    res = base - cent[labels]
    codes = (res + 128).astype(np.uint8)
    offs = np.zeros(nlist + 1, dtype=np.int64)
    offs[1:] = np.cumsum(np.bincount(labels, minlength=nlist))
    cb = np.tile((np.arange(256) - 128).astype(np.float32)[None, :, None], (D, 1, 1))
    idx = wl.Index(N=N, D=D, nlist=nlist, M=D, centroids=cent.astype(np.float32),
                   codebooks=np.ascontiguousarray(cb), list_offsets=offs,
                   codes=np.ascontiguousarray(codes[order]), ids=order.astype(np.int64))
    return base, idx


def brute_knn_int(base, queries, k):
    d = ((base[None, :, :] - queries[:, None, :]) ** 2).sum(-1)        # int64, exact
    ids = np.empty((queries.shape[0], k), dtype=np.int64)
    dist = np.empty((queries.shape[0], k), dtype=np.int64)
    for q in range(queries.shape[0]):
        o = np.lexsort((np.arange(base.shape[0]), d[q]))[:k]
        ids[q], dist[q] = o, d[q][o]
    return ids, dist


def per_query_radii(w, idx, centres, q, keep=0.25, seed=11):
    """A radii[Q][M] input for the per-query-radius tests: the calibrated shared radii,
    each query's row stretched by seeded factors in [0.7, 1.3] (different per query and
    subspace, so that a row or column mix-up shows)."""
    shared = wl.calibrate_radii(w, idx, centres, keep)
    f = np.random.default_rng(seed).uniform(0.7, 1.3, size=(q.shape[0], idx.M)).astype(np.float32)
    return np.ascontiguousarray(shared[None, :] * f)
