"""ctypes front end of the CPU oracle (oracle/ivfpq_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  It takes and returns host numpy arrays, imports
nothing from the GPU package and never touches a GPU.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ivfpq_oracle.cpp")
_LIB = os.path.join(_HERE, "libivfpq_oracle.so")
_lib = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_u64p = ctypes.POINTER(ctypes.c_uint64)
_u8p = ctypes.POINTER(ctypes.c_uint8)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc: -O2, no contraction, no fast-math."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
               "-shared", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: Optional[np.ndarray], ty):
    if a is None:
        return ctypes.cast(None, ty)
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ty)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def coarse(queries, centroids, nprobe: int, metric: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    q, c = _f32(queries), _f32(centroids)
    Q, D = q.shape
    ids = np.empty((Q, nprobe), dtype=np.int32)
    dist = np.empty((Q, nprobe), dtype=np.float32)
    rc = _load().oracle_coarse(ctypes.c_int64(Q), D, c.shape[0], _p(q, _f32p), _p(c, _f32p), nprobe,
                               metric, _p(ids, _i32p), _p(dist, _f32p))
    if rc:
        raise ValueError("oracle_coarse: invalid argument")
    return ids, dist


def _stride(r: np.ndarray, Q: int, M: int) -> int:
    """radii [M] (shared) -> 0, radii [Q][M] (per query) -> M."""
    if r.shape == (M,):
        return 0
    if r.shape == (Q, M):
        return M
    raise ValueError(f"radii must have shape ({M},) or ({Q}, {M})")


def build_lut(queries, centroids, codebooks, probe_ids, radii, mode: int = 0,
              metric: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    q, c, cb, r = _f32(queries), _f32(centroids), _f32(codebooks), _f32(radii)
    pid = np.ascontiguousarray(probe_ids, dtype=np.int32)
    Q, D = q.shape
    M = cb.shape[0]
    nprobe = pid.shape[1]
    lut = np.empty((Q, nprobe, M, 256), dtype=np.float32)
    mask = np.empty((Q, nprobe, M, 4), dtype=np.uint64)
    rc = _load().oracle_build_lut(ctypes.c_int64(Q), D, M, _p(q, _f32p), _p(c, _f32p), _p(cb, _f32p),
                                  _p(pid, _i32p), nprobe, _p(r, _f32p), _stride(r, Q, M), mode, metric,
                                  _p(lut, _f32p), _p(mask, _u64p))
    if rc:
        raise ValueError("oracle_build_lut: invalid argument")
    return lut, mask


def scan_all(queries, index, probe_ids, radii, mode: int = 0,
             metric: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(cand_offsets [Q+1], dist [total], ids [total]) for every candidate."""
    q, r = _f32(queries), _f32(radii)
    pid = np.ascontiguousarray(probe_ids, dtype=np.int32)
    Q, D = q.shape
    nprobe = pid.shape[1]
    offs = np.empty(Q + 1, dtype=np.int64)
    lib = _load()
    args = lambda d, i: (ctypes.c_int64(Q), D, index.M, _p(q, _f32p), _p(index.centroids, _f32p),
                         _p(index.codebooks, _f32p), _p(index.list_offsets, _i64p),
                         _p(index.codes, _u8p), _p(index.ids, _i64p), _p(pid, _i32p), nprobe,
                         _p(r, _f32p), _stride(r, Q, index.M), mode, metric, _p(offs, _i64p), _p(d, _f32p),
                         _p(i, _i64p))
    if lib.oracle_scan_all(*args(None, None)):
        raise ValueError("oracle_scan_all: invalid argument")
    total = int(offs[Q])
    dist = np.empty(total, dtype=np.float32)
    ids = np.empty(total, dtype=np.int64)
    lib.oracle_scan_all(*args(dist, ids))
    return offs, dist, ids


def topk(dist, ids, k: int) -> Tuple[np.ndarray, np.ndarray]:
    d = _f32(dist)
    i = np.ascontiguousarray(ids, dtype=np.int64)
    oi = np.empty(k, dtype=np.int64)
    od = np.empty(k, dtype=np.float32)
    _load().oracle_topk(ctypes.c_int64(d.shape[0]), _p(d, _f32p), _p(i, _i64p), k, _p(oi, _i64p),
                        _p(od, _f32p))
    return oi, od


def search(queries, index, nprobe: int, k: int, radii, threads: int = 1,
           q_range: Optional[Tuple[int, int]] = None, mode: int = 0,
           metric: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Whole search path.  threads > 1 runs the same single-threaded routine on
    disjoint query ranges from Python threads (ctypes releases the GIL)."""
    q, r = _f32(queries), _f32(radii)
    Q, D = q.shape
    lo, hi = q_range if q_range is not None else (0, Q)
    out_ids = np.full((Q, k), -1, dtype=np.int64)
    out_dist = np.full((Q, k), np.inf, dtype=np.float32)
    lib = _load()

    def run(a, b):
        rc = lib.oracle_search(ctypes.c_int64(a), ctypes.c_int64(b), D, index.nlist, index.M,
                               _p(q, _f32p), _p(index.centroids, _f32p), _p(index.codebooks, _f32p),
                               _p(index.list_offsets, _i64p), _p(index.codes, _u8p),
                               _p(index.ids, _i64p), nprobe, k, _p(r, _f32p), _stride(r, Q, index.M), mode, metric,
                               _p(out_ids, _i64p), _p(out_dist, _f32p))
        if rc:
            raise ValueError("oracle_search: invalid argument")

    if threads <= 1:
        run(lo, hi)
    else:
        cuts = np.linspace(lo, hi, threads + 1).astype(np.int64)
        ts = [threading.Thread(target=run, args=(int(cuts[t]), int(cuts[t + 1]))) for t in range(threads)]
        [t.start() for t in ts]
        [t.join() for t in ts]
    return out_ids, out_dist


def exact_knn(base, queries, k: int, metric: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    b, q = _f32(base), _f32(queries)
    N, D = b.shape
    Q = q.shape[0]
    oi = np.empty((Q, k), dtype=np.int64)
    od = np.empty((Q, k), dtype=np.float64)
    _load().oracle_exact_knn(ctypes.c_int64(N), D, _p(b, _f32p), ctypes.c_int64(Q), _p(q, _f32p), k,
                             metric, _p(oi, _i64p), _p(od, _f64p))
    return oi, od


def density_map(proj, lo, cells_per_unit, G: int) -> np.ndarray:
    """[M][G][G] fp64 densities (count / cell area) of projections [n][M][2]."""
    pr, l, c = _f32(proj), _f32(lo), _f32(cells_per_unit)
    n, M, two = pr.shape
    assert two == 2 and l.shape == (M, 2) and c.shape == (M, 2)
    out = np.empty((M, G, G), dtype=np.float64)
    if _load().oracle_density_map(ctypes.c_int64(n), M, _p(pr, _f32p), _p(l, _f32p), _p(c, _f32p), G,
                                  _p(out, _f64p)):
        raise ValueError("oracle_density_map: invalid argument")
    return out


def query_radii(queries, centroids, nearest, lo, cells_per_unit, fmap, coef, fallback,
                scale: float) -> np.ndarray:
    """radii [Q][M] from a per-subspace grid map [M][G][G] and polynomial [M][degree+1]
    (lowest power first), looked up at the residual w.r.t. list nearest[q]."""
    q, c = _f32(queries), _f32(centroids)
    l, cpu, mp, cf, fb = _f32(lo), _f32(cells_per_unit), _f32(fmap), _f32(coef), _f32(fallback)
    near = np.ascontiguousarray(nearest, dtype=np.int32)
    Q, D = q.shape
    M, G = mp.shape[0], mp.shape[1]
    assert mp.shape == (M, G, G) and l.shape == (M, 2) and cpu.shape == (M, 2)
    assert cf.shape[0] == M and fb.shape == (M,) and near.shape == (Q,)
    out = np.empty((Q, M), dtype=np.float32)
    rc = _load().oracle_query_radii(ctypes.c_int64(Q), D, M, _p(q, _f32p), _p(c, _f32p), c.shape[0],
                                    _p(near, _i32p), G, _p(l, _f32p), _p(cpu, _f32p), _p(mp, _f32p),
                                    cf.shape[1] - 1, _p(cf, _f32p), _p(fb, _f32p),
                                    ctypes.c_float(scale), _p(out, _f32p))
    if rc:
        raise ValueError("oracle_query_radii: invalid argument")
    return out
