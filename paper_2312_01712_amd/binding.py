"""Thin ctypes binding of the C-ABI library (include/ivfpq.h).

Argument marshalling only: torch supplies device memory (`data_ptr()`) and the
current stream; every step of the search path runs in the HIP kernels of
`libivfpq_hip.so`.  There is no fallback: if the library is missing and cannot
be built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libivfpq_hip.so")
_lib = None

# every symbol include/ivfpq.h declares
SYMBOLS = [
    "ivfpq_index_create", "ivfpq_index_destroy", "ivfpq_search_workspace_bytes", "ivfpq_search",
    "ivfpq_coarse", "ivfpq_build_lut", "ivfpq_scan_topk", "ivfpq_scan_all", "ivfpq_index_get_info",
    "ivfpq_set_option", "ivfpq_coarse_fallbacks", "ivfpq_last_error",
    "ivfpq_search_ex", "ivfpq_build_lut_ex", "ivfpq_scan_topk_ex", "ivfpq_scan_all_ex",
    "ivfpq_radius_model_create", "ivfpq_radius_model_destroy", "ivfpq_query_radii",
    "ivfpq_search_noalloc", "ivfpq_search_workspace_bytes_ex", "ivfpq_resolve_strategy",
]

SCORE_DISTANCE, SCORE_HIT_COUNT, SCORE_HIT_REWARD = 0, 1, 2
SCAN_AUTO, SCAN_QUERY_MAJOR, SCAN_LIST_MAJOR = 0, 1, 2
METRIC_L2, METRIC_IP = 0, 1

OK, ERR_INVALID_ARGUMENT, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_NO_MEMORY = 0, -1, -2, -3, -4, -5


class IvfpqError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"ivfpq status {status}: {text}")
        self.status = status


class _Desc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int64), ("D", ctypes.c_int32), ("nlist", ctypes.c_int32),
                ("M", ctypes.c_int32), ("ksub", ctypes.c_int32), ("centroids", ctypes.c_void_p),
                ("codebooks", ctypes.c_void_p), ("list_offsets", ctypes.c_void_p),
                ("codes", ctypes.c_void_p), ("ids", ctypes.c_void_p), ("metric", ctypes.c_int32)]


class _Scoring(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("d_query_radii", ctypes.c_void_p), ("strategy", ctypes.c_int32)]


class _Info(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int64), ("D", ctypes.c_int32), ("nlist", ctypes.c_int32),
                ("M", ctypes.c_int32), ("dsub", ctypes.c_int32), ("code_bytes", ctypes.c_int64),
                ("max_list_len", ctypes.c_int64), ("metric", ctypes.c_int32)]


def load_library():
    """Load libivfpq_hip.so, building it first only if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    lib.ivfpq_index_create.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(vp)]
    lib.ivfpq_index_destroy.argtypes = [vp]
    lib.ivfpq_index_destroy.restype = None
    lib.ivfpq_search_workspace_bytes.argtypes = [vp, i64, i32, i32]
    lib.ivfpq_search_workspace_bytes.restype = sz
    lib.ivfpq_search_workspace_bytes_ex.argtypes = [vp, i64, i32, i32, ctypes.POINTER(_Scoring)]
    lib.ivfpq_search_workspace_bytes_ex.restype = sz
    lib.ivfpq_resolve_strategy.argtypes = [vp, i64, i32, i32, ctypes.POINTER(_Scoring)]
    lib.ivfpq_search.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.ivfpq_search_noalloc.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp, vp]
    lib.ivfpq_coarse.argtypes = [vp, vp, i64, i32, vp, vp, vp, sz, vp]
    lib.ivfpq_build_lut.argtypes = [vp, vp, i64, i32, vp, vp, vp, vp, vp]
    lib.ivfpq_scan_topk.argtypes = [vp, vp, i64, i32, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.ivfpq_scan_all.argtypes = [vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp]
    sp = ctypes.POINTER(_Scoring)
    lib.ivfpq_search_ex.argtypes = [vp, vp, i64, i32, i32, vp, sp, vp, vp, vp, sz, vp]
    lib.ivfpq_build_lut_ex.argtypes = [vp, vp, i64, i32, vp, vp, sp, vp, vp, vp]
    lib.ivfpq_scan_topk_ex.argtypes = [vp, vp, i64, i32, vp, i32, vp, sp, vp, vp, vp, sz, vp]
    lib.ivfpq_scan_all_ex.argtypes = [vp, vp, i64, i32, vp, vp, sp, vp, vp, vp, vp, vp]
    lib.ivfpq_radius_model_create.argtypes = [vp, ctypes.POINTER(_RadiusModelDesc), ctypes.POINTER(vp)]
    lib.ivfpq_radius_model_destroy.argtypes = [vp]
    lib.ivfpq_radius_model_destroy.restype = None
    lib.ivfpq_query_radii.argtypes = [vp, vp, vp, i64, vp, i32, ctypes.c_float, vp, vp]
    lib.ivfpq_index_get_info.argtypes = [vp, ctypes.POINTER(_Info)]
    lib.ivfpq_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int]
    lib.ivfpq_coarse_fallbacks.argtypes = [ctypes.c_int]
    lib.ivfpq_coarse_fallbacks.restype = ctypes.c_int64
    lib.ivfpq_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise IvfpqError(rc, load_library().ivfpq_last_error().decode())


def last_error() -> str:
    return load_library().ivfpq_last_error().decode()


def set_option(name: str, value: int):
    _check(load_library().ivfpq_set_option(name.encode(), int(value)))


def coarse_fallbacks(reset: bool = False) -> int:
    n = int(load_library().ivfpq_coarse_fallbacks(1 if reset else 0))
    if n < 0:
        _check(n)
    return n


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, shape=None, device=None, what: str = "tensor") -> torch.Tensor:
    """A tensor the kernels may read or write as it is: on the GPU (the index's, when
    `device` is given), contiguous, of the stated dtype and, when given, shape (None in a
    position leaves that extent free).  The kernels index by these shapes without a bounds
    check of their own, so a mismatch is refused here."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{what}: expected a contiguous CUDA tensor of {dtype}, got "
                         f"{getattr(t, 'dtype', type(t))} on {getattr(t, 'device', 'the host')}")
    if device is not None and t.device.index != device:
        raise ValueError(f"{what}: on cuda:{t.device.index}, the index lives on cuda:{device}")
    if shape is not None:
        if t.dim() != len(shape) or any(e is not None and int(g) != int(e) for g, e in zip(t.shape, shape)):
            raise ValueError(f"{what}: shape {tuple(t.shape)} does not match {tuple(shape)}")
    return t


def _radii(radii, M: int) -> np.ndarray:
    r = np.ascontiguousarray(radii, dtype=np.float32)
    if r.shape != (M,):
        raise ValueError(f"radii must have shape ({M},)")
    return r


def _scoring(mode: int, query_radii: Optional[torch.Tensor], radii, Q: int, M: int, strategy: int = SCAN_AUTO):
    """(host radii pointer or None, ctypes scoring struct or None, objects to keep alive)."""
    keep = []
    qr_ptr = None
    if query_radii is not None:
        qr = _dev(query_radii, torch.float32, (Q, M), what="query_radii")
        qr_ptr = qr.data_ptr()
        keep.append(qr)
    r_ptr = None
    if radii is not None:
        r = _radii(radii, M)
        r_ptr = r.ctypes.data
        keep.append(r)
    sc = None
    if mode != SCORE_DISTANCE or qr_ptr is not None or strategy != SCAN_AUTO:
        sc = _Scoring(mode=int(mode), d_query_radii=qr_ptr, strategy=int(strategy))
        keep.append(sc)
    return r_ptr, (ctypes.byref(sc) if sc is not None else None), keep


class _RadiusModelDesc(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int32), ("grid", ctypes.c_int32), ("degree", ctypes.c_int32),
                ("lo", ctypes.c_void_p), ("cells_per_unit", ctypes.c_void_p), ("map", ctypes.c_void_p),
                ("coef", ctypes.c_void_p), ("fallback", ctypes.c_void_p)]


class RadiusModel:
    """Device copy of a threshold model (`ivfpq_radius_model_create`): per subspace a
    grid map [M][G][G] with its low corner and cells per unit [M][2], polynomial
    coefficients [M][degree+1] (lowest power first) and a fallback radius [M]."""

    def __init__(self, index: "IvfPqIndex", lo, cells_per_unit, fmap, coef, fallback):
        arr = [np.ascontiguousarray(a, dtype=np.float32) for a in (lo, cells_per_unit, fmap, coef, fallback)]
        l, c, mp, cf, fb = arr
        M = mp.shape[0]
        if mp.ndim != 3 or mp.shape[1] != mp.shape[2] or l.shape != (M, 2) or c.shape != (M, 2) \
                or cf.ndim != 2 or cf.shape[0] != M or fb.shape != (M,):
            raise ValueError("radius model arrays have inconsistent shapes")
        desc = _RadiusModelDesc(M=M, grid=mp.shape[1], degree=cf.shape[1] - 1, lo=l.ctypes.data,
                                cells_per_unit=c.ctypes.data, map=mp.ctypes.data, coef=cf.ctypes.data,
                                fallback=fb.ctypes.data)
        handle = ctypes.c_void_p()
        self._h = None
        _check(load_library().ivfpq_radius_model_create(index._h, ctypes.byref(desc), ctypes.byref(handle)))
        self._h = handle
        self.M = M
        del arr

    def close(self):
        if getattr(self, "_h", None):
            load_library().ivfpq_radius_model_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class IvfPqIndex:
    """Device-resident index.  `ivfpq_index_create` copies and re-lays out the
    arrays; the numpy inputs are not kept."""

    def __init__(self, centroids, codebooks, list_offsets, codes, ids=None, metric: int = METRIC_L2):
        lib = load_library()
        cent = np.ascontiguousarray(centroids, dtype=np.float32)
        cb = np.ascontiguousarray(codebooks, dtype=np.float32)
        offs = np.ascontiguousarray(list_offsets, dtype=np.int64)
        if isinstance(codes, torch.Tensor):
            codes_ref, codes_ptr, N = codes, codes.data_ptr(), codes.shape[0]
            assert codes.dtype == torch.uint8 and codes.is_contiguous()
        else:
            codes_ref = np.ascontiguousarray(codes, dtype=np.uint8)
            codes_ptr, N = codes_ref.ctypes.data, codes_ref.shape[0]
        if ids is None:
            ids_ref, ids_ptr = None, None
        elif isinstance(ids, torch.Tensor):
            assert ids.dtype == torch.int64 and ids.is_contiguous()
            ids_ref, ids_ptr = ids, ids.data_ptr()
        else:
            ids_ref = np.ascontiguousarray(ids, dtype=np.int64)
            ids_ptr = ids_ref.ctypes.data
        nlist, D = cent.shape
        M = cb.shape[0]
        desc = _Desc(N=N, D=D, nlist=nlist, M=M, ksub=cb.shape[1], centroids=cent.ctypes.data,
                     codebooks=cb.ctypes.data, list_offsets=offs.ctypes.data,
                     codes=codes_ptr if N > 0 else (codes_ptr or None), ids=ids_ptr, metric=int(metric))
        handle = ctypes.c_void_p()
        self._h = None
        _check(lib.ivfpq_index_create(ctypes.byref(desc), ctypes.byref(handle)))
        self._h = handle
        self.N, self.D, self.nlist, self.M, self.metric = N, D, nlist, M, int(metric)
        self.device = torch.cuda.current_device()
        del codes_ref, ids_ref

    @classmethod
    def from_index(cls, idx, metric: int = METRIC_L2) -> "IvfPqIndex":
        return cls(idx.centroids, idx.codebooks, idx.list_offsets, idx.codes, idx.ids, metric=metric)

    def info(self) -> dict:
        i = _Info()
        _check(load_library().ivfpq_index_get_info(self._h, ctypes.byref(i)))
        return {f: getattr(i, f) for f, _ in _Info._fields_}

    def close(self):
        if getattr(self, "_h", None):
            load_library().ivfpq_index_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- search-side calls -------------------------------------------------
    def workspace_bytes(self, Q: int, nprobe: int, k: int, strategy: int = SCAN_AUTO) -> int:
        sc = _Scoring(mode=SCORE_DISTANCE, d_query_radii=None, strategy=int(strategy))
        return int(load_library().ivfpq_search_workspace_bytes_ex(self._h, Q, nprobe, k, ctypes.byref(sc)))

    def resolve_strategy(self, Q: int, nprobe: int, k: int, mode: int = SCORE_DISTANCE, strategy: int = SCAN_AUTO) -> int:
        """SCAN_QUERY_MAJOR or SCAN_LIST_MAJOR: what a call of this shape runs with."""
        sc = _Scoring(mode=int(mode), d_query_radii=None, strategy=int(strategy))
        rc = int(load_library().ivfpq_resolve_strategy(self._h, Q, nprobe, k, ctypes.byref(sc)))
        if rc < 0:
            _check(rc)
        return rc

    def workspace(self, Q: int, nprobe: int, k: int, strategy: int = SCAN_AUTO) -> torch.Tensor:
        n = max(256, self.workspace_bytes(Q, nprobe, k, strategy))
        return torch.empty(n, dtype=torch.uint8, device="cuda")

    def search(self, queries: torch.Tensor, nprobe: int, k: int, radii, workspace: Optional[torch.Tensor] = None,
               out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None, mode: int = SCORE_DISTANCE,
               query_radii: Optional[torch.Tensor] = None, strategy: int = SCAN_AUTO) -> Tuple[torch.Tensor, torch.Tensor]:
        q = self._queries(queries)
        Q = q.shape[0]
        r_ptr, sc, keep = _scoring(mode, query_radii, radii, Q, self.M, strategy)
        ws = self._workspace(workspace, Q, nprobe, k, strategy)
        ids, dist = self._outputs(out, Q, k, q.device)
        lib = load_library()
        if sc is None:
            _check(lib.ivfpq_search(self._h, q.data_ptr(), Q, nprobe, k, r_ptr, ids.data_ptr(),
                                    dist.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
        else:
            _check(lib.ivfpq_search_ex(self._h, q.data_ptr(), Q, nprobe, k, r_ptr, sc, ids.data_ptr(),
                                       dist.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
        del keep
        return ids, dist

    # ---- argument checks shared by the calls below ---------------------------
    def _queries(self, queries) -> torch.Tensor:
        return _dev(queries, torch.float32, (None, self.D), self.device, "queries")

    def _probes(self, probe_ids, Q: int) -> torch.Tensor:
        return _dev(probe_ids, torch.int32, (Q, None), self.device, "probe_ids")

    def _workspace(self, workspace, Q: int, nprobe: int, k: int, strategy: int = SCAN_AUTO) -> torch.Tensor:
        if workspace is None:
            return self.workspace(Q, nprobe, k, strategy)
        return _dev(workspace, torch.uint8, (None,), self.device, "workspace")

    def _outputs(self, out, Q: int, k: int, device):
        if out is None:
            return (torch.empty((Q, k), dtype=torch.int64, device=device),
                    torch.empty((Q, k), dtype=torch.float32, device=device))
        return (_dev(out[0], torch.int64, (Q, k), self.device, "out ids"),
                _dev(out[1], torch.float32, (Q, k), self.device, "out distances"))

    def search_noalloc(self, queries: torch.Tensor, nprobe: int, k: int, radii,
                       out: Tuple[torch.Tensor, torch.Tensor]) -> Tuple[torch.Tensor, torch.Tensor]:
        """`ivfpq_search_noalloc`: the search whose workspace is the library's own static
        device array; the caller passes inputs and outputs only."""
        q = self._queries(queries)
        Q = q.shape[0]
        ids, dist = self._outputs(out, Q, k, q.device)
        r = _radii(radii, self.M)
        _check(load_library().ivfpq_search_noalloc(self._h, q.data_ptr(), Q, nprobe, k, r.ctypes.data,
                                                   ids.data_ptr(), dist.data_ptr(), _stream()))
        return ids, dist

    def coarse(self, queries: torch.Tensor, nprobe: int, workspace: Optional[torch.Tensor] = None,
               out: Optional[torch.Tensor] = None, with_distances: bool = True):
        """Probe lists [Q][nprobe] int32 (written into `out` when given) and, unless
        with_distances is False, their distances."""
        q = self._queries(queries)
        Q = q.shape[0]
        ws = self._workspace(workspace, Q, nprobe, 1)
        pid = torch.empty((Q, nprobe), dtype=torch.int32, device=q.device) if out is None \
            else _dev(out, torch.int32, (Q, nprobe), self.device, "out probe ids")
        pd = torch.empty((Q, nprobe), dtype=torch.float32, device=q.device) if with_distances else None
        _check(load_library().ivfpq_coarse(self._h, q.data_ptr(), Q, nprobe, pid.data_ptr(),
                                           pd.data_ptr() if pd is not None else None,
                                           ws.data_ptr(), ws.numel(), _stream()))
        return pid, pd

    def query_radii(self, model: RadiusModel, queries: torch.Tensor, probe_ids: torch.Tensor, scale: float = 1.0,
                    out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Per-(query, subspace) radii [Q][M] from the threshold model, looked up at the
        residual w.r.t. the first list of each row of probe_ids."""
        q = self._queries(queries)
        pid = self._probes(probe_ids, q.shape[0])
        Q, nprobe = pid.shape
        r = out if out is not None else torch.empty((Q, self.M), dtype=torch.float32, device=q.device)
        _dev(r, torch.float32, (Q, self.M), self.device, "out radii")
        _check(load_library().ivfpq_query_radii(self._h, model._h, q.data_ptr(), Q, pid.data_ptr(), nprobe,
                                                ctypes.c_float(scale), r.data_ptr(), _stream()))
        return r

    def build_lut(self, queries: torch.Tensor, probe_ids: torch.Tensor, radii, mode: int = SCORE_DISTANCE,
                  query_radii: Optional[torch.Tensor] = None):
        q = self._queries(queries)
        pid = self._probes(probe_ids, q.shape[0])
        Q, nprobe = pid.shape
        r_ptr, sc, keep = _scoring(mode, query_radii, radii, Q, self.M)
        lut = torch.empty((Q, nprobe, self.M, 256), dtype=torch.float32, device=q.device)
        mask = torch.zeros((Q, nprobe, self.M, 4), dtype=torch.int64, device=q.device)
        _check(load_library().ivfpq_build_lut_ex(self._h, q.data_ptr(), Q, nprobe, pid.data_ptr(), r_ptr, sc,
                                                 lut.data_ptr(), mask.data_ptr(), _stream()))
        del keep
        return lut, mask

    def scan_topk(self, queries: torch.Tensor, probe_ids: torch.Tensor, k: int, radii,
                  workspace: Optional[torch.Tensor] = None, mode: int = SCORE_DISTANCE,
                  query_radii: Optional[torch.Tensor] = None,
                  out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None, strategy: int = SCAN_AUTO):
        q = self._queries(queries)
        pid = self._probes(probe_ids, q.shape[0])
        Q, nprobe = pid.shape
        r_ptr, sc, keep = _scoring(mode, query_radii, radii, Q, self.M, strategy)
        ws = self._workspace(workspace, Q, nprobe, k, strategy)
        ids, dist = self._outputs(out, Q, k, q.device)
        _check(load_library().ivfpq_scan_topk_ex(self._h, q.data_ptr(), Q, nprobe, pid.data_ptr(), k, r_ptr, sc,
                                                 ids.data_ptr(), dist.data_ptr(), ws.data_ptr(), ws.numel(),
                                                 _stream()))
        del keep
        return ids, dist

    def scan_all(self, queries: torch.Tensor, probe_ids: torch.Tensor, radii, cand_offsets: torch.Tensor,
                 mode: int = SCORE_DISTANCE, query_radii: Optional[torch.Tensor] = None):
        """Every candidate's (distance, id); cand_offsets [Q+1] int64 on the device."""
        q = self._queries(queries)
        pid = self._probes(probe_ids, q.shape[0])
        Q, nprobe = pid.shape
        offs = _dev(cand_offsets, torch.int64, (Q + 1,), self.device, "cand_offsets")
        r_ptr, sc, keep = _scoring(mode, query_radii, radii, Q, self.M)
        total = int(offs[-1].item()) if Q > 0 else 0
        dist = torch.empty(max(total, 1), dtype=torch.float32, device=q.device)
        ids = torch.empty(max(total, 1), dtype=torch.int64, device=q.device)
        err = torch.empty(1, dtype=torch.int32, device=q.device)
        _check(load_library().ivfpq_scan_all_ex(self._h, q.data_ptr(), Q, nprobe, pid.data_ptr(), r_ptr, sc,
                                                offs.data_ptr(), dist.data_ptr(), ids.data_ptr(), err.data_ptr(),
                                                _stream()))
        del keep
        return dist[:total], ids[:total], err
