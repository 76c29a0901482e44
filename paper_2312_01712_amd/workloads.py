"""Seeded synthetic workloads and the offline IVF-PQ index trainer.

This module produces *inputs only*: base vectors, queries, a trained index
(IVF centroids, residual PQ codebooks, list-sorted codes) and per-subspace
radii.  Both the HIP search path and the CPU oracle consume exactly what is
returned here; neither of them is imported from here and no step of the online
search (filtering, LUT construction, distance calculation, top-k) lives here.

The offline phase follows the paper's Sec. 2.1 ("Inverted File Index",
"Product Quantization") and Algorithm 1 up to the codebook: k-means over the
search points gives C clusters; residuals to the assigned centroid are split in
D/M' sub-vectors and a second k-means per subspace gives E = 256 codebook
entries; a point is encoded by the id of the nearest entry in every subspace.
(The paper writes M for the subspace *dimension*; this code base writes M for
the *number* of subspaces and dsub = D / M for their dimension.)

The paper evaluates on SIFT1M/100M, DEEP1M/100M and TTI1M (Sec. 6.1).  Those
datasets are not available here; the five configurations below are Gaussian
mixtures that take over their shapes (dimension, value range, normalisation,
PQ split), and stand in for them.

k-means details the paper leaves open (initialisation, iteration count, empty
clusters, training subsample) are free choices, because both search paths are
fed the same trained index: D^2-weighted seeding for the IVF centroids (random
distinct points for the PQ codebooks), a fixed number of Lloyd iterations, empty
clusters re-seeded from random points.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional, Tuple

import numpy as np
import torch

KSUB = 256  # codebook entries per subspace (uint8 codes)


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark / test configuration."""
    name: str
    N: int
    D: int
    nlist: int
    M: int
    Q: int
    nprobe: int
    k: int
    family: str            # "gauss" | "sift" | "deep" | "tti"
    n_centres: int
    sigma: float
    keep_frac: float = 0.25   # fraction of codebook entries inside the radius
    query_shift: float = 0.0  # per-centre query/base shift (family "tti")
    seed: int = 0
    kmeans_iters: int = 10

    @property
    def dsub(self) -> int:
        return self.D // self.M


# The five configurations named by the build target, plus scaled-down variants
# of the 100M one for quick iteration and CPU-sized ones for the host tests.
WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    Workload("C1", 100_000, 64, 256, 16, 1_000, 8, 100, "gauss", 256, 0.15),
    Workload("C2", 1_000_000, 128, 1_024, 64, 10_000, 32, 100, "sift", 1_024, 20.0),
    Workload("C3", 1_000_000, 96, 1_024, 48, 10_000, 64, 100, "deep", 2_048, 0.1),
    Workload("C4", 1_000_000, 200, 1_024, 100, 10_000, 64, 100, "tti", 1_024, 0.25,
             query_shift=0.3),
    Workload("C5", 100_000_000, 128, 16_384, 64, 10_000, 64, 100, "sift", 16_384, 20.0,
             kmeans_iters=8),
    Workload("C5_10M", 10_000_000, 128, 4_096, 64, 10_000, 64, 100, "sift", 4_096, 20.0,
             kmeans_iters=8),
    # host-test sized
    Workload("T_gauss", 6_000, 32, 16, 8, 40, 4, 10, "gauss", 16, 0.15),
    Workload("T_sift", 8_000, 32, 24, 16, 32, 6, 20, "sift", 24, 20.0),
    Workload("T_deep", 5_000, 24, 16, 12, 24, 5, 10, "deep", 32, 0.1),
    Workload("T_tti", 5_000, 40, 16, 20, 24, 5, 10, "tti", 16, 0.25, query_shift=0.3),
]}


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------

def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def mixture_centres(w: Workload, device="cpu") -> torch.Tensor:
    """Mixture centres [n_centres][D] fp32 (sub-seed: seed)."""
    g = _gen(w.seed * 1000 + 0, device)
    shape = (w.n_centres, w.D)
    if w.family == "gauss":
        return torch.rand(shape, generator=g, device=device) * 2.0 - 1.0
    if w.family == "sift":
        return torch.rand(shape, generator=g, device=device) * 255.0
    if w.family == "deep":
        c = torch.randn(shape, generator=g, device=device)
        return c / c.norm(dim=1, keepdim=True)
    if w.family == "tti":
        return torch.randn(shape, generator=g, device=device)
    raise ValueError(w.family)


def _draw(w: Workload, centres: torch.Tensor, n: int, g: torch.Generator) -> torch.Tensor:
    device = centres.device
    j = torch.randint(0, centres.shape[0], (n,), generator=g, device=device)
    x = centres[j] + w.sigma * torch.randn((n, w.D), generator=g, device=device)
    if w.family == "sift":
        x = torch.round(torch.clamp(x, 0.0, 255.0))
    elif w.family == "deep":
        x = x / x.norm(dim=1, keepdim=True)
    return x.contiguous()


def base_chunk(w: Workload, centres: torch.Tensor, start: int, count: int) -> torch.Tensor:
    """Base vectors [count][D] for rows start..start+count.  Chunks are drawn
    from per-chunk sub-seeds, so a chunk can be regenerated at will (the 100M
    configuration never holds all base vectors at once).  `start` must be a
    multiple of BASE_CHUNK."""
    assert start % BASE_CHUNK == 0 and count <= BASE_CHUNK
    g = _gen(w.seed * 1000 + 1 + 7919 * (start // BASE_CHUNK + 1), centres.device)
    return _draw(w, centres, count, g)


BASE_CHUNK = 1 << 20


def base_vectors(w: Workload, centres: torch.Tensor) -> torch.Tensor:
    out = [base_chunk(w, centres, s, min(BASE_CHUNK, w.N - s)) for s in range(0, w.N, BASE_CHUNK)]
    return torch.cat(out, 0) if len(out) > 1 else out[0]


def queries(w: Workload, centres: torch.Tensor, n: Optional[int] = None, sub: int = 2) -> torch.Tensor:
    """Held-out queries (sub-seed 2) or calibration queries (sub-seed 3)."""
    device = centres.device
    n = w.Q if n is None else n
    g = _gen(w.seed * 1000 + sub, device)
    c = centres
    if w.query_shift > 0.0:
        gs = _gen(w.seed * 1000 + 5, device)
        c = centres + w.query_shift * torch.randn(centres.shape, generator=gs, device=device)
    return _draw(w, c, n, g)


# ----------------------------------------------------------------------------
# offline trainer
# ----------------------------------------------------------------------------

def _nearest(x: torch.Tensor, c: torch.Tensor, chunk: int = 1 << 16) -> torch.Tensor:
    """argmin_j ||x_i - c_j||^2 by the expanded form, chunked over rows."""
    cc = (c * c).sum(1)
    out = torch.empty(x.shape[0], dtype=torch.int64, device=x.device)
    for s in range(0, x.shape[0], chunk):
        xs = x[s:s + chunk]
        d = cc[None, :] - 2.0 * (xs @ c.T)
        out[s:s + chunk] = d.argmin(1)
    return out


def _seed_centroids(x: torch.Tensor, k: int, g: torch.Generator) -> torch.Tensor:
    """D^2-weighted seeding (k-means++): each new seed is drawn with probability
    proportional to the squared distance to the nearest seed chosen so far.  On
    well-separated mixtures this puts about one seed in every component, which
    plain random seeding does not, and keeps the inverted lists balanced."""
    n, d = x.shape
    c = torch.empty((k, d), dtype=x.dtype, device=x.device)
    first = int(torch.randint(0, n, (1,), generator=g, device=x.device).item())
    c[0] = x[first]
    d2 = ((x - c[0]) ** 2).sum(1)
    # draw all uniforms up front; pick by inverse CDF so that n may exceed multinomial's limit
    u = torch.rand(k, generator=g, device=x.device, dtype=torch.float64)
    for i in range(1, k):
        cdf = torch.cumsum(d2.to(torch.float64), 0)
        j = int(torch.searchsorted(cdf, u[i] * cdf[-1]).clamp(max=n - 1).item())
        c[i] = x[j]
        d2 = torch.minimum(d2, ((x - c[i]) ** 2).sum(1))
    return c


def kmeans(x: torch.Tensor, k: int, iters: int, g: torch.Generator) -> torch.Tensor:
    """D^2-seeded Lloyd k-means; returns centroids [k][d]."""
    n, d = x.shape
    if n < k:
        raise ValueError(f"k-means needs at least k={k} points, got {n}")
    c = _seed_centroids(x, k, g)
    for it in range(iters):
        a = _nearest(x, c)
        sums = torch.zeros((k, d), dtype=torch.float32, device=x.device).index_add_(0, a, x)
        cnt = torch.bincount(a, minlength=k)
        c = sums / cnt.clamp(min=1).to(torch.float32)[:, None]
        if it == iters - 1:
            break
        # clusters that stay (nearly) empty are re-seeded from a random member of one
        # of the largest clusters, so a list that swallowed several mixture components
        # is split instead of starving its neighbours
        small = torch.nonzero(cnt < 0.6 * n / k).reshape(-1)
        if small.numel():
            donors = torch.argsort(cnt, descending=True)[:small.numel()]
            donors = donors[cnt[donors] > 1.5 * n / k]
            perm = torch.randperm(n, generator=g, device=x.device)
            a_perm = a[perm]
            # first occurrence of every donor label in the permuted order
            first = torch.full((k,), n, dtype=torch.int64, device=x.device)
            first.scatter_reduce_(0, a_perm, torch.arange(n, device=x.device), reduce="amin")
            pick = perm[first[donors].clamp(max=n - 1)]
            c[small[:donors.numel()]] = x[pick]
    return c.contiguous()


def _kmeans_batched(x: torch.Tensor, k: int, iters: int, g: torch.Generator) -> torch.Tensor:
    """Independent k-means per leading index: x [M][n][d] -> [M][k][d]."""
    M, n, d = x.shape
    perm = torch.randperm(n, generator=g, device=x.device)[:k]
    c = x[:, perm, :].clone()
    ar = torch.arange(M, device=x.device)[:, None]
    for _ in range(iters):
        dist = (c * c).sum(2)[:, None, :] - 2.0 * torch.bmm(x, c.transpose(1, 2))  # [M][n][k]
        a = dist.argmin(2)                                                        # [M][n]
        flat = (a + ar * k).reshape(-1)
        sums = torch.zeros((M * k, d), dtype=torch.float32, device=x.device)
        sums.index_add_(0, flat, x.reshape(-1, d))
        cnt = torch.bincount(flat, minlength=M * k).to(torch.float32)
        c_new = (sums / cnt.clamp(min=1.0)[:, None]).reshape(M, k, d)
        empty = (cnt == 0).reshape(M, k)
        if bool(empty.any()):
            r = torch.randint(0, n, (M, k), generator=g, device=x.device)
            repl = torch.gather(x, 1, r[:, :, None].expand(M, k, d))
            c_new = torch.where(empty[:, :, None], repl, c_new)
        c = c_new
    return c.contiguous()


def encode(x: torch.Tensor, centroids: torch.Tensor, codebooks: torch.Tensor,
           chunk: int = 1 << 14) -> Tuple[torch.Tensor, torch.Tensor]:
    """Assign each row to its nearest IVF centroid and PQ-encode its residual.

    Returns (labels int64 [n], codes uint8 [n][M])."""
    M, ksub, dsub = codebooks.shape
    labels = _nearest(x, centroids)
    codes = torch.empty((x.shape[0], M), dtype=torch.uint8, device=x.device)
    cb_t = codebooks.transpose(1, 2).contiguous()          # [M][dsub][ksub]
    cb_n = (codebooks * codebooks).sum(2)                   # [M][ksub]
    for s in range(0, x.shape[0], chunk):
        res = x[s:s + chunk] - centroids[labels[s:s + chunk]]
        r = res.reshape(-1, M, dsub).transpose(0, 1)       # [M][n][dsub]
        d = cb_n[:, None, :] - 2.0 * torch.bmm(r, cb_t)    # [M][n][ksub]
        codes[s:s + chunk] = d.argmin(2).transpose(0, 1).to(torch.uint8)
    return labels, codes


@dataclasses.dataclass
class Index:
    """A trained IVF-PQ index on the host (numpy, C-contiguous)."""
    N: int
    D: int
    nlist: int
    M: int
    centroids: np.ndarray     # [nlist][D] fp32
    codebooks: np.ndarray     # [M][256][dsub] fp32
    list_offsets: np.ndarray  # [nlist+1] int64
    codes: np.ndarray         # [N][M] uint8, rows sorted by list
    ids: np.ndarray           # [N] int64 original row ids in the same order

    @property
    def dsub(self) -> int:
        return self.D // self.M


def assemble(labels: torch.Tensor, codes: torch.Tensor, centroids: torch.Tensor,
             codebooks: torch.Tensor) -> Index:
    """Sort codes by list (stable, so ids ascend inside a list) and build CSR offsets."""
    nlist, D = centroids.shape
    M = codebooks.shape[0]
    order = torch.argsort(labels, stable=True)
    counts = torch.bincount(labels, minlength=nlist)
    offs = torch.zeros(nlist + 1, dtype=torch.int64, device=labels.device)
    offs[1:] = torch.cumsum(counts, 0)
    return Index(
        N=int(labels.shape[0]), D=int(D), nlist=int(nlist), M=int(M),
        centroids=np.ascontiguousarray(centroids.cpu().numpy(), dtype=np.float32),
        codebooks=np.ascontiguousarray(codebooks.cpu().numpy(), dtype=np.float32),
        list_offsets=np.ascontiguousarray(offs.cpu().numpy(), dtype=np.int64),
        codes=np.ascontiguousarray(codes[order].cpu().numpy(), dtype=np.uint8),
        ids=np.ascontiguousarray(order.cpu().numpy(), dtype=np.int64),
    )


def train_index(w: Workload, device="cpu", progress=None) -> Tuple[Index, torch.Tensor]:
    """Generate the base set chunk by chunk, train, encode, assemble.

    Returns (index, centres) where centres are the mixture centres (needed to
    regenerate base chunks and to draw queries).  Base vectors are not kept."""
    say = progress or (lambda *_: None)
    centres = mixture_centres(w, device)
    g = _gen(w.seed * 1000 + 4, device)
    # training sample: rows spread over the first chunks
    n_train = min(w.N, max(64 * w.nlist, 65_536))
    n_train = min(n_train, 4 * BASE_CHUNK)
    parts, got, s = [], 0, 0
    while got < n_train:
        c = min(BASE_CHUNK, w.N - s, n_train - got)
        parts.append(base_chunk(w, centres, s, c))
        got += c
        s += BASE_CHUNK
    xt = torch.cat(parts, 0) if len(parts) > 1 else parts[0]
    say(f"[{w.name}] k-means: {w.nlist} lists on {xt.shape[0]} points")
    centroids = kmeans(xt, w.nlist, w.kmeans_iters, g)
    lab = _nearest(xt, centroids)
    n_pq = min(xt.shape[0], 65_536)
    res = (xt[:n_pq] - centroids[lab[:n_pq]]).reshape(n_pq, w.M, w.dsub).transpose(0, 1).contiguous()
    say(f"[{w.name}] PQ k-means: {w.M} x {KSUB} entries on {n_pq} residuals")
    codebooks = _kmeans_batched(res, KSUB, w.kmeans_iters, g)
    del xt, res, lab, parts
    labels = torch.empty(w.N, dtype=torch.int64, device=device)
    codes = torch.empty((w.N, w.M), dtype=torch.uint8, device=device)
    for s in range(0, w.N, BASE_CHUNK):
        c = min(BASE_CHUNK, w.N - s)
        x = base_chunk(w, centres, s, c)
        labels[s:s + c], codes[s:s + c] = encode(x, centroids, codebooks)
        if (s // BASE_CHUNK) % 16 == 0:
            say(f"[{w.name}] encoded {s + c}/{w.N}")
    idx = assemble(labels, codes, centroids, codebooks)
    return idx, centres


def calibrate_radii(w: Workload, index: Index, centres: torch.Tensor, keep_frac: Optional[float] = None,
                    n_cal: int = 1000, metric: int = 0) -> np.ndarray:
    """Per-subspace radius such that about `keep_frac` of the codebook entries
    lie within it of a query residual's projection.

    metric = 1 (inner product, paper Sec. 4.2): the ray starts at the query's own
    projection q_m and entry e has the enlarged sphere of radius^2 r_m^2 + |e|^2, so the
    pooled quantity is |q_m - e|^2 - |e|^2 (clipped at 0) instead of a squared distance.

    Calibration queries (sub-seed 3) are assigned their nprobe nearest lists;
    for each subspace the squared distances from every residual projection to
    every entry are pooled and the keep_frac-quantile is taken as r_m^2.
    keep_frac >= 1 returns +inf (nothing filtered)."""
    kf = w.keep_frac if keep_frac is None else keep_frac
    if kf >= 1.0:
        return np.full(index.M, np.inf, dtype=np.float32)
    device = centres.device
    n_cal = min(n_cal, max(8, 200_000 // (w.nprobe * 1)))
    qc = queries(w, centres, n_cal, sub=3)
    cent = torch.from_numpy(index.centroids).to(device)
    cb = torch.from_numpy(index.codebooks).to(device)
    if metric == 1:
        qm = qc.reshape(-1, index.M, index.dsub)
        radii = np.empty(index.M, dtype=np.float32)
        for m in range(index.M):
            diff = qm[:, m, None, :] - cb[m][None, :, :]
            g = ((diff * diff).sum(2) - (cb[m] * cb[m]).sum(1)[None, :]).reshape(-1)
            kth = max(1, int(math.ceil(kf * g.numel())))
            radii[m] = np.sqrt(np.float32(max(torch.kthvalue(g.cpu(), kth).values.item(), 0.0)))
        return radii
    d = (cent * cent).sum(1)[None, :] - 2.0 * (qc @ cent.T)
    probes = d.topk(min(w.nprobe, index.nlist), dim=1, largest=False).indices  # [n][nprobe]
    res = (qc[:, None, :] - cent[probes]).reshape(-1, index.M, index.dsub)     # [n*nprobe][M][dsub]
    radii = np.empty(index.M, dtype=np.float32)
    for m in range(index.M):
        diff = res[:, m, None, :] - cb[m][None, :, :]
        d2 = (diff * diff).sum(2).reshape(-1)
        kth = max(1, int(math.ceil(kf * d2.numel())))
        r2 = torch.kthvalue(d2.cpu(), kth).values.item()
        radii[m] = np.sqrt(np.float32(r2))
    return radii


def fit_radius_model(w: Workload, index: Index, centres: torch.Tensor, keep_frac: Optional[float] = None,
                     n_cal: int = 512, G: int = 100, n_base: int = 200_000, with_projections: bool = False,
                     target: str = "keep", top: int = 100) -> dict:
    """Offline half of the paper's dynamic threshold (Sec. 4.1, "Determining Proper
    Threshold"): per subspace a G x G density map of the residual projections of
    search points (count / cell area; the paper's G is 100) and a polynomial from the
    density at a projection to the radius it needs.  Here the map stores log(1 +
    density), the polynomial is a quadratic in it fitted by least squares on `n_cal`
    calibration queries.  The radius a projection "needs" (the regression target) is
    either target="top": the paper's -- the radius that contains the entries of the
    query's true `top` nearest neighbours (exact search over the regenerated base
    vectors; each neighbour's entry is measured from the query's residual w.r.t. that
    neighbour's own list) -- or target="keep": the radius that keeps `keep_frac` of
    the 256 entries around the residual w.r.t. the nearest list (no exact search
    needed; for the sizes where one is too slow).  Two-dimensional subspaces only,
    like the paper's.  Returns host arrays in the layout of the library's radius
    model: lo [M][2], cells_per_unit [M][2], map [M][G][G], coef [M][3] (lowest power
    first), fallback [M].  Like the k-means training this is an *input* of the search
    path; the online look-up runs in the library."""
    if index.dsub != 2:
        raise ValueError("the density map needs two-dimensional subspaces")
    kf = w.keep_frac if keep_frac is None else keep_frac
    device = centres.device
    cent = torch.from_numpy(index.centroids).to(device)
    cb = torch.from_numpy(index.codebooks).to(device)
    M = index.M

    def projections(x):
        lab = _nearest(x, cent)
        return (x - cent[lab]).reshape(-1, M, 2)

    base = base_chunk(w, centres, 0, min(BASE_CHUNK, w.N, n_base))
    pb = projections(base)                                     # [n][M][2]
    lo = pb.amin(0)                                            # [M][2]
    span = (pb.amax(0) - lo).clamp(min=1e-12)
    cpu = (float(G) / span).to(torch.float32)                  # cells per unit length

    def cells(p):   # the library's rule: floor((x - lo) * cells_per_unit), clamped to the map
        ij = ((p - lo) * cpu).floor().clamp(0, G - 1).to(torch.int64)
        return ij[..., 0] * G + ij[..., 1]                     # [n][M]

    m_idx = torch.arange(M, device=device)[None, :]
    count = torch.zeros(M * G * G, device=device, dtype=torch.float64)
    count.index_add_(0, (m_idx * G * G + cells(pb)).reshape(-1),
                     torch.ones(pb.shape[0] * M, device=device, dtype=torch.float64))
    area = 1.0 / (cpu[:, 0].double() * cpu[:, 1].double())
    fmap = torch.log1p(count.reshape(M, G * G) / area[:, None]).to(torch.float32)

    qc = queries(w, centres, n_cal, sub=3)
    pc = projections(qc)
    x = torch.gather(fmap, 1, cells(pc).T).T                   # [n][M]
    X = torch.stack([torch.ones_like(x), x, x * x], -1).transpose(0, 1)   # [M][n][3]
    if target == "top":
        truth = exact_knn(w, centres, qc, min(top, w.N))       # ids [n][top]
        row_of_id = np.empty(index.N, dtype=np.int64)
        row_of_id[index.ids] = np.arange(index.N)
        rows = row_of_id[truth]
        lists = np.searchsorted(index.list_offsets, rows, side="right") - 1
        codes = torch.from_numpy(index.codes[rows].astype(np.int64)).to(device)        # [n][top][M]
        ent = cb[torch.arange(M, device=device)[None, None, :], codes]                  # [n][top][M][2]
        res = (qc[:, None, :] - cent[torch.from_numpy(lists).to(device)]).reshape(qc.shape[0], -1, M, 2)
        need = ((res - ent) ** 2).sum(-1).amax(1).sqrt()       # [n][M]: contains every neighbour's entry
    elif target == "keep":
        d2 = ((pc[:, :, None, :] - cb[None]) ** 2).sum(-1)     # [n][M][256]
        kth = max(1, min(KSUB, int(math.ceil(kf * KSUB))))
        need = d2.kthvalue(kth, dim=2).values.sqrt()           # [n][M]
    else:
        raise ValueError("target must be 'top' or 'keep'")
    coef = torch.linalg.lstsq(X.cpu().double(), need.T.cpu().double()[:, :, None]).solution[:, :, 0]
    out = {"lo": lo.cpu().numpy().astype(np.float32), "cells_per_unit": cpu.cpu().numpy(),
           "map": np.ascontiguousarray(fmap.reshape(M, G, G).cpu().numpy()),
           "coef": np.ascontiguousarray(coef.to(torch.float32).numpy()),
           "fallback": need.mean(0).cpu().numpy().astype(np.float32)}
    if with_projections:
        out["projections"] = pb.cpu().numpy()
    return out


def exact_knn(w: Workload, centres: torch.Tensor, q: torch.Tensor, k: int, metric: int = 0) -> np.ndarray:
    """Ground-truth neighbours for recall reporting: ids [Q][k] of the k nearest
    base vectors by squared L2 (paper Sec. 2.1, metric definition), or of the k largest
    inner products (metric = 1), streamed over regenerated base chunks with a running
    top-k (fp32 on `centres.device`)."""
    device = centres.device
    best_d = torch.full((q.shape[0], k), float("inf"), device=device)
    best_i = torch.full((q.shape[0], k), -1, dtype=torch.int64, device=device)
    qq = (q * q).sum(1)[:, None]
    for s in range(0, w.N, BASE_CHUNK):
        c = min(BASE_CHUNK, w.N - s)
        x = base_chunk(w, centres, s, c)
        d = -(q @ x.T) if metric == 1 else qq - 2.0 * (q @ x.T) + (x * x).sum(1)[None, :]
        dk, ik = d.topk(min(k, c), dim=1, largest=False)
        cat_d = torch.cat([best_d, dk], 1)
        cat_i = torch.cat([best_i, ik + s], 1)
        sel = cat_d.topk(k, dim=1, largest=False).indices
        best_d = torch.gather(cat_d, 1, sel)
        best_i = torch.gather(cat_i, 1, sel)
    order = best_d.argsort(1)
    return torch.gather(best_i, 1, order).cpu().numpy()


def recall_at_k(found: np.ndarray, truth: np.ndarray) -> Tuple[float, float]:
    """(k-recall@k, R1@k): mean overlap with the true top-k, and the fraction of
    queries whose true nearest neighbour is among the k returned (paper Sec. 6.1,
    "Metric")."""
    Q, k = truth.shape
    inter = 0
    r1 = 0
    for i in range(Q):
        f = set(int(v) for v in found[i] if v >= 0)
        inter += len(f.intersection(int(v) for v in truth[i]))
        r1 += int(int(truth[i, 0]) in f)
    return inter / float(Q * k), r1 / float(Q)
