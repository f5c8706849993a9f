"""Seeded generators for the synthetic graphs, seed sets and insertion batches.

Everything here is input plumbing.  All randomness comes from
``numpy.random.default_rng(seed)`` with seeds derived from ``BASE_SEED``.  Vertex ids
are randomly permuted with respect to classes/blocks (ids carry no locality), which
is the unfavourable case for caches and the honest one for arrival-order ids.

Conventions
-----------
* A graph is a *symmetric* CSR: ``row_ptr`` int64 [n+1], ``col`` int32 [nnz],
  ``w`` float32 [nnz]; every undirected edge appears in both rows with the same
  float32 weight; no self loops, no duplicate entries.
* A batch holds ``num_new_vertices`` (they get ids n .. n+k-1 in order), undirected
  edges listed once each (``eu``, ``ev``, ``ew``) and newly labelled vertices
  (``seed_vertex``, ``seed_class``).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20260406


@dataclass
class Problem:
    n: int
    C: int
    row_ptr: np.ndarray
    col: np.ndarray
    w: np.ndarray
    seed_vertex: np.ndarray
    seed_class: np.ndarray
    true_class: np.ndarray
    state: dict = field(default_factory=dict)  # generator state for later batches

    @property
    def nnz(self) -> int:
        return int(self.col.shape[0])


@dataclass
class Batch:
    num_new_vertices: int
    eu: np.ndarray
    ev: np.ndarray
    ew: np.ndarray
    seed_vertex: np.ndarray
    seed_class: np.ndarray

    @property
    def num_edges(self) -> int:
        return int(self.eu.shape[0])


# --------------------------------------------------------------------------------------
# heavy deterministic array steps: numpy, or torch on the GPU for the 10M-vertex build
# (same results either way: sorting/searching integers and float64 keys is exact)
# --------------------------------------------------------------------------------------
_BIG = 20_000_000


def _gpu():
    try:
        import torch

        return torch if torch.cuda.is_available() else None
    except ImportError:
        return None


def _argsort(keys: np.ndarray) -> np.ndarray:
    t = _gpu() if keys.shape[0] >= _BIG else None
    if t is None:
        return np.argsort(keys, kind="stable")
    k = t.from_numpy(keys).cuda()
    order = t.sort(k, stable=True).indices
    del k
    return order.cpu().numpy()


def _unique(keys: np.ndarray) -> np.ndarray:
    t = _gpu() if keys.shape[0] >= _BIG else None
    if t is None:
        return np.unique(keys)
    return t.unique(t.from_numpy(keys).cuda(), sorted=True).cpu().numpy()


def _searchsorted_right(cum: np.ndarray, vals: np.ndarray) -> np.ndarray:
    t = _gpu() if vals.shape[0] >= _BIG else None
    if t is None:
        if vals.shape[0] < 100_000:
            return np.searchsorted(cum, vals, side="right")
        # same answers, looked up in ascending order of the queries: neighbouring binary searches then share their
        # path through ``cum`` instead of missing the cache at every level
        order = np.argsort(vals)
        out = np.empty(vals.shape[0], dtype=np.int64)
        out[order] = np.searchsorted(cum, vals[order], side="right")
        return out
    return t.searchsorted(t.from_numpy(cum).cuda(), t.from_numpy(vals).cuda(), right=True).cpu().numpy()


# --------------------------------------------------------------------------------------
# plumbing helpers
# --------------------------------------------------------------------------------------
def edges_to_csr(n: int, eu, ev, ew):
    """Undirected edge list (once each) -> symmetric CSR sorted by (row, col)."""
    eu = np.asarray(eu, dtype=np.int64)
    ev = np.asarray(ev, dtype=np.int64)
    ew = np.asarray(ew, dtype=np.float32)
    src = np.concatenate([eu, ev])
    dst = np.concatenate([ev, eu])
    ww = np.concatenate([ew, ew])
    order = _argsort(src * np.int64(n) + dst)
    src = src[order]
    col = dst[order].astype(np.int32)
    ww = ww[order]
    counts = np.bincount(src, minlength=n)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return row_ptr, col, np.ascontiguousarray(ww)


def _dedupe_undirected(n_total: int, a, b):
    """Drop self loops and duplicate unordered pairs; return (lo, hi) int64 with lo<hi."""
    a = np.asarray(a, dtype=np.int64)
    b = np.asarray(b, dtype=np.int64)
    keep = a != b
    a, b = a[keep], b[keep]
    lo = np.minimum(a, b)
    hi = np.maximum(a, b)
    key = _unique(lo * np.int64(n_total) + hi)
    return key // n_total, key % n_total


def _pick_seeds(rng, candidates: np.ndarray, count: int, true_class: np.ndarray):
    count = int(min(count, candidates.shape[0]))
    sv = np.sort(rng.choice(candidates, size=count, replace=False)).astype(np.int32)
    return sv, true_class[sv].astype(np.int32)


# --------------------------------------------------------------------------------------
# kNN graphs over a Gaussian mixture (stand-in for the paper's embedding kNN graphs)
# --------------------------------------------------------------------------------------
def _knn(Xq: np.ndarray, Xall: np.ndarray, k: int, self_offset: int | None, block: int = 4096):
    """Exact k nearest neighbours (Euclidean) of each row of Xq among the rows of Xall.

    ``self_offset``: row i of Xq is row ``self_offset + i`` of Xall and is excluded.
    Uses torch for the blocked distance/top-k (GPU if there is one); this is input
    construction only.  Returns (idx int64 [q,k], dist float64 [q,k]).
    """
    import torch

    dev = torch.device("cuda" if torch.cuda.is_available() else "cpu")
    A = torch.from_numpy(np.ascontiguousarray(Xall, dtype=np.float32)).to(dev)
    Q = torch.from_numpy(np.ascontiguousarray(Xq, dtype=np.float32)).to(dev)
    a2 = (A * A).sum(1)
    idx_out, d_out = [], []
    for s in range(0, Q.shape[0], block):
        q = Q[s:s + block]
        d2 = (q * q).sum(1, keepdim=True) + a2[None, :] - 2.0 * (q @ A.T)
        if self_offset is not None:
            r = torch.arange(q.shape[0], device=dev)
            d2[r, self_offset + s + r] = float("inf")
        vals, idx = torch.topk(d2, k, dim=1, largest=False)
        idx_out.append(idx.cpu().numpy())
        d_out.append(vals.clamp_min(0).sqrt().double().cpu().numpy())
    return np.concatenate(idx_out), np.concatenate(d_out)


def knn_mixture(n: int, C: int, d: int, k: int, seed_frac: float, seed: int) -> Problem:
    """n points from a C-class Gaussian mixture in R^d (means ~ N(0, 4I), unit covariance),
    symmetrised (union) exact k-NN graph, weights exp(-||x-y||^2 / sigma^2) with sigma the
    median k-NN distance; ``seed_frac`` of the vertices chosen uniformly as seeds."""
    rng = np.random.default_rng(seed)
    means = rng.normal(0.0, 2.0, size=(C, d))
    cls = rng.integers(0, C, size=n)
    X = (means[cls] + rng.normal(size=(n, d))).astype(np.float32)
    idx, dist = _knn(X, X, k, self_offset=0)
    sigma = float(np.median(dist))
    src = np.repeat(np.arange(n, dtype=np.int64), k)
    lo, hi = _dedupe_undirected(n, src, idx.reshape(-1))
    d2 = ((X[lo].astype(np.float64) - X[hi].astype(np.float64)) ** 2).sum(1)
    ew = np.exp(-d2 / sigma ** 2).astype(np.float32)
    ew = np.maximum(ew, np.float32(1e-30))  # weights must stay strictly positive in fp32
    row_ptr, col, w = edges_to_csr(n, lo, hi, ew)
    sv, sc = _pick_seeds(rng, np.arange(n), max(1, round(seed_frac * n)), cls)
    st = dict(kind="knn", rng=rng, means=means, X=X, sigma=sigma, k=k, d=d)
    return Problem(n, C, row_ptr, col, w, sv, sc, cls.astype(np.int32), st)


def knn_mixture_batch(p: Problem, num_new: int, num_seeds: int) -> Batch:
    """``num_new`` fresh points from the same mixture; each links to its k nearest among
    existing + batch points (existing points do not re-pick); ``num_seeds`` of the new
    points are labelled.  Advances ``p.state`` and ``p.n``/``p.true_class``."""
    st = p.state
    rng = st["rng"]
    cls = rng.integers(0, p.C, size=num_new)
    Xb = (st["means"][cls] + rng.normal(size=(num_new, st["d"]))).astype(np.float32)
    Xall = np.concatenate([st["X"], Xb])
    n0 = p.n
    idx, _ = _knn(Xb, Xall, st["k"], self_offset=n0)
    src = np.repeat(np.arange(n0, n0 + num_new, dtype=np.int64), st["k"])
    lo, hi = _dedupe_undirected(n0 + num_new, src, idx.reshape(-1))
    d2 = ((Xall[lo].astype(np.float64) - Xall[hi].astype(np.float64)) ** 2).sum(1)
    ew = np.maximum(np.exp(-d2 / st["sigma"] ** 2).astype(np.float32), np.float32(1e-30))
    new_ids = np.arange(n0, n0 + num_new)
    true_all = np.concatenate([p.true_class, cls.astype(np.int32)])
    sv, sc = _pick_seeds(rng, new_ids, num_seeds, true_all)
    st["X"] = Xall
    p.n = n0 + num_new
    p.true_class = true_all
    return Batch(num_new, lo.astype(np.int32), hi.astype(np.int32), ew, sv, sc)


# --------------------------------------------------------------------------------------
# stochastic block model (planted blocks, uniform weights)
# --------------------------------------------------------------------------------------
def sbm(n: int, C: int, mean_degree: float, in_out_ratio: float, seed_frac: float, seed: int) -> Problem:
    """C equal planted blocks, intra-block edge probability ``in_out_ratio`` x the
    inter-block one, expected mean degree ``mean_degree``, weights ~ U(0.1, 1),
    ``seed_frac`` of vertices labelled with their block."""
    rng = np.random.default_rng(seed)
    block = (rng.permutation(n) % C).astype(np.int32)  # ids carry no block locality
    members = [np.flatnonzero(block == b) for b in range(C)]
    B = n / C
    # mean degree = p_out * (n - B) + p_in * B
    p_out = mean_degree / ((n - B) + in_out_ratio * B)
    p_in = in_out_ratio * p_out
    us, vs = [], []
    for a in range(C):
        na = members[a].shape[0]
        m = rng.binomial(na * (na - 1) // 2, p_in)
        us.append(members[a][rng.integers(0, na, size=m)])
        vs.append(members[a][rng.integers(0, na, size=m)])
        for b in range(a + 1, C):
            nb = members[b].shape[0]
            m = rng.binomial(na * nb, p_out)
            us.append(members[a][rng.integers(0, na, size=m)])
            vs.append(members[b][rng.integers(0, nb, size=m)])
    lo, hi = _dedupe_undirected(n, np.concatenate(us), np.concatenate(vs))
    ew = rng.uniform(0.1, 1.0, size=lo.shape[0]).astype(np.float32)
    row_ptr, col, w = edges_to_csr(n, lo, hi, ew)
    sv, sc = _pick_seeds(rng, np.arange(n), max(1, round(seed_frac * n)), block)
    is_seed = np.zeros(n, dtype=bool)
    is_seed[sv] = True
    st = dict(kind="sbm", rng=rng, in_out_ratio=in_out_ratio, mean_degree=mean_degree, is_seed=is_seed)
    return Problem(n, C, row_ptr, col, w, sv, sc, block, st)


def _members_table(true_class: np.ndarray, C: int):
    order = np.argsort(true_class, kind="stable")
    counts = np.bincount(true_class, minlength=C)
    start = np.zeros(C + 1, dtype=np.int64)
    np.cumsum(counts, out=start[1:])
    return order, start


def sbm_vertex_batch(p: Problem, num_new: int, degree: int, seed_frac: float) -> Batch:
    """``num_new`` new vertices with uniform blocks; each draws ``degree`` neighbours among
    existing + batch vertices, each neighbour from its own block with the probability that
    makes intra-block edges ``in_out_ratio`` x as likely as inter-block ones, otherwise
    from a uniformly chosen other block.  Advances ``p``."""
    st = p.state
    rng = st["rng"]
    C, n0 = p.C, p.n
    r = st["in_out_ratio"]
    p_same = r / (r + (C - 1))
    blk_new = rng.integers(0, C, size=num_new).astype(np.int32)
    true_all = np.concatenate([p.true_class, blk_new])
    order, start = _members_table(true_all, C)
    src = np.repeat(np.arange(n0, n0 + num_new, dtype=np.int64), degree)
    sblk = np.repeat(blk_new.astype(np.int64), degree)
    same = rng.random(src.shape[0]) < p_same
    other = (sblk + rng.integers(1, C, size=src.shape[0])) % C if C > 1 else sblk
    tblk = np.where(same, sblk, other)
    cnt = start[tblk + 1] - start[tblk]
    dst = order[start[tblk] + (rng.random(src.shape[0]) * cnt).astype(np.int64)]
    lo, hi = _dedupe_undirected(n0 + num_new, src, dst)
    ew = rng.uniform(0.1, 1.0, size=lo.shape[0]).astype(np.float32)
    sv, sc = _pick_seeds(rng, np.arange(n0, n0 + num_new), round(seed_frac * num_new), true_all)
    is_seed = np.concatenate([st["is_seed"], np.zeros(num_new, dtype=bool)])
    is_seed[sv] = True
    st["is_seed"] = is_seed
    p.n = n0 + num_new
    p.true_class = true_all
    return Batch(num_new, lo.astype(np.int32), hi.astype(np.int32), ew, sv, sc)


def sbm_edge_batch(p: Problem, num_edges: int, intra_frac: float, num_revealed: int) -> Batch:
    """Edge-only batch: ``num_edges`` new undirected edges between existing vertices
    (``intra_frac`` of them inside a block), plus ``num_revealed`` previously unlabelled
    vertices that become seeds with their block label.  Edges may duplicate existing ones
    (parallel edges are legal: weights add)."""
    st = p.state
    rng = st["rng"]
    C, n = p.C, p.n
    order, start = _members_table(p.true_class, C)
    a = rng.integers(0, n, size=num_edges).astype(np.int64)
    ablk = p.true_class[a].astype(np.int64)
    intra = rng.random(num_edges) < intra_frac
    other = (ablk + rng.integers(1, C, size=num_edges)) % C if C > 1 else ablk
    tblk = np.where(intra, ablk, other)
    cnt = start[tblk + 1] - start[tblk]
    b = order[start[tblk] + (rng.random(num_edges) * cnt).astype(np.int64)]
    lo, hi = _dedupe_undirected(n, a, b)
    ew = rng.uniform(0.1, 1.0, size=lo.shape[0]).astype(np.float32)
    cand = np.flatnonzero(~st["is_seed"])
    sv, sc = _pick_seeds(rng, cand, num_revealed, p.true_class)
    st["is_seed"][sv] = True
    return Batch(0, lo.astype(np.int32), hi.astype(np.int32), ew, sv, sc)


# --------------------------------------------------------------------------------------
# Chung-Lu power-law graph with class-correlated edges
# --------------------------------------------------------------------------------------
def _power_law_degrees(rng, n: int, exponent: float, d_max: int, mean_target: float):
    """Expected degrees from P(d) ~ d^-exponent on [d_min, d_max]; d_min (real-valued) is
    solved by bisection so that the mean is ``mean_target``.  Inverse-CDF sampling."""
    a = exponent - 1.0

    def mean_for(dmin):
        # continuous power law truncated to [dmin, d_max]
        num = (d_max ** (2 - exponent) - dmin ** (2 - exponent)) / (2 - exponent)
        den = (d_max ** (1 - exponent) - dmin ** (1 - exponent)) / (1 - exponent)
        return num / den

    lo, hi = 0.5, float(mean_target)
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if mean_for(mid) < mean_target:
            lo = mid
        else:
            hi = mid
    dmin = 0.5 * (lo + hi)
    u = rng.random(n)
    theta = (dmin ** (-a) - u * (dmin ** (-a) - d_max ** (-a))) ** (-1.0 / a)
    return theta, dmin


def _chung_lu_partners(rng, src_cls: np.ndarray, theta_cum_all, order_cls, start_cls, theta_cum_cls, intra_frac):
    """One partner per entry of ``src_cls`` (the class of the drawing vertex), chosen
    proportional to theta: from that class with probability ``intra_frac``, else from all."""
    m = src_cls.shape[0]
    n = theta_cum_all.shape[0]
    intra = rng.random(m) < intra_frac
    r = rng.random(m)
    dst = _searchsorted_right(theta_cum_all, r * theta_cum_all[-1]).astype(np.int64)
    np.minimum(dst, n - 1, out=dst)
    c = src_cls[intra].astype(np.int64)
    base = np.where(start_cls[c] > 0, theta_cum_cls[np.maximum(start_cls[c] - 1, 0)], 0.0)
    top = theta_cum_cls[start_cls[c + 1] - 1]
    pos = _searchsorted_right(theta_cum_cls, base + r[intra] * (top - base))
    pos = np.clip(pos, start_cls[c], start_cls[c + 1] - 1)
    dst[intra] = order_cls[pos]
    return dst


def chung_lu(n: int, C: int, mean_degree: float, exponent: float, d_max: int, intra_frac: float,
             seed_frac: float, seed: int) -> Problem:
    """Chung-Lu graph: expected degrees from a truncated power law, ~n*mean_degree/2
    undirected edges; each edge's first endpoint ~ theta, its partner from the same class
    with probability ``intra_frac`` (~ theta within the class) else from everyone (~ theta).
    Weights ~ U(0.1, 1).  Duplicates merged, self loops dropped."""
    rng = np.random.default_rng(seed)
    cls = (rng.permutation(n) % C).astype(np.int32)
    theta, dmin = _power_law_degrees(rng, n, exponent, d_max, mean_degree)
    order_cls, start_cls = _members_table(cls, C)
    theta_cum_all = np.cumsum(theta)
    theta_cum_cls = np.cumsum(theta[order_cls])
    m = int(round(n * mean_degree / 2))
    r = rng.random(m)
    src = np.minimum(_searchsorted_right(theta_cum_all, r * theta_cum_all[-1]), n - 1).astype(np.int64)
    dst = _chung_lu_partners(rng, cls[src], theta_cum_all, order_cls, start_cls, theta_cum_cls, intra_frac)
    lo, hi = _dedupe_undirected(n, src, dst)
    ew = rng.uniform(0.1, 1.0, size=lo.shape[0]).astype(np.float32)
    row_ptr, col, w = edges_to_csr(n, lo, hi, ew)
    sv, sc = _pick_seeds(rng, np.arange(n), max(1, round(seed_frac * n)), cls)
    st = dict(kind="chung_lu", rng=rng, theta=theta, dmin=dmin, exponent=exponent, d_max=d_max,
              intra_frac=intra_frac, mean_degree=mean_degree)
    return Problem(n, C, row_ptr, col, w, sv, sc, cls, st)


def chung_lu_vertex_batch(p: Problem, num_new: int, seed_frac: float) -> Batch:
    """``num_new`` new vertices with power-law degrees from the same law; each draws
    round(theta) partners (at least 1) among the *existing* vertices by the class rule."""
    st = p.state
    rng = st["rng"]
    C, n0 = p.C, p.n
    cls_new = rng.integers(0, C, size=num_new).astype(np.int32)
    a = st["exponent"] - 1.0
    u = rng.random(num_new)
    th_new = (st["dmin"] ** (-a) - u * (st["dmin"] ** (-a) - st["d_max"] ** (-a))) ** (-1.0 / a)
    deg = np.maximum(1, np.rint(th_new)).astype(np.int64)
    theta = st["theta"]
    order_cls, start_cls = _members_table(p.true_class, C)
    theta_cum_all = np.cumsum(theta)
    theta_cum_cls = np.cumsum(theta[order_cls])
    src_new = np.repeat(np.arange(num_new, dtype=np.int64), deg)
    true_all = np.concatenate([p.true_class, cls_new])
    dst = _chung_lu_partners(rng, cls_new[src_new], theta_cum_all, order_cls, start_cls, theta_cum_cls,
                             st["intra_frac"])
    lo, hi = _dedupe_undirected(n0 + num_new, src_new + n0, dst)
    ew = rng.uniform(0.1, 1.0, size=lo.shape[0]).astype(np.float32)
    sv, sc = _pick_seeds(rng, np.arange(n0, n0 + num_new), round(seed_frac * num_new), true_all)
    st["theta"] = np.concatenate([theta, th_new])
    p.n = n0 + num_new
    p.true_class = true_all
    return Batch(num_new, lo.astype(np.int32), hi.astype(np.int32), ew, sv, sc)


# --------------------------------------------------------------------------------------
# small random graphs for unit tests
# --------------------------------------------------------------------------------------
def small_random(n: int, C: int, avg_degree: float, num_seeds: int, seed: int, connected: bool = True) -> Problem:
    """Erdos-Renyi-like weighted graph (weights ~ U(0.1, 1)); with ``connected`` a random
    spanning path is added so that every vertex reaches a seed."""
    rng = np.random.default_rng(seed)
    m = int(round(n * avg_degree / 2))
    a = rng.integers(0, n, size=m)
    b = rng.integers(0, n, size=m)
    if connected and n > 1:
        path = rng.permutation(n)
        a = np.concatenate([a, path[:-1]])
        b = np.concatenate([b, path[1:]])
    lo, hi = _dedupe_undirected(n, a, b)
    ew = rng.uniform(0.1, 1.0, size=lo.shape[0]).astype(np.float32)
    row_ptr, col, w = edges_to_csr(n, lo, hi, ew)
    cls = rng.integers(0, C, size=n).astype(np.int32)
    sv, sc = _pick_seeds(rng, np.arange(n), num_seeds, cls)
    is_seed = np.zeros(n, dtype=bool)
    is_seed[sv] = True
    return Problem(n, C, row_ptr, col, w, sv, sc, cls, dict(kind="small", rng=rng, is_seed=is_seed))


def small_random_batch(p: Problem, num_new: int, degree: int, num_new_seeds: int, num_extra_edges: int = 0,
                       num_revealed: int = 0) -> Batch:
    """New vertices with ``degree`` uniform partners each (existing + batch), plus optional
    extra edges between existing vertices and optionally revealed seeds among old vertices."""
    st = p.state
    rng = st["rng"]
    n0 = p.n
    nt = n0 + num_new
    src = np.repeat(np.arange(n0, nt, dtype=np.int64), degree)
    dst = rng.integers(0, nt, size=src.shape[0])
    if num_extra_edges:
        src = np.concatenate([src, rng.integers(0, n0, size=num_extra_edges)])
        dst = np.concatenate([dst, rng.integers(0, n0, size=num_extra_edges)])
    lo, hi = _dedupe_undirected(nt, src, dst)
    ew = rng.uniform(0.1, 1.0, size=lo.shape[0]).astype(np.float32)
    cls_new = rng.integers(0, p.C, size=num_new).astype(np.int32)
    true_all = np.concatenate([p.true_class, cls_new])
    sv, sc = _pick_seeds(rng, np.arange(n0, nt), num_new_seeds, true_all)
    is_seed = np.concatenate([st["is_seed"], np.zeros(num_new, dtype=bool)])
    if num_revealed:
        cand = np.flatnonzero(~is_seed[:n0])
        rv, rc = _pick_seeds(rng, cand, num_revealed, true_all)
        sv = np.concatenate([sv, rv]).astype(np.int32)
        sc = np.concatenate([sc, rc]).astype(np.int32)
    is_seed[sv] = True
    st["is_seed"] = is_seed
    p.n = nt
    p.true_class = true_all
    return Batch(num_new, lo.astype(np.int32), hi.astype(np.int32), ew, sv, sc)


def clustered_batch(p: Problem, num_new: int, mean_cluster: float, intra_degree: int, cross_degree: int,
                    old_degree: int, num_new_seeds: int) -> Batch:
    """New vertices that arrive in groups of similar items (the situation the paper's
    batch-internal sparsified graph is meant for).  The batch is cut into runs of geometric
    length (mean ``mean_cluster``, so singletons occur); a run shares one class.  Each vertex
    draws ``intra_degree`` partners inside its run with strong weights U(0.6,1), ``cross_degree``
    partners anywhere in the batch with weights U(0.05,0.58) (a few above, most below a threshold
    near the mean weight) and ``old_degree`` partners among the existing vertices, 80% of them
    of the run's class, with weights U(0.1,1).  Works on any Problem.  Advances ``p``."""
    st = p.state
    rng = st["rng"]
    C, n0 = p.C, p.n
    nt = n0 + num_new
    cuts = rng.random(num_new) < 1.0 / max(mean_cluster, 1.0)
    if num_new:
        cuts[0] = True
    run_id = np.cumsum(cuts) - 1
    num_runs = int(run_id[-1]) + 1 if num_new else 0
    run_start = np.flatnonzero(cuts)
    run_len = np.diff(np.concatenate([run_start, [num_new]]))
    run_cls = rng.integers(0, C, size=num_runs).astype(np.int32)
    cls_new = run_cls[run_id] if num_new else np.zeros(0, dtype=np.int32)
    ids = np.arange(n0, nt, dtype=np.int64)
    # inside the run
    a1 = np.repeat(ids, intra_degree)
    r1 = np.repeat(run_id, intra_degree)
    b1 = n0 + run_start[r1] + (rng.random(a1.shape[0]) * run_len[r1]).astype(np.int64)
    w1 = rng.uniform(0.6, 1.0, size=a1.shape[0])
    # anywhere in the batch
    a2 = np.repeat(ids, cross_degree)
    b2 = rng.integers(n0, max(nt, n0 + 1), size=a2.shape[0])
    w2 = rng.uniform(0.05, 0.58, size=a2.shape[0])
    # to existing vertices
    a3 = np.repeat(ids, old_degree)
    c3 = np.repeat(cls_new.astype(np.int64), old_degree)
    order, start = _members_table(p.true_class[:n0], C)
    same = rng.random(a3.shape[0]) < 0.8
    cnt = start[c3 + 1] - start[c3]
    same &= cnt > 0
    pick_same = order[np.minimum(start[c3] + (rng.random(a3.shape[0]) * np.maximum(cnt, 1)).astype(np.int64), n0 - 1)]
    b3 = np.where(same, pick_same, rng.integers(0, n0, size=a3.shape[0]))
    w3 = rng.uniform(0.1, 1.0, size=a3.shape[0])
    a = np.concatenate([a1, a2, a3])
    b = np.concatenate([b1, b2, b3])
    ww = np.concatenate([w1, w2, w3])
    keep = a != b
    a, b, ww = a[keep], b[keep], ww[keep]
    lo, hi = np.minimum(a, b), np.maximum(a, b)
    key = lo * np.int64(nt) + hi
    _, first = np.unique(key, return_index=True)  # first listed weight of a repeated pair wins
    lo, hi, ww = lo[first], hi[first], ww[first]
    true_all = np.concatenate([p.true_class, cls_new])
    sv, sc = _pick_seeds(rng, ids, num_new_seeds, true_all)
    is_seed = np.concatenate([st["is_seed"], np.zeros(num_new, dtype=bool)])
    is_seed[sv] = True
    st["is_seed"] = is_seed
    p.n = nt
    p.true_class = true_all
    return Batch(num_new, lo.astype(np.int32), hi.astype(np.int32), ww.astype(np.float32), sv, sc)


def erdos_renyi_single_batch(n: int, mean_degree: float, seed_frac: float, seed: int):
    """The paper's "all unlabelled vertices in one batch" experiment on an Erdos-Renyi graph
    (n vertices, n * mean_degree / 2 uniformly drawn pairs, duplicates and loops dropped, weights
    ~ U(0.1, 1), two classes drawn at random).  The first round(seed_frac * n) ids are the labelled
    vertices; they and the edges among them form the base graph, every other vertex and edge is
    the batch.  Returns (Problem of the base graph, Batch)."""
    rng = np.random.default_rng(seed)
    m = int(round(n * mean_degree / 2.0))
    lo, hi = _dedupe_undirected(n, rng.integers(0, n, size=m), rng.integers(0, n, size=m))
    ew = rng.uniform(0.1, 1.0, size=lo.shape[0]).astype(np.float32)
    cls = rng.integers(0, 2, size=n).astype(np.int32)
    ns = max(1, int(round(seed_frac * n)))
    old = hi < ns  # lo < hi, so both ends are labelled vertices
    row_ptr, col, w = edges_to_csr(ns, lo[old], hi[old], ew[old])
    sv = np.arange(ns, dtype=np.int32)
    st = dict(kind="er", rng=rng, is_seed=np.ones(ns, dtype=bool))
    p = Problem(ns, 2, row_ptr, col, w, sv, cls[:ns].copy(), cls[:ns].copy(), st)
    b = Batch(n - ns, lo[~old].astype(np.int32), hi[~old].astype(np.int32), ew[~old],
              np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.int32))
    return p, b


# --------------------------------------------------------------------------------------
# the five named configurations
# --------------------------------------------------------------------------------------
CONFIGS = {
    # name: (description, builder kwargs)
    "cfg1": dict(kind="knn", n=2_000, C=4, d=16, k=10, seed_frac=0.05, tol=1e-6, max_iter=1000,
                 batches=[dict(num_new=100, num_seeds=5)]),
    "cfg2": dict(kind="knn", n=100_000, C=10, d=64, k=10, seed_frac=0.01, tol=1e-6, max_iter=20000,
                 batches=[dict(num_new=1_000, num_seeds=10)] * 10),
    "cfg3": dict(kind="sbm", n=1_000_000, C=10, mean_degree=20.0, in_out_ratio=8.0, seed_frac=0.01,
                 tol=1e-6, max_iter=20000, batch_fracs=[0.001, 0.01, 0.1], batch_degree=20),
    "cfg4": dict(kind="chung_lu", n=10_000_000, C=50, mean_degree=40.0, exponent=2.1, d_max=50_000,
                 intra_frac=0.8, seed_frac=0.005, tol=1e-6, max_iter=20000, batch_sizes=[10_000, 100_000]),
    "cfg5": dict(kind="sbm-edge-stream", n=1_000_000, C=10, mean_degree=20.0, in_out_ratio=8.0,
                 seed_frac=0.01, tol=1e-6, max_iter=20000, num_batches=100, edges_per_batch=100_000,
                 intra_frac=0.5, revealed_per_batch=1_000),
    # the paper's own setting: binary labels, Erdos-Renyi graph, every unlabelled vertex in one batch
    "cfg6": dict(kind="er-single-batch", n=50_000_000, C=2, mean_degree=5.0, seed_frac=0.01, tol=1e-6,
                 max_iter=100000),
}


def make_config(name: str, scale: float = 1.0) -> Problem:
    """Build the base graph of a named configuration; ``scale`` < 1 shrinks n (same law)."""
    cfg = CONFIGS[name]
    idx = int(name[-1])
    n = max(64, int(round(cfg["n"] * scale)))
    seed = BASE_SEED + idx
    if cfg["kind"] == "knn":
        return knn_mixture(n, cfg["C"], cfg["d"], cfg["k"], cfg["seed_frac"], seed)
    if cfg["kind"] in ("sbm", "sbm-edge-stream"):
        return sbm(n, cfg["C"], cfg["mean_degree"], cfg["in_out_ratio"], cfg["seed_frac"], seed)
    if cfg["kind"] == "chung_lu":
        d_max = max(8, int(round(cfg["d_max"] * min(1.0, scale * 4)))) if scale < 1 else cfg["d_max"]
        return chung_lu(n, cfg["C"], cfg["mean_degree"], cfg["exponent"], d_max, cfg["intra_frac"],
                        cfg["seed_frac"], seed)
    if cfg["kind"] == "er-single-batch":  # base graph = the labelled vertices; the batch holds the rest
        p, b = erdos_renyi_single_batch(n, cfg["mean_degree"], cfg["seed_frac"], seed)
        p.state["single_batch"] = b
        return p
    raise KeyError(name)


def csr_with_batch(n_old: int, row_ptr, col, w, batch: Batch):
    """Symmetric CSR of the graph after an insertion batch (plumbing for large cases: same sort
    path as the generators; parallel edges stay separate entries)."""
    src = np.repeat(np.arange(n_old, dtype=np.int64), np.diff(row_ptr))
    up = src < col
    eu = np.concatenate([src[up], batch.eu.astype(np.int64)])
    ev = np.concatenate([col[up].astype(np.int64), batch.ev.astype(np.int64)])
    ew = np.concatenate([w[up], batch.ew])
    return edges_to_csr(n_old + batch.num_new_vertices, eu, ev, ew)
