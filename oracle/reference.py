"""Plain float64 definitions of what DynLP computes.  TEST INFRASTRUCTURE ONLY.

Notation follows the paper: graph G=(V,E) with symmetric weights w(u,v)>0, labelled
(seed) set V^L with fixed one-hot rows Y_u, unlabelled set V^U, label matrix F (n x C;
the paper's binary scalar F_u is column 1 of the C=2 case), degree d(u)=sum_v w(u,v),
affected set / frontier V_aff, threshold delta (``tol``).

Readings taken where the paper is silent or garbled:
* multi-class: Eq. (1) applied to every column of F with one-hot seed rows;
* Alg. 2 Step 3 threshold: absolute change, max over classes, strict ``>``;
* Alg. 2 Step 3 commit: the computed F'_u is stored whether or not it passed the threshold;
* rows with d(u)=0 never change; parallel edges add their weights;
* an inserted edge affects both endpoints; a vertex that becomes a seed affects its
  neighbours and is itself clamped to one-hot and never updated again;
* a deleted vertex keeps its id as an isolated, unlabelled vertex with the neutral row 1/C; a
  neighbour that loses its last edge keeps the label it had;
* Step 2 for C classes: a supernode's row is its weight share per labelled class, uniform when
  it has no labelled neighbour; the threshold tau acts on each listed batch edge separately.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------------------
# graph model (Section "Preliminaries": weighted undirected graph; Alg. 1 Step 1: update)
# --------------------------------------------------------------------------------------
class Graph:
    """Directed-entry list of a symmetric weighted graph, float64 weights.

    ``insert`` is Alg. 1 Step 1 for insertions: new vertices get ids n..n+k-1 and every new
    undirected edge (u,v,w) is entered in both directions.  Parallel edges are kept as
    separate entries; every formula below is linear in w, so they act as one summed edge.
    """

    def __init__(self, n, row_ptr, col, w, C, seed_vertex, seed_class):
        row_ptr = np.asarray(row_ptr, dtype=np.int64)
        self.n = int(n)
        self.C = int(C)
        self.src = np.repeat(np.arange(self.n, dtype=np.int64), np.diff(row_ptr))
        self.dst = np.asarray(col, dtype=np.int64).copy()
        self.w = np.asarray(w, dtype=np.float64).copy()
        self.seed_class = np.full(self.n, -1, dtype=np.int64)
        self.seed_class[np.asarray(seed_vertex, dtype=np.int64)] = np.asarray(seed_class, dtype=np.int64)

    def insert(self, num_new_vertices, eu, ev, ew, seed_vertex, seed_class):
        eu = np.asarray(eu, dtype=np.int64)
        ev = np.asarray(ev, dtype=np.int64)
        ew = np.asarray(ew, dtype=np.float64)
        self.n += int(num_new_vertices)
        self.src = np.concatenate([self.src, eu, ev])
        self.dst = np.concatenate([self.dst, ev, eu])
        self.w = np.concatenate([self.w, ew, ew])
        self.seed_class = np.concatenate([self.seed_class, np.full(int(num_new_vertices), -1, dtype=np.int64)])
        self.seed_class[np.asarray(seed_vertex, dtype=np.int64)] = np.asarray(seed_class, dtype=np.int64)

    def delete(self, vertices):
        """Alg. 2 Step 1 for Delta^Del: every edge incident to a deleted vertex disappears.  Ids are
        not renumbered: a deleted vertex stays behind as an isolated, unlabelled vertex (it is
        never updated again and can be given edges by a later batch)."""
        dead = np.zeros(self.n, dtype=bool)
        dead[np.asarray(vertices, dtype=np.int64)] = True
        keep = ~(dead[self.src] | dead[self.dst])
        self.src, self.dst, self.w = self.src[keep], self.dst[keep], self.w[keep]
        self.seed_class[dead] = -1

    def csr(self):
        """(row_ptr int64, col int64, w float64), rows in insertion order."""
        order = np.argsort(self.src, kind="stable")
        counts = np.bincount(self.src, minlength=self.n)
        row_ptr = np.zeros(self.n + 1, dtype=np.int64)
        np.cumsum(counts, out=row_ptr[1:])
        return row_ptr, self.dst[order], self.w[order]

    def adjacency(self):
        """list of {v: w} with parallel edges summed (for the pure-Python definitions)."""
        adj = [dict() for _ in range(self.n)]
        for u, v, w in zip(self.src.tolist(), self.dst.tolist(), self.w.tolist()):
            adj[u][v] = adj[u].get(v, 0.0) + w
        return adj


def initial_labels(seed_class, C):
    """Seed rows one-hot Y_u (Eq. 1, second case); unlabelled rows uniform 1/C (the paper
    allows an arbitrary start for unlabelled vertices, Introduction / Step 2 neutral value)."""
    seed_class = np.asarray(seed_class)
    n = seed_class.shape[0]
    F = np.full((n, C), 1.0 / C, dtype=np.float64)
    s = np.flatnonzero(seed_class >= 0)
    F[s] = 0.0
    F[s, seed_class[s]] = 1.0
    return F


# --------------------------------------------------------------------------------------
# Eq. (2): closed-form harmonic solution (dense; tiny graphs only)
# --------------------------------------------------------------------------------------
def harmonic_closed_form(row_ptr, col, w, seed_class, C):
    """F^U = -L_UU^{-1} L_UL F^L with L = D - W (Eq. 2).  Requires every unlabelled vertex
    to reach a seed (else L_UU is singular).  Returns the full n x C matrix."""
    seed_class = np.asarray(seed_class)
    n = seed_class.shape[0]
    Wm = np.zeros((n, n), dtype=np.float64)
    src = np.repeat(np.arange(n), np.diff(row_ptr))
    np.add.at(Wm, (src, np.asarray(col)), np.asarray(w, dtype=np.float64))
    L = np.diag(Wm.sum(axis=1)) - Wm
    lab = np.flatnonzero(seed_class >= 0)
    unl = np.flatnonzero(seed_class < 0)
    F = initial_labels(seed_class, C)
    FL = F[lab]
    L_UU = L[np.ix_(unl, unl)]
    L_UL = L[np.ix_(unl, lab)]
    F[unl] = -np.linalg.solve(L_UU, L_UL @ FL)
    return F


# --------------------------------------------------------------------------------------
# Eq. (1): iterative label propagation ItLP, Jacobi sweeps
# --------------------------------------------------------------------------------------
def itlp_sweep_loops(adj, F, seed_class):
    """One sweep of Eq. (1) written as the definition: loops over vertices, neighbours and
    classes.  ``adj`` is a list of {v: w}.  Reads F^{(k)}, returns F^{(k+1)}."""
    n, C = F.shape
    out = F.copy()
    for u in range(n):
        if seed_class[u] >= 0:
            continue  # F_u = Y_u stays
        d = 0.0
        for v, wuv in adj[u].items():
            d += wuv
        if d == 0.0:
            continue
        for c in range(C):
            acc = 0.0
            for v, wuv in adj[u].items():
                acc += wuv * F[v, c]
            out[u, c] = acc / d
    return out


def itlp_sweep(row_ptr, col, w, F, seed_class):
    """One Jacobi sweep of Eq. (1), vectorised: F^{(k+1)}_u = (1/d(u)) sum_v w(u,v) F^{(k)}_v
    for unlabelled u with d(u)>0; all other rows unchanged."""
    n, C = F.shape
    src = np.repeat(np.arange(n), np.diff(row_ptr))
    d = np.bincount(src, weights=w, minlength=n)
    out = F.copy()
    upd = (np.asarray(seed_class) < 0) & (d > 0)
    for c in range(C):
        num = np.bincount(src, weights=w * F[col, c], minlength=n)
        out[upd, c] = num[upd] / d[upd]
    return out


def itlp_solve(row_ptr, col, w, seed_class, C, tol=1e-10, max_iter=1_000_000, F0=None):
    """ItLP to convergence: sweep until max_u max_c |F^{(k+1)} - F^{(k)}| <= tol.
    Returns (F, sweeps, last_change)."""
    F = initial_labels(seed_class, C) if F0 is None else np.array(F0, dtype=np.float64)
    it, change = 0, np.inf
    while it < max_iter:
        Fn = itlp_sweep(row_ptr, col, w, F, seed_class)
        change = float(np.max(np.abs(Fn - F))) if F.size else 0.0
        F = Fn
        it += 1
        if change <= tol:
            break
    return F, it, change


def itlp_solve_in_place(row_ptr, col, w, seed_class, C, tol=1e-10, max_iter=1_000_000, F0=None, order=None):
    """Eq. (1) applied row after row on one array: a row's new value is visible to the rows that
    come later in the same sweep (what Alg. 2's loop over V_aff does when it runs on a single
    label array).  ``order``: the sequence in which the unlabelled rows are visited (default: by
    id).  Same stop rule as itlp_solve (largest change of a sweep <= tol).  Returns
    (F, sweeps, last_change)."""
    seed_class = np.asarray(seed_class)
    F = initial_labels(seed_class, C) if F0 is None else np.array(F0, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    rows = [u for u in (range(seed_class.shape[0]) if order is None else order)
            if seed_class[u] < 0 and row_ptr[u + 1] > row_ptr[u]]
    change = 0.0
    for sweep in range(1, max_iter + 1):
        change = 0.0
        for u in rows:
            a, b = row_ptr[u], row_ptr[u + 1]
            new = (w[a:b, None] * F[col[a:b]]).sum(axis=0) / w[a:b].sum()
            change = max(change, float(np.max(np.abs(new - F[u]))))
            F[u] = new
        if change <= tol:
            return F, sweep, change
    return F, max_iter, change


# --------------------------------------------------------------------------------------
# how far labels with a known residual are from the fixed point (convergence corollary)
# --------------------------------------------------------------------------------------
def _updatable(row_ptr, col, seed_class):
    """Unlabelled vertices with at least one edge that reach a labelled vertex: the rows on which
    Eq. (1) has a unique fixed point (I - P_UU is invertible there)."""
    seed_class = np.asarray(seed_class)
    return (seed_class < 0) & (np.diff(row_ptr) > 0) & seed_reachable(row_ptr, col, seed_class)


def neumann_solve_dense(row_ptr, col, w, seed_class, b):
    """x = (I - P_UU)^{-1} b by a dense solve, P = D^{-1} W restricted to the updatable rows (tiny
    graphs only); 0 elsewhere.  (I - P_UU)^{-1} = sum_k P_UU^k is the matrix of the paper's
    convergence proof and of Eq. (2)."""
    seed_class = np.asarray(seed_class)
    n = seed_class.shape[0]
    Wm = np.zeros((n, n), dtype=np.float64)
    np.add.at(Wm, (np.repeat(np.arange(n), np.diff(row_ptr)), np.asarray(col)), np.asarray(w, dtype=np.float64))
    U = np.flatnonzero(_updatable(row_ptr, col, seed_class))
    P = Wm[np.ix_(U, U)] / Wm[U].sum(axis=1, keepdims=True)
    x = np.zeros(n, dtype=np.float64)
    x[U] = np.linalg.solve(np.eye(U.size) - P, np.asarray(b, dtype=np.float64)[U])
    return x


def _laplacian_blocks(row_ptr, col, w, seed_class):
    """(U, index of every vertex inside U or -1, d on U, sparse W_UU, sparse W_UL, ids of L) for the
    library solves below (scipy.sparse)."""
    import scipy.sparse as sp

    seed_class = np.asarray(seed_class)
    n = seed_class.shape[0]
    w = np.asarray(w, dtype=np.float64)
    col = np.asarray(col, dtype=np.int64)
    src = np.repeat(np.arange(n, dtype=np.int64), np.diff(row_ptr))
    d = np.bincount(src, weights=w, minlength=n)
    in_U = _updatable(row_ptr, col, seed_class)
    U = np.flatnonzero(in_U)
    pos = np.full(n, -1, dtype=np.int64)
    pos[U] = np.arange(U.size)
    lab = np.flatnonzero(seed_class >= 0)
    lpos = np.full(n, -1, dtype=np.int64)
    lpos[lab] = np.arange(lab.size)
    uu = in_U[src] & in_U[col]
    ul = in_U[src] & (seed_class[col] >= 0)
    W_UU = sp.csr_matrix((w[uu], (pos[src[uu]], pos[col[uu]])), shape=(U.size, U.size))
    W_UL = sp.csr_matrix((w[ul], (pos[src[ul]], lpos[col[ul]])), shape=(U.size, lab.size))
    return U, d[U], W_UU, W_UL, lab


def _cg(A, rhs, x0, rtol, max_iter):
    import scipy.sparse as sp
    import scipy.sparse.linalg as spl

    # Jacobi-preconditioned conjugate gradients on the symmetric positive definite matrix (D - W)_UU
    Minv = sp.diags(1.0 / A.diagonal())
    x, info = spl.cg(A, rhs, x0=x0, rtol=rtol, atol=0.0, maxiter=max_iter, M=Minv)
    if info != 0:
        raise RuntimeError(f"conjugate gradients did not converge (info = {info})")
    return x


def neumann_solve_cg(row_ptr, col, w, seed_class, b, rtol=1e-13, max_iter=20000):
    """x = (I - P_UU)^{-1} b for large graphs: the same system written with the symmetric matrix,
    (D - W)_UU x = D_U b, solved by a library routine (conjugate gradients).  0 outside the
    updatable rows.  Callers certify the result with one step of x <- b + P_UU x."""
    import scipy.sparse as sp

    U, dU, W_UU, _, _ = _laplacian_blocks(row_ptr, col, w, seed_class)
    A = (sp.diags(dU) - W_UU).tocsr()
    b = np.asarray(b, dtype=np.float64)
    x = np.zeros(b.shape[0], dtype=np.float64)
    x[U] = _cg(A, dU * b[U], None, rtol, max_iter)
    return x


def harmonic_solve_cg(row_ptr, col, w, seed_class, C, F_other=None, rtol=1e-13, max_iter=20000):
    """The fixed point of Eq. (1) for large graphs, column by column, from Eq. (2) written with the
    symmetric matrix: (D - W)_UU F_U = W_UL Y_L, solved by a library routine (conjugate
    gradients).  Rows outside the updatable set (labelled, isolated, not connected to any label)
    are taken from ``F_other`` (default: one-hot / uniform start).  Callers certify the result with
    one sweep of Eq. (1): a fixed point does not move."""
    import scipy.sparse as sp

    seed_class = np.asarray(seed_class)
    U, dU, W_UU, W_UL, lab = _laplacian_blocks(row_ptr, col, w, seed_class)
    A = (sp.diags(dU) - W_UU).tocsr()
    F = initial_labels(seed_class, C) if F_other is None else np.array(F_other, dtype=np.float64)
    Y = np.zeros((lab.size, C), dtype=np.float64)
    Y[np.arange(lab.size), seed_class[lab]] = 1.0
    F[lab] = Y
    rhs = W_UL @ Y
    for c in range(C):
        F[U, c] = _cg(A, rhs[:, c], None, rtol, max_iter)
    return F


def recompute_from_scratch(graph: Graph, tol=1e-10, max_iter=1_000_000):
    """Alg. 1 Step 2 with ItLP in place of the dense inverse: labels of the *current* graph
    from the uniform start."""
    row_ptr, col, w = graph.csr()
    return itlp_solve(row_ptr, col, w, graph.seed_class, graph.C, tol, max_iter)


# --------------------------------------------------------------------------------------
# Alg. 2: affected set and Step 3 (frontier-restricted propagation)
# --------------------------------------------------------------------------------------
def affected_set(adj_after, seed_class_after, num_old_vertices, num_new_vertices, eu, ev, new_seed_vertex,
                 deleted=(), adj_before=None):
    """V_aff after Step 1: for each deleted vertex its neighbours in the graph before the batch
    (Alg. 2: V_aff <- V_aff U N(u) for u in Delta^Del; needs ``adj_before``); each inserted
    vertex and its neighbours (V_aff <- V_aff U {u} U N(u)); for edges between existing
    vertices, both endpoints; for a vertex that became a seed, its neighbours.  Seeds and
    isolated vertices are never in the set (they are never updated).  ``adj_after`` is the
    updated graph."""
    A = set()
    for u in np.asarray(deleted, dtype=np.int64).tolist():
        A.update(adj_before[u].keys())
    for u in range(num_old_vertices, num_old_vertices + num_new_vertices):
        A.add(u)
        A.update(adj_after[u].keys())
    for a, b in zip(np.asarray(eu).tolist(), np.asarray(ev).tolist()):
        A.add(a)
        A.add(b)
    for s in np.asarray(new_seed_vertex).tolist():
        A.update(adj_after[s].keys())
    return {u for u in A if seed_class_after[u] < 0 and len(adj_after[u]) > 0}


def _exceeds(new_row, old_row, tol, decide_fp32):
    """Threshold test of Alg. 2 Step 3 (absolute change, max over classes, strict >).
    With ``decide_fp32`` the comparison is carried out in binary32 like the GPU kernel."""
    if decide_fp32:
        r = np.max(np.abs(new_row.astype(np.float32) - old_row.astype(np.float32)))
        return bool(r > np.float32(tol)), float(r)
    r = float(np.max(np.abs(new_row - old_row)))
    return r > tol, r


def step3_propagate(adj, F, seed_class, V_aff, tol, max_iter, decide_fp32=True, trace=None):
    """Alg. 2 Step 3 in synchronous rounds.  Each round: every u in V_aff gets
    F'_u = sum_v alpha_{u,v} F_v from the round-start F (the equivalence of the adjustment
    form and the weighted mean is the paper's Theoretical-analysis section); all F'_u are
    committed; u with change > tol stay and bring in N(u); the others leave.
    ``trace``: a list that receives, per round, (sorted V_aff, sorted rows that moved by more
    than tol, copy of F after the commit).
    Returns (F, rounds, frontier_sizes, max_change_per_round)."""
    F = np.array(F, dtype=np.float64)
    A = set(V_aff)
    sizes, changes = [], []
    rounds = 0
    while A and rounds < max_iter:
        new_rows = {}
        for u in A:
            d = sum(adj[u].values())
            acc = np.zeros(F.shape[1])
            for v, wuv in adj[u].items():
                acc += wuv * F[v]
            new_rows[u] = acc / d
        nxt = set()
        moved = []
        mx = 0.0
        for u, row in new_rows.items():
            big, r = _exceeds(row, F[u], tol, decide_fp32)
            mx = max(mx, r)
            if big:
                moved.append(u)
                nxt.add(u)
                nxt.update(adj[u].keys())
        for u, row in new_rows.items():
            F[u] = row
        if trace is not None:
            trace.append((sorted(A), sorted(moved), F.copy()))
        sizes.append(len(A))
        changes.append(mx)
        A = {u for u in nxt if seed_class[u] < 0 and len(adj[u]) > 0}
        rounds += 1
    return F, rounds, sizes, changes


def step3_update_binary_adjustment(adj, f, seed_class, u):
    """The paper's Step-3 formula exactly as printed for binary scalar labels f_u in [0,1]:
    F'_u = F_u + (0-F_u) W^{L0}/W^{all} + (1-F_u) W^{L1}/W^{all}
               + sum_{v in N(u) \\ (V^{L0} U V^{L1})} (F_v - F_u) w(u,v)/W^{all}."""
    w_all = sum(adj[u].values())
    w_l0 = sum(wuv for v, wuv in adj[u].items() if seed_class[v] == 0)
    w_l1 = sum(wuv for v, wuv in adj[u].items() if seed_class[v] == 1)
    rest = sum((f[v] - f[u]) * wuv / w_all for v, wuv in adj[u].items() if seed_class[v] < 0)
    return f[u] + (0.0 - f[u]) * w_l0 / w_all + (1.0 - f[u]) * w_l1 / w_all + rest


# --------------------------------------------------------------------------------------
# Alg. 2 Step 1 (sparsification + components of G') and Step 2 (label initialisation)
# --------------------------------------------------------------------------------------
def mean_edge_weight(w):
    """The experiments' threshold tau: the average edge weight of the data set.  Every
    undirected edge appears twice in the directed-entry list, so the mean over entries is the
    mean over edges."""
    w = np.asarray(w, dtype=np.float64)
    return float(w.sum() / w.shape[0]) if w.shape[0] else 0.0


def batch_internal_edges(num_old_vertices, num_new_vertices, eu, ev, ew, tau):
    """E' of Alg. 2 Step 1: the batch's edges whose two endpoints are both inserted vertices
    (V' = Delta^Ins) and whose weight exceeds tau (strict: an entry with w <= tau is the one
    the sparsification kernel flags as removed).  Every listed edge is tested on its own
    weight, parallel edges included.  Returns pairs of batch-local ids 0..k-1."""
    lo, hi = int(num_old_vertices), int(num_old_vertices) + int(num_new_vertices)
    out = []
    for a, b, wab in zip(np.asarray(eu).tolist(), np.asarray(ev).tolist(), np.asarray(ew, dtype=np.float64).tolist()):
        if lo <= a < hi and lo <= b < hi and wab > tau:
            out.append((a - lo, b - lo))
    return out


def connected_components(k, edges):
    """FindConnectedComponents(G'(V',E')): comp[i] = index of i's component, components numbered
    in the order of their smallest member (so comp is canonical).  Plain breadth-first search."""
    nbr = [[] for _ in range(k)]
    for a, b in edges:
        nbr[a].append(b)
        nbr[b].append(a)
    comp = np.full(k, -1, dtype=np.int64)
    count = 0
    for s in range(k):
        if comp[s] >= 0:
            continue
        comp[s] = count
        queue = [s]
        while queue:
            nxt = []
            for u in queue:
                for v in nbr[u]:
                    if comp[v] < 0:
                        comp[v] = count
                        nxt.append(v)
            queue = nxt
        count += 1
    return comp, count


def supernode_weights(adj_after, seed_class_after, num_old_vertices, comp, num_components, C):
    """Step 2: W_{c_i}^{L_k} = sum_{u in c_i} sum_{v in L_k} w(u,v), the weight between supernode
    c_i and the supernode of all vertices labelled k (the paper has k in {0,1}; here k < C).
    The sums run over the updated graph's edges, to old and new labelled vertices alike, and
    over every member u of c_i."""
    W = np.zeros((num_components, C), dtype=np.float64)
    for i, c in enumerate(np.asarray(comp).tolist()):
        u = num_old_vertices + i
        for v, wuv in adj_after[u].items():
            if seed_class_after[v] >= 0:
                W[c, seed_class_after[v]] += wuv
    return W


def supernode_label(Wrow):
    """Step 2 initial row of a supernode: class share of its weight to the labelled supernodes,
    W_k / sum_j W_j.  For two classes column 1 is the paper's
    0.5 - W^{L0}/(2(W^{L0}+W^{L1})) + W^{L1}/(2(W^{L0}+W^{L1})).  A supernode with no weight to
    any labelled vertex gets the neutral value (0.5 in the paper, 1/C here)."""
    Wrow = np.asarray(Wrow, dtype=np.float64)
    tot = Wrow.sum()
    if tot <= 0.0:
        return np.full(Wrow.shape[0], 1.0 / Wrow.shape[0])
    return Wrow / tot


def supernode_label_binary_as_printed(w_l0, w_l1):
    """The paper's Step-2 expression for the scalar label, term by term."""
    return 0.5 - w_l0 / (2.0 * (w_l0 + w_l1)) + w_l1 / (2.0 * (w_l0 + w_l1))


def step2_initialise(F, adj_after, seed_class_after, num_old_vertices, num_new_vertices, eu, ev, ew, tau):
    """Steps 1-2 of Alg. 2 for the inserted vertices: components of the sparsified
    batch-internal graph, then every unlabelled member of a component gets the component's
    row.  Labelled inserted vertices are members of their component (their edges count in the
    sums) but keep their one-hot row.  Returns (F with the new rows set, comp, number of
    components, W)."""
    F = np.array(F, dtype=np.float64)
    C = F.shape[1]
    comp, count = connected_components(num_new_vertices,
                                       batch_internal_edges(num_old_vertices, num_new_vertices, eu, ev, ew, tau))
    W = supernode_weights(adj_after, seed_class_after, num_old_vertices, comp, count, C)
    for i in range(num_new_vertices):
        u = num_old_vertices + i
        if seed_class_after[u] < 0:
            F[u] = supernode_label(W[comp[i]])
    return F, comp, count, W


# --------------------------------------------------------------------------------------
# outputs and helpers for comparisons
# --------------------------------------------------------------------------------------
def hard_labels(F):
    """argmax over classes, lowest class index on ties (the paper's 0.5 cut-off for C=2)."""
    return np.argmax(F, axis=1).astype(np.int64)


def top2_margin(F):
    if F.shape[1] == 1:
        return np.full(F.shape[0], np.inf)
    s = np.sort(F, axis=1)
    return s[:, -1] - s[:, -2]


def seed_reachable(row_ptr, col, seed_class):
    """Vertices connected to at least one seed (the convergence corollary needs a connected
    graph with V^L non-empty; on seedless components the harmonic solution is not unique)."""
    seed_class = np.asarray(seed_class)
    n = seed_class.shape[0]
    src = np.repeat(np.arange(n), np.diff(row_ptr))
    col = np.asarray(col)
    reach = seed_class >= 0
    while True:
        grown = reach.copy()
        grown[col[reach[src]]] = True
        if grown.sum() == reach.sum():
            return reach
        reach = grown


def dirichlet_energy(row_ptr, col, w, F):
    """(1/2) sum_{(u,v) in E} w_uv |F_u - F_v|^2 summed over classes (each undirected edge
    once; the CSR lists it twice, hence the extra 1/2)."""
    n = F.shape[0]
    src = np.repeat(np.arange(n), np.diff(row_ptr))
    diff = F[src] - F[col]
    return 0.25 * float(np.sum(np.asarray(w)[:, None] * diff * diff))
