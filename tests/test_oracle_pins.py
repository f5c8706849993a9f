"""Pins for the CPU oracle: it is checked against things that are NOT the oracle itself —
hand-derived closed forms (tests/golden), the dense solve of Eq. (2) versus the iteration of
Eq. (1), the paper's adjustment-form update, invariants, and brute-force set semantics."""
import json
import os

import numpy as np
import pytest

import workloads as W
from oracle import reference as R

GOLD = os.path.join(os.path.dirname(__file__), "golden", "harmonic_cases.json")


def _case_graph(case):
    e = np.array(case["edges"], dtype=np.float64)
    rp, col, w = W.edges_to_csr(case["n"], e[:, 0].astype(np.int64), e[:, 1].astype(np.int64), e[:, 2])
    sc = np.full(case["n"], -1, dtype=np.int64)
    for v, c in case["seeds"]:
        sc[v] = c
    return rp, col, w.astype(np.float64), sc


def _cases():
    return json.load(open(GOLD))["cases"]


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_textbook_values_closed_form_and_itlp(case, oracle_native):
    rp, col, w, sc = _case_graph(case)
    C = case["C"]
    F_cf = R.harmonic_closed_form(rp, col, w, sc, C)
    F_it, _, _ = R.itlp_solve(rp, col, w, sc, C, tol=1e-14)
    F_c, _, _ = oracle_native.itlp_solve(rp, col, w, sc, C, tol=1e-14)
    g = R.Graph(case["n"], rp, col, w, C, [v for v, _ in case["seeds"]], [c for _, c in case["seeds"]])
    adj = g.adjacency()
    F_lp = R.initial_labels(sc, C)
    for _ in range(4000):
        F_lp = R.itlp_sweep_loops(adj, F_lp, sc)
    for u, row in case["expect"].items():
        for F in (F_cf, F_it, F_c, F_lp):
            np.testing.assert_allclose(F[int(u)], row, atol=1e-11, rtol=0)


@pytest.mark.parametrize("n,C,deg,ns,seed", [(40, 2, 3.0, 4, 1), (120, 3, 4.0, 9, 2), (300, 5, 6.0, 20, 3),
                                             (200, 4, 2.2, 6, 4)])
def test_itlp_converges_to_dense_solve(n, C, deg, ns, seed, oracle_native):
    """Eq. (1) iterated to convergence equals Eq. (2) (convergence corollary)."""
    p = W.small_random(n, C, deg, ns, seed)
    sc = np.full(n, -1, dtype=np.int64)
    sc[p.seed_vertex] = p.seed_class
    w = p.w.astype(np.float64)
    F_cf = R.harmonic_closed_form(p.row_ptr, p.col, w, sc, C)
    F_it, it, ch = R.itlp_solve(p.row_ptr, p.col, w, sc, C, tol=1e-13)
    F_c, it_c, _ = oracle_native.itlp_solve(p.row_ptr, p.col, w, sc, C, tol=1e-13)
    assert ch <= 1e-13 and it == it_c
    assert np.max(np.abs(F_it - F_cf)) < 1e-9
    assert np.max(np.abs(F_c - F_cf)) < 1e-9
    # bit-for-bit is not required between numpy and C (different summation order) but nearly
    assert np.max(np.abs(F_c - F_it)) < 1e-12


def test_cfg1_sized_knn_graph_matches_dense_solve(oracle_native):
    """The small named configuration: 2,000-point kNN graph; ItLP vs the dense closed form."""
    p = W.make_config("cfg1")
    sc = np.full(p.n, -1, dtype=np.int64)
    sc[p.seed_vertex] = p.seed_class
    w = p.w.astype(np.float64)
    reach = R.seed_reachable(p.row_ptr, p.col, sc)
    F_c, it, ch = oracle_native.itlp_solve(p.row_ptr, p.col, w, sc, p.C, tol=1e-13, max_iter=2_000_000)
    assert ch <= 1e-13
    if reach.all():
        F_cf = R.harmonic_closed_form(p.row_ptr, p.col, w, sc, p.C)
        assert np.max(np.abs(F_c - F_cf)) < 1e-8
    else:  # restrict the dense solve to the seed-reachable part
        keep = np.flatnonzero(reach)
        remap = -np.ones(p.n, dtype=np.int64)
        remap[keep] = np.arange(keep.size)
        src = np.repeat(np.arange(p.n), np.diff(p.row_ptr))
        m = reach[src]
        rp2, col2, w2 = W.edges_to_csr(keep.size, remap[src[m]][src[m] < p.col[m]], remap[p.col[m]][src[m] < p.col[m]],
                                       w[m][src[m] < p.col[m]])
        F_cf = R.harmonic_closed_form(rp2, col2, w2.astype(np.float64), sc[keep], p.C)
        # float32 round trip of the weights in edges_to_csr is exact (they were float32 already)
        assert np.max(np.abs(F_c[keep] - F_cf)) < 1e-8


def test_three_sweep_implementations_agree(oracle_native):
    p = W.small_random(150, 4, 1.5, 10, 7, connected=False)
    rng = np.random.default_rng(0)
    sc = np.full(p.n, -1, dtype=np.int64)
    sc[p.seed_vertex] = p.seed_class
    F = rng.random((p.n, p.C))
    F /= F.sum(1, keepdims=True)
    F[sc >= 0] = R.initial_labels(sc, p.C)[sc >= 0]
    w = p.w.astype(np.float64)
    g = R.Graph(p.n, p.row_ptr, p.col, w, p.C, p.seed_vertex, p.seed_class)
    a = R.itlp_sweep_loops(g.adjacency(), F, sc)
    b = R.itlp_sweep(p.row_ptr, p.col, w, F, sc)
    c, ch = oracle_native.itlp_sweep(p.row_ptr, p.col, w, F, sc)
    assert np.max(np.abs(a - b)) < 1e-14 and np.max(np.abs(a - c)) < 1e-14
    assert abs(ch - np.max(np.abs(a - F))) < 1e-14
    # isolated rows and seed rows are untouched
    iso = np.diff(p.row_ptr) == 0
    assert iso.any()
    assert np.array_equal(a[iso], F[iso]) and np.array_equal(c[iso], F[iso])
    assert np.array_equal(a[sc >= 0], F[sc >= 0]) and np.array_equal(c[sc >= 0], F[sc >= 0])


def test_sweep_uses_own_row_weights_not_neighbours():
    """Asymmetric-degree trap: vertex 1 has neighbours 0 (w=1) and 2 (w=3); dividing by the
    wrong degree or transposing the gather gives a different value."""
    rp, col, w = W.edges_to_csr(4, [0, 1, 2], [1, 2, 3], [1.0, 3.0, 5.0])
    sc = np.array([0, -1, -1, 1])
    F = np.array([[1, 0], [0.5, 0.5], [0.2, 0.8], [0, 1]], dtype=np.float64)
    out = R.itlp_sweep(rp, col, w.astype(np.float64), F, sc)
    np.testing.assert_allclose(out[1], [(1 * 1 + 3 * 0.2) / 4, (1 * 0 + 3 * 0.8) / 4], atol=1e-15)
    np.testing.assert_allclose(out[2], [(3 * 0.5 + 5 * 0) / 8, (3 * 0.5 + 5 * 1) / 8], atol=1e-15)


def test_paper_adjustment_form_equals_weighted_mean():
    """Alg. 2 Step 3's printed formula (binary scalar labels, seeds contracted into L0/L1)
    gives column 1 of the C=2 matrix update: the equivalence shown in the theory section."""
    p = W.small_random(80, 2, 4.0, 8, 11)
    sc = np.full(p.n, -1, dtype=np.int64)
    sc[p.seed_vertex] = p.seed_class
    rng = np.random.default_rng(5)
    f = rng.random(p.n)
    f[sc == 0] = 0.0
    f[sc == 1] = 1.0
    F = np.stack([1 - f, f], axis=1)
    w = p.w.astype(np.float64)
    g = R.Graph(p.n, p.row_ptr, p.col, w, 2, p.seed_vertex, p.seed_class)
    adj = g.adjacency()
    out = R.itlp_sweep(p.row_ptr, p.col, w, F, sc)
    for u in range(p.n):
        if sc[u] < 0 and adj[u]:
            assert abs(R.step3_update_binary_adjustment(adj, f, sc, u) - out[u, 1]) < 1e-14


def test_invariants_rows_stochastic_seeds_fixed_maximum_principle(oracle_native):
    p = W.small_random(400, 6, 4.0, 25, 21)
    sc = np.full(p.n, -1, dtype=np.int64)
    sc[p.seed_vertex] = p.seed_class
    w = p.w.astype(np.float64)
    F0 = R.initial_labels(sc, p.C)
    F = F0
    for _ in range(30):
        F = R.itlp_sweep(p.row_ptr, p.col, w, F, sc)
        assert np.all(F >= 0) and np.max(np.abs(F.sum(1) - 1)) < 1e-12
        assert np.array_equal(F[sc >= 0], F0[sc >= 0])
    Fs, _, _ = oracle_native.itlp_solve(p.row_ptr, p.col, w, sc, p.C, tol=1e-13)
    assert np.array_equal(Fs[sc >= 0], F0[sc >= 0])
    assert np.all(Fs >= -1e-15) and np.all(Fs <= 1 + 1e-15)
    # harmonic: every unlabelled value lies within the range of its neighbours' values
    for u in np.flatnonzero(sc < 0)[:200]:
        nb = p.col[p.row_ptr[u]:p.row_ptr[u + 1]]
        assert np.all(Fs[u] <= Fs[nb].max(0) + 1e-10) and np.all(Fs[u] >= Fs[nb].min(0) - 1e-10)


def test_solution_minimises_dirichlet_energy(oracle_native):
    p = W.small_random(120, 3, 4.0, 8, 31)
    sc = np.full(p.n, -1, dtype=np.int64)
    sc[p.seed_vertex] = p.seed_class
    w = p.w.astype(np.float64)
    Fs, _, _ = oracle_native.itlp_solve(p.row_ptr, p.col, w, sc, p.C, tol=1e-13)
    e0 = R.dirichlet_energy(p.row_ptr, p.col, w, Fs)
    rng = np.random.default_rng(1)
    for _ in range(20):
        G = Fs + 1e-3 * rng.normal(size=Fs.shape) * (sc < 0)[:, None]
        assert R.dirichlet_energy(p.row_ptr, p.col, w, G) > e0


def test_energy_formula_on_single_edge():
    rp, col, w = W.edges_to_csr(2, [0], [1], [3.0])
    F = np.array([[1.0, 0.0], [0.25, 0.75]])
    # (1/2) * 3 * ((0.75)^2 + (0.75)^2)
    assert abs(R.dirichlet_energy(rp, col, w.astype(np.float64), F) - 0.5 * 3 * 2 * 0.75 ** 2) < 1e-15


def test_fixed_point_independent_of_start_and_incremental_equals_scratch(oracle_native):
    p = W.small_random(250, 3, 4.0, 12, 41)
    g = R.Graph(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class)
    rp, col, w = g.csr()
    F_before, _, _ = oracle_native.itlp_solve(rp, col, w, g.seed_class, p.C, tol=1e-13)
    b = W.small_random_batch(p, 20, 3, 2, num_extra_edges=10, num_revealed=3)
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    rp, col, w = g.csr()
    F_scratch, _, _ = R.recompute_from_scratch(g, tol=1e-13)
    warm = np.concatenate([F_before, np.full((b.num_new_vertices, p.C), 1.0 / p.C)])
    s = np.flatnonzero(g.seed_class >= 0)
    warm[s] = 0
    warm[s, g.seed_class[s]] = 1
    F_warm, _, _ = oracle_native.itlp_solve(rp, col, w, g.seed_class, p.C, tol=1e-13, F0=warm)
    rng = np.random.default_rng(3)
    rnd = rng.random(warm.shape)
    rnd[s] = warm[s]
    F_rnd, _, _ = oracle_native.itlp_solve(rp, col, w, g.seed_class, p.C, tol=1e-13, F0=rnd)
    reach = R.seed_reachable(rp, col, g.seed_class)
    assert np.max(np.abs(F_scratch - F_warm)[reach]) < 1e-9
    assert np.max(np.abs(F_scratch - F_rnd)[reach]) < 1e-9
    F_cf = R.harmonic_closed_form(rp, col, w, g.seed_class, p.C) if reach.all() else None
    if F_cf is not None:
        assert np.max(np.abs(F_scratch - F_cf)) < 1e-9


def test_seedless_component_and_isolated_rows_keep_invariants(oracle_native):
    # component {0,1,2} has a seed; component {3,4} has none; vertex 5 is isolated
    rp, col, w = W.edges_to_csr(6, [0, 1, 3], [1, 2, 4], [1.0, 2.0, 1.0])
    sc = np.array([1, -1, -1, -1, -1, -1])
    reach = R.seed_reachable(rp, col, sc)
    assert reach.tolist() == [True, True, True, False, False, False]
    F, _, _ = oracle_native.itlp_solve(rp, col, w.astype(np.float64), sc, 2, tol=1e-14, max_iter=500)
    np.testing.assert_allclose(F[[1, 2]], [[0, 1], [0, 1]], atol=1e-12)
    np.testing.assert_allclose(F[5], [0.5, 0.5])
    assert np.max(np.abs(F.sum(1) - 1)) < 1e-12


def test_hard_labels_lowest_index_on_ties():
    F = np.array([[0.5, 0.5], [0.2, 0.8], [0.4, 0.4]])
    assert R.hard_labels(F).tolist() == [0, 1, 0]
    F3 = np.array([[0.3, 0.35, 0.35]])
    assert R.hard_labels(F3).tolist() == [1]
    assert abs(R.top2_margin(F3)[0]) < 1e-16


@pytest.mark.parametrize("seed", [21, 22])
def test_in_place_sweeps_share_the_fixed_point_and_need_fewer_sweeps(seed):
    """Updating rows on one array (any visiting order) converges to the same harmonic labels as the
    Jacobi form of Eq. (1): the basis of the library's in-place update mode."""
    p = W.small_random(300, 3, 4.0, 15, seed)
    g = R.Graph(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class)
    rp, col, w = g.csr()
    exact = R.harmonic_closed_form(rp, col, w, g.seed_class, p.C)
    Fj, sweeps_j, _ = R.itlp_solve(rp, col, w, g.seed_class, p.C, tol=1e-11)
    order = np.random.default_rng(seed).permutation(p.n).tolist()
    for o in (None, order, order[::-1]):
        Fg, sweeps_g, _ = R.itlp_solve_in_place(rp, col, w, g.seed_class, p.C, tol=1e-11, order=o)
        assert np.abs(Fg - exact).max() < 1e-8
        assert sweeps_g < sweeps_j
    assert np.abs(Fj - exact).max() < 1e-8


# ---- (I - P_UU)^{-1}: the matrix of the convergence corollary, used for error bounds ------------
def _path(L):
    """Unit path 0-1-...-L with the two ends labelled (classes 0 and 1)."""
    eu = np.arange(L, dtype=np.int64)
    rp, col, w = W.edges_to_csr(L + 1, eu, eu + 1, np.ones(L))
    sc = np.full(L + 1, -1, dtype=np.int32)
    sc[0], sc[L] = 0, 1
    return rp, col, w.astype(np.float64), sc


def test_neumann_solve_on_a_path_gives_the_gamblers_ruin_duration(oracle_native):
    """b = 1: x_i is the expected number of steps of the simple random walk from i to either end of
    the path, i (L - i) (gambler's ruin), so ||(I - P_UU)^{-1}||_inf = L^2 / 4 for even L."""
    L = 12
    rp, col, w, sc = _path(L)
    want = np.array([i * (L - i) for i in range(L + 1)], dtype=np.float64)
    ones = np.ones(L + 1)
    np.testing.assert_allclose(R.neumann_solve_dense(rp, col, w, sc, ones), want, atol=1e-10)
    x, sweeps, last = oracle_native.neumann_solve(rp, col, w, sc, ones, tol=1e-13)
    np.testing.assert_allclose(x, want, atol=1e-9)
    np.testing.assert_allclose(R.neumann_solve_cg(rp, col, w, sc, ones), want, atol=1e-9)
    np.testing.assert_allclose(oracle_native.neumann_solve_cg(rp, col, w, sc, ones), want, atol=1e-9)
    assert x.max() == pytest.approx(L * L / 4)


def test_neumann_solve_three_ways_on_random_weighted_graphs(oracle_native):
    p = W.small_random(300, 3, 3.0, 12, 41, connected=False)  # some vertices reach no label: x = 0 there
    sc = np.full(p.n, -1, dtype=np.int32)
    sc[p.seed_vertex] = p.seed_class
    w = p.w.astype(np.float64)
    b = np.random.default_rng(5).uniform(0.0, 2.0, size=p.n)
    dense = R.neumann_solve_dense(p.row_ptr, p.col, w, sc, b)
    it, sweeps, last = oracle_native.neumann_solve(p.row_ptr, p.col, w, sc, b, tol=1e-14)
    cg = R.neumann_solve_cg(p.row_ptr, p.col, w, sc, b)
    cg_c = oracle_native.neumann_solve_cg(p.row_ptr, p.col, w, sc, b)
    assert np.max(np.abs(dense - it)) < 1e-9 and np.max(np.abs(dense - cg)) < 1e-9 and np.max(np.abs(dense - cg_c)) < 1e-9
    reach = R.seed_reachable(p.row_ptr, p.col, sc)
    upd = (sc < 0) & (np.diff(p.row_ptr) > 0) & reach
    assert np.all(dense[~upd] == 0) and dense[upd].min() > 0 and (~reach).sum() > 0
    # the series sum_k P^k b term by term (what "Neumann" means), 4,000 terms of it
    n = p.n
    Wm = np.zeros((n, n))
    np.add.at(Wm, (np.repeat(np.arange(n), np.diff(p.row_ptr)), p.col), w)
    U = np.flatnonzero(upd)
    P = Wm[np.ix_(U, U)] / Wm[U].sum(1, keepdims=True)
    term, tot = b[U].copy(), b[U].copy()
    for _ in range(4000):
        term = P @ term
        tot += term
    assert np.max(np.abs(tot - dense[U])) < 1e-6 * dense.max()


def test_labels_off_the_fixed_point_differ_from_it_by_the_propagated_residual(oracle_native):
    """F - F* = (I - P_UU)^{-1} (F - T(F)) for ANY label matrix F whose labelled rows are right (T = one
    sweep of Eq. (1)); hence |F - F*| <= (I - P_UU)^{-1} |F - T(F)| row by row and
    ||F - F*||_inf <= ||(I - P_UU)^{-1}||_inf ||F - T(F)||_inf.  This identity is what the GPU tests use to
    bound the distance of a locally stopped run from the exact labels."""
    p = W.small_random(250, 4, 3.5, 10, 43)
    sc = np.full(p.n, -1, dtype=np.int32)
    sc[p.seed_vertex] = p.seed_class
    w = p.w.astype(np.float64)
    exact = R.harmonic_closed_form(p.row_ptr, p.col, w, sc, p.C)
    rng = np.random.default_rng(7)
    F = exact + rng.normal(0.0, 1e-3, size=exact.shape) * (sc < 0)[:, None]
    TF, res = oracle_native.itlp_sweep(p.row_ptr, p.col, w, F, sc)
    r = F - TF
    assert res == pytest.approx(np.max(np.abs(r)))
    for c in range(p.C):
        prop = R.neumann_solve_dense(p.row_ptr, p.col, w, sc, r[:, c])
        np.testing.assert_allclose(prop, (F - exact)[:, c], atol=1e-12)
    bound = R.neumann_solve_dense(p.row_ptr, p.col, w, sc, np.max(np.abs(r), axis=1))
    err = np.max(np.abs(F - exact), axis=1)
    assert np.all(err <= bound + 1e-13)
    H = R.neumann_solve_dense(p.row_ptr, p.col, w, sc, np.ones(p.n)).max()
    assert err.max() <= H * res and H > 1.0
    # the bound is not vacuous: it is within a small factor of the error it bounds
    assert bound.max() <= 50 * err.max()


def test_harmonic_solve_by_conjugate_gradients_is_the_fixed_point_of_eq1(oracle_native):
    """The library solve of (D - W)_UU F_U = W_UL Y_L used as O1 on graphs too large for thousands of sweeps:
    equals Eq. (2) by dense solve, equals ItLP run to convergence, and one sweep of Eq. (1) leaves it alone."""
    p = W.small_random(400, 5, 4.0, 20, 47, connected=False)
    sc = np.full(p.n, -1, dtype=np.int32)
    sc[p.seed_vertex] = p.seed_class
    w = p.w.astype(np.float64)
    cg = R.harmonic_solve_cg(p.row_ptr, p.col, w, sc, p.C)
    cg_c = oracle_native.harmonic_solve_cg(p.row_ptr, p.col, w, sc, p.C)
    assert np.max(np.abs(cg - cg_c)) < 1e-10
    reach = R.seed_reachable(p.row_ptr, p.col, sc)
    it, _, _ = oracle_native.itlp_solve(p.row_ptr, p.col, w, sc, p.C, tol=1e-14, max_iter=1_000_000)
    assert np.max(np.abs(cg - it)[reach]) < 1e-10
    _, moved = oracle_native.itlp_sweep(p.row_ptr, p.col, w, np.where(reach[:, None], cg, it), sc)
    assert moved < 1e-12
    assert np.array_equal(cg[~reach], R.initial_labels(sc, p.C)[~reach])  # left at the start values
    # a class no vertex is labelled with: its column is identically zero (and the library solve must cope with the
    # zero right-hand side)
    z = W.small_random(300, 6, 4.0, 12, 51)
    keep = z.seed_class != 4
    scz = np.full(z.n, -1, dtype=np.int32)
    scz[z.seed_vertex[keep]] = z.seed_class[keep]
    Fz = oracle_native.harmonic_solve_cg(z.row_ptr, z.col, z.w.astype(np.float64), scz, 6)
    Fz_it, _, _ = oracle_native.itlp_solve(z.row_ptr, z.col, z.w.astype(np.float64), scz, 6, tol=1e-14, max_iter=1_000_000)
    rz = R.seed_reachable(z.row_ptr, z.col, scz)
    upd = rz & (scz < 0) & (np.diff(z.row_ptr) > 0)
    assert np.all(Fz[upd, 4] == 0.0) and np.max(np.abs(Fz - Fz_it)[rz]) < 1e-10
    q = W.small_random(120, 3, 3.0, 8, 49)
    scq = np.full(q.n, -1, dtype=np.int32)
    scq[q.seed_vertex] = q.seed_class
    dense = R.harmonic_closed_form(q.row_ptr, q.col, q.w.astype(np.float64), scq, q.C)
    np.testing.assert_allclose(R.harmonic_solve_cg(q.row_ptr, q.col, q.w.astype(np.float64), scq, q.C), dense, atol=1e-11)
    np.testing.assert_allclose(oracle_native.harmonic_solve_cg(q.row_ptr, q.col, q.w.astype(np.float64), scq, q.C), dense, atol=1e-11)
