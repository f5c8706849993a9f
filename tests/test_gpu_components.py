"""GPU parity of the label initialisation of inserted vertices (Alg. 2 Step 1 sparsification +
connected components, Step 2 supernode rows) against the CPU oracle, through the C ABI.

* component ids: bit-exact (they are canonical: numbered by smallest member);
* initial rows: binary32 quotient of binary64 sums vs the oracle's binary64 rows: max-abs <= 1e-6;
* the rounds that follow: same bars as the other batch tests.
"""
import numpy as np
import pytest

import workloads as W
from oracle import native as ON
from oracle import reference as R
import paper_2604_06596_amd as P

pytestmark = pytest.mark.gpu

TOL = 1e-6
INIT_ATOL = 1e-6
ROUNDS_ATOL = 5e-6
O1_ATOL = 1e-4


def _make(p, **kw):
    return P.DynLP(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class, **kw)


def _oracle_init(g, F_before, b, tau):
    """Oracle side: graph update, seed clamp, Steps 1-2.  Returns (rp, col, w, F_init, A0, comp, count, kept)."""
    n_old = g.n
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    F = np.concatenate([F_before, np.full((b.num_new_vertices, g.C), 1.0 / g.C)])
    s = np.asarray(b.seed_vertex, dtype=np.int64)
    F[s] = 0
    F[s, np.asarray(b.seed_class, dtype=np.int64)] = 1
    rp, col, w = g.csr()
    A0 = ON.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex)
    comp, count, kept = ON.components(n_old, b.num_new_vertices, b.eu, b.ev, b.ew, tau)
    F_init, _ = ON.supernode_init(rp, col, w, F, g.seed_class, n_old, comp, count)
    return rp, col, w, F_init, A0, comp, count, kept


def _problem(C, seed, n=5000):
    return W.small_random(n, C, 9.0, 250, seed), W.small_random(n, C, 9.0, 250, seed)


@pytest.mark.parametrize("C,k,mean_cluster", [(2, 800, 6.0), (10, 800, 6.0), (50, 333, 3.0), (10, 1, 1.0), (4, 2500, 40.0)])
def test_components_and_initial_rows_match_the_oracle(C, k, mean_cluster):
    p, p0 = _problem(C, 1200 + C)
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    b = W.clustered_batch(p, k, mean_cluster, 2, 1, 3, max(1, k // 50))
    with _make(p0) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        tau = np.float32(d.mean_edge_weight())
        assert abs(d.mean_edge_weight() - R.mean_edge_weight(g.w)) <= 1e-12 * R.mean_edge_weight(g.w)
        soft0, _ = d.get_labels()
        d.set_initialiser(P.INIT_SUPERNODE, tau)
        d.set_params(TOL, 0)  # no propagation round: the labels read back are the Step-2 rows
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        assert st == 1 and s.iterations == 0
        soft, _ = d.get_labels()
        comp, info = d.last_components()
    rp, col, w, F_init, A0, ocomp, count, kept = _oracle_init(g, soft0.astype(np.float64), b, float(tau))
    assert info.vertices == k and info.kept_edges == kept and info.components == count
    assert np.array_equal(comp, ocomp)
    assert np.max(np.abs(soft - F_init)) <= INIT_ATOL
    assert s.frontier_initial == A0.shape[0]
    if k >= 300:
        assert 1 < count < k  # multi-vertex components and more than one of them


@pytest.mark.parametrize("C,seeds,tau", [(3, 3000, 0.0), (10, 2500, 0.0), (4, 3500, 0.45)])
def test_supernode_sums_with_many_labelled_neighbours_and_one_giant_supernode(C, seeds, tau):
    """Most of the graph labelled and a batch whose internal edges connect nearly all of its vertices (tau = 0:
    one supernode takes almost every contribution): a workgroup's rows then bring far more contributions than its
    LDS list holds, so both the merged atomics and the overflow path carry weight, all onto a handful of sums."""
    p, p0 = (W.small_random(5000, C, 9.0, seeds, 1700 + C), W.small_random(5000, C, 9.0, seeds, 1700 + C))
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    b = W.small_random_batch(p, 4000, 9, 50)
    with _make(p0) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        soft0, _ = d.get_labels()
        d.set_initialiser(P.INIT_SUPERNODE, tau)
        d.set_params(TOL, 0)
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft, _ = d.get_labels()
        comp, info = d.last_components()
    rp, col, w, F_init, A0, ocomp, count, kept = _oracle_init(g, soft0.astype(np.float64), b, float(tau))
    sizes = np.bincount(ocomp)
    labelled = int(np.count_nonzero(g.seed_class[col[rp[p0.n]:]] >= 0))  # contributions of the inserted rows
    print(f"components {count}, largest {sizes.max()} of {b.num_new_vertices}, labelled neighbour entries {labelled}")
    assert sizes.max() > 0.5 * b.num_new_vertices and labelled > 4 * 1024
    assert info.components == count and np.array_equal(comp, ocomp)
    assert np.max(np.abs(soft - F_init)) <= INIT_ATOL


@pytest.mark.parametrize("C", [2, 10])
@pytest.mark.parametrize("R_", [1, 3, 25])
def test_rounds_after_the_supernode_initialisation_match_the_oracle(C, R_):
    p, p0 = _problem(C, 1300 + C)
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    b = W.clustered_batch(p, 500, 6.0, 2, 1, 3, 8)
    with _make(p0) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        tau = np.float32(d.mean_edge_weight())
        soft0, _ = d.get_labels()
        d.set_initialiser(P.INIT_SUPERNODE, tau)
        d.set_params(TOL, R_)
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft, _ = d.get_labels()
        sizes, deltas = d.round_log()
    rp, col, w, F_init, A0, *_ = _oracle_init(g, soft0.astype(np.float64), b, float(tau))
    # Step 3 starts from the binary32 rows the library stored
    F_start = F_init.copy()
    n_old = p0.n
    F_start[n_old:] = F_init[n_old:].astype(np.float32).astype(np.float64)
    o2 = ON.step3_propagate(rp, col, w, F_start, g.seed_class, A0, TOL, R_)
    assert s.iterations == o2["rounds"] == R_ and st == 1
    assert sizes.tolist() == o2["frontier_sizes"].tolist()
    assert np.max(np.abs(soft - o2["F"])) <= ROUNDS_ATOL
    np.testing.assert_allclose(deltas, o2["max_changes"], atol=1e-6)


def test_converged_update_with_supernode_initialisation_matches_exact_labels():
    p, p0 = _problem(4, 1404)
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    batches = [W.clustered_batch(p, 600, 8.0, 2, 1, 3, 10), W.clustered_batch(p, 150, 4.0, 2, 1, 3, 3)]
    with _make(p0) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        tau = np.float32(d.mean_edge_weight())
        d.set_initialiser(P.INIT_SUPERNODE, tau)
        for b in batches:  # the second, smaller batch reuses the first one's scratch
            n_old = g.n
            st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
            assert st == 0
            comp, info = d.last_components()
            g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
            ocomp, count, kept = ON.components(n_old, b.num_new_vertices, b.eu, b.ev, b.ew, float(tau))
            assert np.array_equal(comp, ocomp) and info.components == count and info.kept_edges == kept
            soft, hard = d.get_labels()
            rp, col, w = g.csr()
            exact, _, _ = ON.itlp_solve(rp, col, w, g.seed_class, g.C, tol=1e-11)
            reach = R.seed_reachable(rp, col, g.seed_class)
            assert np.max(np.abs(soft - exact)[reach]) <= O1_ATOL
            clear = reach & (R.top2_margin(exact) > 2 * O1_ATOL)
            assert np.array_equal(hard[clear], R.hard_labels(exact)[clear])


def _path_batch(n_old, k, rng, C):
    """k new vertices strung into one path in a random order of ids, strong weights; first and last
    vertex also attach to an old vertex."""
    order = rng.permutation(k) + n_old
    eu = np.concatenate([order[:-1], [order[0], order[-1]]]).astype(np.int32)
    ev = np.concatenate([order[1:], [0, 1]]).astype(np.int32)
    ew = np.concatenate([np.full(k - 1, 2.0), [0.7, 0.9]]).astype(np.float32)
    return W.Batch(k, eu, ev, ew, np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.int32))


@pytest.mark.parametrize("k", [2, 257, 3000])
def test_one_long_path_is_one_component(k):
    # many hook/jump iterations: exercises the chained loop past its first host round trip
    p0 = W.small_random(600, 3, 5.0, 60, 77)
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    b = _path_batch(p0.n, k, np.random.default_rng(k), p0.C)
    with _make(p0) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        soft0, _ = d.get_labels()
        d.set_initialiser(P.INIT_SUPERNODE, 1.0)
        d.set_params(TOL, 0)
        d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft, _ = d.get_labels()
        comp, info = d.last_components()
    rp, col, w, F_init, A0, ocomp, count, kept = _oracle_init(g, soft0.astype(np.float64), b, 1.0)
    assert count == 1 and info.components == 1 and info.kept_edges == k - 1 == kept
    assert not comp.any() and np.array_equal(comp, ocomp)
    assert info.hook_steps >= 2
    assert np.max(np.abs(soft - F_init)) <= INIT_ATOL
    assert np.ptp(soft[p0.n:], axis=0).max() == 0.0  # one supernode, one row


@pytest.mark.parametrize("tau,expect", [(1e30, "singletons"), (0.0, "all")])
def test_threshold_extremes(tau, expect):
    p, p0 = _problem(3, 1503)
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    b = W.clustered_batch(p, 400, 5.0, 2, 1, 3, 4)
    with _make(p0) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        soft0, _ = d.get_labels()
        d.set_initialiser(P.INIT_SUPERNODE, tau)
        d.set_params(TOL, 0)
        d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft, _ = d.get_labels()
        comp, info = d.last_components()
    rp, col, w, F_init, A0, ocomp, count, kept = _oracle_init(g, soft0.astype(np.float64), b, float(np.float32(tau)))
    assert np.array_equal(comp, ocomp) and info.components == count and info.kept_edges == kept
    if expect == "singletons":
        assert count == 400 and kept == 0 and comp.tolist() == list(range(400))
    else:
        internal = int(((b.eu >= p0.n) & (b.ev >= p0.n)).sum())
        assert kept == internal and count < 100
    assert np.max(np.abs(soft - F_init)) <= INIT_ATOL


def test_batches_without_new_vertices_and_uniform_mode_report_nothing():
    p, p0 = _problem(3, 1603)
    b_edges = W.small_random_batch(p, 0, 0, 0, num_extra_edges=40)
    b_vert = W.small_random_batch(p, 30, 4, 1)
    with _make(p0) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        d.set_initialiser(P.INIT_SUPERNODE, 0.5)
        assert d.apply_batch(0, b_edges.eu, b_edges.ev, b_edges.ew, None, None)[0] == 0
        comp, info = d.last_components()
        assert comp is None and info.vertices == 0 and info.components == 0
        d.set_initialiser(P.INIT_UNIFORM)
        assert d.apply_batch(b_vert.num_new_vertices, b_vert.eu, b_vert.ev, b_vert.ew, b_vert.seed_vertex,
                             b_vert.seed_class)[0] == 0
        comp, info = d.last_components()
        assert comp is None and info.vertices == 0
        with pytest.raises(P.DynLPError):
            d.set_initialiser(7, 0.5)
        with pytest.raises(P.DynLPError):
            d.set_initialiser(P.INIT_SUPERNODE, float("nan"))
        with pytest.raises(P.DynLPError):
            d.set_initialiser(P.INIT_SUPERNODE, -1.0)


def test_all_inserted_vertices_labelled_keeps_their_rows_one_hot():
    p0 = W.small_random(400, 3, 5.0, 40, 91)
    k = 20
    rng = np.random.default_rng(5)
    eu = np.arange(400, 400 + k, dtype=np.int32)
    ev = rng.integers(0, 400, size=k).astype(np.int32)
    eu = np.concatenate([eu, eu[:-1]]).astype(np.int32)
    ev = np.concatenate([ev, np.arange(401, 400 + k)]).astype(np.int32)
    ew = np.full(eu.shape[0], 0.9, dtype=np.float32)
    sv = np.arange(400, 400 + k, dtype=np.int32)
    sc = (np.arange(k) % 3).astype(np.int32)
    with _make(p0) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        d.set_initialiser(P.INIT_SUPERNODE, 0.5)
        assert d.apply_batch(k, eu, ev, ew, sv, sc)[0] == 0
        soft, hard = d.get_labels()
        comp, info = d.last_components()
    assert info.components == 1 and not comp.any()
    assert np.array_equal(soft[400:], np.eye(3, dtype=np.float32)[sc])
    assert np.array_equal(hard[400:], sc)


def test_device_pointer_mode_returns_components_on_the_device():
    import torch

    p, p0 = _problem(5, 1705)
    b = W.clustered_batch(p, 700, 6.0, 2, 1, 3, 7)
    dev = torch.device("cuda:0")
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), dtype=dt, device=dev)
    d = P.DynLP(p0.n, t(p0.row_ptr, torch.int64), t(p0.col, torch.int32), t(p0.w, torch.float32), p0.C,
                t(p0.seed_vertex, torch.int32), t(p0.seed_class, torch.int32), device_ptrs=True)
    with d:
        assert d.static_solve(TOL, 20000)[0] == 0
        tau = np.float32(d.mean_edge_weight())
        d.set_initialiser(P.INIT_SUPERNODE, tau)
        st, _ = d.apply_batch(b.num_new_vertices, t(b.eu, torch.int32), t(b.ev, torch.int32), t(b.ew, torch.float32),
                              t(b.seed_vertex, torch.int32), t(b.seed_class, torch.int32))
        assert st == 0
        comp, info = d.last_components()
        assert comp.is_cuda
        comp = comp.cpu().numpy()
    ocomp, count, kept = ON.components(p0.n, b.num_new_vertices, b.eu, b.ev, b.ew, float(tau))
    assert np.array_equal(comp, ocomp) and info.components == count and info.kept_edges == kept
