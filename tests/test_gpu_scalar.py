"""GPU parity of the binary scalar layout (C = 2 kept as one float per vertex, the paper's own
setting: F_u in [0,1], seeds 0 / 1, neutral 0.5, hard label by the 0.5 cut-off) against the
two-column oracle: column 1 of the oracle's rows is the scalar, column 0 its complement."""
import numpy as np
import pytest

import workloads as W
from oracle import native as ON
from oracle import reference as R
import paper_2604_06596_amd as P

pytestmark = pytest.mark.gpu

TOL = 1e-6
SWEEP_ATOL = 1e-6
ROUNDS_ATOL = 5e-6
O1_ATOL = 1e-4


def _make(p, **kw):
    return P.DynLP(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class, binary_scalar=True, **kw)


def _problem(kind, seed):
    if kind == "random":
        return W.small_random(6000, 2, 8.0, 300, seed)
    if kind == "sbm":
        return W.sbm(30000, 2, 20.0, 8.0, 0.01, seed)
    return W.chung_lu(20000, 2, 12.0, 2.1, 3000, 0.8, 0.02, seed)


def test_scalar_layout_needs_two_classes():
    p = W.small_random(100, 3, 4.0, 10, 1)
    with pytest.raises(P.DynLPError) as ei:
        _make(p)
    assert "binary_scalar" in ei.value.message


@pytest.mark.parametrize("kind", ["random", "sbm", "hub"])
def test_one_sweep_and_static_solve(kind):
    p = _problem(kind, 3100)
    g = R.Graph(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class)
    rp, col, w = g.csr()
    with _make(p) as d:
        soft, hard = d.get_labels()
        F0 = R.initial_labels(g.seed_class, 2)
        assert np.array_equal(soft, F0.astype(np.float32))  # seeds (1,0) / (0,1), others (0.5, 0.5)
        st, s = d.static_solve(0.0, 1)
        soft1, _ = d.get_labels()
        F1, _ = ON.itlp_sweep(rp, col, w, F0, g.seed_class)
        assert np.max(np.abs(soft1 - F1)) <= SWEEP_ATOL
        st, s = d.static_solve(TOL, 20000)
        assert st == 0
        soft, hard = d.get_labels()
        with P.DynLP(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class) as d2:  # two stored columns
            assert d2.static_solve(TOL, 20000)[0] == 0
            soft2, hard2 = d2.get_labels()
    exact, _, _ = ON.itlp_solve(rp, col, w, g.seed_class, 2, tol=1e-12, max_iter=5_000_000)
    reach = R.seed_reachable(rp, col, g.seed_class)
    assert np.max(np.abs(soft - exact)[reach]) <= O1_ATOL
    assert np.max(np.abs(soft - soft2)) <= 5e-6
    assert np.array_equal(soft[:, 0], np.float32(1.0) - soft[:, 1])
    assert np.array_equal(hard, (soft[:, 1] > 0.5).astype(np.int32))
    clear = reach & (R.top2_margin(exact) > 2 * O1_ATOL)
    assert np.array_equal(hard[clear], R.hard_labels(exact)[clear])
    s_idx = np.flatnonzero(g.seed_class >= 0)
    assert np.array_equal(soft[s_idx], R.initial_labels(g.seed_class, 2)[s_idx].astype(np.float32))


@pytest.mark.parametrize("kind", ["random", "sbm", "hub"])
@pytest.mark.parametrize("R_", [1, 3, 25])
def test_first_rounds_of_a_mixed_batch_match_the_oracle(kind, R_):
    p, p0 = _problem(kind, 3200), _problem(kind, 3200)
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    if kind == "random":
        b = W.small_random_batch(p, 250, 7, 5, num_extra_edges=60, num_revealed=3)
    elif kind == "sbm":
        b = W.sbm_vertex_batch(p, 300, 20, 0.01)
    else:
        b = W.chung_lu_vertex_batch(p, 200, 0.02)
    dead = np.random.default_rng(5).choice(p0.n, size=30, replace=False).astype(np.int32)
    with _make(p0) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        soft0, _ = d.get_labels()
        d.set_params(TOL, R_)
        st, s = d.apply_update(dead, b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft, _ = d.get_labels()
        sizes, deltas = d.round_log()
    n_old = g.n
    rp0, col0, _ = g.csr()
    dn = np.concatenate([col0[rp0[u]:rp0[u + 1]] for u in dead])
    g.delete(dead)
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    rp, col, w = g.csr()
    A0 = ON.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex, deleted_neighbours=dn)
    F = np.concatenate([soft0.astype(np.float64), np.full((b.num_new_vertices, 2), 0.5)])
    F[dead] = 0.5
    F[b.seed_vertex] = np.eye(2)[b.seed_class]
    o2 = ON.step3_propagate(rp, col, w, F, g.seed_class, A0, TOL, R_)
    assert s.frontier_initial == len(A0) and s.iterations == o2["rounds"] == R_
    assert sizes.tolist() == o2["frontier_sizes"].tolist()
    assert np.max(np.abs(soft - o2["F"])) <= ROUNDS_ATOL
    np.testing.assert_allclose(deltas, o2["max_changes"], atol=1e-6)


@pytest.mark.parametrize("mode", [P.UPDATE_SYNCHRONOUS, P.UPDATE_IN_PLACE], ids=["synchronous", "in_place"])
def test_supernode_initialisation_and_convergence_in_the_scalar_layout(mode):
    p, p0 = _problem("random", 3300), _problem("random", 3300)
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    b = W.clustered_batch(p, 700, 6.0, 2, 1, 3, 10)
    out = {}
    for max_iter in (0, 20000):  # 0: read the Step-2 rows back; 20000: run to convergence
        with _make(p0) as d:
            d.set_update_mode(mode)
            assert d.static_solve(TOL, 20000)[0] == 0
            soft0, _ = d.get_labels()
            tau = np.float32(d.mean_edge_weight())
            d.set_initialiser(P.INIT_SUPERNODE, tau)
            d.set_params(TOL, max_iter)
            st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
            out[max_iter] = (st, d.get_labels(), d.last_components(), soft0)
    n_old = g.n
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    rp, col, w = g.csr()
    ocomp, count, kept = ON.components(n_old, b.num_new_vertices, b.eu, b.ev, b.ew, float(tau))
    st0, (init_rows, _), (comp, info), soft0 = out[0]  # the labels that context held before the batch
    F = np.concatenate([soft0.astype(np.float64), np.full((b.num_new_vertices, 2), 0.5)])
    F[b.seed_vertex] = np.eye(2)[b.seed_class]
    F_init, _ = ON.supernode_init(rp, col, w, F, g.seed_class, n_old, ocomp, count)
    assert np.array_equal(comp, ocomp) and info.components == count
    assert np.max(np.abs(init_rows - F_init)) <= 1e-6
    assert np.abs(F_init[n_old:, 1] - 0.5).max() > 0.4  # the initialisation moved rows
    st1, (soft, hard), _, _ = out[20000]
    assert st1 == 0
    exact, _, _ = ON.itlp_solve(rp, col, w, g.seed_class, 2, tol=1e-12, max_iter=5_000_000)
    reach = R.seed_reachable(rp, col, g.seed_class)
    assert np.max(np.abs(soft - exact)[reach]) <= O1_ATOL
    clear = reach & (R.top2_margin(exact) > 2 * O1_ATOL)
    assert np.array_equal(hard[clear], R.hard_labels(exact)[clear])
