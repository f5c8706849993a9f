"""GPU parity of the binned rounds (scalar labels; rounds over nearly all vertices run as a scatter pass
into bins of receivers plus a gather pass per bin, with fixed-point accumulation) against the oracle's
synchronous Step 3, against the library's ordinary rounds, and against the exact labels.

``binned_rounds=8`` forces the binned passes with 256 receivers per bin, so that graphs of a few thousand
vertices already span tens of bins and a ragged last one."""
import numpy as np
import pytest

import certify as Cf
import workloads as W
from oracle import native as ON
from oracle import reference as R
import paper_2604_06596_amd as P

pytestmark = pytest.mark.gpu

TOL = 1e-6
ROUNDS_ATOL = 5e-6
O1_ATOL = 1e-4


def _make(p, **kw):
    return P.DynLP(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class, binary_scalar=True, **kw)


def _case(kind, seed):
    """(problem for the batch generator, pristine copy, batch, vertices to delete)"""
    if kind == "random":
        mk = lambda: W.small_random(6007, 2, 8.0, 300, seed)
        p, p0 = mk(), mk()
        b = W.small_random_batch(p, 600, 7, 12, num_extra_edges=60, num_revealed=3)
    else:  # heavy-tailed degrees: hub receivers take thousands of additions into one accumulator
        mk = lambda: W.chung_lu(20000, 2, 12.0, 2.1, 3000, 0.8, 0.02, seed)
        p, p0 = mk(), mk()
        b = W.chung_lu_vertex_batch(p, 2000, 0.02)
    dead = np.random.default_rng(seed).choice(p0.n, size=40, replace=False).astype(np.int32)
    return p0, b, dead


def _oracle_after(p0, b, dead, soft0):
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    n_old = g.n
    rp0, col0, _ = g.csr()
    dn = np.concatenate([col0[rp0[u]:rp0[u + 1]] for u in dead]) if len(dead) else np.zeros(0, np.int32)
    g.delete(dead)
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    rp, col, w = g.csr()
    A0 = ON.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex, deleted_neighbours=dn)
    F = np.concatenate([soft0.astype(np.float64), np.full((b.num_new_vertices, 2), 0.5)])
    F[dead] = 0.5
    F[b.seed_vertex] = np.eye(2)[b.seed_class]
    return g, rp, col, w, F, A0


def _run(p0, b, dead, max_iter, binned, mode=P.UPDATE_SYNCHRONOUS, tol=TOL):
    with _make(p0, binned_rounds=binned) as d:
        d.set_update_mode(mode)
        assert d.static_solve(TOL, 20000)[0] == 0
        soft0, _ = d.get_labels()
        d.set_params(tol, max_iter)
        st, s = d.apply_update(dead, b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft, hard = d.get_labels()
        sizes, deltas = d.round_log()
        kinds = [int(r.staged) for r in d.round_log_full()]
    return dict(st=st, s=s, soft0=soft0, soft=soft, hard=hard, sizes=sizes, deltas=deltas, kinds=kinds)


@pytest.mark.parametrize("kind", ["random", "hub"])
@pytest.mark.parametrize("R_", [12, 40])
def test_binned_rounds_match_the_oracle_round_by_round(kind, R_):
    p0, b, dead = _case(kind, 5100)
    out = _run(p0, b, dead, R_, 8)
    g, rp, col, w, F, A0 = _oracle_after(p0, b, dead, out["soft0"])
    o2 = ON.step3_propagate(rp, col, w, F, g.seed_class, A0, TOL, R_)
    print("round kinds", out["kinds"], "sizes", out["sizes"].tolist())
    assert 3 in out["kinds"], "the case is meant to reach binned rounds"
    assert out["s"].frontier_initial == len(A0) and out["s"].iterations == o2["rounds"] == R_
    assert out["sizes"].tolist() == o2["frontier_sizes"].tolist()
    assert np.max(np.abs(out["soft"] - o2["F"])) <= ROUNDS_ATOL
    np.testing.assert_allclose(out["deltas"], o2["max_changes"], atol=1e-6)
    assert out["s"].rows_updated == o2["rows_updated"] and out["s"].edges_traversed == o2["edges_traversed"]
    # the scalar is a probability and its complement is derived from it
    assert out["soft"].min() >= 0 and out["soft"].max() <= 1
    assert np.array_equal(out["soft"][:, 0], np.float32(1.0) - out["soft"][:, 1])


@pytest.mark.parametrize("kind", ["random", "hub"])
def test_binned_rounds_against_ordinary_rounds_and_twice_the_same(kind):
    """Synchronous mode: binned rounds follow the same V_aff as the ordinary rounds and give the same labels to
    rounding; two runs give identical bits (integer accumulation does not depend on the order of the atomics or
    on where the build step placed an entry)."""
    p0, b, dead = _case(kind, 5200)
    a = _run(p0, b, dead, 60, 8)
    a2 = _run(p0, b, dead, 60, 8)
    c = _run(p0, b, dead, 60, -1)
    assert 3 in a["kinds"] and 3 not in c["kinds"]
    assert np.array_equal(a["soft"], a2["soft"]) and a["sizes"].tolist() == a2["sizes"].tolist()
    assert a["sizes"].tolist() == c["sizes"].tolist()
    # the two contexts also ran their cold starts differently (binned sweeps / ordinary sweeps), each to tol: two
    # label matrices of one graph, each within its own residual certificate of the exact labels
    g, rp, col, w, F, A0 = _oracle_after(p0, b, dead, a["soft0"])
    Cf.check_two_runs(a["soft"], Cf.certificate(rp, col, w, g.seed_class, a["soft"]), c["soft"],
                      Cf.certificate(rp, col, w, g.seed_class, c["soft"]), "binned vs ordinary rounds")


@pytest.mark.parametrize("mode", [P.UPDATE_SYNCHRONOUS, P.UPDATE_IN_PLACE], ids=["synchronous", "in_place"])
@pytest.mark.parametrize("kind", ["random", "hub"])
def test_binned_rounds_converge_to_the_exact_labels(kind, mode):
    p0, b, dead = _case(kind, 5300)
    out = _run(p0, b, dead, 20000, 8, mode=mode)
    g, rp, col, w, F, A0 = _oracle_after(p0, b, dead, out["soft0"])
    assert out["st"] == 0 and 3 in out["kinds"]
    exact, _, _ = ON.itlp_solve(rp, col, w, g.seed_class, 2, tol=1e-12, max_iter=5_000_000)
    reach = R.seed_reachable(rp, col, g.seed_class)
    assert np.max(np.abs(out["soft"] - exact)[reach]) <= O1_ATOL
    clear = reach & (R.top2_margin(exact) > 2 * O1_ATOL)
    assert np.array_equal(out["hard"][clear], R.hard_labels(exact)[clear])
    s_idx = np.flatnonzero(g.seed_class >= 0)
    assert np.array_equal(out["soft"][s_idx], R.initial_labels(g.seed_class, 2)[s_idx].astype(np.float32))


def _many_bins_case():
    mk = lambda: W.small_random(600_001, 2, 4.0, 6000, 5400)
    p, p0 = mk(), mk()
    b = W.small_random_batch(p, 60_000, 7, 600, num_extra_edges=3000, num_revealed=30)
    return p0, b, np.zeros(0, dtype=np.int32)


def test_many_bins_match_the_oracle_round_by_round():
    """660,001 vertices in bins of 256 receivers: 2,579 bins (the scatter pass's per-bin tables in their wide
    instantiation, for more than 2,048 bins) and about 180 chunks of entries; synchronous mode, 10 rounds."""
    p0, b, dead = _many_bins_case()
    R_ = 10
    out = _run(p0, b, dead, R_, 8)
    g, rp, col, w, F, A0 = _oracle_after(p0, b, dead, out["soft0"])
    o2 = ON.step3_propagate(rp, col, w, F, g.seed_class, A0, TOL, R_)
    print("round kinds", out["kinds"], "sizes", out["sizes"].tolist())
    assert out["kinds"].count(3) >= R_ - 2, "the case is meant to run binned rounds"
    assert out["s"].frontier_initial == len(A0) and out["s"].iterations == o2["rounds"] == R_
    assert out["sizes"].tolist() == o2["frontier_sizes"].tolist()
    assert np.max(np.abs(out["soft"] - o2["F"])) <= ROUNDS_ATOL
    np.testing.assert_allclose(out["deltas"], o2["max_changes"], atol=1e-6)
    assert out["s"].rows_updated == o2["rows_updated"] and out["s"].edges_traversed == o2["edges_traversed"]


def test_many_bins_in_place_rounds_of_several_ranges_reach_the_exact_labels():
    """The same graph in the in-place mode: more bins than compute units, so a binned round goes through the graph in
    several ranges, each reading what the ranges before it published in the same round.  Converged labels against
    the exact ones (row-wise residual certificate), and fewer rounds than the synchronous run needs."""
    p0, b, dead = _many_bins_case()
    out = _run(p0, b, dead, 20000, 8, mode=P.UPDATE_IN_PLACE)
    sync = _run(p0, b, dead, 20000, 8, mode=P.UPDATE_SYNCHRONOUS)
    g, rp, col, w, F, A0 = _oracle_after(p0, b, dead, out["soft0"])
    assert out["st"] == 0 and sync["st"] == 0 and 3 in out["kinds"] and 3 in sync["kinds"]
    exact, exact_moved = Cf.exact_labels(rp, col, w, g.seed_class, 2)
    for name, o in (("in-place", out), ("synchronous", sync)):
        cert = Cf.certificate(rp, col, w, g.seed_class, o["soft"])
        err = Cf.check_against_exact(o["soft"], exact, exact_moved, cert, f"many bins, {name}")
        Cf.check_hard(o["hard"], exact, cert)
        assert cert.res <= Cf.local_stop_residual(TOL, o["s"].iterations, Cf.stop_rule_residual(TOL))
        print(f"{name}: {o['s'].iterations} rounds ({o['kinds'].count(3)} binned), err vs exact {err:.2e}")
    assert out["s"].iterations < sync["s"].iterations


@pytest.mark.parametrize("n,deg,new", [(3, 1.0, 1), (50, 3.0, 5), (257, 4.0, 40), (700, 2.2, 300)])
def test_binned_rounds_on_tiny_and_ragged_graphs(n, deg, new):
    """One bin or a few, a last bin that is mostly empty, rows of one entry, vertices without edges: the binned
    rounds must follow the ordinary rounds' V_aff exactly and end at the same labels."""
    mk = lambda: W.small_random(n, 2, deg, max(2, n // 10), 600 + n, connected=(n != 700))
    p, p0 = mk(), mk()
    b = W.small_random_batch(p, new, 2, 1 if new > 1 else 0)
    none = np.zeros(0, np.int32)
    a = _run(p0, b, none, 20000, 8)
    c = _run(p0, b, none, 20000, -1)
    print("kinds", a["kinds"][:12], "sizes", a["sizes"][:12].tolist())
    assert a["st"] == 0 and c["st"] == 0
    assert a["s"].frontier_initial == c["s"].frontier_initial
    k = min(len(a["sizes"]), len(c["sizes"]), 10)
    assert a["sizes"][:k].tolist() == c["sizes"][:k].tolist()
    g, rp, col, w, F, A0 = _oracle_after(p0, b, none, a["soft0"])
    Cf.check_two_runs(a["soft"], Cf.certificate(rp, col, w, g.seed_class, a["soft"]), c["soft"],
                      Cf.certificate(rp, col, w, g.seed_class, c["soft"]), "binned vs ordinary rounds, converged")
    exact, _, _ = ON.itlp_solve(rp, col, w, g.seed_class, 2, tol=1e-12, max_iter=5_000_000)
    reach = R.seed_reachable(rp, col, g.seed_class)
    assert np.max(np.abs(a["soft"] - exact)[reach]) <= O1_ATOL


def test_binned_rounds_across_long_runs_of_vertices_without_entries():
    """Two islands of 400 vertices at the two ends of 180,000 vertex ids, nothing in between: one chunk of entries
    spans far more than 65,535 rows, so the scatter pass cannot address its senders by 16-bit offsets from the chunk's
    first row and reads the 32-bit rows instead.  Round by round against the oracle, then to convergence."""
    rng = np.random.default_rng(5500)
    n, k = 180_000, 400
    isl = [np.arange(k), np.arange(n - k, n)]
    eu, ev = [], []
    for ids in isl:
        a, b = rng.integers(0, k, 1400), rng.integers(0, k, 1400)
        path = rng.permutation(k)
        eu += [ids[a], ids[path[:-1]]]
        ev += [ids[b], ids[path[1:]]]
    eu.append(isl[0][rng.integers(0, k, 6)])
    ev.append(isl[1][rng.integers(0, k, 6)])
    eu, ev = np.concatenate(eu), np.concatenate(ev)
    keep = eu != ev
    key = np.unique(np.minimum(eu, ev)[keep] * n + np.maximum(eu, ev)[keep])
    lo, hi = key // n, key % n
    ew = rng.uniform(0.1, 1.0, lo.shape[0]).astype(np.float32)
    rp, col, w = W.edges_to_csr(n, lo, hi, ew)
    sv = np.sort(np.concatenate([rng.choice(isl[0], 20, replace=False), rng.choice(isl[1], 20, replace=False)])).astype(np.int32)
    sc = (sv >= n // 2).astype(np.int32)
    p0 = W.Problem(n, 2, rp, col, w, sv, sc, np.zeros(n, np.int32))
    new = 60
    bu = np.repeat(np.arange(n, n + new), 4)
    bv = np.concatenate([rng.choice(np.concatenate(isl), 4, replace=False) for _ in range(new)])
    b = W.Batch(new, bu.astype(np.int32), bv.astype(np.int32), rng.uniform(0.1, 1.0, bu.shape[0]).astype(np.float32),
                np.zeros(0, np.int32), np.zeros(0, np.int32))
    none = np.zeros(0, np.int32)
    R_ = 12
    out = _run(p0, b, none, R_, 8)
    g, rp2, col2, w2, F, A0 = _oracle_after(p0, b, none, out["soft0"])
    o2 = ON.step3_propagate(rp2, col2, w2, F, g.seed_class, A0, TOL, R_)
    print("round kinds", out["kinds"], "sizes", out["sizes"].tolist())
    assert 3 in out["kinds"], "the case is meant to reach binned rounds"
    assert out["s"].iterations == o2["rounds"] == R_ and out["sizes"].tolist() == o2["frontier_sizes"].tolist()
    assert np.max(np.abs(out["soft"] - o2["F"])) <= ROUNDS_ATOL
    assert out["s"].rows_updated == o2["rows_updated"] and out["s"].edges_traversed == o2["edges_traversed"]
    full = _run(p0, b, none, 20000, 8)
    assert full["st"] == 0
    exact, _, _ = ON.itlp_solve(rp2, col2, w2, g.seed_class, 2, tol=1e-12, max_iter=5_000_000)
    reach = R.seed_reachable(rp2, col2, g.seed_class)
    cert = Cf.certificate(rp2, col2, w2, g.seed_class, full["soft"])
    Cf.check_against_exact(full["soft"], exact, 1e-12, cert, "islands, converged")
    assert np.all(full["soft"][~reach] == np.float32(0.5))


@pytest.mark.parametrize("kind", ["random", "hub"])
def test_static_solve_with_binned_sweeps(kind):
    """The cold start on scalar labels: every sweep after the first is a binned round over all updatable vertices.
    A fixed number of sweeps equals the same number of oracle sweeps (Eq. (1), Jacobi); run to the stop rule it ends
    at the exact labels, like the ordinary sweeps."""
    p0, _, _ = _case(kind, 5400)
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    rp, col, w = g.csr()
    with _make(p0, binned_rounds=8) as d:
        st, s = d.static_solve(0.0, 9)
        soft9, _ = d.get_labels()
        kinds9 = [int(r.staged) for r in d.round_log_full()]
        sizes9, deltas9 = d.round_log()
    F = R.initial_labels(g.seed_class, 2)
    changes = []
    for _ in range(9):
        F, ch = ON.itlp_sweep(rp, col, w, F, g.seed_class)
        changes.append(ch)
    assert st == 1 and s.iterations == 9 and kinds9 == [0] + [3] * 8
    assert np.max(np.abs(soft9 - F)) <= ROUNDS_ATOL
    np.testing.assert_allclose(deltas9, np.array(changes), atol=1e-6)
    updatable = int(np.count_nonzero((g.seed_class < 0) & (np.diff(rp) > 0)))
    assert sizes9.tolist() == [updatable] * 9
    for mode in (P.UPDATE_SYNCHRONOUS, P.UPDATE_IN_PLACE):
        with _make(p0, binned_rounds=8) as d:
            d.set_update_mode(mode)
            st, s = d.static_solve(TOL, 20000)
            soft, hard = d.get_labels()
            assert st == 0 and s.converged == 1 and 3 in [int(r.staged) for r in d.round_log_full()]
            assert s.final_max_delta <= TOL
        exact, _, _ = ON.itlp_solve(rp, col, w, g.seed_class, 2, tol=1e-12, max_iter=5_000_000)
        reach = R.seed_reachable(rp, col, g.seed_class)
        assert np.max(np.abs(soft - exact)[reach]) <= O1_ATOL
        clear = reach & (R.top2_margin(exact) > 2 * O1_ATOL)
        assert np.array_equal(hard[clear], R.hard_labels(exact)[clear])


def test_binned_rounds_need_the_scalar_layout_and_a_valid_bin_size():
    p = W.small_random(500, 2, 6.0, 30, 7)
    with pytest.raises(P.DynLPError) as ei:
        _make(p, binned_rounds=5)
    assert "binned_rounds" in ei.value.message
    # with n x C rows the option is accepted and ignored
    p3 = W.small_random(3000, 3, 8.0, 150, 8)
    p3b = W.small_random(3000, 3, 8.0, 150, 8)
    b = W.small_random_batch(p3, 300, 7, 5)
    with P.DynLP(p3b.n, p3b.row_ptr, p3b.col, p3b.w, p3b.C, p3b.seed_vertex, p3b.seed_class, binned_rounds=8) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        assert st == 0 and 3 not in [int(r.staged) for r in d.round_log_full()]
