"""Pins for the frontier-restricted propagation (Alg. 2 Steps 1 and 3) of the oracle."""
import numpy as np
import pytest

import workloads as W
from oracle import reference as R


def _setup(n, C, deg, ns, seed, batch_kw):
    p = W.small_random(n, C, deg, ns, seed)
    g = R.Graph(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class)
    rp, col, w = g.csr()
    F_before, _, _ = R.itlp_solve(rp, col, w, g.seed_class, C, tol=1e-13)
    n_old = p.n
    b = W.small_random_batch(p, **batch_kw)
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    F = np.concatenate([F_before, np.full((b.num_new_vertices, C), 1.0 / C)])
    s = np.asarray(b.seed_vertex, dtype=np.int64)
    F[s] = 0
    F[s, np.asarray(b.seed_class)] = 1
    return p, g, b, n_old, F


def _brute_affected(g, b, n_old):
    """V_aff straight from the sentence: inserted vertices and their neighbours; both ends of
    each new edge; neighbours of fresh seeds; never a seed or an isolated vertex."""
    nbr = {u: set() for u in range(g.n)}
    for a, c in zip(g.src.tolist(), g.dst.tolist()):
        nbr[a].add(c)
    A = set()
    for u in range(n_old, g.n):
        A |= {u} | nbr[u]
    for a, c in zip(b.eu.tolist(), b.ev.tolist()):
        A |= {a, c}
    for s in b.seed_vertex.tolist():
        A |= nbr[s]
    return sorted(u for u in A if g.seed_class[u] < 0 and nbr[u])


@pytest.mark.parametrize("kw", [dict(num_new=15, degree=3, num_new_seeds=2),
                                dict(num_new=0, degree=0, num_new_seeds=0, num_extra_edges=12, num_revealed=3),
                                dict(num_new=8, degree=2, num_new_seeds=1, num_extra_edges=5, num_revealed=2)])
def test_affected_set_python_c_and_brute_force_agree(kw, oracle_native):
    p, g, b, n_old, F = _setup(120, 3, 3.0, 8, 5, kw)
    rp, col, w = g.csr()
    A_py = R.affected_set(g.adjacency(), g.seed_class, n_old, b.num_new_vertices, b.eu, b.ev, b.seed_vertex)
    A_c = oracle_native.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex)
    brute = _brute_affected(g, b, n_old)
    assert sorted(A_py) == brute == A_c.tolist()
    assert len(brute) > 0


@pytest.mark.parametrize("tol", [1e-3, 1e-6])
def test_step3_python_sets_equal_c_rounds(tol, oracle_native):
    p, g, b, n_old, F = _setup(150, 3, 3.5, 10, 9, dict(num_new=12, degree=3, num_new_seeds=1, num_extra_edges=6,
                                                        num_revealed=2))
    rp, col, w = g.csr()
    adj = g.adjacency()
    A0 = R.affected_set(adj, g.seed_class, n_old, b.num_new_vertices, b.eu, b.ev, b.seed_vertex)
    Fp, rounds, sizes, changes = R.step3_propagate(adj, F, g.seed_class, A0, tol, 10_000)
    out = oracle_native.step3_propagate(rp, col, w, F, g.seed_class, sorted(A0), tol, 10_000)
    assert rounds == out["rounds"] and sizes == out["frontier_sizes"].tolist()
    assert out["remaining"] == 0
    assert np.max(np.abs(Fp - out["F"])) < 1e-13
    np.testing.assert_allclose(changes, out["max_changes"], atol=1e-7)
    assert out["rows_updated"] == sum(sizes)
    # seeds never move, rows stay stochastic
    s = g.seed_class >= 0
    assert np.array_equal(out["F"][s], F[s])
    assert np.max(np.abs(out["F"].sum(1) - 1)) < 1e-12


def test_step3_first_round_over_all_unlabelled_is_one_itlp_sweep(oracle_native):
    p, g, b, n_old, F = _setup(100, 4, 3.0, 7, 13, dict(num_new=10, degree=3, num_new_seeds=1))
    rp, col, w = g.csr()
    everyone = [u for u in range(g.n) if g.seed_class[u] < 0 and rp[u + 1] > rp[u]]
    out = oracle_native.step3_propagate(rp, col, w, F, g.seed_class, everyone, 1e-6, 1)
    sweep = R.itlp_sweep(rp, col, w, F, g.seed_class)
    assert out["rounds"] == 1 and np.max(np.abs(out["F"] - sweep)) < 1e-14


def test_step3_with_vanishing_threshold_reaches_the_harmonic_solution(oracle_native):
    """delta -> 0: the locally stopped iteration converges to the exact labels of the updated
    graph, i.e. the from-scratch recomputation (Alg. 1)."""
    p, g, b, n_old, F = _setup(200, 3, 4.0, 12, 17, dict(num_new=20, degree=3, num_new_seeds=2, num_extra_edges=8,
                                                         num_revealed=2))
    rp, col, w = g.csr()
    A0 = oracle_native.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex)
    out = oracle_native.step3_propagate(rp, col, w, F, g.seed_class, A0, 1e-13, 1_000_000, decide_fp32=False)
    exact, _, _ = R.recompute_from_scratch(g, tol=1e-14)
    reach = R.seed_reachable(rp, col, g.seed_class)
    assert out["remaining"] == 0
    assert np.max(np.abs(out["F"] - exact)[reach]) < 1e-9


def test_step3_error_grows_with_threshold_and_stays_near_it(oracle_native):
    """The locally stopped answer differs from the exact one by an amount governed by delta:
    monotone in delta and bounded by (expected hitting time of the seed set) x delta."""
    p, g, b, n_old, F = _setup(400, 3, 5.0, 40, 19, dict(num_new=40, degree=4, num_new_seeds=3))
    rp, col, w = g.csr()
    A0 = oracle_native.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex)
    exact, _, _ = R.recompute_from_scratch(g, tol=1e-14)
    reach = R.seed_reachable(rp, col, g.seed_class)
    # ||(I - P_UU)^{-1}||_inf = max expected number of steps to reach a seed
    n = g.n
    Wm = np.zeros((n, n))
    np.add.at(Wm, (np.repeat(np.arange(n), np.diff(rp)), col), w)
    U = np.flatnonzero((g.seed_class < 0) & reach & (Wm.sum(1) > 0))
    P = Wm[np.ix_(U, U)] / Wm[U].sum(1, keepdims=True)
    hit = np.linalg.solve(np.eye(U.size) - P, np.ones(U.size)).max()
    errs = []
    for tol in (1e-3, 1e-5, 1e-7):
        out = oracle_native.step3_propagate(rp, col, w, F, g.seed_class, A0, tol, 1_000_000, decide_fp32=False)
        err = np.max(np.abs(out["F"] - exact)[reach])
        errs.append(err)
        # residual of a dropped row can pile up over a few sub-threshold moves of its
        # neighbours; a factor 4 on the first-order bound covers it on this graph
        assert err <= 4 * hit * tol
    assert errs[0] >= errs[1] >= errs[2]


def test_step3_respects_max_iter(oracle_native):
    p, g, b, n_old, F = _setup(100, 2, 3.0, 5, 23, dict(num_new=10, degree=3, num_new_seeds=1))
    rp, col, w = g.csr()
    A0 = oracle_native.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex)
    out = oracle_native.step3_propagate(rp, col, w, F, g.seed_class, A0, 1e-9, 3)
    assert out["rounds"] == 3 and out["remaining"] > 0


# ---- hand-worked rounds (tests/golden/step3_rounds.json) ---------------------------------------
import json
import os
from fractions import Fraction

_ROUNDS = os.path.join(os.path.dirname(__file__), "golden", "step3_rounds.json")


def _fr(xs):
    return np.array([float(Fraction(x)) for x in xs], dtype=np.float64)


def _rows(f):
    return np.stack([1.0 - f, f], axis=1)


def _golden_setup(case):
    e = np.array(case["edges"], dtype=np.float64).reshape(-1, 3)
    rp, col, w = W.edges_to_csr(case["n_old"], e[:, 0].astype(np.int64), e[:, 1].astype(np.int64), e[:, 2])
    g = R.Graph(case["n_old"], rp, col, w, case["C"], [s[0] for s in case["seeds"]], [s[1] for s in case["seeds"]])
    # the listed start is the exact labelling of the graph before the batch
    exact = R.harmonic_closed_form(rp, col, w, g.seed_class, case["C"])
    np.testing.assert_allclose(exact, _rows(_fr(case["start"])), atol=1e-13)
    b = case["batch"]
    be = np.array(b["edges"], dtype=np.float64).reshape(-1, 3)
    eu, ev, ew = be[:, 0].astype(np.int64), be[:, 1].astype(np.int64), be[:, 2]
    sv = np.array([s[0] for s in b["seeds"]], dtype=np.int64)
    sc = np.array([s[1] for s in b["seeds"]], dtype=np.int64)
    g.insert(b["num_new_vertices"], eu, ev, ew, sv, sc)
    F = np.concatenate([exact, np.full((b["num_new_vertices"], case["C"]), 1.0 / case["C"])])
    F[sv] = 0
    F[sv, sc] = 1
    return g, F, eu, ev, sv


@pytest.mark.parametrize("case", json.load(open(_ROUNDS))["cases"], ids=lambda c: c["name"])
@pytest.mark.parametrize("decide_fp32", [False, True])
def test_hand_worked_rounds(case, decide_fp32, oracle_native):
    """V_aff, the rows that moved and all labels after every round, for both statements of Step 3."""
    g, F0, eu, ev, sv = _golden_setup(case)
    delta = float(Fraction(case["delta"]))
    adj = g.adjacency()
    rp, col, w = g.csr()
    A0 = R.affected_set(adj, g.seed_class, case["n_old"], case["batch"]["num_new_vertices"], eu, ev, sv)
    A0c = oracle_native.affected_set(rp, col, g.seed_class, case["n_old"], eu, ev, sv)
    assert sorted(A0) == case["affected"] == A0c.tolist()
    trace = []
    F, rounds, sizes, changes = R.step3_propagate(adj, F0, g.seed_class, A0, delta, 1000, decide_fp32=decide_fp32,
                                                  trace=trace)
    want = case["rounds"]
    assert rounds == len(want) and sizes == [len(r["V_aff"]) for r in want]
    for t, (r, (A, moved, Ft)) in enumerate(zip(want, trace)):
        assert A == r["V_aff"] and moved == r["moved"], f"round {t + 1}"
        np.testing.assert_allclose(Ft, _rows(_fr(r["f"])), atol=1e-14, err_msg=f"round {t + 1}")
    # the C loop, stopped after t rounds for every t: same labels, same |V_aff| per round, and the size of the
    # V_aff that remains is that of the next listed round
    for t in range(1, len(want) + 1):
        out = oracle_native.step3_propagate(rp, col, w, F0, g.seed_class, A0c, delta, t, decide_fp32=decide_fp32)
        assert out["rounds"] == t
        assert out["frontier_sizes"].tolist() == [len(r["V_aff"]) for r in want[:t]]
        np.testing.assert_allclose(out["F"], _rows(_fr(want[t - 1]["f"])), atol=1e-14)
        assert out["remaining"] == (len(want[t]["V_aff"]) if t < len(want) else 0)
        assert out["rows_updated"] == sum(len(r["V_aff"]) for r in want[:t])
    out = oracle_native.step3_propagate(rp, col, w, F0, g.seed_class, A0c, delta, 1000, decide_fp32=decide_fp32)
    assert out["rounds"] == len(want) and out["remaining"] == 0


@pytest.mark.parametrize("kw", [dict(num_new=25, degree=4, num_new_seeds=2),
                                dict(num_new=0, degree=0, num_new_seeds=0, num_extra_edges=40, num_revealed=3),
                                dict(num_new=10, degree=3, num_new_seeds=1, num_extra_edges=30, num_revealed=2)])
def test_csr_with_batch_is_the_graph_update_of_the_oracle(kw):
    """workloads.csr_with_batch builds the updated CSR the full-size GPU tests hand to the oracle; it must be
    the same graph as the oracle's own update (Alg. 1 Step 1): per row the same multiset of (neighbour, weight),
    parallel edges kept as separate entries."""
    p = W.small_random(160, 3, 4.0, 9, 31)
    n_old = p.n  # the batch generator advances p.n
    b = W.small_random_batch(p, **kw)
    # make sure parallel edges occur: repeat some batch edges, and re-insert an edge the base graph already has
    dup = slice(0, min(5, b.num_edges))
    u0 = int(np.flatnonzero(np.diff(p.row_ptr) > 0)[0])
    eu = np.concatenate([b.eu, b.eu[dup], [u0]]).astype(b.eu.dtype)
    ev = np.concatenate([b.ev, b.ev[dup], [p.col[p.row_ptr[u0]]]]).astype(b.ev.dtype)
    ew = np.concatenate([b.ew, b.ew[dup] * np.float32(0.5), [np.float32(0.25)]]).astype(b.ew.dtype)
    b2 = W.Batch(num_new_vertices=b.num_new_vertices, eu=eu, ev=ev, ew=ew, seed_vertex=b.seed_vertex, seed_class=b.seed_class)
    g = R.Graph(n_old, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class)
    g.insert(b2.num_new_vertices, b2.eu, b2.ev, b2.ew, b2.seed_vertex, b2.seed_class)
    rp_o, col_o, w_o = g.csr()
    rp_w, col_w, w_w = W.csr_with_batch(n_old, p.row_ptr, p.col, p.w, b2)
    assert rp_w.tolist() == rp_o.tolist() and rp_w[-1] == p.col.shape[0] + 2 * b2.num_edges
    for u in range(g.n):
        a = sorted(zip(col_o[rp_o[u]:rp_o[u + 1]].tolist(), np.asarray(w_o[rp_o[u]:rp_o[u + 1]], dtype=np.float64).tolist()))
        c = sorted(zip(col_w[rp_w[u]:rp_w[u + 1]].tolist(), np.asarray(w_w[rp_w[u]:rp_w[u + 1]], dtype=np.float64).tolist()))
        assert a == c, u
    # at least one row really holds a parallel edge
    assert any(len(set(col_o[rp_o[u]:rp_o[u + 1]].tolist())) < rp_o[u + 1] - rp_o[u] for u in range(g.n))
