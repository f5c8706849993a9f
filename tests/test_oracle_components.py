"""Pins for the oracle's Alg. 2 Step 1 (sparsified batch-internal graph, its connected
components) and Step 2 (supernode label initialisation)."""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import connected_components as scipy_cc

import workloads as W
from oracle import native as N
from oracle import reference as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "supernode_cases.json")


def _cases():
    return json.load(open(GOLDEN))["cases"]


def _build(case):
    """Graph after the batch (old vertices have no edges among themselves in these cases)."""
    n_old, k, C = case["n_old"], case["k"], case["C"]
    g = R.Graph(n_old, np.zeros(n_old + 1, dtype=np.int64), [], [], C, [], [])
    e = np.array(case["edges"], dtype=np.float64).reshape(-1, 3)
    sv = [s[0] for s in case["seeds"]]
    sc = [s[1] for s in case["seeds"]]
    g.insert(k, e[:, 0].astype(np.int64), e[:, 1].astype(np.int64), e[:, 2], sv, sc)
    return g, e


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_hand_worked_supernode_cases(case):
    g, e = _build(case)
    n_old, k, C = case["n_old"], case["k"], case["C"]
    F0 = R.initial_labels(g.seed_class, C)
    F, comp, count, Wm = R.step2_initialise(F0, g.adjacency(), g.seed_class, n_old, k, e[:, 0].astype(int),
                                            e[:, 1].astype(int), e[:, 2], case["tau"])
    got = [sorted((n_old + np.flatnonzero(comp == c)).tolist()) for c in range(count)]
    assert got == case["components"]  # numbered by smallest member, as listed
    for u, row in case["rows"].items():
        np.testing.assert_allclose(F[int(u)], row, rtol=0, atol=1e-15)
    np.testing.assert_array_equal(F[:n_old], F0[:n_old])  # Step 2 touches inserted rows only
    # the C implementation agrees
    c2, cnt2, _ = N.components(n_old, k, e[:, 0], e[:, 1], e[:, 2], case["tau"])
    rp, col, w = g.csr()
    F2, W2 = N.supernode_init(rp, col, w, F0, g.seed_class, n_old, c2, cnt2)
    np.testing.assert_array_equal(c2, comp)
    np.testing.assert_allclose(F2, F, rtol=0, atol=1e-15)
    np.testing.assert_allclose(W2, Wm, rtol=0, atol=1e-15)


def test_two_roots_are_renumbered_densely():
    # the kernel-design section's second example: parents {0, 2} survive and are renumbered 0, 1
    comp, count = R.connected_components(4, [(0, 1), (2, 3)])
    assert count == 2 and comp.tolist() == [0, 0, 1, 1]
    comp, count = R.connected_components(5, [(4, 1), (3, 0)])  # numbering follows the smallest member
    assert count == 3 and comp.tolist() == [0, 1, 2, 0, 1]


def test_threshold_is_strict_and_only_batch_internal_edges_count():
    eu, ev, ew = [10, 10, 11, 3], [11, 12, 12, 12], [0.5, 0.500001, 0.2, 9.0]
    assert R.batch_internal_edges(10, 3, eu, ev, ew, 0.5) == [(0, 2)]
    assert R.batch_internal_edges(10, 3, eu, ev, ew, 0.1) == [(0, 1), (0, 2), (1, 2)]
    assert R.batch_internal_edges(10, 3, eu, ev, ew, 10.0) == []
    # parallel batch edges are tested one by one, not summed
    assert R.batch_internal_edges(0, 2, [0, 0], [1, 1], [0.3, 0.3], 0.5) == []


def test_mean_edge_weight():
    # undirected weights 1, 2, 6 listed in both directions
    assert R.mean_edge_weight([1, 2, 6, 1, 2, 6]) == 3.0
    assert R.mean_edge_weight([]) == 0.0


def _closure_components(k, edges):
    """Brute force from the definition: i ~ j iff j is reachable from i (boolean closure)."""
    A = np.eye(k, dtype=bool)
    for a, b in edges:
        A[a, b] = A[b, a] = True
    for _ in range(k):
        A = (A.astype(np.int64) @ A.astype(np.int64)) > 0
    first = np.array([int(np.flatnonzero(A[i])[0]) for i in range(k)])  # smallest reachable id
    roots = sorted(set(first.tolist()))
    return np.array([roots.index(f) for f in first])


@pytest.mark.parametrize("seed", range(6))
def test_components_match_brute_force_closure(seed):
    rng = np.random.default_rng(100 + seed)
    k = int(rng.integers(2, 13))
    m = int(rng.integers(0, 2 * k))
    edges = [(int(a), int(b)) for a, b in rng.integers(0, k, size=(m, 2)) if a != b]
    comp, count = R.connected_components(k, edges)
    want = _closure_components(k, edges)
    np.testing.assert_array_equal(comp, want)
    assert count == want.max() + 1


@pytest.mark.parametrize("k,m,seed", [(50, 30, 1), (400, 350, 2), (3000, 2500, 3), (3000, 9000, 4), (1, 0, 5)])
def test_components_match_the_library_routine(k, m, seed):
    rng = np.random.default_rng(seed)
    n_old = 17
    a = rng.integers(0, n_old + k, size=m)
    b = rng.integers(0, n_old + k, size=m)
    keep = a != b
    a, b = a[keep], b[keep]
    w = rng.uniform(0.0, 1.0, size=a.shape[0])
    tau = 0.4
    edges = R.batch_internal_edges(n_old, k, a, b, w, tau)
    comp, count = R.connected_components(k, edges)
    sel = (a >= n_old) & (b >= n_old) & (w > tau)
    M = sp.coo_matrix((np.ones(sel.sum()), (a[sel] - n_old, b[sel] - n_old)), shape=(k, k))
    cnt_lib, lab = scipy_cc(M, directed=False)
    assert count == cnt_lib and len(edges) == int(sel.sum())
    # same partition: the map between the two labelings is a bijection
    pairs = set(zip(comp.tolist(), lab.tolist()))
    assert len(pairs) == count
    # canonical numbering: component ids appear in ascending order of first occurrence
    firsts = [int(np.flatnonzero(comp == c)[0]) for c in range(count)]
    assert firsts == sorted(firsts)
    c2, cnt2, kept = N.components(n_old, k, a, b, w, tau)
    np.testing.assert_array_equal(c2, comp)
    assert cnt2 == count and kept == len(edges)


def test_binary_row_equals_the_printed_expression():
    rng = np.random.default_rng(7)
    for w0, w1 in rng.uniform(0.0, 5.0, size=(20, 2)).tolist() + [[0.0, 2.0], [3.0, 0.0]]:
        row = R.supernode_label([w0, w1])
        assert abs(row[1] - R.supernode_label_binary_as_printed(w0, w1)) < 1e-15
        assert abs(row[0] + row[1] - 1.0) < 1e-15
    np.testing.assert_array_equal(R.supernode_label([0.0, 0.0]), [0.5, 0.5])  # the paper's neutral value
    np.testing.assert_array_equal(R.supernode_label([0.0, 0.0, 0.0, 0.0]), [0.25] * 4)


def _clustered(seed, n=300, C=3, k=200):
    p = W.small_random(n, C, 4.0, 20, seed)
    g = R.Graph(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class)
    tau = R.mean_edge_weight(g.w)
    n_old = p.n
    b = W.clustered_batch(p, k, 6.0, 2, 1, 3, 5)
    return p, g, b, n_old, tau


@pytest.mark.parametrize("seed", [11, 12])
def test_step2_invariants_on_a_clustered_batch(seed):
    p, g, b, n_old, tau = _clustered(seed)
    rp, col, w = g.csr()
    F_before, _, _ = R.itlp_solve(rp, col, w, g.seed_class, p.C, tol=1e-12)
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    F0 = np.concatenate([F_before, np.full((b.num_new_vertices, p.C), 1.0 / p.C)])
    F0[b.seed_vertex] = np.eye(p.C)[b.seed_class]
    adj = g.adjacency()
    F, comp, count, Wm = R.step2_initialise(F0, adj, g.seed_class, n_old, b.num_new_vertices, b.eu, b.ev, b.ew, tau)
    assert 1 < count < b.num_new_vertices  # the batch really has multi-vertex components and several of them
    np.testing.assert_allclose(F.sum(axis=1), 1.0, atol=1e-12)
    np.testing.assert_array_equal(F[:n_old], F0[:n_old])
    new_unl = np.array([u for u in range(n_old, g.n) if g.seed_class[u] < 0])
    for c in range(count):
        rows = F[[u for u in new_unl if comp[u - n_old] == c]]
        if len(rows):
            assert np.ptp(rows, axis=0).max() == 0.0  # one value per supernode
    np.testing.assert_array_equal(F[b.seed_vertex], np.eye(p.C)[b.seed_class])
    # total weight conservation: sum of W = weight of all (inserted vertex -> labelled vertex) entries
    tot = sum(wuv for u in range(n_old, g.n) for v, wuv in adj[u].items() if g.seed_class[v] >= 0)
    assert abs(Wm.sum() - tot) < 1e-9
    # the C implementation agrees on the same inputs
    c2, cnt2, _ = N.components(n_old, b.num_new_vertices, b.eu, b.ev, b.ew, tau)
    rp2, col2, w2 = g.csr()
    F2, W2 = N.supernode_init(rp2, col2, w2, F0, g.seed_class, n_old, c2, cnt2)
    np.testing.assert_array_equal(c2, comp)
    np.testing.assert_allclose(F2, F, atol=1e-14)


def test_initialisation_changes_the_start_not_the_fixed_point():
    p, g, b, n_old, tau = _clustered(13)
    rp, col, w = g.csr()
    F_before, _, _ = R.itlp_solve(rp, col, w, g.seed_class, p.C, tol=1e-13)
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    F0 = np.concatenate([F_before, np.full((b.num_new_vertices, p.C), 1.0 / p.C)])
    F0[b.seed_vertex] = np.eye(p.C)[b.seed_class]
    adj = g.adjacency()
    A = R.affected_set(adj, g.seed_class, n_old, b.num_new_vertices, b.eu, b.ev, b.seed_vertex)
    F1, *_ = R.step2_initialise(F0, adj, g.seed_class, n_old, b.num_new_vertices, b.eu, b.ev, b.ew, tau)
    assert np.abs(F1 - F0).max() > 0.05
    Fa, ra, _, _ = R.step3_propagate(adj, F0, g.seed_class, A, 1e-10, 100000, decide_fp32=False)
    Fb, rb, _, _ = R.step3_propagate(adj, F1, g.seed_class, A, 1e-10, 100000, decide_fp32=False)
    rp2, col2, w2 = g.csr()
    exact = R.harmonic_closed_form(rp2, col2, w2, g.seed_class, p.C)
    reach = R.seed_reachable(rp2, col2, g.seed_class)
    assert np.abs(Fa - exact)[reach].max() < 1e-7
    assert np.abs(Fb - exact)[reach].max() < 1e-7
