"""Pins for vertex deletions in the oracle (Alg. 2 Step 1 for Delta^Del, then Step 3)."""
import json
import os

import numpy as np
import pytest

import workloads as W
from oracle import native as N
from oracle import reference as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "deletion_cases.json")


def _graph(case):
    e = np.array(case["edges"], dtype=np.float64).reshape(-1, 3)
    rp, col, w = W.edges_to_csr(case["n"], e[:, 0].astype(np.int64), e[:, 1].astype(np.int64), e[:, 2])
    sv = [s[0] for s in case["seeds"]]
    sc = [s[1] for s in case["seeds"]]
    return R.Graph(case["n"], rp, col, w, case["C"], sv, sc)


def _closed_form_reachable(g):
    """Eq. (2) on the part of the graph that reaches a seed (elsewhere L_UU is singular); other
    rows come back as NaN."""
    rp, col, w = g.csr()
    reach = R.seed_reachable(rp, col, g.seed_class)
    idx = np.flatnonzero(reach)
    new_id = np.full(g.n, -1, dtype=np.int64)
    new_id[idx] = np.arange(idx.shape[0])
    keep = reach[g.src]  # a reachable vertex only has reachable neighbours
    once = keep & (g.src < g.dst)
    srp, scol, sw = W.edges_to_csr(idx.shape[0], new_id[g.src[once]], new_id[g.dst[once]], g.w[once])
    Fs = R.harmonic_closed_form(srp, scol, sw.astype(np.float64), g.seed_class[idx], g.C)
    F = np.full((g.n, g.C), np.nan)
    F[idx] = Fs
    return F, reach


@pytest.mark.parametrize("case", json.load(open(GOLDEN))["cases"], ids=lambda c: c["name"])
def test_hand_worked_deletions(case):
    g = _graph(case)
    C = case["C"]
    rp, col, w = g.csr()
    F_before = R.harmonic_closed_form(rp, col, w, g.seed_class, C)
    adj_before = g.adjacency()
    g.delete(case["delete"])
    adj = g.adjacency()
    for u in case["delete"]:
        assert not adj[u] and g.seed_class[u] == -1
        assert all(u not in adj[v] for v in range(g.n))
    A = R.affected_set(adj, g.seed_class, g.n, 0, [], [], [], deleted=case["delete"], adj_before=adj_before)
    assert sorted(A) == case["affected"]
    rp, col, w = g.csr()
    exact, _ = _closed_form_reachable(g)
    for u, row in case["expect"].items():
        np.testing.assert_allclose(exact[int(u)], row, atol=1e-12)
    # Step 3 from the labels held before the batch reaches the same rows
    F0 = F_before.copy()
    F0[case["delete"]] = 1.0 / C
    F, rounds, _, _ = R.step3_propagate(adj, F0, g.seed_class, A, 1e-13, 100000, decide_fp32=False)
    for u, row in case["expect"].items():
        np.testing.assert_allclose(F[int(u)], row, atol=1e-9)
    # the C implementation of the affected set agrees
    dn = [v for u in case["delete"] for v in adj_before[u]]
    A2 = N.affected_set(rp, col, g.seed_class, g.n, [], [], [], deleted_neighbours=dn)
    assert A2.tolist() == case["affected"]


def _random_case(seed, n=120, C=3):
    p = W.small_random(n, C, 4.0, 12, seed)
    return p, R.Graph(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_delete_equals_rebuilding_the_graph_without_those_vertices(seed):
    p, g = _random_case(seed)
    rng = np.random.default_rng(seed)
    dead = rng.choice(p.n, size=9, replace=False)
    dead[0] = p.seed_vertex[0]  # one of them is a seed
    g.delete(dead)
    # independent construction: filter the original edge list, drop the deleted seeds
    src = np.repeat(np.arange(p.n), np.diff(p.row_ptr))
    keep = ~(np.isin(src, dead) | np.isin(p.col, dead))
    once = keep & (src < p.col)
    rp2, col2, w2 = W.edges_to_csr(p.n, src[once], p.col[once], p.w[once])
    ks = ~np.isin(p.seed_vertex, dead)
    g2 = R.Graph(p.n, rp2, col2, w2, p.C, p.seed_vertex[ks], p.seed_class[ks])
    assert np.array_equal(g.seed_class, g2.seed_class)
    a1, a2 = g.adjacency(), g2.adjacency()
    assert all(a1[u].keys() == a2[u].keys() and all(abs(a1[u][v] - a2[u][v]) < 1e-12 for v in a1[u]) for u in range(p.n))
    F1, reach = _closed_form_reachable(g)
    F2, reach2 = _closed_form_reachable(g2)
    assert np.array_equal(reach, reach2)
    np.testing.assert_allclose(F1[reach], F2[reach], atol=1e-10)


def _brute_affected(adj_before, adj_after, seed_class, n_old, k, eu, ev, new_seeds, deleted):
    A = set()
    for u in deleted:
        A |= set(adj_before[u])
    for u in range(n_old, n_old + k):
        A |= {u} | set(adj_after[u])
    for a, b in zip(eu, ev):
        A |= {int(a), int(b)}
    for s in new_seeds:
        A |= set(adj_after[int(s)])
    return sorted(u for u in A if seed_class[u] < 0 and adj_after[u])


@pytest.mark.parametrize("seed", [4, 5])
def test_mixed_batch_deletions_first_then_insertions(seed):
    p, g = _random_case(seed, n=200)
    rp, col, w = g.csr()
    F_before = R.harmonic_closed_form(rp, col, w, g.seed_class, p.C)
    rng = np.random.default_rng(seed)
    unl = np.flatnonzero(g.seed_class < 0)
    dead = rng.choice(unl, size=10, replace=False)
    n_old = p.n
    b = W.small_random_batch(p, 15, 3, 2, num_extra_edges=8)
    # one inserted edge re-attaches a deleted id
    b.eu = np.concatenate([b.eu, [dead[0]]]).astype(np.int32)
    b.ev = np.concatenate([b.ev, [n_old + 1]]).astype(np.int32)
    b.ew = np.concatenate([b.ew, [0.5]]).astype(np.float32)
    adj_before = g.adjacency()
    g.delete(dead)
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    adj = g.adjacency()
    A = R.affected_set(adj, g.seed_class, n_old, b.num_new_vertices, b.eu, b.ev, b.seed_vertex, deleted=dead,
                       adj_before=adj_before)
    want = _brute_affected(adj_before, adj, g.seed_class, n_old, b.num_new_vertices, b.eu, b.ev, b.seed_vertex, dead)
    assert sorted(A) == want
    assert dead[0] in A and n_old + 1 in adj[dead[0]]
    rp, col, w = g.csr()
    dn = [v for u in dead for v in adj_before[u]]
    A2 = N.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex, deleted_neighbours=dn)
    assert A2.tolist() == want
    # Step 3 from the old labels converges to the exact labels of the new graph
    F0 = np.concatenate([F_before, np.full((b.num_new_vertices, p.C), 1.0 / p.C)])
    F0[dead] = 1.0 / p.C
    F0[b.seed_vertex] = np.eye(p.C)[b.seed_class]
    o = N.step3_propagate(rp, col, w, F0, g.seed_class, A2, 1e-12, 200000, decide_fp32=False)
    exact, reach = _closed_form_reachable(g)
    assert np.abs(o["F"] - exact)[reach].max() < 1e-8
