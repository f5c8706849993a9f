"""Long seeded sequences of mixed calls on one context: insertion batches (new vertices, edges between old
vertices, revealed seeds, edges to ids deleted earlier), updates with deletions, storage compaction, switches of the
update mode, of the final check and of the initialiser, tolerance changes - in a random but fixed order.  After every
call that changes the graph:

* the stored graph equals the oracle's `Graph` after the same calls (row lengths, entries as multisets, seed classes,
  degrees);
* |V_aff| after Step 1 equals the oracle's affected set;
* the converged labels are within their residual certificate of the exact labels of that graph (tests/certify.py),
  seeds exactly one-hot, hard labels equal to the exact argmax wherever the
  margin is clear;
* the residual respects what the stop rules of the calls so far imply.

The point is the interplay the single-feature tests do not reach: rows relocated after a compaction, a batch that
re-attaches deleted ids, binned rounds (scalar layout, bins of 256 receivers) after deletions have emptied rows, mode
switches in the middle of a history."""
import numpy as np
import pytest

import certify as Cf
import workloads as W
from oracle import native as ON
from oracle import reference as R
import paper_2604_06596_amd as P

pytestmark = pytest.mark.gpu


def _rows(rp, col, w):
    return [sorted(zip(col[rp[u]:rp[u + 1]].tolist(), np.asarray(w[rp[u]:rp[u + 1]], dtype=np.float32).tolist()))
            for u in range(len(rp) - 1)]


def _check_graph(d, g):
    rp, col, w, deg, sc = d.export_graph()
    orp, ocol, ow = g.csr()
    assert rp.tolist() == orp.tolist()
    assert _rows(rp, col, w) == _rows(orp, ocol, ow)
    assert sc.tolist() == g.seed_class.tolist()
    np.testing.assert_allclose(deg, np.bincount(g.src, weights=g.w, minlength=g.n), rtol=1e-5, atol=0)


@pytest.mark.parametrize("layout,C,seed", [("rows", 5, 11), ("rows", 2, 12), ("rows", 12, 15), ("scalar-binned", 2, 13), ("scalar-binned", 2, 16), ("scalar", 2, 14)])
def test_random_sequence_of_calls(layout, C, seed):
    rng = np.random.default_rng(9000 + seed)
    mk = lambda: W.small_random(3001, C, 7.0, 150, 9100 + seed)
    p, p0 = mk(), mk()
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, C, p0.seed_vertex, p0.seed_class)
    kw = {}
    if layout.startswith("scalar"):
        kw = dict(binary_scalar=True, binned_rounds=8 if layout == "scalar-binned" else -1)
    tol = 1e-6
    final_check = False
    history = []
    with P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, C, p0.seed_vertex, p0.seed_class, slack_factor=1.05, **kw) as d:
        assert d.static_solve(tol, 50000)[0] == 0
        implied = Cf.stop_rule_residual(tol)  # what the calls so far allow the residual to be
        deleted_before = np.zeros(0, dtype=np.int32)
        for step in range(70):
            op = rng.choice(["insert", "insert", "update", "compact", "mode", "check", "init", "tol"])
            history.append(str(op))
            if op == "compact":
                soft_a, _ = d.get_labels()
                d.compact_storage()
                soft_b, _ = d.get_labels()
                assert np.array_equal(soft_a, soft_b)
                _check_graph(d, g)
                continue
            if op == "mode":
                d.set_update_mode(int(rng.integers(0, 2)))
                continue
            if op == "check":
                final_check = bool(rng.integers(0, 2))
                d.set_final_check(final_check)
                continue
            if op == "init":
                if rng.integers(0, 2):
                    d.set_initialiser(P.INIT_SUPERNODE, float(np.float32(d.mean_edge_weight())))
                else:
                    d.set_initialiser(P.INIT_UNIFORM)
                continue
            if op == "tol":
                tol = float(rng.choice([1e-6, 1e-5, 3e-6]))
                d.set_params(tol, 50000)
                continue
            n_old = g.n
            b = W.small_random_batch(p, int(rng.integers(1, 120)), int(rng.integers(1, 8)), int(rng.integers(0, 4)),
                                     num_extra_edges=int(rng.integers(0, 40)), num_revealed=int(rng.integers(0, 3)))
            if deleted_before.size and rng.integers(0, 2):  # give an id deleted earlier an edge again
                b.eu = np.concatenate([b.eu, [int(deleted_before[0])]]).astype(np.int32)
                b.ev = np.concatenate([b.ev, [n_old]]).astype(np.int32)
                b.ew = np.concatenate([b.ew, [0.7]]).astype(np.float32)
            dead = np.zeros(0, dtype=np.int32)
            if op == "update":
                dead = rng.choice(n_old, size=int(rng.integers(1, 60)), replace=False).astype(np.int32)
                dead = np.setdiff1d(dead, np.concatenate([b.eu, b.ev, b.seed_vertex])).astype(np.int32)
            rp0, col0, _ = g.csr()
            dn = (np.concatenate([col0[rp0[u]:rp0[u + 1]] for u in dead]) if dead.size else np.zeros(0, np.int32))
            if dead.size:
                st, s = d.apply_update(dead, b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
                g.delete(dead)
                deleted_before = dead
            else:
                st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
            assert st == 0 and s.converged == 1, history
            g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
            _check_graph(d, g)
            rp, col, w = g.csr()
            sc = g.seed_class
            A0 = ON.affected_set(rp, col, sc, n_old, b.eu, b.ev, b.seed_vertex, deleted_neighbours=dn)
            assert s.frontier_initial == len(A0), history
            soft, hard = d.get_labels()
            exact, _, _ = ON.itlp_solve(rp, col, w, sc, C, tol=1e-13, max_iter=10_000_000)
            cert = Cf.certificate(rp, col, w, sc, soft)
            Cf.check_against_exact(soft, exact, 1e-13, cert, f"step {step} ({op}, {len(dead)} deleted)")
            Cf.check_hard(hard, exact, cert)
            implied = (Cf.stop_rule_residual(tol) if final_check else Cf.local_stop_residual(tol, s.iterations, implied))
            assert cert.res <= implied, (history, cert.res, implied)
            s_idx = np.flatnonzero(sc >= 0)
            assert np.array_equal(soft[s_idx], R.initial_labels(sc, C)[s_idx].astype(np.float32))
            assert soft.min() >= 0 and np.max(np.abs(soft.sum(1) - 1)) < 1e-5
        print(layout, "calls:", " ".join(history))
