"""Storage compaction of the mutable CSR: rows laid out again with fresh slack; nothing a caller can
observe changes (graph in stored order, labels, later batches), the pool's used part shrinks."""
import numpy as np
import pytest

import workloads as W
from oracle import native as ON
from oracle import reference as R
import paper_2604_06596_amd as P

pytestmark = pytest.mark.gpu

TOL = 1e-6


def test_compaction_keeps_graph_and_labels_and_later_batches_still_match_the_oracle():
    p = W.small_random(6000, 4, 8.0, 300, 5100)
    p0 = W.small_random(6000, 4, 8.0, 300, 5100)
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    rng = np.random.default_rng(3)
    with P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class, slack_factor=1.05) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        used0, cap0 = d.storage_info()
        for _ in range(3):  # little slack: many rows relocate; a seventh of the vertices is deleted each time
            b = W.small_random_batch(p, 300, 8, 3, num_extra_edges=400)
            dead = rng.choice(g.n, size=900, replace=False).astype(np.int32)
            st, s = d.apply_update(dead, b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
            assert st == 0
            g.delete(dead)
            g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        used1, _ = d.storage_info()
        before_graph = d.export_graph()
        before_soft, before_hard = d.get_labels()
        d.compact_storage()
        used2, cap2 = d.storage_info()
        assert used0 < used1 and used2 < used1 and used2 <= cap2
        after_graph = d.export_graph()
        assert all(np.array_equal(a, b) for a, b in zip(before_graph, after_graph))
        soft, hard = d.get_labels()
        assert np.array_equal(soft, before_soft) and np.array_equal(hard, before_hard)
        # a further batch behaves as usual
        b = W.small_random_batch(p, 200, 6, 2, num_extra_edges=100)
        n_old = g.n
        d.set_params(TOL, 3)
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft2, _ = d.get_labels()
        sizes, _ = d.round_log()
        g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        rp, col, w = g.csr()
        A0 = ON.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex)
        F = np.concatenate([soft.astype(np.float64), np.full((b.num_new_vertices, g.C), 1.0 / g.C)])
        F[b.seed_vertex] = np.eye(g.C)[b.seed_class]
        o2 = ON.step3_propagate(rp, col, w, F, g.seed_class, A0, TOL, 3)
        assert sizes.tolist() == o2["frontier_sizes"].tolist()
        assert np.max(np.abs(soft2 - o2["F"])) <= 5e-6
        print(f"pool entries in use: after create {used0}, after three batches {used1}, after compaction {used2}")


def test_compaction_of_empty_and_tiny_graphs():
    rp = np.zeros(1, dtype=np.int64)
    with P.DynLP(0, rp, np.zeros(0, np.int32), np.zeros(0, np.float32), 2, None, None) as d:
        d.compact_storage()
        assert d.storage_info()[0] == 0
    p = W.small_random(50, 2, 3.0, 5, 1)
    with P.DynLP(p.n, p.row_ptr, p.col, p.w, 2, p.seed_vertex, p.seed_class) as d:
        g0 = d.export_graph()
        d.compact_storage()
        d.compact_storage()
        assert all(np.array_equal(a, b) for a, b in zip(g0, d.export_graph()))
        assert d.static_solve(TOL, 10000)[0] == 0
