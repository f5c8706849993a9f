"""The optional device allocator of dynlp_options (alloc / dealloc): every device array of a context comes from it
and goes back to it; an allocator that runs out of memory surfaces as DYNLP_ERR_OOM, except for the arrays of the
binned rounds, whose absence only costs speed.  The failures are produced on the host (the allocator returns 0):
no kernel is ever launched on memory that was not handed out."""
import numpy as np
import pytest
import torch

import certify as Cf
import workloads as W
from oracle import reference as R
import paper_2604_06596_amd as P

pytestmark = pytest.mark.gpu

TOL = 1e-6


class TorchAllocator:
    """Device memory from torch's caching allocator; ``refuse(nbytes)`` may veto a request."""

    def __init__(self):
        self.live = {}
        self.calls = 0
        self.refuse = lambda nbytes: False
        self.refused = 0

    def alloc(self, nbytes):
        self.calls += 1
        if self.refuse(nbytes):
            self.refused += 1
            return 0
        t = torch.empty(max(1, nbytes), dtype=torch.uint8, device="cuda:0")
        self.live[t.data_ptr()] = t
        return t.data_ptr()

    def free(self, ptr):
        assert ptr in self.live, "the library frees only what the allocator handed out"
        del self.live[ptr]


def _problem(C):
    mk = lambda: W.small_random(5000, C, 8.0, 250, 7100 + C)
    p, p0 = mk(), mk()
    b = W.small_random_batch(p, 500, 7, 10, num_extra_edges=50, num_revealed=2)
    return p0, b


def _run(p0, b, **kw):
    with P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class, **kw) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft, hard = d.get_labels()
        kinds = [int(r.staged) for r in d.round_log_full()]
    return st, s, soft, hard, kinds


@pytest.mark.parametrize("C", [2, 10])
def test_every_device_array_comes_from_the_allocator_and_goes_back(C):
    p0, b = _problem(C)
    a = TorchAllocator()
    st, s, soft, hard, _ = _run(p0, b, allocator=a, slack_factor=1.01)  # little slack: the batch regrows the pool
    assert st == 0 and a.calls > 10
    assert not a.live, "destroy returns everything"
    st2, s2, soft2, hard2, _ = _run(p0, b, slack_factor=1.01)
    assert np.array_equal(soft, soft2) and np.array_equal(hard, hard2) and s.iterations == s2.iterations


def test_an_allocator_without_memory_gives_oom_and_an_unusable_context():
    p0, b = _problem(10)
    a = TorchAllocator()
    with P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class, allocator=a) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        a.refuse = lambda nbytes: True  # from now on nothing can be allocated (the batch's device copies come first)
        with pytest.raises(P.DynLPError) as ei:
            d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        assert ei.value.status == -2 and "allocation" in ei.value.message
        a.refuse = lambda nbytes: False
        with pytest.raises(P.DynLPError) as ei:
            d.get_labels()
        assert ei.value.status == -4  # the context may only be destroyed now
    assert not a.live
    # creation itself
    a2 = TorchAllocator()
    a2.refuse = lambda nbytes: a2.calls > 3
    with pytest.raises(P.DynLPError) as ei:
        P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class, allocator=a2)
    assert ei.value.status == -2 and not a2.live


def test_without_memory_for_the_binned_arrays_the_rounds_are_ordinary_ones():
    """Scalar labels with binned rounds switched on, and an allocator that refuses every request of 160,000 bytes or
    more once the context exists (the per-entry arrays of the binned rounds are that large here; the batch's own
    device copies are not): cold start and batch run as ordinary sweeps and rounds and end at the same labels."""
    p0, b = _problem(2)
    a = TorchAllocator()
    d = P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, 2, p0.seed_vertex, p0.seed_class, binary_scalar=True, binned_rounds=8,
                allocator=a, reserve_vertices=2000, reserve_edges=20000)
    with d:
        a.refuse = lambda nbytes: nbytes >= 160000
        st0, s0 = d.static_solve(TOL, 20000)
        kinds0 = [int(r.staged) for r in d.round_log_full()]
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        kinds = [int(r.staged) for r in d.round_log_full()]
        soft, hard = d.get_labels()
    assert st0 == 0 and st == 0 and a.refused >= 2
    assert 3 not in kinds0 and 3 not in kinds
    assert not a.live
    st2, s2, soft2, hard2, kinds2 = _run(p0, b, binary_scalar=True, binned_rounds=8)
    assert 3 in kinds2
    # ordinary rounds and binned rounds are two locally stopped runs on one graph: each within its own residual
    # certificate of the exact labels, hence within the sum of the two of each other
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, 2, p0.seed_vertex, p0.seed_class)
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    rp, col, w = g.csr()
    Cf.check_two_runs(soft, Cf.certificate(rp, col, w, g.seed_class, soft), soft2,
                      Cf.certificate(rp, col, w, g.seed_class, soft2), "ordinary vs binned rounds")


def test_without_memory_for_the_half_edge_ranks_the_insertion_takes_its_second_atomic():
    """The insertion keeps, per half-edge, what the counting atomic returned (its place among the entries appended to
    its row) so that the writing pass needs no atomic of its own.  That array is optional: refused, the writing pass
    counts again.  Either way the appended entries are sorted afterwards, so graph and labels agree bit for bit."""
    p0, b = _problem(10)
    m = int(b.eu.shape[0])
    a = TorchAllocator()
    with P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class, allocator=a) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        a.refuse = lambda nbytes: nbytes == 3 * m * 4
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft, hard = d.get_labels()
        graph = d.export_graph()
    assert st == 0 and a.refused == 1 and not a.live
    with P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class) as d2:
        assert d2.static_solve(TOL, 20000)[0] == 0
        st2, s2 = d2.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft2, hard2 = d2.get_labels()
        graph2 = d2.export_graph()
    assert st2 == 0 and s.iterations == s2.iterations and s.frontier_initial == s2.frontier_initial
    for x, y in zip(graph, graph2):
        assert np.array_equal(x, y)
    assert np.array_equal(soft, soft2) and np.array_equal(hard, hard2)


def test_calls_that_change_nothing_survive_an_allocator_without_memory():
    """dynlp_get_labels, dynlp_export_graph, dynlp_mean_edge_weight and dynlp_compact_storage only need temporary
    arrays (compaction: the new layout beside the old one).  When the allocator refuses them they return
    DYNLP_ERR_OOM, hand back what they had already taken, and leave the context usable and unchanged."""
    p0, b = _problem(10)
    a = TorchAllocator()
    with P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class, allocator=a) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        soft, hard = d.get_labels()
        graph = d.export_graph()
        mean = d.mean_edge_weight()
        held = set(a.live)
        for refuse in (lambda nbytes: True, lambda nbytes: nbytes > 100_000):  # nothing at all / only small arrays
            a.refuse = refuse
            for call in (d.get_labels, d.export_graph, d.mean_edge_weight, d.compact_storage):
                if call == d.mean_edge_weight and not refuse(8192):
                    continue  # its only array is a few KB
                with pytest.raises(P.DynLPError) as ei:
                    call()
                assert ei.value.status == -2 and "allocation" in ei.value.message
                assert set(a.live) == held, "a failed call hands back whatever it had already allocated"
        a.refuse = lambda nbytes: False
        soft2, hard2 = d.get_labels()
        assert np.array_equal(soft, soft2) and np.array_equal(hard, hard2)
        assert d.mean_edge_weight() == mean
        d.compact_storage()
        for x, y in zip(graph, d.export_graph()):
            assert np.array_equal(x, y)
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        assert st == 0
    assert not a.live
