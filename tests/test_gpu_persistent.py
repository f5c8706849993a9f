"""Several rounds per launch (dynlp_options.persistent_rounds; k_rounds_persistent: a grid of resident workgroups
with a bounded barrier between rounds): the rounds must be the oracle's rounds - same V_aff every round, same
labels to rounding - whether they run one per launch or many, in both update modes; a barrier that is given up
(forced from the host with a spin limit of one poll) must leave complete rounds behind and the batch must finish
with ordinary launches at the same labels."""
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


def _case(kind, C):
    if kind == "random":
        mk = lambda: W.small_random(5000, C, 9.0, 250, 1900 + C)
        p, p0 = mk(), mk()
        b = W.small_random_batch(p, 250, 7, 5, num_extra_edges=60, num_revealed=3)
    elif kind == "sbm":
        p, p0 = W.sbm(30000, C, 20.0, 8.0, 0.01, 1777), W.sbm(30000, C, 20.0, 8.0, 0.01, 1777)
        b = W.sbm_vertex_batch(p, 300, 20, 0.01)
    else:  # hubs: rows of more than 128 entries get a workgroup each
        p, p0 = (W.chung_lu(20000, C, 12.0, 2.1, 3000, 0.8, 0.02, 1098) for _ in range(2))
        b = W.chung_lu_vertex_batch(p, 200, 0.02)
    return p0, b


def _oracle_start(p0, b, soft0):
    g = R.Graph(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class)
    n_old = g.n
    g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    rp, col, w = g.csr()
    F = np.concatenate([soft0.astype(np.float64), np.full((b.num_new_vertices, g.C), 1.0 / g.C)])
    F[b.seed_vertex] = np.eye(g.C)[b.seed_class]
    A0 = ON.affected_set(rp, col, g.seed_class, n_old, b.eu, b.ev, b.seed_vertex)
    return g, rp, col, w, F, A0


def _run(p0, b, max_iter, mode=P.UPDATE_SYNCHRONOUS, tol=TOL, **kw):
    with P.DynLP(p0.n, p0.row_ptr, p0.col, p0.w, p0.C, p0.seed_vertex, p0.seed_class, **kw) as d:
        d.set_update_mode(mode)
        assert d.static_solve(TOL, 20000)[0] == 0
        soft0, _ = d.get_labels()
        d.set_params(tol, max_iter)
        st, s = d.apply_batch(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
        soft, hard = d.get_labels()
        sizes, deltas = d.round_log()
        kinds = [int(r.staged) for r in d.round_log_full()]
    return dict(st=st, s=s, soft0=soft0, soft=soft, hard=hard, sizes=sizes, deltas=deltas, kinds=kinds)


@pytest.mark.parametrize("kind,C", [("random", 10), ("random", 50), ("random", 2), ("sbm", 10), ("hub", 3)])
@pytest.mark.parametrize("R_", [3, 33, 70])
def test_rounds_inside_one_launch_match_the_oracle_round_by_round(kind, C, R_):
    """Cut both sides after R rounds (inside the first launch, just past one launch of 32 rounds, past two)."""
    p0, b = _case(kind, C)
    out = _run(p0, b, R_, persistent_rounds=1)
    g, rp, col, w, F, A0 = _oracle_start(p0, b, out["soft0"])
    o2 = ON.step3_propagate(rp, col, w, F, g.seed_class, A0, TOL, R_)
    print("kinds", out["kinds"][:6], "...", "sizes", out["sizes"][:8].tolist())
    assert out["kinds"][0] == 0 and set(out["kinds"][1:]) == {4}, "the rounds after the first are meant to share launches"
    assert out["s"].iterations == o2["rounds"] == R_ and out["st"] == 1
    assert out["sizes"].tolist() == o2["frontier_sizes"].tolist()
    assert np.max(np.abs(out["soft"] - o2["F"])) <= ROUNDS_ATOL
    np.testing.assert_allclose(out["deltas"], o2["max_changes"], atol=1e-6)
    assert out["s"].edges_traversed == o2["edges_traversed"] and out["s"].rows_updated == o2["rows_updated"]


@pytest.mark.parametrize("kind,C", [("random", 10), ("sbm", 10), ("hub", 3)])
def test_synchronous_batches_are_bit_identical_with_one_round_per_launch(kind, C):
    p0, b = _case(kind, C)
    a = _run(p0, b, 20000, persistent_rounds=1)
    c = _run(p0, b, 20000, persistent_rounds=-1)
    assert a["st"] == 0 and c["st"] == 0 and 4 in a["kinds"] and 4 not in c["kinds"]
    assert np.array_equal(a["soft"], c["soft"]) and np.array_equal(a["hard"], c["hard"])
    assert a["sizes"].tolist() == c["sizes"].tolist()
    a2 = _run(p0, b, 20000, persistent_rounds=1)
    assert np.array_equal(a["soft"], a2["soft"])


@pytest.mark.parametrize("kind,C", [("random", 10), ("sbm", 10), ("hub", 3)])
def test_in_place_batches_reach_the_exact_labels(kind, C):
    p0, b = _case(kind, C)
    out = _run(p0, b, 20000, mode=P.UPDATE_IN_PLACE, persistent_rounds=1)
    assert out["st"] == 0 and 4 in out["kinds"]
    g, rp, col, w, F, A0 = _oracle_start(p0, b, out["soft0"])
    assert out["s"].frontier_initial == len(A0) == out["sizes"][0]
    exact, exact_moved = Cf.exact_labels(rp, col, w, g.seed_class, g.C)
    cert = Cf.certificate(rp, col, w, g.seed_class, out["soft"])
    Cf.check_against_exact(out["soft"], exact, exact_moved, cert, f"{kind} C={C}, in place, many rounds per launch")
    Cf.check_hard(out["hard"], exact, cert)
    assert cert.res <= Cf.local_stop_residual(TOL, out["s"].iterations, Cf.stop_rule_residual(TOL))


@pytest.mark.parametrize("mode", [P.UPDATE_SYNCHRONOUS, P.UPDATE_IN_PLACE], ids=["synchronous", "in_place"])
def test_a_barrier_that_is_given_up_leaves_complete_rounds_and_the_batch_finishes_with_ordinary_launches(mode):
    """A spin limit of one poll makes workgroups give up at the first barrier unless every other workgroup has
    already arrived: the launch ends after a complete round, the library notices, and the rest of the batch runs one
    round per launch.  Every kernel exits normally."""
    p0, b = _case("sbm", 10)
    a = _run(p0, b, 20000, mode=mode, persistent_rounds=1, persistent_spin_limit=1)
    c = _run(p0, b, 20000, mode=mode, persistent_rounds=-1)
    assert a["st"] == 0 and c["st"] == 0
    print("kinds", a["kinds"][:12])
    assert a["kinds"].count(4) >= 1 and 2 in a["kinds"], "one short persistent launch, then ordinary fused rounds"
    if mode == P.UPDATE_SYNCHRONOUS:
        assert np.array_equal(a["soft"], c["soft"]) and a["sizes"].tolist() == c["sizes"].tolist()
    else:
        g, rp, col, w, F, A0 = _oracle_start(p0, b, a["soft0"])
        Cf.check_two_runs(a["soft"], Cf.certificate(rp, col, w, g.seed_class, a["soft"]), c["soft"],
                          Cf.certificate(rp, col, w, g.seed_class, c["soft"]), "given-up barrier vs ordinary launches")


def test_the_limit_cycle_safeguard_still_ends_a_batch_that_shares_launches():
    """The strongly tied pair of test_gpu_parity (rounds that repeat exactly): the library leaves the persistent
    stretch and the averaged staged rounds end the batch."""
    p = W.small_random(400, 2, 6.0, 40, 4242)
    a_ = int(p.seed_vertex[np.flatnonzero(p.seed_class == 0)[0]])
    b_ = int(p.seed_vertex[np.flatnonzero(p.seed_class == 1)[0]])
    u, v = p.n, p.n + 1
    with P.DynLP(p.n, p.row_ptr, p.col, p.w, 2, p.seed_vertex, p.seed_class, persistent_rounds=1) as d:
        assert d.static_solve(TOL, 20000)[0] == 0
        d.set_params(TOL, 20000)
        st, s = d.apply_batch(2, np.array([u, u, v], np.int32), np.array([v, a_, b_], np.int32),
                              np.array([1.0, 0.001, 0.001], np.float32))
        soft, hard = d.get_labels()
        kinds = [int(r.staged) for r in d.round_log_full()]
    assert st == 0 and s.converged == 1 and s.iterations < 8000
    assert 4 in kinds and kinds[-1] == 1
    gap = 0.0005 / 2.001
    assert abs(soft[u, 1] - (0.5 - gap)) <= 1e-4 and abs(soft[v, 1] - (0.5 + gap)) <= 1e-4
