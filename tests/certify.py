"""Error certificates for label matrices the GPU library returns (test helper; calls only the oracle).

Why: Alg. 2 Step 3 stops row by row (a row leaves V_aff once it moves by <= tol), so a converged batch update is
*not* within a fixed multiple of tol of the exact harmonic labels, and the paper gives no bound.  What is known
exactly is the identity behind its convergence corollary: with T = one sweep of Eq. (1) and r = F - T(F),

    F - F* = (I - P_UU)^{-1} r     hence     |F - F*|_u <= ((I - P_UU)^{-1} |r|)_u      (row by row)
                                   and       ||F - F*||_inf <= H * ||r||_inf,  H = ||(I - P_UU)^{-1}||_inf

for ANY F whose labelled rows are right (pinned on the CPU by
test_labels_off_the_fixed_point_differ_from_it_by_the_propagated_residual).  The tests therefore
  * measure r with one float64 oracle sweep over the GPU's labels,
  * compute the row-wise bound and H with the oracle's Neumann-series solve, and
  * assert that the GPU's distance from the exact labels respects them,
and they bound ||r||_inf itself by what the arithmetic of each stop rule gives:

  stop_rule_residual(tol)          a static solve, or a batch that ended with dynlp_set_final_check on, ends with a
                                   sweep / round over ALL rows that moved none by more than tol.  Synchronous rows:
                                   F_end = T32(F_prev), |F_end - F_prev| <= tol, so |F_end - T(F_end)| <=
                                   |T32(F_prev) - T(F_prev)| + |T(F_prev) - T(F_end)| <= SWEEP_ATOL + tol (T is an
                                   average: it does not expand the max norm).  In-place rows: the rows written after
                                   row u in that last sweep each moved by <= tol, same bound.  Sweeps that store the
                                   mean of old and new row (the limit-cycle safeguard) test half the move: 2 * tol.
  local_stop_residual(tol, rounds, before)
                                   a batch in the paper's mode.  After its last update a row's residual is <= tol +
                                   SWEEP_ATOL (else a neighbour moved by more than tol in that round and the row would
                                   have been brought back); in every later round its neighbours each move by <= tol
                                   (same reason), which changes its weighted mean by <= tol.  Rows the batch never
                                   touched start from the residual `before` the batch.  Hence
                                   ||r||_inf <= before + (rounds + 1) * tol + SWEEP_ATOL: loose, but a consequence of
                                   the rule, not of a measurement.

SWEEP_ATOL = 1e-6 is the float32-vs-float64 bar of one row update (a tree-shaped sum of <= ~50 products of values
<= 1: relative error <= (log2 k + 3) * 2^-24).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from oracle import native as ON
from oracle import reference as R

SWEEP_ATOL = 1e-6


def stop_rule_residual(tol: float, averaged: bool = False) -> float:
    return (2.0 if averaged else 1.0) * tol + SWEEP_ATOL


def local_stop_residual(tol: float, rounds: int, before: float) -> float:
    return before + (rounds + 1) * tol + SWEEP_ATOL


@dataclass
class Certificate:
    res: float            # ||F - T(F)||_inf over the updatable rows (float64 oracle sweep)
    H: float              # ||(I - P_UU)^{-1}||_inf
    rowwise: np.ndarray   # (I - P_UU)^{-1} max_c |r|: bound on max_c |F - F*| per row (0 outside the updatable rows)
    updatable: np.ndarray # unlabelled, at least one edge, connected to a labelled vertex
    reach: np.ndarray     # connected to a labelled vertex
    refined: np.ndarray   # T(F): the labels after the oracle's sweep
    slack: float          # what the Neumann solves themselves may be off by

    @property
    def bound(self) -> float:
        return float(self.rowwise.max()) if self.rowwise.size else 0.0


def _neumann(rp, col, w, sc, b, n):
    """(I - P_UU)^{-1} b and how far the returned vector is from satisfying its own equation."""
    if n <= 4000:
        x, _, last = ON.neumann_solve(rp, col, w, sc, b, tol=1e-13, max_iter=5_000_000)
    else:
        x = ON.neumann_solve_cg(rp, col, w, sc, b)
    # one step of x <- b + P_UU x from the result: the move is the solve's own residual
    _, _, last = ON.neumann_solve(rp, col, w, sc, b, tol=0.0, max_iter=1, x0=x)
    return x, last


def certificate(rp, col, w, sc, soft) -> Certificate:
    sc = np.asarray(sc, dtype=np.int32)
    n = sc.shape[0]
    w = np.asarray(w, dtype=np.float64)
    F = np.asarray(soft, dtype=np.float64)
    TF, _ = ON.itlp_sweep(rp, col, w, F, sc)
    reach = R.seed_reachable(rp, col, sc)
    upd = (sc < 0) & (np.diff(rp) > 0) & reach
    r = np.max(np.abs(F - TF), axis=1) * upd
    e, miss_e = _neumann(rp, col, w, sc, r, n)
    h, miss_h = _neumann(rp, col, w, sc, upd.astype(np.float64), n)
    H = float(h.max()) if n else 0.0
    # a solve whose own residual is `miss` is within H * miss of the true solution
    slack = H * (miss_e + miss_h * float(r.max() if n else 0.0)) + 1e-12
    return Certificate(res=float(r.max()) if n else 0.0, H=H, rowwise=e, updatable=upd, reach=reach, refined=TF,
                       slack=slack)


def exact_labels(rp, col, w, sc, C):
    """O1: the fixed point of Eq. (1).  ItLP from the oracle's own start on small graphs; on large ones the library
    solve of Eq. (2), certified by one sweep of Eq. (1) (a fixed point does not move).  Returns (F*, how far one
    sweep moves it)."""
    sc = np.asarray(sc, dtype=np.int32)
    w = np.asarray(w, dtype=np.float64)
    if sc.shape[0] <= 4000:
        F, _, _ = ON.itlp_solve(rp, col, w, sc, C, tol=1e-13, max_iter=10_000_000)
    else:
        F = ON.harmonic_solve_cg(rp, col, w, sc, C)
    reach = R.seed_reachable(rp, col, sc)
    TF, _ = ON.itlp_sweep(rp, col, w, F, sc)
    moved = float(np.max(np.abs(TF - F)[reach])) if F.size else 0.0
    return F, moved


def check_against_exact(soft, exact, exact_moved, cert: Certificate, what: str = "") -> float:
    """The GPU's rows against the exact ones: row by row within the certificate, and in norm within H * res.
    ``exact_moved``: how far one sweep moves ``exact`` (its own distance from the fixed point is <= H * that)."""
    err_rows = np.max(np.abs(np.asarray(soft, dtype=np.float64) - exact), axis=1)
    own = cert.H * exact_moved + cert.slack
    ok = err_rows[cert.reach] <= cert.rowwise[cert.reach] * (1 + 1e-9) + own
    err = float(err_rows[cert.reach].max()) if cert.reach.any() else 0.0
    print(f"{what}: max|F_gpu - F_exact| = {err:.3e}; certificate: residual {cert.res:.3e}, H = {cert.H:.1f}, "
          f"row-wise bound max {cert.bound:.3e}, H * residual = {cert.H * cert.res:.3e}")
    assert bool(ok.all()), f"{what}: {int((~ok).sum())} rows further from the exact labels than their residual allows"
    assert err <= cert.H * cert.res + own
    return err


def check_hard(hard, exact, cert: Certificate, extra: float = 0.0):
    """Hard labels must equal the exact argmax wherever the exact top-2 margin exceeds twice what the row can be
    off by (then no column can overtake another)."""
    allow = cert.rowwise * (1 + 1e-9) + cert.slack + extra
    clear = cert.reach & (R.top2_margin(exact) > 2.0 * allow)
    assert np.array_equal(np.asarray(hard)[clear], R.hard_labels(exact)[clear])
    return int(clear.sum())


def check_two_runs(soft_a, cert_a: Certificate, soft_b, cert_b: Certificate, what: str = "") -> float:
    """Two label matrices of one graph (the GPU's and the oracle's Step-3 loop's, or two GPU modes): each is within
    its certificate of the same fixed point, so they are within the sum of each other, row by row."""
    d_rows = np.max(np.abs(np.asarray(soft_a, dtype=np.float64) - np.asarray(soft_b, dtype=np.float64)), axis=1)
    allow = (cert_a.rowwise + cert_b.rowwise) * (1 + 1e-9) + cert_a.slack + cert_b.slack
    m = cert_a.reach
    d = float(d_rows[m].max()) if m.any() else 0.0
    print(f"{what}: max difference {d:.3e} (allowed row by row, max {float(allow[m].max()) if m.any() else 0.0:.3e})")
    assert bool((d_rows[m] <= allow[m]).all())
    return d
