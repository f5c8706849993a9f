"""ctypes access to the plain-C oracle (``c/dynlp_oracle.c``).  TEST INFRASTRUCTURE ONLY.

``build()`` compiles the C file with gcc into ``oracle/_dynlp_oracle.so``; ``lib()`` loads it
(building it first if it is absent).  The wrappers only marshal numpy arrays.
"""
from __future__ import annotations

import ctypes as ct
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "c", "dynlp_oracle.c")
_SO = os.path.join(_HERE, "_dynlp_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-std=c11", "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = ct.CDLL(_SO)
        i64, f64, p = ct.c_int64, ct.c_double, ct.c_void_p
        L.oracle_num_threads.restype = ct.c_int
        L.oracle_set_num_threads.argtypes = [ct.c_int]
        L.oracle_itlp_sweep.restype = f64
        L.oracle_itlp_sweep.argtypes = [i64, p, p, p, ct.c_int, p, p, p]
        L.oracle_itlp_solve.restype = i64
        L.oracle_itlp_solve.argtypes = [i64, p, p, p, ct.c_int, p, p, p, f64, i64, p]
        L.oracle_neumann_solve.restype = i64
        L.oracle_neumann_solve.argtypes = [i64, p, p, p, p, p, p, p, f64, i64, p]
        L.oracle_laplacian_cg.restype = i64
        L.oracle_laplacian_cg.argtypes = [i64, p, p, p, p, ct.c_int, p, p, f64, i64, p]
        L.oracle_affected_set.restype = i64
        L.oracle_affected_set.argtypes = [i64, p, p, p, i64, i64, p, p, i64, p, p, p]
        L.oracle_step3.restype = i64
        L.oracle_step3.argtypes = [i64, p, p, p, ct.c_int, p, p, p, i64, f64, i64, ct.c_int, p, p, i64, p, p]
        L.oracle_components.restype = i64
        L.oracle_components.argtypes = [i64, i64, i64, p, p, p, f64, p, p]
        L.oracle_supernode_init.restype = None
        L.oracle_supernode_init.argtypes = [i64, p, p, p, ct.c_int, p, i64, p, i64, p, p]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ct.c_void_p)


def _csr(row_ptr, col, w):
    return (np.ascontiguousarray(row_ptr, dtype=np.int64), np.ascontiguousarray(col, dtype=np.int32),
            np.ascontiguousarray(w, dtype=np.float64))


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(t: int) -> None:
    lib().oracle_set_num_threads(int(t))


def itlp_sweep(row_ptr, col, w, F, seed_class):
    """One Jacobi sweep of Eq. (1).  Returns (F_new, max_change)."""
    rp, cl, ww = _csr(row_ptr, col, w)
    F = np.ascontiguousarray(F, dtype=np.float64)
    sc = np.ascontiguousarray(seed_class, dtype=np.int32)
    out = np.empty_like(F)
    ch = lib().oracle_itlp_sweep(F.shape[0], _ptr(rp), _ptr(cl), _ptr(ww), F.shape[1], _ptr(sc), _ptr(F), _ptr(out))
    return out, float(ch)


def itlp_solve(row_ptr, col, w, seed_class, C, tol=1e-10, max_iter=1_000_000, F0=None):
    """ItLP to convergence.  Returns (F, sweeps, last_change)."""
    from .reference import initial_labels

    rp, cl, ww = _csr(row_ptr, col, w)
    sc = np.ascontiguousarray(seed_class, dtype=np.int32)
    F = initial_labels(sc, C) if F0 is None else np.array(F0, dtype=np.float64, order="C")
    tmp = np.empty_like(F)
    last = ct.c_double(0.0)
    it = lib().oracle_itlp_solve(F.shape[0], _ptr(rp), _ptr(cl), _ptr(ww), C, _ptr(sc), _ptr(F), _ptr(tmp),
                                 float(tol), int(max_iter), ct.byref(last))
    return F, int(it), float(last.value)


def neumann_solve(row_ptr, col, w, seed_class, b, tol=1e-12, max_iter=10_000_000, x0=None):
    """x = (I - P_UU)^{-1} b by the iteration x <- b + P_UU x (zero on labelled and isolated vertices, and on
    vertices that reach no labelled vertex, where the series has no limit: b is taken as 0 there).
    Returns (x, sweeps, last_change)."""
    from .reference import seed_reachable

    rp, cl, ww = _csr(row_ptr, col, w)
    sc = np.ascontiguousarray(seed_class, dtype=np.int32)
    b = np.array(b, dtype=np.float64, order="C")
    b[~seed_reachable(rp, cl, sc)] = 0.0
    x = np.zeros_like(b) if x0 is None else np.array(x0, dtype=np.float64, order="C")
    tmp = np.empty_like(x)
    last = ct.c_double(0.0)
    it = lib().oracle_neumann_solve(sc.shape[0], _ptr(rp), _ptr(cl), _ptr(ww), _ptr(sc), _ptr(b), _ptr(x), _ptr(tmp),
                                    float(tol), int(max_iter), ct.byref(last))
    return x, int(it), float(last.value)


def _updatable_mask(rp, cl, sc):
    from .reference import seed_reachable

    return ((sc < 0) & (np.diff(rp) > 0) & seed_reachable(rp, cl, sc)).astype(np.uint8)


def _laplacian_cg(rp, cl, ww, in_U, B, X, rtol, max_iter):
    worst = ct.c_double(0.0)
    k = B.shape[1]
    assert X.shape == B.shape and X.shape[0] == in_U.shape[0]
    out = X
    for c0 in range(0, k, 64):  # the C routine advances up to 64 systems at once
        Bc = np.ascontiguousarray(B[:, c0:c0 + 64])
        Xc = np.ascontiguousarray(X[:, c0:c0 + 64])
        it = lib().oracle_laplacian_cg(in_U.shape[0], _ptr(rp), _ptr(cl), _ptr(ww), _ptr(in_U), Bc.shape[1], _ptr(Bc),
                                       _ptr(Xc), float(rtol), int(max_iter), ct.byref(worst))
        if it < 0 or worst.value > rtol:
            raise RuntimeError(f"conjugate gradients stopped after {it} iterations at relative residual {worst.value:.2e}")
        out[:, c0:c0 + 64] = Xc
    return out


def neumann_solve_cg(row_ptr, col, w, seed_class, b, rtol=1e-13, max_iter=100_000):
    """x = (I - P_UU)^{-1} b from the symmetric form (D - W)_UU x = D_U b by conjugate gradients (0 outside the
    updatable rows).  For graphs where the series iteration of neumann_solve needs too many sweeps."""
    rp, cl, ww = _csr(row_ptr, col, w)
    sc = np.ascontiguousarray(seed_class, dtype=np.int32)
    n = sc.shape[0]
    in_U = _updatable_mask(rp, cl, sc)
    deg = np.bincount(np.repeat(np.arange(n), np.diff(rp)), weights=ww, minlength=n)
    B = (deg * np.asarray(b, dtype=np.float64) * in_U).reshape(n, 1)
    X = np.zeros((n, 1), dtype=np.float64)
    return _laplacian_cg(rp, cl, ww, in_U, B, X, rtol, max_iter)[:, 0]


def harmonic_solve_cg(row_ptr, col, w, seed_class, C, rtol=1e-13, max_iter=100_000):
    """The fixed point of Eq. (1) from Eq. (2) in symmetric form, (D - W)_UU F_U = W_UL Y_L, all C columns by
    conjugate gradients.  Rows outside the updatable set keep their start values (one-hot / uniform)."""
    from .reference import initial_labels

    rp, cl, ww = _csr(row_ptr, col, w)
    sc = np.ascontiguousarray(seed_class, dtype=np.int32)
    n = sc.shape[0]
    in_U = _updatable_mask(rp, cl, sc)
    F = initial_labels(sc, C)
    # B_u = sum over labelled neighbours v of w(u,v) Y_v
    src = np.repeat(np.arange(n), np.diff(rp))
    lab = sc[cl] >= 0
    B = np.zeros((n, C), dtype=np.float64)
    np.add.at(B, (src[lab], sc[cl[lab]]), ww[lab])
    B *= in_U[:, None]
    X = np.full((n, C), 1.0 / C, dtype=np.float64) * in_U[:, None]
    X = _laplacian_cg(rp, cl, ww, in_U, B, np.ascontiguousarray(X), rtol, max_iter)
    F[in_U > 0] = X[in_U > 0]
    return F


def affected_set(row_ptr, col, seed_class, n_old, eu, ev, new_seed_vertex, deleted_neighbours=None):
    """V_aff of a batch on the already-updated CSR; ascending int32 ids.  ``deleted_neighbours``:
    the vertices that were adjacent to a deleted vertex before the batch (Alg. 2 adds N(u) for
    every deleted u); they join the set under the same rule as everyone else (unlabelled and not
    isolated in the updated graph)."""
    rp = np.ascontiguousarray(row_ptr, dtype=np.int64)
    cl = np.ascontiguousarray(col, dtype=np.int32)
    sc = np.ascontiguousarray(seed_class, dtype=np.int32)
    n = sc.shape[0]
    eu = np.ascontiguousarray(eu, dtype=np.int32)
    ev = np.ascontiguousarray(ev, dtype=np.int32)
    sv = np.ascontiguousarray(new_seed_vertex, dtype=np.int32)
    flag = np.empty(max(n, 1), dtype=np.uint8)
    out = np.empty(max(n, 1), dtype=np.int32)
    cnt = lib().oracle_affected_set(n, _ptr(rp), _ptr(cl), _ptr(sc), int(n_old), eu.shape[0], _ptr(eu), _ptr(ev),
                                    sv.shape[0], _ptr(sv), _ptr(flag), _ptr(out))
    A = out[:cnt].copy()
    if deleted_neighbours is not None and len(deleted_neighbours):
        extra = np.unique(np.asarray(deleted_neighbours, dtype=np.int64))
        ok = (sc[extra] < 0) & (np.diff(rp)[extra] > 0)
        A = np.union1d(A, extra[ok].astype(np.int32)).astype(np.int32)
    return A


def step3_propagate(row_ptr, col, w, F, seed_class, V_aff, tol, max_iter, decide_fp32=True, record=4096):
    """Alg. 2 Step 3.  Returns dict(F, rounds, frontier_sizes, max_changes, rows_updated,
    edges_traversed, remaining)."""
    rp, cl, ww = _csr(row_ptr, col, w)
    F = np.array(F, dtype=np.float64, order="C")
    sc = np.ascontiguousarray(seed_class, dtype=np.int32)
    A0 = np.ascontiguousarray(V_aff, dtype=np.int32)
    sizes = np.zeros(record, dtype=np.int64)
    changes = np.zeros(record, dtype=np.float64)
    totals = np.zeros(2, dtype=np.int64)
    rem = ct.c_int64(0)
    rounds = lib().oracle_step3(F.shape[0], _ptr(rp), _ptr(cl), _ptr(ww), F.shape[1], _ptr(sc), _ptr(F), _ptr(A0),
                                A0.shape[0], float(tol), int(max_iter), int(bool(decide_fp32)), _ptr(sizes),
                                _ptr(changes), record, _ptr(totals), ct.byref(rem))
    k = min(int(rounds), record)
    return dict(F=F, rounds=int(rounds), frontier_sizes=sizes[:k].copy(), max_changes=changes[:k].copy(),
                rows_updated=int(totals[0]), edges_traversed=int(totals[1]), remaining=int(rem.value))


def components(n_old, k, eu, ev, ew, tau):
    """Components of the sparsified batch-internal graph (Alg. 2 Step 1).  Returns
    (comp int32[k], number of components, |E'|)."""
    eu = np.ascontiguousarray(eu, dtype=np.int32)
    ev = np.ascontiguousarray(ev, dtype=np.int32)
    ew = np.ascontiguousarray(ew, dtype=np.float64)
    comp = np.empty(max(int(k), 1), dtype=np.int32)
    kept = ct.c_int64(0)
    cnt = lib().oracle_components(int(n_old), int(k), eu.shape[0], _ptr(eu), _ptr(ev), _ptr(ew), float(tau),
                                  _ptr(comp), ct.byref(kept))
    return comp[:int(k)].copy(), int(cnt), int(kept.value)


def supernode_init(row_ptr, col, w, F, seed_class, n_old, comp, num_comp):
    """Alg. 2 Step 2 on the updated CSR.  Returns (F with the inserted unlabelled rows set, W)."""
    rp, cl, ww = _csr(row_ptr, col, w)
    F = np.array(F, dtype=np.float64, order="C")
    sc = np.ascontiguousarray(seed_class, dtype=np.int32)
    comp = np.ascontiguousarray(comp, dtype=np.int32)
    W = np.zeros((max(int(num_comp), 1), F.shape[1]), dtype=np.float64)
    lib().oracle_supernode_init(F.shape[0], _ptr(rp), _ptr(cl), _ptr(ww), F.shape[1], _ptr(sc), int(n_old),
                                _ptr(comp), int(num_comp), _ptr(W), _ptr(F))
    return F, W[:int(num_comp)]
