"""CPU oracle for dynamic batched label propagation (DynLP).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, float64 statement of what
the GPU library must compute, written from the paper's equations.  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import it.
It shares no code with ``paper_2604_06596_amd`` and neither imports the other.

Contents
--------
``reference``  numpy / pure-Python definitions: closed-form harmonic solution (Eq. 2),
               Jacobi label propagation ItLP (Eq. 1), graph update + recompute (Alg. 1),
               the frontier-restricted propagation of Alg. 2 Step 3, argmax labels.
``native``     the same ItLP sweep / solve and Step-3 loop in plain C (``c/dynlp_oracle.c``),
               for graphs too large for the Python loops; checked against ``reference``.

Pinned by ``tests/test_oracle_*.py`` against closed forms (path = linear interpolation,
series-conductance voltage divider, star, complete graph), the dense solve of Eq. (2),
the paper's adjustment-form update (Alg. 2 Step 3 formula), row-stochastic / seed / maximum
principle invariants, and brute-force set semantics of the frontier loop on tiny graphs.

Parity unpinned: the paper's own worked numbers (the u9 trajectory of its example figure,
the tau=5 index set of its sparsification figure) live only in figures that are not part of
the text, so nothing here is checked against them.
"""
