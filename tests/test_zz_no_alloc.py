"""The entry point that allocates nothing (dynlp_get_labels_static) against dynlp_get_labels, through the
C ABI: two calls in a row, the second on a smaller input (the static staging array keeps the first call's
contents), both pointer modes, the binary scalar layout, and the rejection of requests beyond the array."""
import numpy as np
import pytest
import torch

import workloads as W
import paper_2604_06596_amd as P

pytestmark = pytest.mark.gpu


def _solved(n, C, deg, ns, seed, **kw):
    p = W.small_random(n, C, deg, ns, seed)
    d = P.DynLP(p.n, p.row_ptr, p.col, p.w, p.C, p.seed_vertex, p.seed_class, **kw)
    st, _ = d.static_solve(1e-6, 5000)
    assert st == 0
    return d


def _same(d):
    soft, hard = d.get_labels()
    if torch.is_tensor(soft):
        soft, hard = soft.cpu().numpy(), hard.cpu().numpy()
    s2, h2 = d.get_labels_static()
    assert s2.shape == soft.shape and h2.shape == hard.shape
    assert np.array_equal(s2.view(np.uint32), soft.view(np.uint32))  # bit for bit
    assert np.array_equal(h2, hard)
    # one output at a time uses the same staging area from its start
    assert np.array_equal(d.get_labels_static(soft=False)[1], hard)
    assert np.array_equal(d.get_labels_static(hard=False)[0].view(np.uint32), soft.view(np.uint32))
    return soft, hard


def test_two_calls_in_a_row_the_second_on_a_smaller_input():
    big = _solved(6000, 7, 6.0, 120, 3)
    small = _solved(900, 3, 4.0, 30, 4)
    try:
        soft_b, hard_b = _same(big)
        soft_s, hard_s = _same(small)  # reuses the array that still holds the larger call's rows
        assert soft_s.shape[0] < soft_b.shape[0]
        _same(big)
    finally:
        big.destroy()
        small.destroy()


def test_device_pointer_contexts_and_scalar_layout():
    p = W.small_random(3000, 2, 5.0, 60, 9)
    dv = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dt).cuda()
    d = P.DynLP(p.n, dv(p.row_ptr, torch.int64), dv(p.col, torch.int32), dv(p.w, torch.float32), 2,
                dv(p.seed_vertex, torch.int32), dv(p.seed_class, torch.int32), device_ptrs=True, binary_scalar=True)
    try:
        assert d.static_solve(1e-6, 5000)[0] == 0
        _same(d)
    finally:
        d.destroy()


def test_requests_beyond_the_static_array_are_rejected_and_smaller_ones_still_work():
    n, C = 400_000, 10  # soft alone: 16,000,000 bytes; with hard: 17.6 MB > 16 MiB
    rp = np.zeros(n + 1, dtype=np.int64)
    e = np.zeros(0, dtype=np.int32)
    d = P.DynLP(n, rp, e, np.zeros(0, dtype=np.float32), C, np.array([5], dtype=np.int32), np.array([3], dtype=np.int32))
    try:
        cap = d.static_scratch_bytes
        assert cap == 16 << 20 and n * C * 4 + n * 4 > cap >= n * C * 4
        with pytest.raises(P.DynLPError) as ei:
            d.get_labels_static()
        assert ei.value.status == -1 and "static scratch" in ei.value.message
        soft, _ = d.get_labels_static(hard=False)  # fits on its own
        ref, hard_ref = d.get_labels()
        assert np.array_equal(soft, ref)
        assert np.array_equal(d.get_labels_static(soft=False)[1], hard_ref)
        assert hard_ref[5] == 3 and soft[5, 3] == 1.0
    finally:
        d.destroy()
