"""C-ABI checks that need no GPU: the library loads, exports what the header declares, and
rejects bad arguments before touching a device."""
import ctypes as ct
import os
import re

import numpy as np
import pytest

import paper_2604_06596_amd as P
from paper_2604_06596_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(P.library_path()):
        P.build()
    return B.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dynlp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dynlp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == names


def test_stats_and_options_layout_match_header():
    # field order and sizes as declared in include/dynlp.h (natural alignment)
    assert ct.sizeof(B.Stats) == 4 + 4 + 4 + 4 + 8 * 6 + 4 * 5 + 4 + 8
    assert B.Stats.rows_updated.offset == 16
    assert B.Stats.ms_update_kernel.offset == 64
    assert B.Options.stream.offset == 8 and B.Options.slack_factor.offset == 20
    assert B.Options.alloc.offset == 48 and B.Options.binary_scalar.offset == 72 and ct.sizeof(B.Options) == 96 and B.Options.persistent_rounds.offset == 80 and B.Options.ingest_chunk_edges.offset == 88


def _tiny():
    # path 0-1-2
    rp = np.array([0, 1, 3, 4], dtype=np.int64)
    col = np.array([1, 0, 2, 1], dtype=np.int32)
    w = np.array([1, 1, 2, 2], dtype=np.float32)
    return rp, col, w


@pytest.mark.parametrize("mutate,needle", [
    (lambda a: a.update(C=0), "num_classes"),
    (lambda a: a.update(C=65), "num_classes"),
    (lambda a: a.update(n=-1), "n must be"),
    (lambda a: a.update(rp=np.array([0, 2, 1, 4], dtype=np.int64)), "row_ptr"),
    (lambda a: a.update(rp=np.array([1, 1, 3, 4], dtype=np.int64)), "row_ptr"),
    (lambda a: a.update(col=np.array([1, 0, 3, 1], dtype=np.int32)), "neighbour id"),
    (lambda a: a.update(col=np.array([0, 0, 2, 1], dtype=np.int32)), "self loop"),
    (lambda a: a.update(w=np.array([1, 1, 0, 2], dtype=np.float32)), "weight"),
    (lambda a: a.update(w=np.array([1, np.inf, 2, 2], dtype=np.float32)), "weight"),
    (lambda a: a.update(w=np.array([1, np.nan, 2, 2], dtype=np.float32)), "weight"),
    (lambda a: a.update(sv=np.array([3], dtype=np.int32)), "seed vertex"),
    (lambda a: a.update(sc=np.array([2], dtype=np.int32)), "seed class"),
    (lambda a: a.update(sv=np.array([0, 0], dtype=np.int32), sc=np.array([0, 1], dtype=np.int32)), "two different"),
    (lambda a: a.update(group_lanes=5), "group_lanes"),
    (lambda a: a.update(C=3, binary_scalar=True), "binary_scalar"),
])
def test_create_rejects_bad_arguments_without_a_gpu(lib, mutate, needle):
    rp, col, w = _tiny()
    a = dict(n=3, rp=rp, col=col, w=w, C=2, sv=np.array([0], dtype=np.int32), sc=np.array([1], dtype=np.int32),
             group_lanes=0, binary_scalar=False)
    mutate(a)
    with pytest.raises(B.DynLPError) as ei:
        P.DynLP(a["n"], a["rp"], a["col"], a["w"], a["C"], a["sv"], a["sc"], group_lanes=a["group_lanes"],
                binary_scalar=a["binary_scalar"])
    assert ei.value.status == -1
    assert needle in ei.value.message


def test_null_handles_are_rejected(lib):
    assert lib.dynlp_static_solve(None, 1e-4, 10, None) == -1
    assert lib.dynlp_apply_batch(None, 0, 0, None, None, None, 0, None, None, None) == -1
    assert lib.dynlp_get_labels(None, None, None) == -1
    assert lib.dynlp_num_vertices(None) == -1
    assert lib.dynlp_last_error(None) is not None
    lib.dynlp_destroy(None)
    out = ct.c_void_p()
    assert lib.dynlp_create(None, 0, None, None, None, 2, 0, None, None, None) == -1
    assert lib.dynlp_create(ct.byref(out), 3, None, None, None, 2, 0, None, None, None) == -1
    assert not out


def test_valid_arguments_without_gpu_fail_loudly_not_silently(lib):
    import torch

    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    rp, col, w = _tiny()
    with pytest.raises(B.DynLPError) as ei:
        P.DynLP(3, rp, col, w, 2, np.array([0], dtype=np.int32), np.array([1], dtype=np.int32))
    assert ei.value.status == -3 and "no usable GPU" in ei.value.message


def test_missing_library_raises(tmp_path):
    with pytest.raises(FileNotFoundError):
        B.load_library(str(tmp_path / "libdynlp.so"))


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_06596_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|#include\s+\"[^\"]*oracle", text, flags=re.M), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert not re.search(r"^\s*(from|import)\s+paper_2604_06596_amd", text, flags=re.M), f


def test_init_info_layout_and_null_handles(lib):
    assert ct.sizeof(B.InitInfo) == 32 and B.InitInfo.hook_steps.offset == 24 and B.InitInfo.ms.offset == 28
    assert lib.dynlp_set_initialiser(None, 1, 0.5) == -1
    assert lib.dynlp_mean_edge_weight(None, None) == -1
    assert lib.dynlp_last_components(None, 0, None, None) == -1


def test_round_info_layout_matches_header():
    assert ct.sizeof(B.RoundInfo) == 64  # 60 bytes of fields, padded to the 8-byte alignment
    assert B.RoundInfo.max_delta.offset == 40 and B.RoundInfo.group_lanes.offset == 56


def test_device_pointer_mode_refuses_host_arrays_before_calling_the_library():
    rp, col, w = _tiny()
    with pytest.raises(TypeError):
        P.DynLP(3, rp, col, w, 2, np.array([0], dtype=np.int32), np.array([1], dtype=np.int32), device_ptrs=True)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_new_entry_points_reject_null_handles(lib):
    assert lib.dynlp_apply_update(None, 0, None, 0, 0, None, None, None, 0, None, None, None) == -1
    assert lib.dynlp_set_update_mode(None, 0) == -1
    assert lib.dynlp_storage_info(None, None, None) == -1
    assert lib.dynlp_compact_storage(None) == -1
    assert lib.dynlp_stream_bandwidth(None, 1 << 20, 1, None, None) == -1
