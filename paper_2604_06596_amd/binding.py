"""ctypes binding of libdynlp (argument marshalling only; same names as include/dynlp.h).

Host mode (default): arrays are numpy arrays.  Device mode (``device_ptrs=True``): arrays are
torch tensors on the GPU (only ``.data_ptr()`` is used); outputs are returned as torch tensors.
"""
from __future__ import annotations

import ctypes as ct
import os

import numpy as np

from .build import library_path

STATUS = {0: "DYNLP_OK", 1: "DYNLP_NOT_CONVERGED", -1: "DYNLP_ERR_INVALID_ARG", -2: "DYNLP_ERR_OOM",
          -3: "DYNLP_ERR_DEVICE", -4: "DYNLP_ERR_STATE"}
MAX_CLASSES = 64


class DynLPError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status
        self.message = message


class Stats(ct.Structure):
    _fields_ = [("iterations", ct.c_int32), ("converged", ct.c_int32), ("final_max_delta", ct.c_float),
                ("rows_updated", ct.c_int64), ("edges_traversed", ct.c_int64), ("frontier_initial", ct.c_int64),
                ("frontier_peak", ct.c_int64), ("rows_relocated", ct.c_int64), ("update_launches", ct.c_int64),
                ("ms_update_kernel", ct.c_float), ("ms_insert", ct.c_float), ("ms_seed", ct.c_float),
                ("ms_iterate", ct.c_float), ("ms_total", ct.c_float), ("final_checks", ct.c_int32),
                ("ingest_chunks", ct.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class RoundInfo(ct.Structure):
    _fields_ = [("rows_short", ct.c_int64), ("rows_long", ct.c_int64), ("entries_short", ct.c_int64),
                ("entries_long", ct.c_int64), ("rows_moved", ct.c_int64), ("max_delta", ct.c_float),
                ("ms_update", ct.c_float), ("reserved", ct.c_float), ("staged", ct.c_int32), ("group_lanes", ct.c_int32)]


class InitInfo(ct.Structure):
    _fields_ = [("vertices", ct.c_int64), ("kept_edges", ct.c_int64), ("components", ct.c_int64),
                ("hook_steps", ct.c_int32), ("ms", ct.c_float)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


INIT_UNIFORM, INIT_SUPERNODE = 0, 1
UPDATE_SYNCHRONOUS, UPDATE_IN_PLACE = 0, 1

_ALLOC_FN = ct.CFUNCTYPE(ct.c_void_p, ct.c_size_t, ct.c_void_p)
_DEALLOC_FN = ct.CFUNCTYPE(None, ct.c_void_p, ct.c_void_p)


class Options(ct.Structure):
    _fields_ = [("device", ct.c_int32), ("stream", ct.c_void_p), ("ptrs_on_device", ct.c_int32),
                ("slack_factor", ct.c_float), ("reserve_vertices", ct.c_int64), ("reserve_edges", ct.c_int64),
                ("time_kernels", ct.c_int32), ("group_lanes", ct.c_int32), ("alloc", _ALLOC_FN),
                ("dealloc", _DEALLOC_FN), ("alloc_user", ct.c_void_p), ("binary_scalar", ct.c_int32),
                ("binned_rounds", ct.c_int32), ("persistent_rounds", ct.c_int32), ("persistent_spin_limit", ct.c_int32),
                ("ingest_chunk_edges", ct.c_int64)]


EXPORTS = ["dynlp_default_options", "dynlp_create", "dynlp_static_solve", "dynlp_set_params", "dynlp_apply_batch",
           "dynlp_get_labels", "dynlp_num_vertices", "dynlp_num_entries", "dynlp_num_classes", "dynlp_export_graph",
           "dynlp_round_log", "dynlp_last_error", "dynlp_destroy", "dynlp_set_initialiser",
           "dynlp_mean_edge_weight", "dynlp_last_components", "dynlp_set_update_mode", "dynlp_apply_update", "dynlp_storage_info",
           "dynlp_compact_storage", "dynlp_stream_bandwidth", "dynlp_get_labels_static", "dynlp_static_scratch_bytes",
           "dynlp_set_final_check", "dynlp_gather_bandwidth"]

_lib = None


def load_library(path: str | None = None):
    """Load libdynlp.so.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2604_06596_amd.build` "
                                "(or __graft_entry__.build()); DynLP has no CPU fallback")
    # PyTorch ships its own libamdhip64.so.7.  A process must not run two HIP runtimes, so torch is
    # imported first: the loader then binds libdynlp's libamdhip64.so.7 dependency to the copy that
    # is already resident, and tensors, streams and this library share one runtime.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ct.CDLL(path)
    p, i32, i64, f32 = ct.c_void_p, ct.c_int32, ct.c_int64, ct.c_float
    L.dynlp_default_options.argtypes = [ct.POINTER(Options)]
    L.dynlp_default_options.restype = None
    L.dynlp_create.argtypes = [ct.POINTER(p), i64, p, p, p, i32, i64, p, p, ct.POINTER(Options)]
    L.dynlp_create.restype = ct.c_int
    L.dynlp_static_solve.argtypes = [p, f32, i32, ct.POINTER(Stats)]
    L.dynlp_static_solve.restype = ct.c_int
    L.dynlp_set_params.argtypes = [p, f32, i32]
    L.dynlp_set_params.restype = ct.c_int
    L.dynlp_apply_batch.argtypes = [p, i64, i64, p, p, p, i64, p, p, ct.POINTER(Stats)]
    L.dynlp_apply_batch.restype = ct.c_int
    L.dynlp_apply_update.argtypes = [p, i64, p, i64, i64, p, p, p, i64, p, p, ct.POINTER(Stats)]
    L.dynlp_apply_update.restype = ct.c_int
    L.dynlp_get_labels.argtypes = [p, p, p]
    L.dynlp_get_labels.restype = ct.c_int
    L.dynlp_get_labels_static.argtypes = [p, p, p]
    L.dynlp_get_labels_static.restype = ct.c_int
    L.dynlp_static_scratch_bytes.argtypes = []
    L.dynlp_static_scratch_bytes.restype = i64
    for name in ("dynlp_num_vertices", "dynlp_num_entries"):
        getattr(L, name).argtypes = [p]
        getattr(L, name).restype = i64
    L.dynlp_num_classes.argtypes = [p]
    L.dynlp_num_classes.restype = i32
    L.dynlp_export_graph.argtypes = [p, p, p, p, p, p]
    L.dynlp_export_graph.restype = ct.c_int
    L.dynlp_round_log.argtypes = [p, i64, ct.POINTER(RoundInfo)]
    L.dynlp_round_log.restype = i64
    L.dynlp_storage_info.argtypes = [p, ct.POINTER(i64), ct.POINTER(i64)]
    L.dynlp_storage_info.restype = ct.c_int
    L.dynlp_stream_bandwidth.argtypes = [p, i64, i32, ct.POINTER(ct.c_double), ct.POINTER(ct.c_double)]
    L.dynlp_stream_bandwidth.restype = ct.c_int
    L.dynlp_gather_bandwidth.argtypes = [p, i64, i32, i64, i32, ct.POINTER(ct.c_double), ct.POINTER(ct.c_double)]
    L.dynlp_gather_bandwidth.restype = ct.c_int
    L.dynlp_compact_storage.argtypes = [p]
    L.dynlp_compact_storage.restype = ct.c_int
    L.dynlp_set_update_mode.argtypes = [p, i32]
    L.dynlp_set_update_mode.restype = ct.c_int
    L.dynlp_set_final_check.argtypes = [p, i32]
    L.dynlp_set_final_check.restype = ct.c_int
    L.dynlp_set_initialiser.argtypes = [p, i32, f32]
    L.dynlp_set_initialiser.restype = ct.c_int
    L.dynlp_mean_edge_weight.argtypes = [p, ct.POINTER(ct.c_double)]
    L.dynlp_mean_edge_weight.restype = ct.c_int
    L.dynlp_last_components.argtypes = [p, i64, p, ct.POINTER(InitInfo)]
    L.dynlp_last_components.restype = ct.c_int
    L.dynlp_last_error.argtypes = [p]
    L.dynlp_last_error.restype = ct.c_char_p
    L.dynlp_destroy.argtypes = [p]
    L.dynlp_destroy.restype = None
    _lib = L
    return L


def _is_torch(a) -> bool:
    return a is not None and type(a).__module__.startswith("torch")


class DynLP:
    """One context of the library.  Method names mirror the C entry points."""

    def __init__(self, n, row_ptr, col, w, num_classes, seed_vertex, seed_class, *, device=0, stream=None,
                 device_ptrs=False, slack_factor=1.25, reserve_vertices=0, reserve_edges=0, time_kernels=False,
                 group_lanes=0, binary_scalar=False, binned_rounds=0, allocator=None, library=None,
                 ingest_chunk_edges=0, persistent_rounds=0, persistent_spin_limit=0):
        """``allocator``: optional object with ``alloc(nbytes) -> device address (0 = no memory)`` and
        ``free(address)``; the library then takes all its device arrays from it (dynlp_options.alloc / dealloc)."""
        self._L = load_library(library)
        self._h = ct.c_void_p()
        self.device_ptrs = bool(device_ptrs)
        self.device = int(device)
        self._keep = []
        opt = Options()
        self._L.dynlp_default_options(ct.byref(opt))
        opt.device = int(device)
        opt.stream = ct.c_void_p(int(stream) if stream else 0)
        opt.ptrs_on_device = 1 if device_ptrs else 0
        opt.slack_factor = float(slack_factor)
        opt.reserve_vertices = int(reserve_vertices)
        opt.reserve_edges = int(reserve_edges)
        opt.time_kernels = 1 if time_kernels else 0
        opt.group_lanes = int(group_lanes)
        opt.binary_scalar = 1 if binary_scalar else 0
        opt.binned_rounds = int(binned_rounds)
        opt.ingest_chunk_edges = int(ingest_chunk_edges)
        opt.persistent_rounds = int(persistent_rounds)
        opt.persistent_spin_limit = int(persistent_spin_limit)
        if allocator is not None:
            # the callbacks must outlive the context
            self._alloc_cb = _ALLOC_FN(lambda nbytes, user: int(allocator.alloc(int(nbytes))) or None)
            self._dealloc_cb = _DEALLOC_FN(lambda ptr, user: allocator.free(int(ptr or 0)))
            opt.alloc = self._alloc_cb
            opt.dealloc = self._dealloc_cb
        nseeds = 0 if seed_vertex is None else int(len(seed_vertex))
        st = self._L.dynlp_create(ct.byref(self._h), int(n), self._in(row_ptr, np.int64), self._in(col, np.int32),
                                  self._in(w, np.float32), int(num_classes), nseeds, self._in(seed_vertex, np.int32),
                                  self._in(seed_class, np.int32), ct.byref(opt))
        self._keep.clear()
        if st != 0:
            msg = self._L.dynlp_last_error(None).decode()
            self._h = ct.c_void_p()
            raise DynLPError(st, msg)

    # -- marshalling -----------------------------------------------------------------------------
    def _in(self, a, dtype):
        """Pointer to an input array of the given dtype (host numpy or device torch)."""
        if a is None:
            return None
        if self.device_ptrs:
            if not _is_torch(a):
                raise TypeError("device_ptrs=True needs torch tensors on the GPU")
            import torch

            want = {np.int64: torch.int64, np.int32: torch.int32, np.float32: torch.float32}[dtype]
            if a.dtype != want or not a.is_cuda or not a.is_contiguous():
                raise TypeError(f"expected a contiguous CUDA tensor of {want}")
            self._keep.append(a)
            return ct.c_void_p(a.data_ptr()) if a.numel() else None
        arr = np.ascontiguousarray(a, dtype=dtype)
        self._keep.append(arr)
        return arr.ctypes.data_as(ct.c_void_p) if arr.size else None

    def _out(self, shape, dtype):
        if self.device_ptrs:
            import torch

            t = torch.empty(shape, dtype={np.int64: torch.int64, np.int32: torch.int32,
                                          np.float32: torch.float32}[dtype], device=f"cuda:{self.device}")
            return t, (ct.c_void_p(t.data_ptr()) if t.numel() else None)
        a = np.empty(shape, dtype=dtype)
        return a, (a.ctypes.data_as(ct.c_void_p) if a.size else None)

    def _check(self, st, ok=(0,)):
        if st not in ok:
            raise DynLPError(st, self._L.dynlp_last_error(self._h).decode())
        return st

    # -- the C entry points ----------------------------------------------------------------------
    def static_solve(self, tol, max_iter):
        """dynlp_static_solve.  Returns (status, Stats); status 1 = max_iter reached."""
        s = Stats()
        st = self._check(self._L.dynlp_static_solve(self._h, float(tol), int(max_iter), ct.byref(s)), ok=(0, 1))
        return st, s

    def set_params(self, tol, max_iter):
        self._check(self._L.dynlp_set_params(self._h, float(tol), int(max_iter)))

    def storage_info(self):
        """dynlp_storage_info.  Returns (pool entries in use, pool capacity)."""
        used, cap = ct.c_int64(0), ct.c_int64(0)
        self._check(self._L.dynlp_storage_info(self._h, ct.byref(used), ct.byref(cap)))
        return int(used.value), int(cap.value)

    def stream_bandwidth(self, nbytes=1 << 30, repetitions=10):
        """dynlp_stream_bandwidth: (GB/s of a plain copy, read + written; GB/s of a read-only pass)."""
        cp, rd = ct.c_double(0.0), ct.c_double(0.0)
        self._check(self._L.dynlp_stream_bandwidth(self._h, int(nbytes), int(repetitions), ct.byref(cp), ct.byref(rd)))
        return float(cp.value), float(rd.value)

    def gather_bandwidth(self, table_rows, row_bytes, gathers, repetitions=5):
        """dynlp_gather_bandwidth: (rows gathered per second, GB/s) for random whole-row reads of row_bytes bytes."""
        per_s, gbs = ct.c_double(0.0), ct.c_double(0.0)
        self._check(self._L.dynlp_gather_bandwidth(self._h, int(table_rows), int(row_bytes), int(gathers), int(repetitions),
                                                   ct.byref(per_s), ct.byref(gbs)))
        return float(per_s.value), float(gbs.value)

    def compact_storage(self):
        """dynlp_compact_storage."""
        self._check(self._L.dynlp_compact_storage(self._h))

    def set_update_mode(self, mode):
        """dynlp_set_update_mode: UPDATE_SYNCHRONOUS or UPDATE_IN_PLACE."""
        self._check(self._L.dynlp_set_update_mode(self._h, int(mode)))

    def set_final_check(self, on=True):
        """dynlp_set_final_check: end every batch with a round over all rows that moves none by more than tol."""
        self._check(self._L.dynlp_set_final_check(self._h, 1 if on else 0))

    def set_initialiser(self, mode, tau=0.0):
        """dynlp_set_initialiser: INIT_UNIFORM or INIT_SUPERNODE with threshold tau."""
        self._check(self._L.dynlp_set_initialiser(self._h, int(mode), float(tau)))

    def mean_edge_weight(self):
        """dynlp_mean_edge_weight."""
        out = ct.c_double(0.0)
        self._check(self._L.dynlp_mean_edge_weight(self._h, ct.byref(out)))
        return float(out.value)

    def last_components(self, want_comp=True):
        """dynlp_last_components.  Returns (comp [vertices] int32 or None, InitInfo)."""
        info = InitInfo()
        self._check(self._L.dynlp_last_components(self._h, 0, None, ct.byref(info)))
        if not want_comp or info.vertices == 0:
            return None, info
        comp, cp = self._out((int(info.vertices),), np.int32)
        self._check(self._L.dynlp_last_components(self._h, int(info.vertices), cp, ct.byref(info)))
        return comp, info

    def apply_batch(self, num_new_vertices, eu, ev, ew, seed_vertex=None, seed_class=None):
        """dynlp_apply_batch.  Returns (status, Stats)."""
        s = Stats()
        m = 0 if eu is None else int(len(eu))
        ns = 0 if seed_vertex is None else int(len(seed_vertex))
        st = self._L.dynlp_apply_batch(self._h, int(num_new_vertices), m, self._in(eu, np.int32),
                                       self._in(ev, np.int32), self._in(ew, np.float32), ns,
                                       self._in(seed_vertex, np.int32), self._in(seed_class, np.int32), ct.byref(s))
        self._keep.clear()
        self._check(st, ok=(0, 1))
        return st, s

    def apply_update(self, deleted_vertex, num_new_vertices=0, eu=None, ev=None, ew=None, seed_vertex=None,
                     seed_class=None):
        """dynlp_apply_update (deletions, then insertions).  Returns (status, Stats)."""
        s = Stats()
        nd = 0 if deleted_vertex is None else int(len(deleted_vertex))
        m = 0 if eu is None else int(len(eu))
        ns = 0 if seed_vertex is None else int(len(seed_vertex))
        st = self._L.dynlp_apply_update(self._h, nd, self._in(deleted_vertex, np.int32), int(num_new_vertices), m,
                                        self._in(eu, np.int32), self._in(ev, np.int32), self._in(ew, np.float32), ns,
                                        self._in(seed_vertex, np.int32), self._in(seed_class, np.int32), ct.byref(s))
        self._keep.clear()
        self._check(st, ok=(0, 1))
        return st, s

    def get_labels(self, soft=True, hard=True):
        """dynlp_get_labels.  Returns (soft [n, C] float32 or None, hard [n] int32 or None)."""
        n, C = self.num_vertices, self.num_classes
        so, sp = self._out((n, C), np.float32) if soft else (None, None)
        ho, hp = self._out((n,), np.int32) if hard else (None, None)
        self._check(self._L.dynlp_get_labels(self._h, sp, hp))
        return so, ho

    def get_labels_static(self, soft=True, hard=True):
        """dynlp_get_labels_static: as get_labels, but into host (numpy) arrays in either pointer mode and
        without any device allocation.  Returns (soft [n, C] float32 or None, hard [n] int32 or None)."""
        n, C = self.num_vertices, self.num_classes
        so = np.empty((n, C), dtype=np.float32) if soft else None
        ho = np.empty((n,), dtype=np.int32) if hard else None
        sp = so.ctypes.data_as(ct.c_void_p) if soft and so.size else None
        hp = ho.ctypes.data_as(ct.c_void_p) if hard and ho.size else None
        self._check(self._L.dynlp_get_labels_static(self._h, sp, hp))
        return so, ho

    @property
    def static_scratch_bytes(self):
        return int(self._L.dynlp_static_scratch_bytes())

    @property
    def num_vertices(self):
        return int(self._L.dynlp_num_vertices(self._h))

    @property
    def num_entries(self):
        return int(self._L.dynlp_num_entries(self._h))

    @property
    def num_classes(self):
        return int(self._L.dynlp_num_classes(self._h))

    def export_graph(self):
        """dynlp_export_graph.  Returns (row_ptr, col, w, degree, seed_class)."""
        n, nnz = self.num_vertices, self.num_entries
        rp, rpp = self._out((n + 1,), np.int64)
        col, colp = self._out((nnz,), np.int32)
        w, wp = self._out((nnz,), np.float32)
        deg, degp = self._out((n,), np.float32)
        sc, scp = self._out((n,), np.int32)
        self._check(self._L.dynlp_export_graph(self._h, rpp, colp, wp, degp, scp))
        return rp, col, w, deg, sc

    def round_log_full(self):
        """dynlp_round_log.  Returns the list of RoundInfo structures of the last solve / batch."""
        rounds = int(self._L.dynlp_round_log(self._h, 0, None))
        if rounds <= 0:
            return []
        buf = (RoundInfo * rounds)()
        self._L.dynlp_round_log(self._h, rounds, buf)
        return list(buf)

    def round_log(self, kernel_ms=False):
        """Per-round (frontier sizes int64, max change float32[, row-update device time in ms])."""
        info = self.round_log_full()
        sizes = np.array([r.rows_short + r.rows_long for r in info], dtype=np.int64)
        delta = np.array([r.max_delta for r in info], dtype=np.float32)
        if kernel_ms:
            return sizes, delta, np.array([r.ms_update for r in info], dtype=np.float32)
        return sizes, delta

    def destroy(self):
        if self._h:
            self._L.dynlp_destroy(self._h)
            self._h = ct.c_void_p()

    close = destroy

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()
