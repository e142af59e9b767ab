"""ctypes binding of libdgn: the same entry points as ``include/dgn.h``, argument marshalling only.

Device memory comes from PyTorch (``torch.empty(..., device="cuda")``) and the HIP stream from
``torch.cuda.current_stream()``; every step of the path runs in the library's kernels.  There is no
fallback: if ``libdgn.so`` has not been built the import fails.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_int, c_int32, c_int64, c_size_t, c_void_p

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdgn.so")

DGN_OK = 0
DGN_ERR_INVALID_ARG = -1
DGN_ERR_NULL_PTR = -2
DGN_ERR_TOO_LARGE = -3
DGN_ERR_ID_OUT_OF_RANGE = -4
DGN_ERR_TOO_MANY_SETS = -5
DGN_ERR_WORKSPACE_TOO_SMALL = -6
DGN_ERR_NOT_TOPOLOGICAL = -7
DGN_ERR_HIP = -8
DGN_ERR_BAD_CSR = -9

EXPORTS = [
    "dgn_graph_build_workspace", "dgn_graph_build", "dgn_graph_from_csr_workspace", "dgn_graph_from_csr",
    "dgn_graph_get_csr", "dgn_graph_get_sizes", "dgn_graph_destroy", "dgn_prune_workspace", "dgn_prune",
    "dgn_prune_words", "dgn_keep_compact", "dgn_keep_compact_static_limits", "dgn_keep_compact_static", "dgn_backward_prune_workspace", "dgn_backward_prune", "dgn_inplace_workspace",
    "dgn_inplace", "dgn_inplace_kept", "dgn_ignore_mask", "dgn_per_set_lists_workspace", "dgn_per_set_lists",
    "dgn_target_digest_workspace", "dgn_target_digest", "dgn_calibrate", "dgn_selftest_wave_ops", "dgn_strerror",
    "dgn_version",
    "dgn_last_hip_error",
]


class dgn_coo_desc(ctypes.Structure):
    _fields_ = [("num_ops", c_int64), ("num_tensors", c_int64), ("nnz_in", c_int64), ("nnz_out", c_int64),
                ("in_op", c_void_p), ("in_tensor", c_void_p), ("out_op", c_void_p), ("out_tensor", c_void_p),
                ("num_graphs", c_int32), ("graph_op_offsets", c_void_p), ("graph_tensor_offsets", c_void_p)]


class dgn_csr_desc(ctypes.Structure):
    _fields_ = [("num_ops", c_int64), ("num_tensors", c_int64), ("nnz_in", c_int64), ("nnz_out", c_int64),
                ("in_rowptr", c_void_p), ("in_idx", c_void_p), ("out_rowptr", c_void_p), ("out_idx", c_void_p),
                ("num_graphs", c_int32), ("graph_op_offsets", c_void_p), ("graph_tensor_offsets", c_void_p)]


class dgn_options(ctypes.Structure):
    _fields_ = [("validate", c_int32), ("recompute_keep", c_int32), ("traversal", c_int32),
                ("profile", c_int32), ("defer_percent", c_int32), ("max_queue_entries", c_int32),
                ("defer_start_shift", c_int32), ("defer_floor_shift", c_int32), ("incremental", c_int32),
                ("recycle", c_int32)]


class dgn_stats(ctypes.Structure):
    _fields_ = [("levels", c_int64), ("tensor_visits", c_int64), ("max_frontier", c_int64),
                ("launches", c_int64), ("level_launches", c_int64), ("level_trace", c_void_p),
                ("level_trace_cap", c_int64), ("reserved", c_int64), ("recycled", c_int64),
                ("atomic_updates", c_int64), ("phase_ms", ctypes.c_float * 8)]

class dgn_machine_rates(ctypes.Structure):
    _fields_ = [("random_load_gps", ctypes.c_float), ("random_atomic_gps", ctypes.c_float),
                ("random_store_gps", ctypes.c_float), ("dependent_load_ns", ctypes.c_float),
                ("dependent_atomic_ns", ctypes.c_float), ("same_address_atomic_ns", ctypes.c_float),
                ("launch_floor_us", ctypes.c_float), ("launch_back_to_back_us", ctypes.c_float),
                ("copy_gbs", ctypes.c_float), ("random_atomic_noreturn_gps", ctypes.c_float),
                ("random_load_and_atomic_gps", ctypes.c_float), ("run_atomic_gps", ctypes.c_float),
                ("reserved", ctypes.c_float * 4), ("buffer_bytes", c_int64)]

    def as_dict(self):
        return {n: round(float(getattr(self, n)), 3) for n, _ in self._fields_[:12]} | {"buffer_bytes": int(self.buffer_bytes)}


PHASES = ["clear", "seed", "traverse", "count", "scan", "scatter", "total"]


class DgnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {dgn_strerror(code)} ({code})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                          f"(python __graft_entry__.py at the repository root); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    lib.dgn_strerror.restype = c_char_p
    lib.dgn_strerror.argtypes = [c_int]
    lib.dgn_version.restype = c_int
    lib.dgn_last_hip_error.restype = c_int
    lib.dgn_graph_build_workspace.argtypes = [POINTER(dgn_coo_desc), POINTER(c_size_t), POINTER(c_size_t)]
    lib.dgn_graph_from_csr_workspace.argtypes = [POINTER(dgn_csr_desc), POINTER(c_size_t), POINTER(c_size_t)]
    lib.dgn_graph_build.argtypes = [POINTER(dgn_coo_desc), c_void_p, c_size_t, c_void_p, c_size_t,
                                    POINTER(dgn_options), c_void_p, POINTER(c_void_p)]
    lib.dgn_graph_from_csr.argtypes = [POINTER(dgn_csr_desc), c_void_p, c_size_t, c_void_p, c_size_t,
                                       POINTER(dgn_options), c_void_p, POINTER(c_void_p)]
    lib.dgn_graph_get_csr.argtypes = [c_void_p] + [POINTER(c_void_p)] * 6
    lib.dgn_graph_get_sizes.argtypes = [c_void_p] + [POINTER(c_int64)] * 4 + [POINTER(c_int32)]
    lib.dgn_graph_destroy.argtypes = [c_void_p]
    lib.dgn_graph_destroy.restype = None
    lib.dgn_prune_workspace.argtypes = [c_void_p, c_int32, POINTER(c_size_t)]
    lib.dgn_prune.argtypes = [c_void_p, c_int32, c_int64] + [c_void_p] * 9 + [c_void_p, c_size_t,
                              POINTER(dgn_options), POINTER(dgn_stats), c_void_p]
    lib.dgn_prune_words.argtypes = [c_void_p, c_int64, c_int64] + [c_void_p] * 9 + [c_void_p, c_size_t,
                                    POINTER(dgn_options), POINTER(dgn_stats), c_void_p]
    lib.dgn_keep_compact.argtypes = [c_void_p] + [c_void_p] * 7 + [c_void_p, c_size_t, c_void_p]
    lib.dgn_keep_compact_static.argtypes = [c_void_p] + [c_void_p] * 7 + [c_void_p]
    lib.dgn_keep_compact_static_limits.argtypes = [POINTER(c_int64), POINTER(c_size_t)]
    lib.dgn_backward_prune_workspace.argtypes = [c_void_p, POINTER(c_size_t)]
    lib.dgn_backward_prune.argtypes = [c_void_p, c_int32] + [c_void_p] * 9 + [c_void_p, c_size_t,
                                       POINTER(dgn_options), POINTER(dgn_stats), c_void_p]
    lib.dgn_ignore_mask.argtypes = [c_void_p] * 8
    lib.dgn_per_set_lists_workspace.argtypes = [c_int64, POINTER(c_size_t)]
    lib.dgn_per_set_lists.argtypes = [c_void_p, c_void_p, c_int64, c_void_p, c_void_p, c_int64, c_void_p, c_size_t,
                                      c_void_p]
    lib.dgn_target_digest_workspace.argtypes = [POINTER(c_size_t)]
    lib.dgn_target_digest.argtypes = [c_void_p, c_int32, c_int64, c_void_p, c_void_p, POINTER(ctypes.c_uint64), c_void_p,
                                      c_size_t, c_void_p]
    lib.dgn_calibrate.argtypes = [c_void_p, c_size_t, POINTER(dgn_machine_rates), c_void_p]
    lib.dgn_selftest_wave_ops.argtypes = [c_void_p, c_size_t, c_void_p]
    lib.dgn_inplace_workspace.argtypes = [c_void_p, POINTER(c_size_t)]
    lib.dgn_inplace.argtypes = [c_void_p, c_void_p, ctypes.c_uint64, c_void_p, c_void_p, c_void_p, c_size_t,
                                POINTER(c_int32), c_void_p]
    lib.dgn_inplace_kept.argtypes = [c_void_p, c_void_p, ctypes.c_uint64, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                     c_size_t, POINTER(c_int32), c_void_p]
    return lib


_lib = _load()


def _dp(t):
    """Device (or host) pointer of a tensor / numpy array, or NULL."""
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        return t.data_ptr() if t.numel() else None
    if isinstance(t, np.ndarray):
        return t.ctypes.data if t.size else None
    return int(t)


def _stream(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if isinstance(stream, torch.cuda.Stream) else int(stream)


def _check(rc: int, where: str):
    if rc != DGN_OK:
        raise DgnError(rc, where)


def dgn_strerror(code: int) -> str:
    return _lib.dgn_strerror(code).decode()


def dgn_version() -> int:
    return _lib.dgn_version()


def dgn_last_hip_error() -> int:
    return _lib.dgn_last_hip_error()


def make_coo_desc(num_ops, num_tensors, in_op, in_tensor, out_op, out_tensor, num_graphs=1,
                  graph_op_offsets=None, graph_tensor_offsets=None, nnz_in=None, nnz_out=None):
    """Fill a ``dgn_coo_desc``; offsets are HOST int64 numpy arrays (kept alive by the caller)."""
    d = dgn_coo_desc()
    d.num_ops, d.num_tensors = num_ops, num_tensors
    d.nnz_in = int(in_op.numel()) if nnz_in is None else nnz_in
    d.nnz_out = int(out_op.numel()) if nnz_out is None else nnz_out
    d.in_op, d.in_tensor, d.out_op, d.out_tensor = _dp(in_op), _dp(in_tensor), _dp(out_op), _dp(out_tensor)
    d.num_graphs = num_graphs
    d.graph_op_offsets, d.graph_tensor_offsets = _dp(graph_op_offsets), _dp(graph_tensor_offsets)
    return d


def make_csr_desc(num_ops, num_tensors, in_rowptr, in_idx, out_rowptr, out_idx, num_graphs=1,
                  graph_op_offsets=None, graph_tensor_offsets=None):
    d = dgn_csr_desc()
    d.num_ops, d.num_tensors = num_ops, num_tensors
    d.nnz_in, d.nnz_out = int(in_idx.numel()), int(out_idx.numel())
    d.in_rowptr, d.in_idx, d.out_rowptr, d.out_idx = _dp(in_rowptr), _dp(in_idx), _dp(out_rowptr), _dp(out_idx)
    d.num_graphs = num_graphs
    d.graph_op_offsets, d.graph_tensor_offsets = _dp(graph_op_offsets), _dp(graph_tensor_offsets)
    return d


def dgn_graph_build_workspace(desc: dgn_coo_desc):
    g, s = c_size_t(0), c_size_t(0)
    rc = _lib.dgn_graph_build_workspace(ctypes.byref(desc) if desc is not None else None, ctypes.byref(g),
                                        ctypes.byref(s))
    return rc, g.value, s.value


def dgn_graph_from_csr_workspace(desc: dgn_csr_desc):
    g, s = c_size_t(0), c_size_t(0)
    rc = _lib.dgn_graph_from_csr_workspace(ctypes.byref(desc) if desc is not None else None, ctypes.byref(g),
                                           ctypes.byref(s))
    return rc, g.value, s.value


def _opt(options):
    return ctypes.byref(options) if options is not None else None


def dgn_graph_build(desc, graph_mem, graph_bytes, scratch, scratch_bytes, options=None, stream=None):
    """Returns (rc, handle)."""
    h = c_void_p(None)
    rc = _lib.dgn_graph_build(ctypes.byref(desc), _dp(graph_mem), graph_bytes, _dp(scratch), scratch_bytes,
                              _opt(options), _stream(stream), ctypes.byref(h))
    return rc, h.value


def dgn_graph_from_csr(desc, graph_mem, graph_bytes, scratch, scratch_bytes, options=None, stream=None):
    h = c_void_p(None)
    rc = _lib.dgn_graph_from_csr(ctypes.byref(desc), _dp(graph_mem), graph_bytes, _dp(scratch), scratch_bytes,
                                 _opt(options), _stream(stream), ctypes.byref(h))
    return rc, h.value


def dgn_graph_get_csr(handle):
    """Returns (rc, dict of raw device addresses)."""
    ptrs = [c_void_p(None) for _ in range(6)]
    rc = _lib.dgn_graph_get_csr(handle, *[ctypes.byref(p) for p in ptrs])
    names = ["in_rowptr", "in_idx", "out_rowptr", "out_idx", "prod_rowptr", "prod_idx"]
    return rc, {n: p.value for n, p in zip(names, ptrs)}


def dgn_graph_get_sizes(handle):
    v = [c_int64(0) for _ in range(4)]
    g = c_int32(0)
    rc = _lib.dgn_graph_get_sizes(handle, *[ctypes.byref(x) for x in v], ctypes.byref(g))
    return rc, dict(num_ops=v[0].value, num_tensors=v[1].value, nnz_in=v[2].value, nnz_out=v[3].value,
                    num_graphs=g.value)


def dgn_graph_destroy(handle):
    _lib.dgn_graph_destroy(handle)


def dgn_prune_workspace(handle, num_sets: int):
    s = c_size_t(0)
    rc = _lib.dgn_prune_workspace(handle, num_sets, ctypes.byref(s))
    return rc, s.value


def dgn_prune(handle, num_sets, num_targets, tgt_rowptr, tgt_idx, tensor_mask, op_mask, op_flag, kept_ops,
              kept_masks, kept_count, per_query_count, scratch, scratch_bytes, options=None, stats=None,
              stream=None) -> int:
    return _lib.dgn_prune(handle, num_sets, num_targets, _dp(tgt_rowptr), _dp(tgt_idx), _dp(tensor_mask),
                          _dp(op_mask), _dp(op_flag), _dp(kept_ops), _dp(kept_masks), _dp(kept_count),
                          _dp(per_query_count), _dp(scratch), scratch_bytes, _opt(options),
                          ctypes.byref(stats) if stats is not None else None, _stream(stream))


def dgn_prune_words(handle, num_sets, num_targets, tgt_rowptr, tgt_idx, tensor_mask, op_mask, op_flag, kept_ops,
                    kept_masks, kept_count, per_query_count, scratch, scratch_bytes, options=None, stats=None,
                    stream=None) -> int:
    return _lib.dgn_prune_words(handle, num_sets, num_targets, _dp(tgt_rowptr), _dp(tgt_idx), _dp(tensor_mask),
                                _dp(op_mask), _dp(op_flag), _dp(kept_ops), _dp(kept_masks), _dp(kept_count),
                                _dp(per_query_count), _dp(scratch), scratch_bytes, _opt(options),
                                ctypes.byref(stats) if stats is not None else None, _stream(stream))


def dgn_keep_compact(handle, tensor_mask_in, op_mask, op_flag, kept_ops, kept_masks, kept_count,
                     per_query_count, scratch, scratch_bytes, stream=None) -> int:
    return _lib.dgn_keep_compact(handle, _dp(tensor_mask_in), _dp(op_mask), _dp(op_flag), _dp(kept_ops),
                                 _dp(kept_masks), _dp(kept_count), _dp(per_query_count), _dp(scratch),
                                 scratch_bytes, _stream(stream))


def dgn_keep_compact_static_limits():
    """Returns (return code, largest num_ops, bytes of the library's static device array)."""
    m, b = c_int64(0), c_size_t(0)
    rc = _lib.dgn_keep_compact_static_limits(ctypes.byref(m), ctypes.byref(b))
    return rc, m.value, b.value


def dgn_keep_compact_static(handle, tensor_mask_in, op_mask, op_flag, kept_ops, kept_masks, kept_count,
                            per_query_count, stream=None) -> int:
    return _lib.dgn_keep_compact_static(handle, _dp(tensor_mask_in), _dp(op_mask), _dp(op_flag), _dp(kept_ops),
                                        _dp(kept_masks), _dp(kept_count), _dp(per_query_count), _stream(stream))


def dgn_backward_prune_workspace(handle):
    s = c_size_t(0)
    rc = _lib.dgn_backward_prune_workspace(handle, ctypes.byref(s))
    return rc, s.value


def dgn_backward_prune(handle, num_pairs, obj, wrt, tensor_mask, op_mask, op_flag, kept_ops, kept_masks,
                       kept_count, per_query_count, scratch, scratch_bytes, options=None, stats=None,
                       stream=None) -> int:
    return _lib.dgn_backward_prune(handle, num_pairs, _dp(obj), _dp(wrt), _dp(tensor_mask), _dp(op_mask),
                                   _dp(op_flag), _dp(kept_ops), _dp(kept_masks), _dp(kept_count),
                                   _dp(per_query_count), _dp(scratch), scratch_bytes, _opt(options),
                                   ctypes.byref(stats) if stats is not None else None, _stream(stream))


def dgn_ignore_mask(handle, tensor_mask, kept_ops, kept_masks, kept_count, ignore_mask, ignore_count,
                    stream=None) -> int:
    return _lib.dgn_ignore_mask(handle, _dp(tensor_mask), _dp(kept_ops), _dp(kept_masks), _dp(kept_count),
                                _dp(ignore_mask), _dp(ignore_count), _stream(stream))


def dgn_per_set_lists_workspace(num_kept: int):
    s = c_size_t(0)
    rc = _lib.dgn_per_set_lists_workspace(num_kept, ctypes.byref(s))
    return rc, s.value


def dgn_per_set_lists(kept_ops, kept_masks, num_kept, set_rowptr, set_ops, set_ops_capacity, scratch,
                      scratch_bytes, stream=None) -> int:
    return _lib.dgn_per_set_lists(_dp(kept_ops), _dp(kept_masks), num_kept, _dp(set_rowptr), _dp(set_ops),
                                  set_ops_capacity, _dp(scratch), scratch_bytes, _stream(stream))


def dgn_target_digest_workspace():
    s = c_size_t(0)
    rc = _lib.dgn_target_digest_workspace(ctypes.byref(s))
    return rc, s.value


def dgn_target_digest(handle, num_sets, num_targets, tgt_rowptr, tgt_idx, scratch, scratch_bytes, stream=None):
    """Returns (return code, (digest word 0, digest word 1))."""
    out = (ctypes.c_uint64 * 2)()
    rc = _lib.dgn_target_digest(handle, num_sets, num_targets, _dp(tgt_rowptr), _dp(tgt_idx), out, _dp(scratch),
                                scratch_bytes, _stream(stream))
    return rc, (int(out[0]), int(out[1]))


def dgn_selftest_wave_ops(buffer, nbytes, stream=None) -> int:
    return int(_lib.dgn_selftest_wave_ops(_dp(buffer), nbytes, _stream(stream)))


def dgn_calibrate(buffer, nbytes, stream=None):
    """Returns (return code, dgn_machine_rates)."""
    out = dgn_machine_rates()
    rc = _lib.dgn_calibrate(_dp(buffer), nbytes, ctypes.byref(out), _stream(stream))
    return rc, out


def dgn_inplace_workspace(handle):
    s = c_size_t(0)
    rc = _lib.dgn_inplace_workspace(handle, ctypes.byref(s))
    return rc, s.value


def dgn_inplace(handle, op_mask, select, rename, renamed_count, scratch, scratch_bytes, stream=None):
    """Returns (return code, pointer-doubling rounds run)."""
    rounds = c_int32(0)
    rc = _lib.dgn_inplace(handle, _dp(op_mask), ctypes.c_uint64(select & (2**64 - 1)), _dp(rename),
                          _dp(renamed_count), _dp(scratch), scratch_bytes, ctypes.byref(rounds), _stream(stream))
    return rc, rounds.value


def dgn_inplace_kept(handle, op_mask, select, kept_ops, kept_count, rename, renamed_count, scratch, scratch_bytes,
                     stream=None):
    """Returns (return code, pointer-doubling rounds run)."""
    rounds = c_int32(0)
    rc = _lib.dgn_inplace_kept(handle, _dp(op_mask), ctypes.c_uint64(select & (2**64 - 1)), _dp(kept_ops), _dp(kept_count),
                               _dp(rename), _dp(renamed_count), _dp(scratch), scratch_bytes, ctypes.byref(rounds),
                               _stream(stream))
    return rc, rounds.value


# ------------------------------------------------------------------------------------------------
# Buffer owners (allocation and marshalling only -- no arithmetic of the method happens here)
# ------------------------------------------------------------------------------------------------
def _view(addr, count, dtype, keep):
    """Wrap ``count`` elements at raw device address ``addr`` inside the tensor ``keep``."""
    if count == 0:
        return torch.empty(0, dtype=dtype, device=keep.device)
    off = addr - keep.data_ptr()
    nbytes = count * torch.empty(0, dtype=dtype).element_size()
    return keep[off:off + nbytes].view(dtype)


class DeviceGraph:
    """Owns graph_mem for one built graph; frees the handle on ``close()``."""

    def __init__(self, handle, graph_mem, keep_alive, sizes):
        self.handle = handle
        self.graph_mem = graph_mem
        self._keep = keep_alive
        self.__dict__.update(sizes)

    @classmethod
    def from_coo(cls, g, validate=False, device="cuda"):
        """``g``: any object with the fields of ``graphgen.Graph`` (host numpy arrays)."""
        dev = torch.device(device)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
        in_op, in_t, out_op, out_t = t(g.in_op), t(g.in_tensor), t(g.out_op), t(g.out_tensor)
        oo = None if g.graph_op_offsets is None else np.ascontiguousarray(g.graph_op_offsets, dtype=np.int64)
        to = None if g.graph_tensor_offsets is None else np.ascontiguousarray(g.graph_tensor_offsets, dtype=np.int64)
        desc = make_coo_desc(g.num_ops, g.num_tensors, in_op, in_t, out_op, out_t, g.num_graphs, oo, to)
        rc, gb, sb = dgn_graph_build_workspace(desc)
        _check(rc, "dgn_graph_build_workspace")
        graph_mem = torch.empty(gb, dtype=torch.uint8, device=dev)
        scratch = torch.empty(sb, dtype=torch.uint8, device=dev)
        opts = dgn_options(validate=1 if validate else 0)
        rc, h = dgn_graph_build(desc, graph_mem, gb, scratch, sb, opts)
        _check(rc, "dgn_graph_build")
        del scratch
        rc, sizes = dgn_graph_get_sizes(h)
        _check(rc, "dgn_graph_get_sizes")
        return cls(h, graph_mem, (), sizes)

    @classmethod
    def from_csr(cls, num_ops, num_tensors, in_rowptr, in_idx, out_rowptr, out_idx, num_graphs=1,
                 graph_op_offsets=None, graph_tensor_offsets=None, validate=False):
        """CSR arrays are device int32 tensors, borrowed for the life of the graph."""
        desc = make_csr_desc(num_ops, num_tensors, in_rowptr, in_idx, out_rowptr, out_idx, num_graphs,
                             graph_op_offsets, graph_tensor_offsets)
        rc, gb, sb = dgn_graph_from_csr_workspace(desc)
        _check(rc, "dgn_graph_from_csr_workspace")
        dev = in_rowptr.device
        graph_mem = torch.empty(gb, dtype=torch.uint8, device=dev)
        scratch = torch.empty(sb, dtype=torch.uint8, device=dev)
        opts = dgn_options(validate=1 if validate else 0)
        rc, h = dgn_graph_from_csr(desc, graph_mem, gb, scratch, sb, opts)
        _check(rc, "dgn_graph_from_csr")
        rc, sizes = dgn_graph_get_sizes(h)
        _check(rc, "dgn_graph_get_sizes")
        return cls(h, graph_mem, (in_rowptr, in_idx, out_rowptr, out_idx), sizes)

    def csr(self):
        """The built adjacency as int32 tensors (views into graph_mem; borrowed arrays are returned as given)."""
        rc, p = dgn_graph_get_csr(self.handle)
        _check(rc, "dgn_graph_get_csr")
        P, T, Ein, Eout = self.num_ops, self.num_tensors, self.nnz_in, self.nnz_out
        out = {}
        if self._keep:
            out["in_rowptr"], out["in_idx"], out["out_rowptr"], out["out_idx"] = self._keep
        else:
            out["in_rowptr"] = _view(p["in_rowptr"], P + 1, torch.int32, self.graph_mem)
            out["in_idx"] = _view(p["in_idx"], Ein, torch.int32, self.graph_mem)
            out["out_rowptr"] = _view(p["out_rowptr"], P + 1, torch.int32, self.graph_mem)
            out["out_idx"] = _view(p["out_idx"], Eout, torch.int32, self.graph_mem)
        out["prod_rowptr"] = _view(p["prod_rowptr"], T + 1, torch.int32, self.graph_mem)
        out["prod_idx"] = _view(p["prod_idx"], Eout, torch.int32, self.graph_mem)
        return out

    def close(self):
        if self.handle:
            dgn_graph_destroy(self.handle)
            self.handle = None

    def __del__(self):
        self.close()


class PruneBuffers:
    """All caller-owned buffers of one ``dgn_prune`` call, allocated once and reusable."""

    def __init__(self, graph: DeviceGraph, num_sets: int, device=None, recycle: bool = True):
        """``recycle``: from the second ``prune`` on, tell the library that these buffers still hold what the
        previous call wrote (``dgn_options.recycle``), so that it zeroes only that instead of everything.
        The outputs are then read-only for the caller; pass ``False`` to write to them between calls."""
        dev = graph.graph_mem.device if device is None else torch.device(device)
        P, T, G = graph.num_ops, graph.num_tensors, graph.num_graphs
        self.recycle, self._scratch_defined = bool(recycle), False
        rc, sb = dgn_prune_workspace(graph.handle, num_sets)
        _check(rc, "dgn_prune_workspace")
        self.graph, self.num_sets = graph, num_sets
        self.scratch_bytes = sb
        self.scratch = torch.empty(sb, dtype=torch.uint8, device=dev)
        # int64 storage for the 64-bit masks (torch has no general uint64 support); bit patterns are what matter
        self.tensor_mask = torch.empty(T, dtype=torch.int64, device=dev)
        self.op_mask = torch.empty(P, dtype=torch.int64, device=dev)
        self.op_flag = torch.empty(P, dtype=torch.uint8, device=dev)
        self.kept_ops = torch.empty(P, dtype=torch.int32, device=dev)
        self.kept_masks = torch.empty(P, dtype=torch.int64, device=dev)
        self.kept_count = torch.empty(1 + (G + 1 if G > 1 else 0), dtype=torch.int64, device=dev)
        self.per_query_count = torch.empty(64 * (G if G > 1 else 1), dtype=torch.int64, device=dev)

    def prune(self, tgt_rowptr, tgt_idx, options=None, stats=None, stream=None) -> int:
        """``tgt_rowptr`` / ``tgt_idx``: device int32 tensors. Returns the library's return code."""
        if options is not None:
            options = dgn_options.from_buffer_copy(options)      # the caller's object stays as it is
            options.recycle = 0
        if self.recycle and self._scratch_defined:
            if options is None:
                options = dgn_options()
            options.recycle = 1
        rc = dgn_prune(self.graph.handle, self.num_sets, int(tgt_idx.numel()), tgt_rowptr, tgt_idx,
                       self.tensor_mask, self.op_mask, self.op_flag, self.kept_ops, self.kept_masks,
                       self.kept_count, self.per_query_count, self.scratch, self.scratch_bytes, options,
                       stats, stream)
        self._scratch_defined = rc == DGN_OK  # after an error everything is cleared next time
        return rc

    def keep_compact(self, tensor_mask_in, stream=None) -> int:
        self._scratch_defined = False         # op_mask no longer goes with the log of the last prune
        return dgn_keep_compact(self.graph.handle, tensor_mask_in, self.op_mask, self.op_flag, self.kept_ops,
                                self.kept_masks, self.kept_count, self.per_query_count, self.scratch,
                                self.scratch_bytes, stream)

    def to_host(self):
        """Copy every output to numpy (uint64 views of the masks)."""
        torch.cuda.synchronize()
        n = int(self.kept_count[0].item())
        u = lambda t: t.cpu().numpy().view(np.uint64)
        return dict(tensor_mask=u(self.tensor_mask), op_mask=u(self.op_mask), op_flag=self.op_flag.cpu().numpy(),
                    kept_ops=self.kept_ops[:n].cpu().numpy(), kept_masks=u(self.kept_masks[:n]),
                    kept_count=self.kept_count.cpu().numpy(), per_query_count=self.per_query_count.cpu().numpy())


class TransactionCache:
    """Results of ``dgn_prune`` kept by (graph, number of sets, digest of the target sets) -- the transactions of
    Sec. 4.1 of the paper: asking again for a function that exists builds nothing new.  The digest is computed on
    the device (``dgn_target_digest``); a hit costs that and a dictionary look-up, a miss prunes into the least
    recently used of at most ``capacity`` buffer sets.  Buffers handed out stay valid until ``capacity`` other
    target sets have been asked for since."""

    def __init__(self, graph: DeviceGraph, num_sets: int, capacity: int = 2, device=None):
        self.graph, self.num_sets, self.capacity = graph, num_sets, max(1, int(capacity))
        self._device = device
        self._entries = {}                    # digest -> PruneBuffers, oldest first
        rc, sb = dgn_target_digest_workspace()
        _check(rc, "dgn_target_digest_workspace")
        dev = graph.graph_mem.device if device is None else torch.device(device)
        self._scratch, self._scratch_bytes = torch.empty(sb, dtype=torch.uint8, device=dev), sb
        self.hits = self.misses = 0

    def digest(self, tgt_rowptr, tgt_idx, stream=None):
        rc, d = dgn_target_digest(self.graph.handle, self.num_sets, int(tgt_idx.numel()), tgt_rowptr, tgt_idx,
                                  self._scratch, self._scratch_bytes, stream)
        _check(rc, "dgn_target_digest")
        return d

    def prune(self, tgt_rowptr, tgt_idx, options=None, stream=None) -> "PruneBuffers":
        """The buffers that hold the result for these target sets (pruned now, or found)."""
        key = self.digest(tgt_rowptr, tgt_idx, stream)
        buf = self._entries.pop(key, None)
        if buf is not None:
            self.hits += 1
        else:
            self.misses += 1
            if len(self._entries) >= self.capacity:
                _, buf = next(iter(self._entries.items()))            # least recently used: its buffers are recycled
                del self._entries[next(iter(self._entries))]
            else:
                buf = PruneBuffers(self.graph, self.num_sets, self._device)
            _check(buf.prune(tgt_rowptr, tgt_idx, options=options, stream=stream), "dgn_prune")
        self._entries[key] = buf                                       # most recently used last
        return buf


class InplaceBuffers:
    """Caller-owned buffers of one ``dgn_inplace`` call (rename dictionary, count, scratch)."""

    def __init__(self, graph: DeviceGraph, device=None):
        dev = graph.graph_mem.device if device is None else torch.device(device)
        rc, sb = dgn_inplace_workspace(graph.handle)
        _check(rc, "dgn_inplace_workspace")
        self.graph = graph
        self.scratch_bytes = sb
        self.scratch = torch.empty(sb, dtype=torch.uint8, device=dev)
        self.rename = torch.empty(graph.num_tensors, dtype=torch.int32, device=dev)
        self.renamed_count = torch.empty(1, dtype=torch.int64, device=dev)
        self.rounds = 0

    def run(self, op_mask, select: int = 2**64 - 1, stream=None, kept_ops=None, kept_count=None) -> int:
        """``op_mask``: device int64 tensor holding K (as written by ``PruneBuffers.prune``); with ``kept_ops`` and
        ``kept_count`` of the same prune the pass visits the kept operators only."""
        if kept_ops is not None and kept_count is not None:
            rc, self.rounds = dgn_inplace_kept(self.graph.handle, op_mask, select, kept_ops, kept_count, self.rename,
                                               self.renamed_count, self.scratch, self.scratch_bytes, stream)
        else:
            rc, self.rounds = dgn_inplace(self.graph.handle, op_mask, select, self.rename, self.renamed_count,
                                          self.scratch, self.scratch_bytes, stream)
        return rc


class BackwardPruneBuffers(PruneBuffers):
    """Buffers of one ``dgn_backward_prune`` call: the same outputs as ``PruneBuffers``, larger scratch."""

    def __init__(self, graph: DeviceGraph, num_pairs: int = 64, device=None, recycle: bool = True):
        super().__init__(graph, num_pairs, device, recycle)
        self._backward_defined = False        # the scratch buffer was last written by backward_prune
        rc, sb = dgn_backward_prune_workspace(graph.handle)
        _check(rc, "dgn_backward_prune_workspace")
        self.scratch_bytes = sb
        self.scratch = torch.empty(sb, dtype=torch.uint8, device=self.scratch.device)

    def prune(self, *args, **kwargs) -> int:
        self._backward_defined = False        # an ordinary prune lays the scratch buffer out its own way
        return super().prune(*args, **kwargs)

    def keep_compact(self, *args, **kwargs) -> int:
        self._backward_defined = False
        return super().keep_compact(*args, **kwargs)

    def backward_prune(self, obj, wrt, options=None, stats=None, stream=None) -> int:
        """``obj`` / ``wrt``: device int32 tensors of equal length (the pairs)."""
        self._scratch_defined = False         # the scratch buffer is laid out differently by this call
        if options is not None:
            options = dgn_options.from_buffer_copy(options)
            options.recycle = 0
        if self.recycle and self._backward_defined:
            if options is None:
                options = dgn_options()
            options.recycle = 1
        rc = dgn_backward_prune(self.graph.handle, int(obj.numel()), obj, wrt, self.tensor_mask, self.op_mask,
                                self.op_flag, self.kept_ops, self.kept_masks, self.kept_count,
                                self.per_query_count, self.scratch, self.scratch_bytes, options, stats, stream)
        self._backward_defined = rc == DGN_OK     # after an error everything is cleared next time
        return rc


class ReadoutBuffers:
    """Buffers for ``dgn_ignore_mask`` and ``dgn_per_set_lists`` on the result held by a ``PruneBuffers``."""

    def __init__(self, result: PruneBuffers):
        dev = result.tensor_mask.device
        self.result = result
        self.ignore_mask = torch.empty(result.graph.num_tensors, dtype=torch.int64, device=dev)
        self.ignore_count = torch.empty(1, dtype=torch.int64, device=dev)
        self.set_rowptr = torch.empty(65, dtype=torch.int64, device=dev)
        self.set_ops = None
        self._scratch = None

    def ignore(self, stream=None) -> int:
        r = self.result
        return dgn_ignore_mask(r.graph.handle, r.tensor_mask, r.kept_ops, r.kept_masks, r.kept_count,
                               self.ignore_mask, self.ignore_count, stream)

    def per_set_lists(self, stream=None) -> int:
        """Sizes ``set_ops`` from the result's counts (two small read-backs), then runs the call."""
        r = self.result
        num_kept = int(r.kept_count[0].item())
        total = int(r.per_query_count.sum().item())
        rc, sb = dgn_per_set_lists_workspace(num_kept)
        if rc:
            return rc
        if self._scratch is None or self._scratch.numel() < sb:
            self._scratch = torch.empty(sb, dtype=torch.uint8, device=self.set_rowptr.device)
        if self.set_ops is None or self.set_ops.numel() < max(total, 1):
            self.set_ops = torch.empty(max(total, 1), dtype=torch.int32, device=self.set_rowptr.device)
        return dgn_per_set_lists(r.kept_ops, r.kept_masks, num_kept, self.set_rowptr, self.set_ops, total,
                                 self._scratch, self._scratch.numel(), stream)
