"""ctypes front end of the CPU oracle (``forward_prune.c``, ``backward_prune.c``, ``inplace.c``,
``postprocess.c``, ``transaction.c``) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the bench's ``cpu_baseline`` leg may import this package; the
product path never does.  It imports nothing from the GPU package.

Every function here is a thin marshalling layer: all arithmetic is in the C files, which follow
Algorithm 1, the removal rule of Sec. 2.1, the creation-order rule of Sec. 3.2, Algorithm 2
(Sec. 2.3) and Algorithm 3 (Sec. 2.4) of the paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("forward_prune.c", "backward_prune.c", "inplace.c",
                                             "postprocess.c", "transaction.c")]
_LIB = os.path.join(_HERE, "liboracle.so")
_LIB_SAN = os.path.join(_HERE, "liboracle_san.so")
_lib = None


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no threading).  ``sanitize``: a second library built with
    AddressSanitizer and UndefinedBehaviorSanitizer (any finding aborts the process); a process that loads it must
    have been started with the ASan runtime preloaded (see ``tests/test_oracle_sanitized.py``)."""
    lib = _LIB_SAN if sanitize else _LIB
    flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] \
        if sanitize else ["-O2"]
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < max(os.path.getmtime(f) for f in _SRCS):
        tmp = lib + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *flags, "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", *_SRCS, "-o", tmp])
        os.replace(tmp, lib)
    return lib


def _load():
    global _lib
    if _lib is None:
        # ORACLE_SANITIZE=1: run on the sanitizer build (the oracle's own arithmetic is the same source)
        _lib = ctypes.CDLL(build(sanitize=os.environ.get("ORACLE_SANITIZE") == "1"))
        _lib.orc_certificate.restype = ctypes.c_int64
        _lib.orc_child_sets.restype = ctypes.c_int64
        _lib.orc_per_set_lists.restype = ctypes.c_int64
        _lib.orc_mix64.restype = ctypes.c_uint64
        _lib.orc_mix64.argtypes = [ctypes.c_uint64]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


i64 = ctypes.c_int64
i32 = ctypes.c_int32


@dataclass
class Adjacency:
    num_ops: int
    num_tensors: int
    in_rowptr: np.ndarray
    in_idx: np.ndarray
    out_rowptr: np.ndarray
    out_idx: np.ndarray
    prod_rowptr: np.ndarray
    prod_idx: np.ndarray


def build_csr(n_rows: int, row, col):
    row, col = _c(row, np.int32), _c(col, np.int32)
    rowptr = np.empty(n_rows + 1, np.int32)
    idx = np.empty(row.shape[0], np.int32)
    rc = _load().orc_build_csr(i64(n_rows), i64(row.shape[0]), _p(row), _p(col), _p(rowptr), _p(idx))
    if rc:
        raise ValueError("orc_build_csr: id out of range")
    return rowptr, idx


def build_adjacency(num_ops, num_tensors, in_op, in_tensor, out_op, out_tensor) -> Adjacency:
    in_rowptr, in_idx = build_csr(num_ops, in_op, in_tensor)
    out_rowptr, out_idx = build_csr(num_ops, out_op, out_tensor)
    prod_rowptr = np.empty(num_tensors + 1, np.int32)
    prod_idx = np.empty(out_idx.shape[0], np.int32)
    rc = _load().orc_build_producers(i64(num_ops), i64(num_tensors), _p(out_rowptr), _p(out_idx),
                                     _p(prod_rowptr), _p(prod_idx))
    if rc:
        raise ValueError("orc_build_producers: tensor id out of range")
    return Adjacency(num_ops, num_tensors, in_rowptr, in_idx, out_rowptr, out_idx, prod_rowptr, prod_idx)


def mark(adj: Adjacency, num_sets: int, tgt_rowptr, tgt_idx, M: Optional[np.ndarray] = None):
    """Algorithm 1 for every target set; returns (M, parent_edges_per_set)."""
    tgt_rowptr, tgt_idx = _c(tgt_rowptr, np.int32), _c(tgt_idx, np.int32)
    total = tgt_rowptr.shape[0] - 1
    if M is None:
        M = np.zeros(adj.num_tensors, np.uint64)
    edges = np.zeros(total, np.int64)
    rc = _load().orc_forward_prune(i64(adj.num_ops), i64(adj.num_tensors), _p(adj.in_rowptr),
                                   _p(adj.in_idx), _p(adj.prod_rowptr), _p(adj.prod_idx), i64(total),
                                   i32(num_sets), _p(tgt_rowptr), _p(tgt_idx), _p(M), _p(edges))
    if rc:
        raise ValueError("orc_forward_prune: bad argument")
    return M, edges


def keep(adj: Adjacency, M: np.ndarray):
    K = np.empty(adj.num_ops, np.uint64)
    flag = np.empty(adj.num_ops, np.uint8)
    _load().orc_keep(i64(adj.num_ops), _p(adj.out_rowptr), _p(adj.out_idx), _p(M), _p(K), _p(flag))
    return K, flag


def compact(K: np.ndarray, num_graphs: int = 1, graph_op_offsets=None):
    P = K.shape[0]
    batched = num_graphs > 1 and graph_op_offsets is not None
    kept_ops = np.empty(P, np.int32)
    kept_masks = np.empty(P, np.uint64)
    kept_count = np.zeros(1 + (num_graphs + 1 if batched else 0), np.int64)
    pq = np.zeros(64 * (num_graphs if batched else 1), np.int64)
    off = _c(graph_op_offsets, np.int64) if batched else None
    _load().orc_compact(i64(P), _p(K), i32(num_graphs), _p(off), _p(kept_ops), _p(kept_masks),
                        _p(kept_count), _p(pq))
    n = int(kept_count[0])
    return kept_ops[:n].copy(), kept_masks[:n].copy(), kept_count, pq


def seed_masks(num_tensors: int, num_sets: int, tgt_rowptr, tgt_idx) -> np.ndarray:
    tgt_rowptr, tgt_idx = _c(tgt_rowptr, np.int32), _c(tgt_idx, np.int32)
    S = np.zeros(num_tensors, np.uint64)
    rc = _load().orc_seed_masks(i64(num_tensors), i64(tgt_rowptr.shape[0] - 1), i32(num_sets),
                                _p(tgt_rowptr), _p(tgt_idx), _p(S))
    if rc:
        raise ValueError("orc_seed_masks: target id out of range")
    return S


def reverse_sweep(adj: Adjacency, S: np.ndarray):
    M = S.copy()
    K = np.empty(adj.num_ops, np.uint64)
    _load().orc_reverse_sweep(i64(adj.num_ops), _p(adj.in_rowptr), _p(adj.in_idx), _p(adj.out_rowptr),
                              _p(adj.out_idx), _p(M), _p(K))
    return M, K


def certificate(adj: Adjacency, S: np.ndarray, M: np.ndarray, K: np.ndarray) -> int:
    """Number of violated fixed-point equations (0 proves M, K correct on a DAG)."""
    R = S.copy()
    return int(_load().orc_certificate(i64(adj.num_ops), i64(adj.num_tensors), _p(adj.in_rowptr),
                                       _p(adj.in_idx), _p(adj.out_rowptr), _p(adj.out_idx),
                                       _p(_c(M, np.uint64)), _p(_c(K, np.uint64)), _p(R)))


@dataclass
class PruneResult:
    tensor_mask: np.ndarray      # M  [T] uint64
    op_mask: np.ndarray          # K  [P] uint64
    op_flag: np.ndarray          # [P] uint8
    kept_ops: np.ndarray         # ascending operator ids
    kept_masks: np.ndarray
    kept_count: np.ndarray       # [1] or [1 + G + 1]
    per_query_count: np.ndarray  # [64] or [G*64]
    parent_edges: np.ndarray


def forward_prune(adj: Adjacency, num_sets: int, tgt_rowptr, tgt_idx, num_graphs: int = 1,
                  graph_op_offsets=None) -> PruneResult:
    """Whole path: Algorithm 1 per set, removal rule, ordered compaction."""
    M, edges = mark(adj, num_sets, tgt_rowptr, tgt_idx)
    K, flag = keep(adj, M)
    kept_ops, kept_masks, kept_count, pq = compact(K, num_graphs, graph_op_offsets)
    return PruneResult(M, K, flag, kept_ops, kept_masks, kept_count, pq, edges)


def child_sets(adj: Adjacency, K: np.ndarray, select: int = 2**64 - 1):
    """Child(x) of every tensor in the graph left by the prune (Sec. 2.2 graph model, Sec. 2.4):
    (child_rowptr, child_idx, in_graph)."""
    K = _c(K, np.uint64)
    cap = 0
    kept = (K & np.uint64(select)) != 0
    din = np.diff(adj.in_rowptr).astype(np.int64)
    dout = np.diff(adj.out_rowptr).astype(np.int64)
    cap = int((din[kept] * dout[kept]).sum())
    child_rowptr = np.empty(adj.num_tensors + 1, np.int32)
    child_idx = np.empty(max(cap, 1), np.int32)
    in_graph = np.empty(adj.num_tensors, np.uint8)
    n = _load().orc_child_sets(i64(adj.num_ops), i64(adj.num_tensors), _p(adj.in_rowptr), _p(adj.in_idx),
                               _p(adj.out_rowptr), _p(adj.out_idx), _p(K), ctypes.c_uint64(select),
                               _p(child_rowptr), _p(child_idx), i64(cap), _p(in_graph))
    if n < 0:
        raise MemoryError("orc_child_sets")
    return child_rowptr, child_idx[:n].copy(), in_graph


def inplace(adj: Adjacency, K: np.ndarray, select: int = 2**64 - 1) -> np.ndarray:
    """Algorithm 3 on the pruned graph: rename dictionary RD as an int32 array over tensors
    (ancestor id, -1 for tensors outside the graph)."""
    child_rowptr, child_idx, in_graph = child_sets(adj, K, select)
    RD = np.empty(adj.num_tensors, np.int32)
    _load().orc_inplace(i64(adj.num_tensors), _p(child_rowptr), _p(child_idx), _p(in_graph), _p(RD))
    return RD


def consumers(adj: Adjacency):
    """tensor -> consumer operators (ascending operator id), as a CSR: the transpose of the input CSR."""
    op_of_edge = np.repeat(np.arange(adj.num_ops, dtype=np.int32), np.diff(adj.in_rowptr))
    return build_csr(adj.num_tensors, adj.in_idx, op_of_edge)


def backward_mark(adj: Adjacency, obj, wrt) -> np.ndarray:
    """Algorithm 2 for up to 64 (objective, derivative target) pairs: bit i of M[x] = m_x of pair i."""
    obj, wrt = _c(obj, np.int32), _c(wrt, np.int32)
    assert obj.shape == wrt.shape
    cons_rowptr, cons_idx = consumers(adj)
    M = np.zeros(adj.num_tensors, np.uint64)
    V = np.empty(max(adj.num_tensors, 1), np.uint8)
    rc = _load().orc_backward_prune(i64(adj.num_tensors), _p(cons_rowptr), _p(cons_idx), _p(adj.out_rowptr),
                                    _p(adj.out_idx), i32(obj.shape[0]), _p(obj), _p(wrt), _p(M), _p(V))
    if rc:
        raise ValueError("orc_backward_prune: bad argument")
    return M


def backward_prune(adj: Adjacency, obj, wrt, num_graphs: int = 1, graph_op_offsets=None) -> PruneResult:
    """Algorithm 2, then the same removal rule and ordered compaction as the forward prune."""
    M = backward_mark(adj, obj, wrt)
    K, flag = keep(adj, M)
    kept_ops, kept_masks, kept_count, pq = compact(K, num_graphs, graph_op_offsets)
    return PruneResult(M, K, flag, kept_ops, kept_masks, kept_count, pq, np.zeros(0, np.int64))


def ignore_mask(adj: Adjacency, K: np.ndarray, M: np.ndarray) -> np.ndarray:
    """Sec. 3.2: bit q of ignore[t] iff t is written by an operator kept for set q and is not coloured for q."""
    out = np.empty(adj.num_tensors, np.uint64)
    _load().orc_ignore_mask(i64(adj.num_ops), i64(adj.num_tensors), _p(adj.out_rowptr), _p(adj.out_idx),
                            _p(_c(K, np.uint64)), _p(_c(M, np.uint64)), _p(out))
    return out


def per_set_lists(K: np.ndarray):
    """Sec. 3.2: for every set q the ascending ids of the operators kept for it: (set_rowptr[65], set_ops)."""
    K = _c(K, np.uint64)
    total = int(sum(int(np.count_nonzero((K >> np.uint64(q)) & np.uint64(1))) for q in range(64)))
    rowptr = np.empty(65, np.int64)
    ops = np.empty(max(total, 1), np.int32)
    n = _load().orc_per_set_lists(i64(K.shape[0]), _p(K), _p(rowptr), _p(ops))
    assert n == total
    return rowptr, ops[:n].copy()


def mix64(z: int) -> int:
    """Output function of SplitMix64 (the digest's mixing step)."""
    return int(_load().orc_mix64(ctypes.c_uint64(z & (2**64 - 1))))


def target_digest(num_sets: int, tgt_rowptr, tgt_idx):
    """128-bit digest of the target sets as ``dgn_prune`` receives them (key of a transaction, Sec. 4.1);
    returns two Python ints."""
    rp, ix = _c(tgt_rowptr, np.int32), _c(tgt_idx, np.int32)
    out = np.zeros(2, dtype=np.uint64)
    _load().orc_target_digest(i32(num_sets), i64(len(rp) - 1), _p(rp), i64(len(ix)), _p(ix), _p(out))
    return int(out[0]), int(out[1])
