"""Seeded synthetic tensor/operator DAG generators.

This module only *describes inputs*: operators in creation (topological) order,
each with a list of input tensors and a list of output tensors, and target
sets.  It contains none of the pruning method's arithmetic and is the one
module shared by the CPU oracle's tests and the GPU path's tests/bench.

Every random quantity is a pure function of ``(seed, stream, counter)``
through a SplitMix64-style 64-bit mixer, so any element can be regenerated
independently and results do not depend on numpy's own generators.

Conventions (all generators):
  * graph inputs take the lowest tensor ids of their graph;
  * operator outputs are numbered consecutively in creation order after them;
  * inputs are drawn with replacement (duplicate edges stay);
  * COO arrays are emitted operator-major, ``int32``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 170708265

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)
_STREAM_MUL = _U64(0xD6E8FEB86659FD93)

# stream ids: one per random quantity
S_NOUT, S_FANIN, S_SRC, S_SKIP, S_SKIPLEN, S_REC, S_TGT_N, S_TGT, S_PERM = range(1, 10)
S_PAIR_OBJ, S_PAIR_WRT = 10, 11


def rng_u64(seed: int, stream: int, counters) -> np.ndarray:
    """SplitMix64 finaliser of ``seed ^ stream*C + (counter+1)*golden`` (uint64 array)."""
    c = np.asarray(counters).astype(_U64, copy=False)
    with np.errstate(over="ignore"):
        x = _U64(seed & 0xFFFFFFFFFFFFFFFF) ^ (_U64(stream) * _STREAM_MUL)
        z = x + (c + _U64(1)) * _GOLDEN
        z = (z ^ (z >> _U64(30))) * _M1
        z = (z ^ (z >> _U64(27))) * _M2
        z = z ^ (z >> _U64(31))
    return z


def rng_below(seed: int, stream: int, counters, n) -> np.ndarray:
    """Integers in ``[0, n)`` (``n`` scalar or array, each < 2**32) as int64."""
    z = rng_u64(seed, stream, counters) >> _U64(32)
    nn = np.asarray(n).astype(_U64, copy=False)
    return ((z * nn) >> _U64(32)).astype(np.int64)


def rng_unit(seed: int, stream: int, counters) -> np.ndarray:
    """Doubles in ``[0, 1)`` with 53 random bits."""
    return (rng_u64(seed, stream, counters) >> _U64(11)).astype(np.float64) * (1.0 / (1 << 53))


@dataclass
class Graph:
    """Operators as two COO edge lists (operator reads tensor / operator writes tensor)."""

    num_ops: int
    num_tensors: int
    in_op: np.ndarray
    in_tensor: np.ndarray
    out_op: np.ndarray
    out_tensor: np.ndarray
    num_graphs: int = 1
    graph_op_offsets: Optional[np.ndarray] = None      # int64 [G+1]
    graph_tensor_offsets: Optional[np.ndarray] = None  # int64 [G+1]
    name: str = ""

    @property
    def nnz_in(self) -> int:
        return int(self.in_op.shape[0])

    @property
    def nnz_out(self) -> int:
        return int(self.out_op.shape[0])


@dataclass
class Targets:
    """``num_sets`` target sets per graph, CSR over ``G*num_sets`` sets, global tensor ids."""

    num_sets: int
    tgt_rowptr: np.ndarray  # int32 [G*Q+1]
    tgt_idx: np.ndarray     # int32


def _excl_cumsum(a: np.ndarray) -> np.ndarray:
    out = np.zeros(a.shape[0] + 1, dtype=np.int64)
    np.cumsum(a, out=out[1:])
    return out


def _expand(counts: np.ndarray):
    """Row index and within-row slot for every element of a ragged layout."""
    rowptr = _excl_cumsum(counts)
    n = int(rowptr[-1])
    row = np.repeat(np.arange(counts.shape[0], dtype=np.int64), counts)
    slot = np.arange(n, dtype=np.int64) - rowptr[row]
    return row, slot, rowptr


def _outputs_consecutive(n_out: np.ndarray, first_free: int):
    """Number outputs consecutively from ``first_free``; returns (first_out[P+1], out_op, out_tensor)."""
    first_out = _excl_cumsum(n_out) + first_free
    out_op, slot, _ = _expand(n_out)
    out_tensor = first_out[out_op] + slot
    return first_out, out_op, out_tensor


def _i32(a) -> np.ndarray:
    a = np.asarray(a)
    assert a.size == 0 or (a.min() >= 0 and a.max() < 2**31 - 1)
    return np.ascontiguousarray(a, dtype=np.int32)


# --------------------------------------------------------------------------
# Family 0: layered random DAG with a sliding window of recent tensors
# --------------------------------------------------------------------------
def layered(num_ops: int, seed: int, num_inputs: int = 16, window: int = 64,
            fan_max: int = 3, out_max: int = 2, name: str = "layered") -> Graph:
    ops = np.arange(num_ops, dtype=np.int64)
    n_out = 1 + rng_below(seed, S_NOUT, ops, out_max)
    first_out, out_op, out_tensor = _outputs_consecutive(n_out, num_inputs)
    fan = 1 + rng_below(seed, S_FANIN, ops, fan_max)
    in_op, slot, _ = _expand(fan)
    produced = first_out[in_op] - num_inputs
    pool = num_inputs + np.minimum(window, produced)
    r = rng_below(seed, S_SRC, in_op * fan_max + slot, pool)
    in_tensor = np.where(r < num_inputs, r, first_out[in_op] - 1 - (r - num_inputs))
    return Graph(num_ops, int(first_out[-1]), _i32(in_op), _i32(in_tensor), _i32(out_op),
                 _i32(out_tensor), name=name)


def targets_tail(g: Graph, seed: int, num_sets: int, per_set_min: int, per_set_max: int,
                 tail_fraction: float) -> Targets:
    """Each set: U{min..max} tensors uniform (with replacement) from the last ``tail_fraction`` of ids."""
    q = np.arange(num_sets, dtype=np.int64)
    n = per_set_min + rng_below(seed, S_TGT_N, q, per_set_max - per_set_min + 1)
    row, slot, rowptr = _expand(n)
    span = max(1, int(g.num_tensors * tail_fraction))
    lo = g.num_tensors - span
    idx = lo + rng_below(seed, S_TGT, row * 1024 + slot, span)
    return Targets(num_sets, _i32(rowptr), _i32(idx))


# --------------------------------------------------------------------------
# Family 1: CNN-training-shaped DAG (layers with skip edges)
# --------------------------------------------------------------------------
def cnn(num_layers: int, width: int, seed: int, skip_prob: float = 0.2, skip_min: int = 2,
        skip_max: int = 32, fan_max: int = 3, out_max: int = 2, name: str = "cnn"):
    num_ops = num_layers * width
    ops = np.arange(num_ops, dtype=np.int64)
    n_out = 1 + rng_below(seed, S_NOUT, ops, out_max)
    first_out, out_op, out_tensor = _outputs_consecutive(n_out, width)  # `width` graph inputs = layer -1
    # tensor range of layer l (index l+1; entry 0 is the graph-input layer)
    layer_start = np.empty(num_layers + 2, dtype=np.int64)
    layer_start[0] = 0
    layer_start[1:] = first_out[np.arange(num_layers + 1, dtype=np.int64) * width]
    fan = 1 + rng_below(seed, S_FANIN, ops, fan_max)
    in_op, slot, _ = _expand(fan)
    cnt = in_op * fan_max + slot
    layer = in_op // width
    is_skip = rng_unit(seed, S_SKIP, cnt) < skip_prob
    s = skip_min + rng_below(seed, S_SKIPLEN, cnt, skip_max - skip_min + 1)
    src_layer = np.maximum(layer - np.where(is_skip, s, 1), -1) + 1  # index into layer_start
    lo = layer_start[src_layer]
    n = layer_start[src_layer + 1] - lo
    in_tensor = lo + rng_below(seed, S_SRC, cnt, n)
    g = Graph(num_ops, int(first_out[-1]), _i32(in_op), _i32(in_tensor), _i32(out_op),
              _i32(out_tensor), name=name)
    return g, layer_start


def targets_range(seed: int, num_sets: int, per_set_min: int, per_set_max: int, lo: int, hi: int,
                  extra_first=None) -> Targets:
    """Each set: U{min..max} tensors uniform over ids ``[lo, hi)``; set 0 optionally gets extra ids first."""
    q = np.arange(num_sets, dtype=np.int64)
    n = per_set_min + rng_below(seed, S_TGT_N, q, per_set_max - per_set_min + 1)
    row, slot, rowptr = _expand(n)
    idx = lo + rng_below(seed, S_TGT, row * 1024 + slot, hi - lo)
    if extra_first is not None:
        extra = np.asarray(extra_first, dtype=np.int64)
        idx = np.concatenate([extra, idx])
        rowptr = rowptr + extra.shape[0]
        rowptr[0] = 0
    return Targets(num_sets, _i32(rowptr), _i32(idx))


# --------------------------------------------------------------------------
# Family 2: unrolled RNN
# --------------------------------------------------------------------------
def rnn(num_steps: int, ops_per_step: int, seed: int, rec_prob: float = 0.1, num_inputs: int = 16,
        window: int = 64, fan_max: int = 3, name: str = "rnn") -> Graph:
    num_ops = num_steps * ops_per_step
    ops = np.arange(num_ops, dtype=np.int64)
    j = ops % ops_per_step
    fan = 1 + rng_below(seed, S_FANIN, ops, fan_max)
    has_rec = (ops >= ops_per_step) & (rng_unit(seed, S_REC, ops) < rec_prob)
    tot = fan + has_rec
    in_op, slot, _ = _expand(tot)
    jj = j[in_op]
    pool = num_inputs + np.minimum(window, jj)
    r = rng_below(seed, S_SRC, in_op * fan_max + np.minimum(slot, fan_max - 1), pool)
    own = num_inputs + in_op  # tensor id of this op's output
    intra = np.where(r < num_inputs, r, own - 1 - (r - num_inputs))
    is_rec = slot >= fan[in_op]
    in_tensor = np.where(is_rec, own - ops_per_step, intra)
    out_op = ops
    out_tensor = num_inputs + ops
    return Graph(num_ops, num_inputs + num_ops, _i32(in_op), _i32(in_tensor), _i32(out_op),
                 _i32(out_tensor), name=name)


# --------------------------------------------------------------------------
# Family 3: power-law fan-in, sources uniform over all earlier tensors
# --------------------------------------------------------------------------
def zipf_cdf(s: float, cap: int) -> np.ndarray:
    w = np.arange(1, cap + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def powerlaw(num_ops: int, seed: int, zipf_s: float = 2.1, fan_cap: int = 64, out_max: int = 3,
             num_inputs: int = 16, name: str = "powerlaw", chunk: int = 1 << 24) -> Graph:
    ops = np.arange(num_ops, dtype=np.int64)
    n_out = 1 + rng_below(seed, S_NOUT, ops, out_max)
    first_out, out_op, out_tensor = _outputs_consecutive(n_out, num_inputs)
    cdf = zipf_cdf(zipf_s, fan_cap)
    fan = np.minimum(np.searchsorted(cdf, rng_unit(seed, S_FANIN, ops), side="right"),
                     fan_cap - 1).astype(np.int64) + 1
    rowptr = _excl_cumsum(fan)
    nnz = int(rowptr[-1])
    in_op = np.empty(nnz, dtype=np.int32)
    in_tensor = np.empty(nnz, dtype=np.int32)
    # chunked over operators to bound temporaries
    for a in range(0, num_ops, chunk):
        b = min(num_ops, a + chunk)
        row = np.repeat(np.arange(a, b, dtype=np.int64), fan[a:b])
        e0, e1 = int(rowptr[a]), int(rowptr[b])
        slot = np.arange(e0, e1, dtype=np.int64) - rowptr[row]
        in_op[e0:e1] = row
        in_tensor[e0:e1] = rng_below(seed, S_SRC, row * fan_cap + slot, first_out[row])
    return Graph(num_ops, int(first_out[-1]), in_op, in_tensor, _i32(out_op), _i32(out_tensor),
                 name=name)


# --------------------------------------------------------------------------
# Family 4: packed batch of independent layered graphs
# --------------------------------------------------------------------------
def batch_layered(num_graphs: int, ops_per_graph: int, seed0: int, num_sets: int = 64,
                  per_set: int = 4, tail_fraction: float = 0.1, num_inputs: int = 16,
                  window: int = 64, fan_max: int = 3, out_max: int = 2, name: str = "batch"):
    """``num_graphs`` graphs, graph g generated by :func:`layered` / :func:`targets_tail` with seed
    ``seed0 + g``, concatenated with id offsets into one packed graph."""
    in_ops, in_ts, out_ops, out_ts, t_idx = [], [], [], [], []
    op_off = np.arange(num_graphs + 1, dtype=np.int64) * ops_per_graph
    t_off = np.zeros(num_graphs + 1, dtype=np.int64)
    for g in range(num_graphs):
        gr = layered(ops_per_graph, seed0 + g, num_inputs, window, fan_max, out_max)
        tg = targets_tail(gr, seed0 + g, num_sets, per_set, per_set, tail_fraction)
        in_ops.append(gr.in_op.astype(np.int64) + op_off[g])
        in_ts.append(gr.in_tensor.astype(np.int64) + t_off[g])
        out_ops.append(gr.out_op.astype(np.int64) + op_off[g])
        out_ts.append(gr.out_tensor.astype(np.int64) + t_off[g])
        t_idx.append(tg.tgt_idx.astype(np.int64) + t_off[g])
        t_off[g + 1] = t_off[g] + gr.num_tensors
    graph = Graph(num_graphs * ops_per_graph, int(t_off[-1]), _i32(np.concatenate(in_ops)),
                  _i32(np.concatenate(in_ts)), _i32(np.concatenate(out_ops)),
                  _i32(np.concatenate(out_ts)), num_graphs, op_off, t_off, name)
    rowptr = np.arange(num_graphs * num_sets + 1, dtype=np.int64) * per_set
    return graph, Targets(num_sets, _i32(rowptr), _i32(np.concatenate(t_idx)))


# --------------------------------------------------------------------------
# The five named workloads, optionally scaled down for quick tests
# --------------------------------------------------------------------------
def config(k: int, scale: float = 1.0):
    """Return ``(Graph, Targets)`` for workload ``k`` in 0..4; ``scale`` < 1 shrinks the op count."""
    seed = BASE_SEED + 1000 * k
    if k == 0:
        g = layered(max(8, int(2000 * scale)), seed, name="cfg0-layered")
        return g, targets_tail(g, seed, 1, 4, 4, 0.10)
    if k == 1:
        layers = max(4, int(500 * scale))
        g, layer_start = cnn(layers, 400, seed, name="cfg1-cnn")
        lo = int(layer_start[max(0, layers - 50) + 1])
        return g, targets_range(seed, 64, 1, 8, lo, g.num_tensors)
    if k == 2:
        steps = max(2, int(10000 * scale))
        g = rnn(steps, 1000, seed, name="cfg2-rnn")
        return g, targets_range(seed, 1, 32, 32, 16, g.num_tensors, extra_first=[g.num_tensors - 1])
    if k == 3:
        g = powerlaw(max(64, int(50_000_000 * scale)), seed, name="cfg3-powerlaw")
        return g, targets_tail(g, seed, 64, 1, 16, 0.05)
    if k == 4:
        ng = max(1, int(4096 * scale))
        return batch_layered(ng, 20000, BASE_SEED + 4000, name="cfg4-batch")
    raise ValueError(f"no such config: {k}")


def backward_pairs(g: Graph, seed: int, num_pairs: int = 64, num_sources: int = 16,
                   tail_fraction: float = 0.05):
    """(objective, derivative target) pairs for the backward prune: the objective of pair i is one of
    the first ``num_sources`` tensors of the graph (its graph inputs: every route starts at one),
    the derivative target is uniform over the last ``tail_fraction`` of the tensor ids.  Returns two
    int32 arrays of ``num_pairs`` ids."""
    i = np.arange(num_pairs, dtype=np.int64)
    obj = rng_below(seed, S_PAIR_OBJ, i, max(1, min(num_sources, g.num_tensors)))
    span = max(1, int(g.num_tensors * tail_fraction))
    wrt = g.num_tensors - span + rng_below(seed, S_PAIR_WRT, i, span)
    return _i32(obj), _i32(wrt)


# --------------------------------------------------------------------------
# Input transformations used by tests (no effect on the graph's meaning)
# --------------------------------------------------------------------------
def permutation_keys(n: int, seed: int) -> np.ndarray:
    """The uint64 keys whose stable argsort is ``permutation(n, seed)`` (a caller with a faster sort may use them)."""
    return rng_u64(seed, S_PERM, np.arange(n, dtype=np.int64))


def permutation(n: int, seed: int) -> np.ndarray:
    """Seeded permutation of ``range(n)`` (argsort of counter-based keys; ties impossible in practice)."""
    return np.argsort(permutation_keys(n, seed), kind="stable").astype(np.int64)


def shuffle_coo(g: Graph, seed: int) -> Graph:
    """Same edges, COO order shuffled by seeded permutations (for the CSR-builder tests)."""
    pi = permutation(g.nnz_in, seed)
    po = permutation(g.nnz_out, seed + 1)
    return Graph(g.num_ops, g.num_tensors, g.in_op[pi].copy(), g.in_tensor[pi].copy(),
                 g.out_op[po].copy(), g.out_tensor[po].copy(), g.num_graphs, g.graph_op_offsets,
                 g.graph_tensor_offsets, g.name + "-shuffled")


def relabel_tensors(g: Graph, t: Targets, seed: int):
    """Rename tensor ids by a seeded permutation (single graphs only). Returns (Graph, Targets, perm)
    with ``perm[old] = new``."""
    assert g.num_graphs == 1
    perm = permutation(g.num_tensors, seed)
    g2 = Graph(g.num_ops, g.num_tensors, g.in_op.copy(), _i32(perm[g.in_tensor]), g.out_op.copy(),
               _i32(perm[g.out_tensor]), name=g.name + "-relabelled")
    return g2, Targets(t.num_sets, t.tgt_rowptr.copy(), _i32(perm[t.tgt_idx])), perm
