"""Pins for the CPU oracle of Algorithm 2 (Backward Prune, Sec. 2.3).  Expected values come from
hand-worked cases, from enumerating every route, and from boolean matrix closure -- never from the
oracle itself."""
import numpy as np
import pytest

import graphgen as gg
from helpers import (graph_from_ops, load_backward_examples, marks_by_closure, marks_by_route_enumeration,
                     random_small_graph)


def _adj(oracle, g):
    return oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)


@pytest.mark.parametrize("case", load_backward_examples(), ids=lambda c: c["name"][:40])
def test_hand_worked_cases(oracle, case):
    g = case["graph"]
    r = oracle.backward_prune(_adj(oracle, g), case["obj"], case["wrt"])
    assert r.tensor_mask.tolist() == case["M"].tolist()
    assert r.kept_ops.tolist() == case["kept"].tolist()
    # the two definitions agree with the hand-worked values as well
    assert marks_by_route_enumeration(case["ops"], g.num_tensors, case["obj"], case["wrt"]).tolist() == case["M"].tolist()
    assert marks_by_closure(case["ops"], g.num_tensors, case["obj"], case["wrt"]).tolist() == case["M"].tolist()


@pytest.mark.parametrize("seed", range(30))
def test_small_random_graphs_against_both_definitions(oracle, seed):
    rng = np.random.default_rng(500 + seed)
    g, ops = random_small_graph(rng, int(rng.integers(1, 14)), multi_producer=bool(seed % 3 == 0))
    n = int(rng.integers(1, 65))
    obj = rng.integers(0, g.num_tensors, n).astype(np.int32)
    wrt = rng.integers(0, g.num_tensors, n).astype(np.int32)
    M = oracle.backward_mark(_adj(oracle, g), obj, wrt)
    assert M.tolist() == marks_by_route_enumeration(ops, g.num_tensors, obj, wrt).tolist()
    assert M.tolist() == marks_by_closure(ops, g.num_tensors, obj, wrt).tolist()


@pytest.mark.parametrize("seed", range(10))
def test_medium_random_graphs_against_closure(oracle, seed):
    rng = np.random.default_rng(900 + seed)
    g, ops = random_small_graph(rng, int(rng.integers(50, 300)), multi_producer=bool(seed % 2))
    obj = rng.integers(0, max(1, g.num_tensors // 4), 64).astype(np.int32)
    wrt = rng.integers(0, g.num_tensors, 64).astype(np.int32)
    M = oracle.backward_mark(_adj(oracle, g), obj, wrt)
    assert M.tolist() == marks_by_closure(ops, g.num_tensors, obj, wrt).tolist()


def test_pairs_are_independent_and_deep_chains_do_not_overflow(oracle):
    n = 200_000
    g = graph_from_ops([([i], [i + 1]) for i in range(n)], n + 1)
    adj = _adj(oracle, g)
    obj = np.asarray([0, 1000, 5, n], np.int32)
    wrt = np.asarray([n, 2000, 5, 0], np.int32)
    M = oracle.backward_mark(adj, obj, wrt)
    ids = np.arange(n + 1)
    expect = np.ones(n + 1, np.uint64) | (((ids >= 1000) & (ids <= 2000)).astype(np.uint64) << np.uint64(1))
    assert np.array_equal(M, expect)
    for i in range(4):                                    # bit i of the batch = the pair run alone
        alone = oracle.backward_mark(adj, obj[i:i + 1], wrt[i:i + 1])
        assert np.array_equal((M >> np.uint64(i)) & np.uint64(1), alone)


@pytest.mark.parametrize("cfg,scale", [(0, 1.0), (1, 0.1), (2, 0.01), (3, 0.002)])
def test_marked_set_is_inside_both_reachabilities(oracle, cfg, scale):
    """On the workload families: marked(pair) = coloured set of the forward prune with target x_wrt,
    restricted to what x_obj reaches; checked through properties that need no second traversal."""
    g, _ = gg.config(cfg, scale)
    adj = _adj(oracle, g)
    obj, wrt = gg.backward_pairs(g, gg.BASE_SEED + 1000 * cfg, 64, 400 if cfg == 1 else 16)
    r = oracle.backward_prune(adj, obj, wrt)
    M = r.tensor_mask
    # ancestors of x_wrt by Algorithm 1 (pinned separately): the marked set of pair i is inside them
    rowptr = np.arange(65, dtype=np.int32)
    anc, _ = oracle.mark(adj, 64, rowptr, wrt)
    assert not np.any(M & ~anc)
    bits = np.uint64(1) << np.arange(64, dtype=np.uint64)
    connected = (anc[obj] & bits) != 0
    connected &= obj != wrt
    assert np.array_equal((M[obj] & bits) != 0, connected)           # x_obj is marked iff it leads to x_wrt
    assert np.array_equal((M[wrt] & bits) != 0, connected)           # and then so is x_wrt
    assert connected.sum() >= 8
    # path-closure: a marked non-objective node has a marked parent, a marked non-target node a marked child
    prod_of = adj.prod_rowptr
    sample = np.flatnonzero(M)[:: max(1, int(np.count_nonzero(M)) // 500)]
    cons_rowptr, cons_idx = oracle.consumers(adj)
    for x in sample.tolist():
        up = np.uint64(0)
        for p in range(prod_of[x], prod_of[x + 1]):
            o = adj.prod_idx[p]
            for e in range(adj.in_rowptr[o], adj.in_rowptr[o + 1]):
                up |= M[adj.in_idx[e]]
        down = np.uint64(0)
        for c in range(cons_rowptr[x], cons_rowptr[x + 1]):
            o = cons_idx[c]
            for e in range(adj.out_rowptr[o], adj.out_rowptr[o + 1]):
                down |= M[adj.out_idx[e]]
        is_obj = np.bitwise_or.reduce(bits[obj == x]) if np.any(obj == x) else np.uint64(0)
        is_wrt = np.bitwise_or.reduce(bits[wrt == x]) if np.any(wrt == x) else np.uint64(0)
        assert not (M[x] & ~(up | is_obj)), x
        assert not (M[x] & ~(down | is_wrt)), x
