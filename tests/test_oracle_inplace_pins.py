"""Pins for the CPU oracle of Algorithm 3 (in-place structures, Sec. 2.4).  None of them calls the
oracle to produce an expected value: they use hand-worked cases, a characterisation of the result
that does not walk in node order, and structural invariants."""
import numpy as np
import pytest

import graphgen as gg
from helpers import (load_inplace_examples, random_small_graph, rename_by_reachability, single_child_links,
                     targets_from_sets)


def _adj(oracle, g):
    return oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)


@pytest.mark.parametrize("case", load_inplace_examples(), ids=lambda c: c["name"][:40])
def test_hand_worked_cases(oracle, case):
    g = case["graph"]
    rd = oracle.inplace(_adj(oracle, g), case["K"], case["select"])
    assert rd.tolist() == case["rename"].tolist()


def test_long_chain_is_one_structure(oracle):
    n = 5000
    ops = [([i], [i + 1]) for i in range(n)]
    from helpers import graph_from_ops
    g = graph_from_ops(ops, n + 1)
    rd = oracle.inplace(_adj(oracle, g), np.ones(n, np.uint64))
    assert (rd == 0).all()
    # cut the chain by removing one operator: two structures, the cut leaves both ends in the graph
    K = np.ones(n, np.uint64)
    K[1234] = 0
    rd = oracle.inplace(_adj(oracle, g), K)
    assert (rd[:1235] == 0).all() and (rd[1235:] == 1235).all()


@pytest.mark.parametrize("seed", range(40))
def test_matches_reachability_characterisation(oracle, seed):
    rng = np.random.default_rng(1000 + seed)
    g, _ = random_small_graph(rng, int(rng.integers(1, 60)), multi_producer=bool(seed % 3 == 0))
    if seed % 2:                                     # node order must not have to be topological
        g, _, _ = gg.relabel_tensors(g, targets_from_sets([[0]]), seed)
    K = rng.integers(0, 4, g.num_ops).astype(np.uint64)
    for select in (1, 2, 3):
        kept = (K & np.uint64(select)) != 0
        rd = oracle.inplace(_adj(oracle, g), K, select)
        assert rd.tolist() == rename_by_reachability(g, kept).tolist()


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_invariants_on_pruned_configs(oracle, cfg):
    g, tg = gg.config(cfg, scale=0.05 if cfg else 1.0)
    adj = _adj(oracle, g)
    res = oracle.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx)
    rd = oracle.inplace(adj, res.op_mask)
    kept = res.op_mask != 0
    in_graph, link = single_child_links(g, kept)
    assert ((rd >= 0) == in_graph).all()
    present = np.flatnonzero(in_graph)
    assert (rd[rd[present]] == rd[present]).all()            # an ancestor is its own ancestor
    # a renamed node was entered from a single-child parent that carries the same ancestor
    has_parent_with = set()
    for p in present:
        if link[p] >= 0:
            has_parent_with.add((int(link[p]), int(rd[p])))
    renamed = present[rd[present] != present]
    assert len(renamed) > 0
    for v in renamed:
        assert (int(v), int(rd[v])) in has_parent_with
    # a node that no single-child parent points to keeps its own name
    pointed = set(int(link[p]) for p in present if link[p] >= 0)
    for v in present:
        if int(v) not in pointed:
            assert rd[v] == v
