"""Pins for the oracle's ignore mask and per-set operator lists (Sec. 3.2): hand-worked values and
properties that follow from the definitions; no expected value comes from the oracle itself."""
import numpy as np
import pytest

import graphgen as gg
from helpers import graph_from_ops, load_worked_example, targets_from_sets


def _adj(oracle, g):
    return oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)


def test_hand_worked_split(oracle):
    # x -> Split -> (p, q); p -> ReLU -> r; q -> Tanh -> s.   Tensors x p q r s = 0..4.
    g = graph_from_ops([([0], [1, 2]), ([1], [3]), ([2], [4])], 5)
    adj = _adj(oracle, g)
    # set 0 wants r, set 1 wants s, set 2 wants p (hand-worked from Sec. 2.1 / 2.2 / 3.2):
    #   set 0 colours x p r, keeps Split and ReLU; q is computed by Split but unused -> ignore
    #   set 1 colours x q s, keeps Split and Tanh; p ignore
    #   set 2 colours x p,   keeps Split;          q ignore
    r = oracle.forward_prune(adj, 3, *_sets([[3], [4], [1]]))
    assert r.tensor_mask.tolist() == [7, 5, 2, 1, 2]
    assert r.op_mask.tolist() == [7, 1, 2]
    ig = oracle.ignore_mask(adj, r.op_mask, r.tensor_mask)
    assert ig.tolist() == [0, 2, 5, 0, 0]
    rowptr, ops = oracle.per_set_lists(r.op_mask)
    assert rowptr[:4].tolist() == [0, 2, 4, 5] and (rowptr[4:] == 5).all()
    assert ops.tolist() == [0, 1, 0, 2, 0]


def _sets(sets):
    tg = targets_from_sets(sets)
    return tg.tgt_rowptr, tg.tgt_idx


def test_paper_example_has_no_ignored_tensor(oracle):
    # f = x*sin(a*x+b): every operator has one output, so a kept operator's output is always coloured
    g, tid, cases = load_worked_example()
    adj = _adj(oracle, g)
    for c in cases:
        r = oracle.forward_prune(adj, c["targets"].num_sets, c["targets"].tgt_rowptr, c["targets"].tgt_idx)
        assert not oracle.ignore_mask(adj, r.op_mask, r.tensor_mask).any()


@pytest.mark.parametrize("cfg,scale", [(0, 1.0), (1, 0.2), (3, 0.002), (4, 0.0005)])
def test_properties_on_configs(oracle, cfg, scale):
    g, tg = gg.config(cfg, scale)
    adj = _adj(oracle, g)
    r = oracle.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx, g.num_graphs, g.graph_op_offsets)
    ig = oracle.ignore_mask(adj, r.op_mask, r.tensor_mask)
    assert not (ig & r.tensor_mask).any()                       # never both coloured and ignored for one set
    # tensor-side statement of the same mask: OR of K over the producers, minus the colours
    prodK = np.zeros(g.num_tensors, np.uint64)
    np.bitwise_or.at(prodK, g.out_tensor, r.op_mask[g.out_op])
    assert np.array_equal(ig, prodK & ~r.tensor_mask)
    if cfg in (0, 1, 3):
        assert ig.any()                                         # multi-output operators exist in these families
    rowptr, ops = oracle.per_set_lists(r.op_mask)
    if g.num_graphs == 1:
        assert np.array_equal(np.diff(rowptr), r.per_query_count)
    for q in (0, 1, tg.num_sets - 1, 63):
        lst = ops[rowptr[q]:rowptr[q + 1]]
        assert np.all(np.diff(lst) > 0)                         # creation order, no repeats
        assert np.array_equal(lst, np.flatnonzero((r.op_mask >> np.uint64(q)) & np.uint64(1)))
    assert np.array_equal(np.unique(ops), r.kept_ops)           # union of the lists = the kept list
