"""GPU parity of the transaction key (``dgn_target_digest``; Sec. 4.1 of the paper) against the oracle's, bit for
bit, and the cache of prune results built on it."""
import numpy as np
import pytest

import graphgen as gg
from helpers import targets_from_sets
from test_gpu_parity import assert_same, oracle_prune

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dgn():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1707_08265_amd as d
    return d


def _gpu_digest(dgn, dg, t):
    import torch
    cache = dgn.TransactionCache(dg, t.num_sets)
    return cache.digest(torch.from_numpy(t.tgt_rowptr).cuda(), torch.from_numpy(t.tgt_idx).cuda())


def test_digest_matches_the_oracle(dgn, oracle):
    g, tg = gg.config(3, 0.004)
    dg = dgn.DeviceGraph.from_coo(g)
    cases = [tg,
             targets_from_sets([[]], 1),                                         # one empty set: three words
             targets_from_sets([[5], [], [], [7, 7, 2]], 4),                     # empty sets, a duplicate
             gg.targets_range(11, 64, 0, 3, 0, g.num_tensors),                   # ragged, some sets empty
             gg.targets_range(12, 64, 20000, 20000, 0, g.num_tensors),           # 1.28 M targets: every block loops
             gg.targets_range(13, 7, 1, 300, 0, g.num_tensors)]
    seen = set()
    for i, t in enumerate(cases):
        got = _gpu_digest(dgn, dg, t)
        want = oracle.target_digest(t.num_sets, t.tgt_rowptr, t.tgt_idx)
        assert got == want, f"case {i}: {got} != {want}"
        seen.add(got)
    assert len(seen) == len(cases)


def test_digest_of_a_packed_batch_counts_every_graphs_sets(dgn, oracle):
    g, tg = gg.config(4, 0.002)                             # 8 graphs x 64 sets: 513 row pointers
    dg = dgn.DeviceGraph.from_coo(g)
    assert _gpu_digest(dgn, dg, tg) == oracle.target_digest(tg.num_sets, tg.tgt_rowptr, tg.tgt_idx)


def test_cache_returns_existing_results_and_prunes_new_ones(dgn, oracle):
    import torch
    g, tg = gg.config(3, 0.01)
    dg = dgn.DeviceGraph.from_coo(g)
    adj, _ = oracle_prune(oracle, g, tg)
    draws = [tg] + [gg.targets_range(100 + i, tg.num_sets, 1, 6, 0, g.num_tensors) for i in range(3)]
    ref = [oracle.forward_prune(adj, t.num_sets, t.tgt_rowptr, t.tgt_idx, g.num_graphs, g.graph_op_offsets) for t in draws]
    dev = [(torch.from_numpy(t.tgt_rowptr).cuda(), torch.from_numpy(t.tgt_idx).cuda()) for t in draws]
    cache = dgn.TransactionCache(dg, tg.num_sets, capacity=2)
    b0 = cache.prune(*dev[0])
    assert_same(b0.to_host(), ref[0], "first")
    assert (cache.hits, cache.misses) == (0, 1)
    assert cache.prune(*dev[0]) is b0 and (cache.hits, cache.misses) == (1, 1)        # the same function again
    # equal target sets in other device arrays are the same transaction
    again = (dev[0][0].clone(), dev[0][1].clone())
    assert cache.prune(*again) is b0 and cache.hits == 2
    b1 = cache.prune(*dev[1])
    assert b1 is not b0
    assert_same(b1.to_host(), ref[1], "second")
    assert_same(b0.to_host(), ref[0], "first, untouched by the second")
    # a third set of targets takes over the least recently used buffers (those of draw 0) and recycles them
    assert cache.prune(*dev[1]) is b1
    assert cache.prune(*dev[0]) is b0                                                    # now draw 1 is the older one
    b2 = cache.prune(*dev[2])
    assert b2 is b1 and cache.misses == 3
    assert_same(b2.to_host(), ref[2], "third, in recycled buffers")
    b3 = cache.prune(*dev[1])                                                            # draw 1 was evicted: pruned again
    assert cache.misses == 4 and b3 is b0
    assert_same(b3.to_host(), ref[1], "second again")
    # one target id changed: another transaction
    idx = draws[3].tgt_idx.copy()
    idx[0] = (idx[0] + 1) % g.num_tensors
    changed = gg.Targets(draws[3].num_sets, draws[3].tgt_rowptr, idx)
    k1 = cache.digest(*dev[3])
    k2 = cache.digest(torch.from_numpy(changed.tgt_rowptr).cuda(), torch.from_numpy(changed.tgt_idx).cuda())
    assert k1 != k2
