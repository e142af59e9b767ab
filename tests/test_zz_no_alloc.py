"""The entry point that allocates nothing (``dgn_keep_compact_static``: removal rule + ordered compaction with the
passes' scratch in an array of the library's own code object) against ``dgn_keep_compact``, which takes its
scratch from the caller, and against the oracle: two calls in a row through the C ABI, the second on a
smaller graph, so that the second call runs over what the first one left in the shared array."""
import numpy as np
import pytest

import graphgen as gg

pytestmark = pytest.mark.gpu

NAMES = ("op_mask", "op_flag", "kept_ops", "kept_masks", "kept_count", "per_query_count")


@pytest.fixture(scope="module")
def dgn():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1707_08265_amd as d
    return d


def _both_ways(d, orc, g, tg, what):
    import torch
    print(f"no-alloc entry point, {what}: P={g.num_ops} T={g.num_tensors} graphs={g.num_graphs}", flush=True)
    adj = orc.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    ref = orc.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx, g.num_graphs, g.graph_op_offsets)
    dg = d.DeviceGraph.from_coo(g)
    M = torch.from_numpy(ref.tensor_mask.view(np.int64)).cuda()
    # the existing entry point, scratch from the caller
    a = d.PruneBuffers(dg, tg.num_sets)
    assert a.keep_compact(M) == 0
    want = a.to_host()
    # the new one: outputs only (every output buffer starts dirty)
    b = d.PruneBuffers(dg, tg.num_sets)
    for t in (b.op_mask, b.op_flag, b.kept_ops, b.kept_masks, b.kept_count, b.per_query_count):
        t.fill_(-1 if t.dtype != torch.uint8 else 255)
    rc = d.dgn_keep_compact_static(dg.handle, M, b.op_mask, b.op_flag, b.kept_ops, b.kept_masks, b.kept_count,
                                   b.per_query_count)
    assert rc == 0, d.dgn_strerror(rc)
    got = b.to_host()
    for name in NAMES:
        assert np.array_equal(got[name], want[name]), f"{what}: {name} differs from dgn_keep_compact"
        assert np.array_equal(got[name], getattr(ref, name)), f"{what}: {name} differs from the oracle"
    return int(got["kept_count"][0])


def test_static_scratch_entry_point_matches_the_caller_scratch_one(dgn, oracle):
    rc, max_ops, nbytes = dgn.dgn_keep_compact_static_limits()
    assert rc == 0 and max_ops == 1 << 26 and 0 < nbytes < 16 << 20
    # first a graph of many tiles with a ragged tail, then a smaller one of another family over the same array
    g1, t1 = gg.config(3, 0.01)              # 500 000 operators, 64 sets
    k1 = _both_ways(dgn, oracle, g1, t1, "first call")
    g2, t2 = gg.config(1, 0.37)              # 74 000 operators, 64 sets, most of them kept
    k2 = _both_ways(dgn, oracle, g2, t2, "second call, smaller")
    assert k1 > 0 and k2 > 0
    # a packed batch (per-graph offsets and counts; few graphs: the replicated counters of the array are used)
    g3, t3 = gg.config(4, 8 / 4096)
    _both_ways(dgn, oracle, g3, t3, "third call, packed batch")


def test_static_scratch_entry_point_rejects_what_it_cannot_take(dgn):
    assert dgn.dgn_keep_compact_static(None, None, None, None, None, None, None, None, stream=0) == dgn.DGN_ERR_NULL_PTR
