"""GPU parity of Backward Prune (Algorithm 2): marked masks, operator masks, flags, the compacted list
and the counts of the HIP path, through the C ABI binding, against the CPU oracle, bit for bit."""
import numpy as np
import pytest

import graphgen as gg
from helpers import graph_from_ops, load_backward_examples, random_small_graph

pytestmark = pytest.mark.gpu

NAMES = ("tensor_mask", "op_mask", "op_flag", "kept_ops", "kept_masks", "kept_count", "per_query_count")


@pytest.fixture(scope="module")
def dgn():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1707_08265_amd as d
    return d


def _adj(orc, g):
    return orc.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)


def gpu_backward(d, g, obj, wrt, buf=None, dg=None, stats=None, **knobs):
    import torch
    dg = dg or d.DeviceGraph.from_coo(g)
    buf = buf or d.BackwardPruneBuffers(dg, 64)
    opts = d.dgn_options(**knobs) if knobs else None
    rc = buf.backward_prune(torch.from_numpy(obj).cuda(), torch.from_numpy(wrt).cuda(), options=opts, stats=stats)
    assert rc == 0, d.dgn_strerror(rc)
    return dg, buf, buf.to_host()


def assert_same(out, ref, what):
    for name in NAMES:
        assert np.array_equal(out[name], getattr(ref, name)), f"{what}: {name} differs"


@pytest.mark.parametrize("case", load_backward_examples(), ids=lambda c: c["name"][:40])
def test_hand_worked_cases(dgn, case):
    _, _, out = gpu_backward(dgn, case["graph"], case["obj"], case["wrt"])
    assert out["tensor_mask"].tolist() == case["M"].tolist()
    assert out["kept_ops"].tolist() == case["kept"].tolist()


@pytest.mark.parametrize("seed", range(12))
def test_random_small_graphs(dgn, oracle, seed):
    rng = np.random.default_rng(8000 + seed)
    g, _ = random_small_graph(rng, int(rng.integers(1, 500)), multi_producer=bool(seed % 3 == 0))
    n = int(rng.integers(1, 65))
    obj = rng.integers(0, max(1, g.num_tensors // 3), n).astype(np.int32)
    wrt = rng.integers(0, g.num_tensors, n).astype(np.int32)
    _, _, out = gpu_backward(dgn, g, obj, wrt)
    assert_same(out, oracle.backward_prune(_adj(oracle, g), obj, wrt), f"seed {seed}")


@pytest.mark.parametrize("k,scale", [(0, 1.0), (1, 1.0), (2, 0.02), (3, 0.005)])
def test_parity_configs(dgn, oracle, k, scale):
    g, _ = gg.config(k, scale)
    obj, wrt = gg.backward_pairs(g, gg.BASE_SEED + 1000 * k, 64, 400 if k == 1 else 16)
    print(f"config {k} scale {scale}: P={g.num_ops} T={g.num_tensors}", flush=True)
    st = dgn.dgn_stats()
    dg, buf, out = gpu_backward(dgn, g, obj, wrt, stats=st)
    ref = oracle.backward_prune(_adj(oracle, g), obj, wrt)
    assert_same(out, ref, f"cfg{k}")
    assert int(ref.kept_count[0]) > 0 and st.reserved >= 3
    # same buffers again, other pairs (dirty buffers), and a different traversal schedule for the first stage
    obj2, wrt2 = gg.backward_pairs(g, 77 + k, 33, 400 if k == 1 else 16, tail_fraction=0.5)
    _, _, out2 = gpu_backward(dgn, g, obj2, wrt2, buf=buf, dg=dg, defer_percent=100)
    assert_same(out2, oracle.backward_prune(_adj(oracle, g), obj2, wrt2), f"cfg{k} second call")


def test_recycled_buffers_over_a_sequence_of_calls(dgn, oracle):
    """The buffers of a backward prune recycle like those of a prune: stage one zeroes what the previous call set
    -- its own masks and, through the same log and kept list, the caller's marked masks and K.  Other pairs every
    time, an ordinary prune and a failed call in between; every result against the oracle."""
    import torch
    g, tg = gg.config(3, 0.01)
    adj = _adj(oracle, g)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.BackwardPruneBuffers(dg, 64)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    def run(seed, n):
        obj, wrt = gg.backward_pairs(g, seed, n, 16, tail_fraction=0.3)
        rc = buf.backward_prune(up(obj), up(wrt))
        assert rc == 0, dgn.dgn_strerror(rc)
        assert_same(buf.to_host(), oracle.backward_prune(adj, obj, wrt), f"pairs seed {seed}")
    run(1, 64)
    run(2, 64)
    run(3, 17)
    run(4, 64)
    # an ordinary prune through the same object lays the scratch buffer out differently
    assert buf.prune(up(tg.tgt_rowptr), up(tg.tgt_idx)) == 0
    run(5, 64)
    run(6, 64)
    # a call that fails half way (an objective out of range is found after stage one)
    bad = np.asarray([0, g.num_tensors + 5], np.int32)
    assert buf.backward_prune(up(bad), up(np.asarray([3, 4], np.int32))) == dgn.DGN_ERR_ID_OUT_OF_RANGE
    run(7, 64)
    run(8, 64)


def test_deep_chain_and_edge_cases(dgn, oracle):
    import torch
    n = 20_000
    g = graph_from_ops([([i], [i + 1]) for i in range(n)], n + 1)
    obj = np.asarray([0, 1000, 5, n, 7], np.int32)
    wrt = np.asarray([n, 2000, 5, 0, 8], np.int32)
    st = dgn.dgn_stats()
    dg, buf, out = gpu_backward(dgn, g, obj, wrt, stats=st)
    assert_same(out, oracle.backward_prune(_adj(oracle, g), obj, wrt), "chain")
    # the forward stage repeats whole passes over stage one's kept list until one adds nothing: on a chain a pass gets
    # as far as the waves that happen to run in list order carry it, so the count is bounded by the groups of 64
    print(f"chain of {n}: {int(st.reserved)} forward passes", flush=True)
    assert 1 <= st.reserved <= n // 64 + 64
    # bad ids are reported, not followed
    bad = np.asarray([0, n + 5], np.int32)
    rc = buf.backward_prune(torch.from_numpy(bad).cuda(), torch.from_numpy(np.asarray([3, 4], np.int32)).cuda())
    assert rc == dgn.DGN_ERR_ID_OUT_OF_RANGE
    rc = buf.backward_prune(torch.from_numpy(np.asarray([3, 4], np.int32)).cuda(), torch.from_numpy(bad).cuda())
    assert rc == dgn.DGN_ERR_ID_OUT_OF_RANGE
    rc = dgn.dgn_backward_prune(dg.handle, 0, buf.kept_ops, buf.kept_ops, buf.tensor_mask, buf.op_mask, buf.op_flag,
                                buf.kept_ops, buf.kept_masks, buf.kept_count, buf.per_query_count, buf.scratch,
                                buf.scratch_bytes)
    assert rc == dgn.DGN_ERR_TOO_MANY_SETS
    rc = dgn.dgn_backward_prune(dg.handle, 2, buf.kept_ops, buf.kept_ops, buf.tensor_mask, buf.op_mask, buf.op_flag,
                                buf.kept_ops, buf.kept_masks, buf.kept_count, buf.per_query_count, buf.scratch,
                                buf.scratch_bytes - 1)
    assert rc == dgn.DGN_ERR_WORKSPACE_TOO_SMALL
    # and the buffers still work afterwards
    _, _, out = gpu_backward(dgn, g, obj, wrt, buf=buf, dg=dg)
    assert_same(out, oracle.backward_prune(_adj(oracle, g), obj, wrt), "chain again")


def test_relabelled_tensors(dgn, oracle):
    from helpers import targets_from_sets
    g, _ = gg.config(1, 0.1)
    obj, wrt = gg.backward_pairs(g, 5, 64, 400)
    g2, tg2, perm = gg.relabel_tensors(g, targets_from_sets([obj.tolist(), wrt.tolist()]), 99)
    obj2, wrt2 = tg2.tgt_idx[:64].copy(), tg2.tgt_idx[64:].copy()
    _, _, out = gpu_backward(dgn, g2, obj2, wrt2)
    ref = oracle.backward_prune(_adj(oracle, g2), obj2, wrt2)
    assert_same(out, ref, "relabelled")
    _, _, out0 = gpu_backward(dgn, g, obj, wrt)
    assert np.array_equal(out["tensor_mask"][perm], out0["tensor_mask"])
    assert np.array_equal(out["kept_ops"], out0["kept_ops"])


def test_full_size_config3_sampled_pairs(dgn, oracle):
    """Full size: all 64 pairs on the GPU; the oracle (one graph-wide search per pair) checks two of
    them bit for bit, the rest through properties that hold for every pair."""
    g, _ = gg.config(3, 1.0)
    obj, wrt = gg.backward_pairs(g, gg.BASE_SEED + 3000, 64, 16)
    print(f"config 3 full size: P={g.num_ops} T={g.num_tensors}", flush=True)
    st = dgn.dgn_stats()
    _, _, out = gpu_backward(dgn, g, obj, wrt, stats=st)
    M = out["tensor_mask"]
    print(f"marked tensors {np.count_nonzero(M)}, kept operators {int(out['kept_count'][0])}, "
          f"forward passes {st.reserved}", flush=True)
    adj = _adj(oracle, g)
    bits = np.uint64(1) << np.arange(64, dtype=np.uint64)
    connected = (M[obj] & bits) != 0
    assert np.array_equal((M[wrt] & bits) != 0, connected) and connected.sum() >= 8
    sample = [int(np.flatnonzero(connected)[0]), int(np.flatnonzero(connected)[-1])]
    for i in sample:
        print(f"oracle on pair {i}", flush=True)
        ref = oracle.backward_mark(adj, obj[i:i + 1], wrt[i:i + 1])
        assert np.array_equal((M >> np.uint64(i)) & np.uint64(1), ref), f"pair {i}"
    K, flag = oracle.keep(adj, M)                                  # removal rule and compaction from the GPU's marks
    kept_ops, kept_masks, kept_count, pq = oracle.compact(K)
    assert np.array_equal(out["op_mask"], K) and np.array_equal(out["op_flag"], flag)
    assert np.array_equal(out["kept_ops"], kept_ops) and np.array_equal(out["kept_masks"], kept_masks)
    assert np.array_equal(out["kept_count"], kept_count) and np.array_equal(out["per_query_count"], pq)


@pytest.mark.parametrize("k,scale", [(1, 0.3), (3, 0.1)])
def test_flag_array_of_the_caller_absent_or_unaligned(dgn, oracle, k, scale):
    """The first stage keeps a byte per kept operator in the caller's op_flag when that is 8-byte aligned, else in
    scratch memory, and the last count pass reads those bytes instead of all of K: the result must not depend on
    where they live (config 3 at five million operators takes the flag-driven count pass)."""
    import torch
    g, _ = gg.config(k, scale)
    n_pairs = 64 if k == 1 else 4                           # (the oracle searches the whole graph once per pair)
    obj, wrt = gg.backward_pairs(g, 99 + k, n_pairs, 400 if k == 1 else 16)
    ref = oracle.backward_prune(_adj(oracle, g), obj, wrt)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.BackwardPruneBuffers(dg, n_pairs)
    own = buf.op_flag
    for how in ("aligned", "none", "unaligned", "aligned"):
        if how == "none":
            buf.op_flag = None
        elif how == "unaligned":
            store = torch.zeros(g.num_ops + 8, dtype=torch.uint8, device="cuda")
            buf.op_flag = store[1:1 + g.num_ops]
        else:
            buf.op_flag = own
        for rep in range(2):                                # the second call recycles what the first left
            rc = buf.backward_prune(torch.from_numpy(obj).cuda(), torch.from_numpy(wrt).cuda())
            assert rc == 0, dgn.dgn_strerror(rc)
            torch.cuda.synchronize()
            n = int(buf.kept_count[0].item())
            assert np.array_equal(buf.tensor_mask.cpu().numpy().view(np.uint64), ref.tensor_mask), how
            assert np.array_equal(buf.op_mask.cpu().numpy().view(np.uint64), ref.op_mask), how
            assert np.array_equal(buf.kept_ops[:n].cpu().numpy(), ref.kept_ops), how
            assert np.array_equal(buf.per_query_count.cpu().numpy(), ref.per_query_count), how
            if buf.op_flag is not None:
                assert np.array_equal(buf.op_flag.cpu().numpy(), ref.op_flag), how
