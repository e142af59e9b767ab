"""GPU parity of repeated prunes that recycle their buffers (``dgn_options.recycle``): a prune that finds the
previous result of the same graph in place zeroes only what that result set.  Every call is compared with the
CPU oracle, bit for bit, with target sets that change from call to call so that a word left over from the
previous result would show."""
import numpy as np
import pytest

import graphgen as gg
from helpers import random_small_graph, targets_from_sets
from test_gpu_parity import assert_same, oracle_prune

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dgn():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1707_08265_amd as d
    return d


def _draws(g, tg, n):
    """The config's own targets, then other draws: other tensors, other set sizes, from other parts of the graph."""
    Q = tg.num_sets
    out = [tg]
    for i in range(1, n):
        lo = (g.num_tensors * (i % 4)) // 5
        out.append(gg.targets_range(9000 + 17 * i, Q, 1, 3 + 5 * (i % 3), lo, g.num_tensors))
    return out


def _prune(dgn, buf, t, **knobs):
    import torch
    st = dgn.dgn_stats()
    opts = dgn.dgn_options(**knobs) if knobs else None
    rc = buf.prune(torch.from_numpy(t.tgt_rowptr).cuda(), torch.from_numpy(t.tgt_idx).cuda(), options=opts, stats=st)
    assert rc == 0, dgn.dgn_strerror(rc)
    return st


@pytest.mark.parametrize("k,scale", [(0, 1.0), (1, 0.2), (2, 0.02), (3, 0.02)])
def test_recycled_prunes_match_the_oracle(dgn, oracle, k, scale):
    g, tg = gg.config(k, scale)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, tg.num_sets)                 # recycles from its second call on
    adj, _ = oracle_prune(oracle, g, tg)
    seen = []
    for i, t in enumerate(_draws(g, tg, 6)):
        st = _prune(dgn, buf, t)
        ref = oracle.forward_prune(adj, t.num_sets, t.tgt_rowptr, t.tgt_idx, g.num_graphs, g.graph_op_offsets)
        assert_same(buf.to_host(), ref, f"cfg{k} call {i}")
        seen.append(int(st.recycled))
    print(f"cfg{k}: recycled per call {seen}", flush=True)
    # call 0 has no flag, call 1 finds no log yet; from then on the previous result is found -- unless a prune
    # coloured so much of the graph that its log did not hold it
    assert seen[0] == 0 and seen[1] == 0
    assert k == 0 or k == 2 or all(seen[2:]), seen


def test_recycled_prunes_of_a_graph_large_enough_for_the_flag_driven_count_pass(dgn, oracle):
    """Above four million operators the count pass reads the keep flags the traversal wrote (a byte per
    operator) instead of all of K; recycled buffers must hand it flags with nothing left over."""
    g, tg = gg.config(3, 0.1)                               # five million operators
    assert g.num_ops >= 1 << 22
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, tg.num_sets)
    adj, _ = oracle_prune(oracle, g, tg)
    seen = []
    for i, t in enumerate(_draws(g, tg, 4)):
        st = _prune(dgn, buf, t)
        ref = oracle.forward_prune(adj, t.num_sets, t.tgt_rowptr, t.tgt_idx, g.num_graphs, g.graph_op_offsets)
        assert_same(buf.to_host(), ref, f"call {i}")
        seen.append(int(st.recycled))
    assert seen == [0, 0, 1, 1]
    # the same without a flag array of the caller's: the library keeps the flags in its scratch buffer
    import torch
    keep = buf.op_flag
    buf.op_flag = None
    st = _prune(dgn, buf, tg)
    buf.op_flag = keep
    out = buf.to_host()
    ref = oracle.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx, g.num_graphs, g.graph_op_offsets)
    assert np.array_equal(out["op_mask"], ref.op_mask) and np.array_equal(out["kept_ops"], ref.kept_ops)
    assert np.array_equal(out["per_query_count"], ref.per_query_count)
    torch.cuda.synchronize()


def test_flag_bytes_in_scratch_are_cleared_even_when_the_count_pass_does_not_read_them(dgn, oracle):
    """The keep flags live in the scratch buffer when the caller gives no flag array.  A call with the stand-alone
    removal-rule pass does not read them, but with ``recycle`` it leaves a header that names them: the call that
    finds the header zeroes them at the kept operators only, so everything else must have been cleared by the call
    that wrote it.  Sequence over a scratch buffer that starts as all 0xFF: stand-alone pass, stand-alone pass +
    recycle, recycle (the flag-driven count pass: five million operators), each against the oracle."""
    import torch
    g, tg = gg.config(3, 0.1)
    assert g.num_ops >= 1 << 22
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, tg.num_sets, recycle=False)
    buf.scratch.fill_(255)
    adj, _ = oracle_prune(oracle, g, tg)
    draws = _draws(g, tg, 3)
    seq = [dict(recompute_keep=1), dict(recompute_keep=1, recycle=1), dict(recycle=1)]
    recycled = []
    for i, (t, knobs) in enumerate(zip(draws, seq)):
        st = dgn.dgn_stats()
        rc = dgn.dgn_prune(dg.handle, t.num_sets, len(t.tgt_idx), torch.from_numpy(t.tgt_rowptr).cuda(),
                           torch.from_numpy(t.tgt_idx).cuda(), buf.tensor_mask, buf.op_mask, None, buf.kept_ops,
                           buf.kept_masks, buf.kept_count, buf.per_query_count, buf.scratch, buf.scratch_bytes,
                           options=dgn.dgn_options(**knobs), stats=st)
        assert rc == 0, dgn.dgn_strerror(rc)
        out = buf.to_host()
        ref = oracle.forward_prune(adj, t.num_sets, t.tgt_rowptr, t.tgt_idx, g.num_graphs, g.graph_op_offsets)
        for name in ("tensor_mask", "op_mask", "kept_count", "kept_ops", "kept_masks", "per_query_count"):
            assert np.array_equal(out[name], getattr(ref, name)), f"call {i} {knobs}: {name}"
        recycled.append(int(st.recycled))
    assert recycled == [0, 0, 1], recycled


def test_recycled_prunes_of_a_small_packed_batch(dgn, oracle):
    """Eight packed graphs go through the frontier traversal (the per-graph sweep starts at 64 graphs): the log,
    the per-graph kept offsets and the per-graph set counts must all survive recycling."""
    g, tg = gg.config(4, 0.002)
    assert 1 < g.num_graphs < 64
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, tg.num_sets)
    adj, _ = oracle_prune(oracle, g, tg)
    Q, G = tg.num_sets, g.num_graphs
    draws = [tg]
    for i in range(1, 4):                                   # other targets, each inside its own graph
        sets = []
        for gi in range(G):
            lo, hi = int(g.graph_tensor_offsets[gi]), int(g.graph_tensor_offsets[gi + 1])
            one = gg.targets_range(500 + 10 * i + gi, Q, 0, 3, lo, hi)
            sets += [list(one.tgt_idx[one.tgt_rowptr[q]:one.tgt_rowptr[q + 1]]) for q in range(Q)]
        rowptr = np.concatenate([[0], np.cumsum([len(x) for x in sets])]).astype(np.int32)
        draws.append(gg.Targets(Q, rowptr, np.asarray([t for x in sets for t in x], np.int32)))
    seen = []
    for i, t in enumerate(draws):
        st = _prune(dgn, buf, t)
        ref = oracle.forward_prune(adj, Q, t.tgt_rowptr, t.tgt_idx, G, g.graph_op_offsets)
        assert_same(buf.to_host(), ref, f"call {i}")
        seen.append(int(st.recycled))
    assert seen == [0, 0, 1, 1]


def test_swept_batches_ignore_the_flag_and_clear_what_they_must(dgn, oracle):
    """64 graphs and more are swept graph by graph: no log is kept, the flag has no effect, and since the sweep
    stores K of every operator only M is cleared -- buffers full of an earlier result, or of garbage, must not
    show in the next one."""
    g, tg = gg.config(4, 0.02)
    assert g.num_graphs >= 64
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, tg.num_sets)
    adj, ref = oracle_prune(oracle, g, tg)
    Q, G = tg.num_sets, g.num_graphs
    # a second draw: every other set of every graph empty
    cnt = np.diff(tg.tgt_rowptr)
    cnt2 = cnt.copy()
    cnt2[::2] = 0
    rowptr2 = np.concatenate([[0], np.cumsum(cnt2)]).astype(np.int32)
    idx2 = np.concatenate([tg.tgt_idx[tg.tgt_rowptr[s]:tg.tgt_rowptr[s] + cnt2[s]] for s in range(len(cnt))] +
                          [np.zeros(0, np.int32)]).astype(np.int32)
    t2 = gg.Targets(Q, rowptr2, idx2)
    ref2 = oracle.forward_prune(adj, Q, t2.tgt_rowptr, t2.tgt_idx, G, g.graph_op_offsets)
    for i, (t, r) in enumerate([(tg, ref), (t2, ref2), (tg, ref)]):
        if i == 2:
            buf.op_mask.fill_(-1)                           # K is not cleared by the library: the sweep must store all of it
            buf.op_flag.fill_(7)
        st = _prune(dgn, buf, t)
        assert int(st.recycled) == 0
        assert_same(buf.to_host(), r, f"call {i}")


@pytest.mark.parametrize("multi", [False, True])
def test_random_graphs_random_call_sequences(dgn, oracle, multi):
    """Small random graphs with the awkward cases (operators without inputs or outputs, duplicate edges, several
    producers of a tensor), each pruned several times through the same buffers for random target sets and with
    random schedule knobs, queue caps that force the overflow path, the stand-alone keep pass and incremental
    calls mixed in: every call against the oracle."""
    rng = np.random.default_rng(4242 + multi)
    for trial in range(12):
        P = int(rng.integers(1, 3000)) if trial % 3 else int(rng.integers(1, 60))
        g, _ = random_small_graph(rng, P, num_inputs=int(rng.integers(1, 6)), multi_producer=multi)
        Q = int(rng.integers(1, 65))
        dg = dgn.DeviceGraph.from_coo(g)
        buf = dgn.PruneBuffers(dg, Q)
        adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
        prev_sets = None
        for call in range(5):
            incremental = prev_sets is not None and rng.random() < 0.2
            if incremental:                                 # earlier sets plus more targets: a superset, set by set
                sets = [s + [int(rng.integers(0, g.num_tensors)) for _ in range(int(rng.integers(0, 3)))] for s in prev_sets]
            else:
                sets = [[int(rng.integers(0, g.num_tensors)) for _ in range(int(rng.integers(0, 5)))] for _ in range(Q)]
            t = targets_from_sets(sets)
            knobs = {}
            if incremental:
                knobs["incremental"] = 1
            r = rng.random()
            if r < 0.2:
                knobs["traversal"] = int(rng.integers(1, 3))
            elif r < 0.4:
                knobs["defer_percent"] = int(rng.integers(30, 99))
                knobs["defer_floor_shift"] = int(rng.integers(1, 12))
            elif r < 0.5:
                knobs["max_queue_entries"] = int(rng.integers(1, 64))
            elif r < 0.6 and not incremental:
                knobs["recompute_keep"] = 1
            _prune(dgn, buf, t, **knobs)
            ref = oracle.forward_prune(adj, Q, t.tgt_rowptr, t.tgt_idx)
            assert_same(buf.to_host(), ref, f"multi={multi} trial {trial} call {call} {knobs}")
            prev_sets = sets


def test_recycle_survives_schedule_knobs_and_the_standalone_keep_pass(dgn, oracle):
    g, tg = gg.config(3, 0.02)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, tg.num_sets)
    adj, _ = oracle_prune(oracle, g, tg)
    knobs = [dict(), dict(), dict(defer_percent=60), dict(recompute_keep=1), dict(traversal=1), dict(traversal=2),
             dict(defer_percent=95, defer_floor_shift=14), dict()]
    for i, (t, kn) in enumerate(zip(_draws(g, tg, len(knobs)), knobs)):
        st = _prune(dgn, buf, t, **kn)
        ref = oracle.forward_prune(adj, t.num_sets, t.tgt_rowptr, t.tgt_idx, g.num_graphs, g.graph_op_offsets)
        assert_same(buf.to_host(), ref, f"call {i} {kn}")
        assert int(st.recycled) == (1 if i >= 2 else 0), (i, kn)


def test_queue_overflow_and_incremental_calls_fall_back_to_a_full_clear(dgn, oracle):
    """A prune whose frontier queue overflowed (its log misses what the fix-up sweeps coloured) and an
    incremental prune (which keeps no log) must not be recycled from: the call after them clears everything."""
    g, tg = gg.config(3, 0.02)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, tg.num_sets)
    adj, _ = oracle_prune(oracle, g, tg)
    ts = _draws(g, tg, 8)
    plan = [dict(), dict(), dict(), dict(max_queue_entries=64), dict(), dict(), "incremental", dict(), dict()]
    want = [0, 0, 1, 1, 0, 1, 0, 0, 1]
    prev = None
    for i, kn in enumerate(plan):
        if kn == "incremental":                             # the same targets plus one more set's worth
            t = prev
            st = _prune(dgn, buf, t, incremental=1)
        else:
            t = ts[i % len(ts)]
            st = _prune(dgn, buf, t, **kn)
        ref = oracle.forward_prune(adj, t.num_sets, t.tgt_rowptr, t.tgt_idx, g.num_graphs, g.graph_op_offsets)
        assert_same(buf.to_host(), ref, f"call {i} {kn}")
        assert int(st.recycled) == want[i], (i, kn, int(st.recycled))
        prev = t


def test_a_prune_that_fills_the_log_is_not_recycled_from(dgn, oracle):
    """Everything upstream of the last tensors of a long, thin graph: the prune colours most of the graph through
    the few log segments the single-workgroup kernel writes, the log overflows, and the next call clears
    everything; results stay exact throughout."""
    g = gg.layered(200000, 31)                              # frontiers stay below the width of one workgroup
    t_all = gg.targets_range(5, 1, 64, 64, g.num_tensors - 200, g.num_tensors)
    t_few = gg.targets_range(6, 1, 2, 2, 16, 400)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, 1)
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    seq = [t_few, t_few, t_all, t_few, t_few, t_few]
    seen = []
    for i, t in enumerate(seq):
        st = _prune(dgn, buf, t)
        ref = oracle.forward_prune(adj, 1, t.tgt_rowptr, t.tgt_idx)
        assert_same(buf.to_host(), ref, f"call {i}")
        seen.append(int(st.recycled))
    coloured = int(np.count_nonzero(oracle.forward_prune(adj, 1, t_all.tgt_rowptr, t_all.tgt_idx).tensor_mask))
    print(f"recycled per call {seen}; the large prune colours {coloured} of {g.num_tensors} tensors", flush=True)
    assert coloured > g.num_tensors // 4                    # more than the whole log holds
    assert seen == [0, 0, 1, 0, 1, 1]                       # call 3 follows the prune that overflowed its log


def test_other_buffers_or_another_graph_are_not_mistaken_for_the_previous_result(dgn, oracle):
    import torch
    g, tg = gg.config(3, 0.01)
    g2, tg2 = gg.config(3, 0.011)
    dg, dg2 = dgn.DeviceGraph.from_coo(g), dgn.DeviceGraph.from_coo(g2)
    buf = dgn.PruneBuffers(dg, tg.num_sets)
    adj, ref = oracle_prune(oracle, g, tg)
    for _ in range(3):
        st = _prune(dgn, buf, tg)
    assert int(st.recycled) == 1
    # the same scratch buffer with other output buffers: nothing to recycle, and the result is still right
    other = dgn.PruneBuffers(dg, tg.num_sets)
    other.scratch, other.scratch_bytes, other._scratch_defined = buf.scratch, buf.scratch_bytes, True
    other.tensor_mask.fill_(-1)
    other.op_mask.fill_(-1)
    st = _prune(dgn, other, tg)
    assert int(st.recycled) == 0
    assert_same(other.to_host(), ref, "other buffers")
    # the first buffers again: the header now names the other ones
    buf.tensor_mask.fill_(-1)
    buf.op_mask.fill_(-1)
    st = _prune(dgn, buf, tg)
    assert int(st.recycled) == 0
    assert_same(buf.to_host(), ref, "first buffers again")
    # another graph through a scratch buffer that is large enough for both
    if g2.num_tensors >= g.num_tensors:
        big = dgn.PruneBuffers(dg2, tg2.num_sets)
        _prune(dgn, big, tg2)
        _prune(dgn, big, tg2)
        small = dgn.PruneBuffers(dg, tg.num_sets)
        small.scratch, small.scratch_bytes, small._scratch_defined = big.scratch, big.scratch_bytes, True
        small.tensor_mask.fill_(-1)
        small.op_mask.fill_(-1)
        st = _prune(dgn, small, tg)
        assert int(st.recycled) == 0
        assert_same(small.to_host(), ref, "scratch last used for another graph")
    torch.cuda.synchronize()


def test_two_host_threads_prune_the_same_graph_on_their_own_streams(dgn, oracle):
    """The graph handle is shared (its launch-layout hints are the only thing calls write to it), buffers,
    scratch and stream are each thread's own: the calls may overlap on the GPU and every result must still be
    the oracle's."""
    import threading
    import torch
    g, tg = gg.config(1, 0.3)
    dg = dgn.DeviceGraph.from_coo(g)
    adj, _ = oracle_prune(oracle, g, tg)
    draws = _draws(g, tg, 5)
    refs = [oracle.forward_prune(adj, t.num_sets, t.tgt_rowptr, t.tgt_idx, g.num_graphs, g.graph_op_offsets) for t in draws]
    dev_targets = [(torch.from_numpy(t.tgt_rowptr).cuda(), torch.from_numpy(t.tgt_idx).cuda()) for t in draws]
    torch.cuda.synchronize()
    failures = []

    def worker(k):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                buf = dgn.PruneBuffers(dg, tg.num_sets)
                order = list(range(len(draws))) if k == 0 else list(reversed(range(len(draws))))
                for rep in range(3):
                    for i in order:
                        rc = buf.prune(*dev_targets[i], stream=stream)
                        assert rc == 0, dgn.dgn_strerror(rc)
                        stream.synchronize()
                        assert_same(buf.to_host(), refs[i], f"thread {k} rep {rep} draw {i}")
        except Exception as e:      # noqa: BLE001 -- reported by the main thread
            failures.append(f"thread {k}: {e!r}")

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not failures, failures
