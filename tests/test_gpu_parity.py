"""GPU parity: the HIP path, called through the C ABI binding, against the CPU oracle, bit for bit
(all arithmetic is integer / bitwise, so the bar is exact equality of masks, flags, counts and the
compacted order)."""
import numpy as np
import pytest

import graphgen as gg
from helpers import graph_from_ops, load_worked_example, random_small_graph, targets_from_sets

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dgn():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1707_08265_amd as d
    return d


def gpu_prune(d, g, tg, recompute_keep=False, validate=False, stats=None, **knobs):
    import torch
    dg = d.DeviceGraph.from_coo(g, validate=validate)
    buf = d.PruneBuffers(dg, tg.num_sets)
    rowptr = torch.from_numpy(tg.tgt_rowptr).cuda()
    idx = torch.from_numpy(tg.tgt_idx).cuda()
    opts = d.dgn_options(recompute_keep=1 if recompute_keep else 0, **knobs)
    rc = buf.prune(rowptr, idx, options=opts, stats=stats)
    assert rc == 0, d.dgn_strerror(rc)
    out = buf.to_host()
    return dg, buf, out


def oracle_prune(orc, g, tg):
    adj = orc.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    return adj, orc.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx, g.num_graphs, g.graph_op_offsets)


def assert_same(out, r, what=""):
    assert np.array_equal(out["tensor_mask"], r.tensor_mask), f"{what}: coloured-tensor masks differ"
    assert np.array_equal(out["op_mask"], r.op_mask), f"{what}: operator keep masks differ"
    assert np.array_equal(out["op_flag"], r.op_flag), f"{what}: keep flags differ"
    assert np.array_equal(out["kept_count"], r.kept_count), f"{what}: kept counts differ"
    assert np.array_equal(out["kept_ops"], r.kept_ops), f"{what}: compacted order differs"
    assert np.array_equal(out["kept_masks"], r.kept_masks), f"{what}: compacted masks differ"
    assert np.array_equal(out["per_query_count"], r.per_query_count), f"{what}: per-set counts differ"


def test_worked_example(dgn, oracle):
    g, tid, cases = load_worked_example()
    for c in cases:
        _, _, out = gpu_prune(dgn, g, c["targets"])
        assert np.array_equal(out["tensor_mask"], c["M"]), c["name"]
        assert np.array_equal(out["op_mask"], c["K"]), c["name"]
        assert np.array_equal(out["kept_ops"], c["kept"]), c["name"]
        assert np.array_equal(out["per_query_count"][: len(c["pq"])], c["pq"]), c["name"]
    _, _, out = gpu_prune(dgn, g, cases[0]["targets"])
    assert out["tensor_mask"][tid["b"]] == 0          # Sec. 2.2: b must not be marked


# sizes the oracle finishes in seconds, spanning many tiles and ragged tails
CASES = [(0, 1.0), (1, 1.0), (2, 0.02), (3, 0.02), (4, 0.002)]


@pytest.mark.parametrize("k,scale", CASES)
def test_parity_configs(dgn, oracle, k, scale):
    g, tg = gg.config(k, scale)
    print(f"config {k} scale {scale}: P={g.num_ops} T={g.num_tensors} E={g.nnz_in}+{g.nnz_out}", flush=True)
    st = dgn.dgn_stats()
    dg, buf, out = gpu_prune(dgn, g, tg, stats=st)
    adj, r = oracle_prune(oracle, g, tg)
    assert_same(out, r, f"cfg{k}")
    assert st.levels > 0 and st.tensor_visits >= int(r.kept_count[0])      # every kept operator is expanded
    # stand-alone removal-rule pass gives the same K as the traversal accumulated
    _, _, out2 = gpu_prune(dgn, g, tg, recompute_keep=True)
    assert_same(out2, r, f"cfg{k} recompute_keep")


@pytest.mark.parametrize("k,scale", [(1, 0.2), (3, 0.004), (4, 0.001)])
def test_csr_builder_parity_on_shuffled_coo(dgn, oracle, k, scale):
    g, tg = gg.config(k, scale)
    gs = gg.shuffle_coo(g, 11 + k)
    adj = oracle.build_adjacency(gs.num_ops, gs.num_tensors, gs.in_op, gs.in_tensor, gs.out_op, gs.out_tensor)
    dg = dgn.DeviceGraph.from_coo(gs, validate=True)
    csr = {n: v.cpu().numpy() for n, v in dg.csr().items()}
    for name in ("in_rowptr", "in_idx", "out_rowptr", "out_idx", "prod_rowptr", "prod_idx"):
        assert np.array_equal(csr[name], getattr(adj, name)), name
    # and the prune result on the shuffled input is the same
    _, _, out = gpu_prune(dgn, gs, tg)
    _, r = oracle_prune(oracle, g, tg)
    assert_same(out, r, "shuffled")


def test_sort_of_many_tiles_and_of_few_distinct_keys(dgn, oracle):
    """The radix sort keeps its slot tables per tile, per group of 16 tiles and per chunk of groups: an edge list of
    > 64 groups (8.4 M edges) makes a chunk hold several groups, with a ragged last chunk, group and tile.  And a
    graph of few operators with thousands of inputs each (duplicates included) leaves most digits of a pass empty
    and the others crowded."""
    g, _ = gg.config(3, 0.1)                                   # 5 M operators, ~13 M input edges, ~10 M output edges
    assert g.nnz_in > 64 * 16 * 8192 and g.nnz_out > 64 * 16 * 8192
    gs = gg.shuffle_coo(g, 23)
    adj = oracle.build_adjacency(gs.num_ops, gs.num_tensors, gs.in_op, gs.in_tensor, gs.out_op, gs.out_tensor)
    dg = dgn.DeviceGraph.from_coo(gs)
    csr = {n: v.cpu().numpy() for n, v in dg.csr().items()}
    for name in ("in_rowptr", "in_idx", "out_rowptr", "out_idx", "prod_rowptr", "prod_idx"):
        assert np.array_equal(csr[name], getattr(adj, name)), name
    del dg, csr, adj

    rng = np.random.default_rng(29)
    P, T, fan = 700, 60000, 3000
    in_op = np.repeat(np.arange(P, dtype=np.int32), fan)
    in_tensor = rng.integers(0, T - P, size=P * fan).astype(np.int32)      # with repeats inside an operator
    out_op = np.arange(P, dtype=np.int32)
    out_tensor = (T - P + out_op).astype(np.int32)
    few = gg.Graph(P, T, in_op, in_tensor, out_op, out_tensor, name="few-keys")
    fs = gg.shuffle_coo(few, 31)
    adj = oracle.build_adjacency(P, T, fs.in_op, fs.in_tensor, fs.out_op, fs.out_tensor)
    dg = dgn.DeviceGraph.from_coo(fs)
    csr = {n: v.cpu().numpy() for n, v in dg.csr().items()}
    for name in ("in_rowptr", "in_idx", "out_rowptr", "out_idx", "prod_rowptr", "prod_idx"):
        assert np.array_equal(csr[name], getattr(adj, name)), name


@pytest.mark.parametrize("offset", [1, 2, 3])
def test_coo_arrays_at_unaligned_addresses(dgn, oracle, offset):
    """The builder reads the edge lists 16 bytes at a time where their addresses allow it: arrays that start 4, 8 or
    12 bytes past such an address, with ragged lengths, must give the same adjacency -- recorded operator by
    operator (the one-pass path) and shuffled (the sort and the row-pointer pass)."""
    import torch
    rng = np.random.default_rng(40 + offset)
    g0, _ = random_small_graph(rng, 3000 + offset, num_inputs=4)
    for variant in ("ordered", "shuffled"):
        g = g0 if variant == "ordered" else gg.shuffle_coo(g0, 7)
        adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)

        def shifted(a):
            buf = torch.zeros(len(a) + 8, dtype=torch.int32, device="cuda")
            view = buf[offset:offset + len(a)]
            view.copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)))
            assert view.data_ptr() % 16 == 4 * offset
            return view

        in_op, in_t, out_op, out_t = shifted(g.in_op), shifted(g.in_tensor), shifted(g.out_op), shifted(g.out_tensor)
        desc = dgn.make_coo_desc(g.num_ops, g.num_tensors, in_op, in_t, out_op, out_t)
        rc, gb, sb = dgn.dgn_graph_build_workspace(desc)
        assert rc == 0
        graph_mem = torch.empty(gb, dtype=torch.uint8, device="cuda")
        scratch = torch.empty(sb, dtype=torch.uint8, device="cuda")
        rc, h = dgn.dgn_graph_build(desc, graph_mem, gb, scratch, sb, dgn.dgn_options())
        assert rc == 0, dgn.dgn_strerror(rc)
        rc, sizes = dgn.dgn_graph_get_sizes(h)
        assert rc == 0
        dg = dgn.DeviceGraph(h, graph_mem, (), sizes)
        csr = {n: v.cpu().numpy() for n, v in dg.csr().items()}
        for name in ("in_rowptr", "in_idx", "out_rowptr", "out_idx", "prod_rowptr", "prod_idx"):
            assert np.array_equal(csr[name], getattr(adj, name)), f"{variant}, offset {offset}: {name}"


def test_from_csr_and_keep_compact(dgn, oracle):
    import torch
    g, tg = gg.config(1, 0.3)
    adj, r = oracle_prune(oracle, g, tg)
    c = lambda a: torch.from_numpy(a).cuda()
    dg = dgn.DeviceGraph.from_csr(g.num_ops, g.num_tensors, c(adj.in_rowptr), c(adj.in_idx), c(adj.out_rowptr),
                                  c(adj.out_idx), validate=True)
    csr = dg.csr()
    assert np.array_equal(csr["prod_rowptr"].cpu().numpy(), adj.prod_rowptr)
    assert np.array_equal(csr["prod_idx"].cpu().numpy(), adj.prod_idx)
    buf = dgn.PruneBuffers(dg, tg.num_sets)
    assert buf.prune(c(tg.tgt_rowptr), c(tg.tgt_idx)) == 0
    assert_same(buf.to_host(), r, "from_csr")
    # removal rule + compaction alone, from the oracle's coloured masks
    buf2 = dgn.PruneBuffers(dg, tg.num_sets)
    M = torch.from_numpy(r.tensor_mask.view(np.int64)).cuda()
    assert buf2.keep_compact(M) == 0
    out = buf2.to_host()
    for name, ref in (("op_mask", r.op_mask), ("op_flag", r.op_flag), ("kept_ops", r.kept_ops),
                      ("kept_masks", r.kept_masks), ("kept_count", r.kept_count),
                      ("per_query_count", r.per_query_count)):
        assert np.array_equal(out[name], ref), name


@pytest.mark.parametrize("multi", [False, True])
def test_random_small_graphs(dgn, oracle, multi):
    rng = np.random.default_rng(77 + multi)
    for trial in range(25):
        P = int(rng.integers(1, 300))
        g, ops = random_small_graph(rng, P, num_inputs=int(rng.integers(1, 6)), multi_producer=multi)
        Q = int(rng.integers(1, 65))
        sets = [[int(rng.integers(0, g.num_tensors)) for _ in range(int(rng.integers(0, 5)))] for _ in range(Q)]
        tg = targets_from_sets(sets)
        _, _, out = gpu_prune(dgn, g, tg)
        _, r = oracle_prune(oracle, g, tg)
        assert_same(out, r, f"trial {trial} multi={multi}")


def test_edge_cases(dgn, oracle):
    import torch
    # empty target sets: everything zero, nothing kept
    g, _ = gg.config(0)
    tg = targets_from_sets([[], [], []])
    _, _, out = gpu_prune(dgn, g, tg)
    assert not out["tensor_mask"].any() and not out["op_mask"].any() and out["kept_count"][0] == 0
    assert not out["per_query_count"].any() and len(out["kept_ops"]) == 0
    # a graph with no operators at all
    g0 = gg.Graph(0, 5, *(np.zeros(0, np.int32) for _ in range(4)))
    _, _, out = gpu_prune(dgn, g0, targets_from_sets([[3], [3, 4]]))
    assert list(out["tensor_mask"]) == [0, 0, 0, 3, 2] and out["kept_count"][0] == 0
    # 64 sets all holding the same tensor; zero-input and zero-output operators; duplicate edges
    gz = graph_from_ops([([], [1]), ([1, 1], [2]), ([2], []), ([0, 2], [3])], 4)
    tz = targets_from_sets([[3]] * 64)
    _, _, out = gpu_prune(dgn, gz, tz)
    _, r = oracle_prune(oracle, gz, tz)
    assert_same(out, r, "all-64-sets")
    assert out["tensor_mask"][3] == np.uint64(0xFFFFFFFFFFFFFFFF) and list(out["kept_ops"]) == [0, 1, 3]
    # target id out of range is reported, the valid ones are still processed
    dg = dgn.DeviceGraph.from_coo(gz)
    buf = dgn.PruneBuffers(dg, 1)
    rc = buf.prune(torch.tensor([0, 2], dtype=torch.int32).cuda(), torch.tensor([3, 99], dtype=torch.int32).cuda())
    assert rc == dgn.DGN_ERR_ID_OUT_OF_RANGE
    # an edge naming a tensor that does not exist is refused at build time
    bad = gg.Graph(1, 2, np.array([0], np.int32), np.array([5], np.int32), np.array([0], np.int32),
                   np.array([1], np.int32))
    with pytest.raises(dgn.DgnError) as ei:
        dgn.DeviceGraph.from_coo(bad)
    assert ei.value.code == dgn.DGN_ERR_ID_OUT_OF_RANGE
    # non-topological operator order is caught by validation
    cyc = graph_from_ops([([2], [1]), ([1], [2])], 3)
    with pytest.raises(dgn.DgnError) as ei:
        dgn.DeviceGraph.from_coo(cyc, validate=True)
    assert ei.value.code == dgn.DGN_ERR_NOT_TOPOLOGICAL


def test_deep_chain_many_levels(dgn, oracle):
    n = 3000                      # one frontier level per operator
    ops = np.arange(n, dtype=np.int32)
    g = gg.Graph(n, n + 1, ops, ops, ops, ops + 1)
    tg = targets_from_sets([[n], [n // 2]])
    st = dgn.dgn_stats()
    _, _, out = gpu_prune(dgn, g, tg, stats=st)
    _, r = oracle_prune(oracle, g, tg)
    assert_same(out, r, "chain")
    assert st.levels >= n


def test_relabelled_tensors(dgn, oracle):
    g, tg = gg.config(1, 0.1)
    g2, tg2, perm = gg.relabel_tensors(g, tg, 5)
    _, _, out = gpu_prune(dgn, g2, tg2)
    _, r = oracle_prune(oracle, g, tg)
    assert np.array_equal(out["tensor_mask"][perm], r.tensor_mask)
    assert np.array_equal(out["op_mask"], r.op_mask) and np.array_equal(out["kept_ops"], r.kept_ops)


def test_buffers_are_reusable_and_outputs_fully_rewritten(dgn, oracle):
    import torch
    g, tg = gg.config(1, 0.1)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, tg.num_sets)
    for t in (buf.tensor_mask, buf.op_mask, buf.kept_masks, buf.per_query_count, buf.kept_count):
        t.fill_(-1)
    buf.op_flag.fill_(7)
    buf.scratch.fill_(0xAB)
    c = lambda a: torch.from_numpy(a).cuda()
    _, r = oracle_prune(oracle, g, tg)
    for _ in range(3):                         # same buffers, dirty from the previous call
        assert buf.prune(c(tg.tgt_rowptr), c(tg.tgt_idx)) == 0
        assert_same(buf.to_host(), r, "reuse")
    # then a different, smaller query in the same buffers
    tg1 = targets_from_sets([[int(tg.tgt_idx[0])]])
    buf1 = dgn.PruneBuffers(dg, 1)
    assert buf1.prune(c(tg1.tgt_rowptr), c(tg1.tgt_idx)) == 0
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    assert_same(buf1.to_host(), oracle.forward_prune(adj, 1, tg1.tgt_rowptr, tg1.tgt_idx), "single")


@pytest.mark.parametrize("k,scale", [(1, 0.5), (3, 0.01), (4, 0.001)])
def test_schedule_knobs_do_not_change_results(dgn, oracle, k, scale):
    """Deferral decay, forced one-launch-per-level traversal and a tiny frontier queue (which forces
    the overflow fix-up sweeps) are schedules only: the fixed point is unique."""
    g, tg = gg.config(k, scale)
    _, r = oracle_prune(oracle, g, tg)
    for knobs in (dict(defer_percent=100), dict(defer_percent=50), dict(defer_percent=95),
                  dict(traversal=1), dict(traversal=1, defer_percent=60), dict(traversal=2), dict(traversal=2, defer_percent=70),
                  dict(traversal=2, defer_percent=90, defer_start_shift=3, defer_floor_shift=14),
                  dict(max_queue_entries=1000), dict(max_queue_entries=37, traversal=1)):
        st = dgn.dgn_stats()
        _, _, out = gpu_prune(dgn, g, tg, stats=st, **knobs)
        assert_same(out, r, f"cfg{k} {knobs}")


# ---- the workloads at their full sizes, in the launch configuration bench.py times ---------------
def _full_size_check(dgn, oracle, k, sampled_graphs=None):
    import torch
    g, tg = gg.config(k, 1.0)
    print(f"config {k} full size: P={g.num_ops} T={g.num_tensors} E={g.nnz_in}+{g.nnz_out}", flush=True)
    dg, buf, out = gpu_prune(dgn, g, tg)
    del dg, buf
    torch.cuda.empty_cache()
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    # (1) the O(E) fixed-point certificate proves M and K as a whole (unique solution on a DAG)
    S = oracle.seed_masks(g.num_tensors, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx)
    assert oracle.certificate(adj, S, out["tensor_mask"], out["op_mask"]) == 0
    # (2) properties of the compacted outputs that hold at any size
    assert np.array_equal(out["op_flag"], (out["op_mask"] != 0).astype(np.uint8))
    assert np.array_equal(out["kept_ops"], np.nonzero(out["op_mask"])[0].astype(np.int32))
    assert np.array_equal(out["kept_masks"], out["op_mask"][out["kept_ops"]])
    assert out["kept_count"][0] == len(out["kept_ops"])
    if sampled_graphs is None:
        # (3) element by element against Algorithm 1 itself
        r = oracle.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx, g.num_graphs, g.graph_op_offsets)
        assert_same(out, r, f"cfg{k} full size")
    else:
        # (3') Algorithm 1 on sampled graphs of the packed batch, one by one
        Q = tg.num_sets
        for gi in sampled_graphs:
            one = gg.layered(20000, gg.BASE_SEED + 4000 + gi)
            t1 = gg.targets_tail(one, gg.BASE_SEED + 4000 + gi, Q, 4, 4, 0.10)
            _, r1 = oracle_prune(oracle, one, t1)
            ta, tb = g.graph_tensor_offsets[gi], g.graph_tensor_offsets[gi + 1]
            oa, ob = g.graph_op_offsets[gi], g.graph_op_offsets[gi + 1]
            assert np.array_equal(out["tensor_mask"][ta:tb], r1.tensor_mask), gi
            assert np.array_equal(out["op_mask"][oa:ob], r1.op_mask), gi
            assert np.array_equal(out["per_query_count"][gi * 64:(gi + 1) * 64], r1.per_query_count), gi
            a, b = out["kept_count"][1 + gi], out["kept_count"][2 + gi]
            assert np.array_equal(out["kept_ops"][a:b] - oa, r1.kept_ops), gi
        # (4) the per-graph outputs of EVERY graph, recounted from K: kept_count[1 + g] = kept operators below graph g's
        # first operator; per_query_count[g*64 + q] = operators of graph g with bit q of K
        kept_below = np.concatenate(([0], np.cumsum(out["op_mask"] != 0)))[g.graph_op_offsets]
        assert np.array_equal(out["kept_count"][1:], kept_below.astype(np.int64))
        pq = np.zeros((g.num_graphs, 64), dtype=np.int64)
        graph_of = np.repeat(np.arange(g.num_graphs), np.diff(g.graph_op_offsets))
        for q in range(Q):
            has = ((out["op_mask"] >> np.uint64(q)) & np.uint64(1)).astype(bool)
            pq[:, q] = np.bincount(graph_of[has], minlength=g.num_graphs)
        assert np.array_equal(out["per_query_count"].reshape(g.num_graphs, 64), pq)


def test_full_size_config2_unrolled_rnn(dgn, oracle):
    _full_size_check(dgn, oracle, 2)


def test_full_size_config3_power_law_50m(dgn, oracle):
    _full_size_check(dgn, oracle, 3)


def test_full_size_config4_packed_batch(dgn, oracle):
    _full_size_check(dgn, oracle, 4, sampled_graphs=[0, 1, 777, 2048, 4095])


def _pack(graphs_and_sets, Q):
    """Concatenate (Graph, list-of-Q-target-lists) pairs into one packed batch with global ids."""
    in_op, in_t, out_op, out_t, sets = [], [], [], [], []
    op_off, t_off = [0], [0]
    for g, s in graphs_and_sets:
        in_op.append(g.in_op.astype(np.int64) + op_off[-1]); in_t.append(g.in_tensor.astype(np.int64) + t_off[-1])
        out_op.append(g.out_op.astype(np.int64) + op_off[-1]); out_t.append(g.out_tensor.astype(np.int64) + t_off[-1])
        sets += [[t + t_off[-1] for t in one] for one in s]
        op_off.append(op_off[-1] + g.num_ops); t_off.append(t_off[-1] + g.num_tensors)
    cat = lambda xs: np.concatenate(xs).astype(np.int32) if xs else np.zeros(0, np.int32)
    g = gg.Graph(op_off[-1], t_off[-1], cat(in_op), cat(in_t), cat(out_op), cat(out_t), len(graphs_and_sets),
                 np.asarray(op_off, np.int64), np.asarray(t_off, np.int64), "packed")
    return g, targets_from_sets(sets, Q)


def test_packed_batches_use_the_per_graph_sweep(dgn, oracle):
    """Batches of >= 64 topologically numbered graphs take the one-wave-per-graph sweep; same results."""
    # equal-sized layered graphs
    g, tg = gg.batch_layered(96, 700, 4242, num_sets=64)
    st = dgn.dgn_stats()
    _, _, out = gpu_prune(dgn, g, tg, stats=st)
    _, r = oracle_prune(oracle, g, tg)
    assert_same(out, r, "batch 96x700")
    assert st.levels == 0                     # no frontier levels were run
    _, _, out = gpu_prune(dgn, g, tg, recompute_keep=True)
    assert_same(out, r, "batch 96x700 recompute_keep")
    _, _, out = gpu_prune(dgn, g, tg, traversal=1)          # and the generic traversal agrees
    assert_same(out, r, "batch 96x700 generic")
    # ragged graphs with awkward operators (no inputs, no outputs, duplicate edges), some graphs empty
    rng = np.random.default_rng(5)
    Q = 7
    parts = []
    for i in range(130):
        P = int(rng.integers(0, 200))
        gi, _ = random_small_graph(rng, P, num_inputs=int(rng.integers(1, 5)), multi_producer=False)
        parts.append((gi, [[int(rng.integers(0, gi.num_tensors)) for _ in range(int(rng.integers(0, 4)))]
                           for _ in range(Q)]))
    g, tg = _pack(parts, Q)
    st = dgn.dgn_stats()
    _, _, out = gpu_prune(dgn, g, tg, validate=True, stats=st)
    _, r = oracle_prune(oracle, g, tg)
    assert_same(out, r, "ragged batch")
    assert st.levels == 0
    # graphs whose operator order is NOT topological fall back to the frontier traversal
    parts = []
    for i in range(70):
        gi, _ = random_small_graph(rng, int(rng.integers(1, 80)), num_inputs=3, multi_producer=True)
        parts.append((gi, [[int(rng.integers(0, gi.num_tensors))] for _ in range(3)]))
    g, tg = _pack(parts, 3)
    _, _, out = gpu_prune(dgn, g, tg)
    _, r = oracle_prune(oracle, g, tg)
    assert_same(out, r, "non-topological batch")


def _rewriting_graph(rng, num_ops, num_inputs):
    """Operators in topological order where some tensors have several producers: an operator may write again to a
    tensor that nobody has read yet (so every reader still comes after every writer), often one created many
    operators earlier."""
    ops, n_t, unread = [], num_inputs, []
    for _ in range(num_ops):
        ins = [int(rng.integers(max(0, n_t - 40), n_t)) for _ in range(int(rng.integers(1, 4)))]
        unread = [t for t in unread if t not in ins]
        outs = []
        for _ in range(int(rng.integers(1, 3))):
            if unread and rng.random() < 0.3:
                y = unread[int(rng.integers(0, len(unread)))]
                if y not in outs:
                    outs.append(y)
                    continue
            outs.append(n_t)
            unread.append(n_t)
            n_t += 1
        ops.append((ins, outs))
    return graph_from_ops(ops, n_t, "rewriting"), ops


def test_swept_batches_with_tensors_written_by_several_operators(dgn, oracle):
    """The per-graph sweep fetches a group's tensor words while the group before it is still being worked on; a
    tensor written again by an operator of an earlier group is the case where that word was stored by this very
    sweep.  Graphs of several groups each, re-written tensors in the same and in different groups."""
    rng = np.random.default_rng(77)
    Q = 5
    parts, rewritten = [], 0
    for i in range(80):
        gi, ops = _rewriting_graph(rng, int(rng.integers(100, 700)), 4)
        writers = np.bincount(np.concatenate([np.asarray(o[1], np.int64) for o in ops]), minlength=gi.num_tensors)
        rewritten += int((writers > 1).sum())
        parts.append((gi, [[int(rng.integers(gi.num_tensors // 2, gi.num_tensors)) for _ in range(int(rng.integers(1, 4)))]
                           for _ in range(Q)]))
    assert rewritten > 1000
    g, tg = _pack(parts, Q)
    st = dgn.dgn_stats()
    _, _, out = gpu_prune(dgn, g, tg, validate=True, stats=st)       # the order is topological: validation passes
    _, r = oracle_prune(oracle, g, tg)
    assert_same(out, r, "swept batch with re-written tensors")
    assert st.levels == 0                                            # and the sweep was taken
    _, _, out = gpu_prune(dgn, g, tg, traversal=1)
    assert_same(out, r, "the same through the frontier traversal")


def _hub_graph(rng, num_ops, num_inputs, wide):
    """Topological operator list with hub tensors (each read by dozens of the operators that follow it, far more
    than the sweep registers per producer) and, with ``wide``, operators of up to 12 inputs, so that 64
    consecutive operators can have more input edges than the sweep's tables take."""
    ops, n_t, hub = [], num_inputs, 0
    for o in range(num_ops):
        n_in = int(rng.choice([6, 9, 12])) if wide and rng.random() < 0.6 else int(rng.integers(1, 4))
        ins = [hub if rng.random() < 0.45 else int(rng.integers(max(0, n_t - 40), n_t)) for _ in range(n_in)]
        outs = list(range(n_t, n_t + int(rng.integers(1, 3))))
        n_t += len(outs)
        if o % 37 == 0:
            hub = outs[0]
        ops.append((ins, outs))
    return graph_from_ops(ops, n_t, "hubs"), ops


@pytest.mark.parametrize("wide", [False, True])
def test_swept_batches_with_hub_tensors_and_wide_operators(dgn, oracle, wide):
    """The sweep's side paths: a producer with more in-group readers than it registers (masks resolved lane by
    lane instead of by relaxation) and groups with too many input edges for the tables (walked one operator at
    a time, straight to memory), mixed with ordinary groups in the same graphs."""
    rng = np.random.default_rng(91 + wide)
    Q = 64
    parts = []
    for i in range(72):
        gi, ops = _hub_graph(rng, int(rng.integers(130, 500)), 3, wide)
        parts.append((gi, [[int(rng.integers(gi.num_tensors // 3, gi.num_tensors)) for _ in range(int(rng.integers(0, 3)))]
                           for _ in range(Q)]))
    readers = np.bincount(parts[0][0].in_tensor, minlength=parts[0][0].num_tensors)
    assert readers.max() > 12                                        # hubs exist
    if wide:
        fan_in = np.bincount(parts[0][0].in_op, minlength=parts[0][0].num_ops)
        assert max(fan_in[i:i + 64].sum() for i in range(0, len(fan_in) - 63)) > 256
    g, tg = _pack(parts, Q)
    st = dgn.dgn_stats()
    _, _, out = gpu_prune(dgn, g, tg, validate=True, stats=st)
    _, r = oracle_prune(oracle, g, tg)
    assert_same(out, r, f"swept batch with hubs (wide={wide})")
    assert st.levels == 0


def test_more_than_64_sets_run_word_by_word(dgn, oracle):
    """150 target sets on one graph: three words of 64, 64 and 22 sets, each equal to the oracle's run
    of Algorithm 1 on exactly those sets."""
    import torch
    g, _ = gg.config(1, 0.3)
    n_sets = 150
    tg = gg.targets_tail(g, 4242, n_sets, 1, 5, 0.2)
    dg = dgn.DeviceGraph.from_coo(g)
    P, T, W = g.num_ops, g.num_tensors, 3
    rc, sb = dgn.dgn_prune_workspace(dg.handle, 64)
    assert rc == 0
    dev = "cuda"
    M = torch.empty(W * T, dtype=torch.int64, device=dev)
    K = torch.empty(W * P, dtype=torch.int64, device=dev)
    flag = torch.empty(W * P, dtype=torch.uint8, device=dev)
    kept = torch.empty(W * P, dtype=torch.int32, device=dev)
    kmask = torch.empty(W * P, dtype=torch.int64, device=dev)
    count = torch.empty(W, dtype=torch.int64, device=dev)
    pq = torch.empty(W * 64, dtype=torch.int64, device=dev)
    scratch = torch.empty(sb, dtype=torch.uint8, device=dev)
    st = dgn.dgn_stats()
    rc = dgn.dgn_prune_words(dg.handle, n_sets, int(tg.tgt_idx.shape[0]), torch.from_numpy(tg.tgt_rowptr).cuda(),
                             torch.from_numpy(tg.tgt_idx).cuda(), M, K, flag, kept, kmask, count, pq, scratch, sb,
                             None, st)
    assert rc == 0, dgn.dgn_strerror(rc)
    torch.cuda.synchronize()
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    u = lambda t: t.cpu().numpy().view(np.uint64)
    levels = 0
    for w in range(W):
        lo, hi = 64 * w, min(64 * (w + 1), n_sets)
        rowptr = (tg.tgt_rowptr[lo:hi + 1] - tg.tgt_rowptr[lo]).astype(np.int32)
        idx = tg.tgt_idx[tg.tgt_rowptr[lo]:tg.tgt_rowptr[hi]]
        ref = oracle.forward_prune(adj, hi - lo, rowptr, idx)
        n = int(count[w].item())
        assert n == int(ref.kept_count[0])
        assert np.array_equal(u(M[w * T:(w + 1) * T]), ref.tensor_mask), f"word {w}"
        assert np.array_equal(u(K[w * P:(w + 1) * P]), ref.op_mask), f"word {w}"
        assert np.array_equal(flag[w * P:(w + 1) * P].cpu().numpy(), ref.op_flag), f"word {w}"
        assert np.array_equal(kept[w * P:w * P + n].cpu().numpy(), ref.kept_ops), f"word {w}"
        assert np.array_equal(u(kmask[w * P:w * P + n]), ref.kept_masks), f"word {w}"
        assert np.array_equal(pq[w * 64:(w + 1) * 64].cpu().numpy(), ref.per_query_count), f"word {w}"
    assert st.levels > 3 and st.launches > 3
    # a packed batch is refused, and so is a set count below one
    rc = dgn.dgn_prune_words(dg.handle, 0, 0, torch.from_numpy(tg.tgt_rowptr).cuda(), None, M, K, flag, kept, kmask,
                             count, pq, scratch, sb)
    assert rc == dgn.DGN_ERR_TOO_MANY_SETS


def _prefix_graph(g, num_ops):
    """The first num_ops operators of g (creation order) as a graph of their own, with the tensors they use."""
    keep_in, keep_out = g.in_op < num_ops, g.out_op < num_ops
    T = int(max(g.in_tensor[keep_in].max(initial=0), g.out_tensor[keep_out].max(initial=0))) + 1
    return gg.Graph(num_ops, T, g.in_op[keep_in].copy(), g.in_tensor[keep_in].copy(), g.out_op[keep_out].copy(),
                    g.out_tensor[keep_out].copy(), name=g.name + "-prefix")


@pytest.mark.parametrize("k,scale", [(0, 1.0), (1, 0.5), (2, 0.02), (3, 0.02), (4, 0.002)])
def test_incremental_prune_adds_target_sets(dgn, oracle, k, scale):
    """Pruning for some sets and then adding the others incrementally gives the one-shot result."""
    import torch
    g, tg = gg.config(k, scale)
    Q = tg.num_sets
    n_sets = len(tg.tgt_rowptr) - 1
    # first call: every other set is empty; second call (incremental): all sets
    rowptr1 = tg.tgt_rowptr.copy()
    cnt = np.diff(tg.tgt_rowptr)
    cnt1 = cnt.copy()
    cnt1[1::2] = 0
    if n_sets == 1:
        cnt1[0] = max(1, cnt[0] // 2)                       # a single set: only some of its targets first
    rowptr1 = np.concatenate([[0], np.cumsum(cnt1)]).astype(np.int32)
    idx1 = np.concatenate([tg.tgt_idx[tg.tgt_rowptr[s]:tg.tgt_rowptr[s] + cnt1[s]] for s in range(n_sets)] +
                          [np.zeros(0, np.int32)]).astype(np.int32)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, Q)
    rc = buf.prune(torch.from_numpy(rowptr1).cuda(), torch.from_numpy(idx1).cuda())
    assert rc == 0
    adj, _ = oracle_prune(oracle, g, tg)
    part = oracle.forward_prune(adj, Q, rowptr1, idx1, g.num_graphs, g.graph_op_offsets)
    assert_same(buf.to_host(), part, f"cfg{k} first part")
    st = dgn.dgn_stats()
    rc = buf.prune(torch.from_numpy(tg.tgt_rowptr).cuda(), torch.from_numpy(tg.tgt_idx).cuda(),
                   options=dgn.dgn_options(incremental=1), stats=st)
    assert rc == 0
    _, full = oracle_prune(oracle, g, tg)
    assert_same(buf.to_host(), full, f"cfg{k} incremental")
    # adding nothing new changes nothing and traverses nothing
    rc = buf.prune(torch.from_numpy(tg.tgt_rowptr).cuda(), torch.from_numpy(tg.tgt_idx).cuda(),
                   options=dgn.dgn_options(incremental=1, recompute_keep=1), stats=st)
    assert rc == 0 and (st.tensor_visits == 0 or g.num_graphs > 1)
    assert_same(buf.to_host(), full, f"cfg{k} incremental, nothing new")


def test_incremental_prune_of_an_extended_graph(dgn, oracle):
    """A recorded graph grows by appended operators (an unrolled loop gets one more step): the result for
    the shorter graph, zero-extended, plus the new targets gives the result of pruning the longer graph."""
    import torch
    g, tg = gg.config(2, 0.02)                              # 200 steps of 1000 operators
    P_old = g.num_ops - 3000                                # the graph before its last three steps
    g_old = _prefix_graph(g, P_old)
    old_targets = gg.targets_range(777, 1, 20, 20, 16, g_old.num_tensors)
    dg_old = dgn.DeviceGraph.from_coo(g_old)
    b_old = dgn.PruneBuffers(dg_old, 1)
    assert b_old.prune(torch.from_numpy(old_targets.tgt_rowptr).cuda(), torch.from_numpy(old_targets.tgt_idx).cuda()) == 0
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, 1)
    buf.tensor_mask.zero_()
    buf.op_mask.zero_()
    buf.tensor_mask[: g_old.num_tensors] = b_old.tensor_mask
    buf.op_mask[:P_old] = b_old.op_mask
    new_idx = np.asarray([g.num_tensors - 1, g.num_tensors - 500], np.int32)        # targets in the appended steps
    rc = buf.prune(torch.from_numpy(np.asarray([0, 2], np.int32)).cuda(), torch.from_numpy(new_idx).cuda(),
                   options=dgn.dgn_options(incremental=1))
    assert rc == 0
    all_idx = np.concatenate([old_targets.tgt_idx, new_idx]).astype(np.int32)
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    ref = oracle.forward_prune(adj, 1, np.asarray([0, len(all_idx)], np.int32), all_idx)
    assert_same(buf.to_host(), ref, "extended graph")


@pytest.mark.parametrize("which", ["in", "out", "none"])
def test_csr_builder_skips_only_the_sorts_it_may_skip(dgn, oracle, which):
    """Edges that already come in row order are copied, not sorted; any mix of ordered and shuffled edge
    lists must give the same adjacency as the oracle's stable sort."""
    g, tg = gg.config(3, 0.004)
    gs = gg.shuffle_coo(g, 5)
    if which == "in":                                       # only the input edges are shuffled
        mixed = gg.Graph(g.num_ops, g.num_tensors, gs.in_op, gs.in_tensor, g.out_op, g.out_tensor, name="mixed")
    elif which == "out":                                    # only the output edges are shuffled
        mixed = gg.Graph(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, gs.out_op, gs.out_tensor, name="mixed")
    else:                                                   # nothing shuffled, but tensor ids permuted: the
        mixed, tg, _ = gg.relabel_tensors(g, tg, 3)         # producer lists still need their sort
    adj = oracle.build_adjacency(mixed.num_ops, mixed.num_tensors, mixed.in_op, mixed.in_tensor, mixed.out_op,
                                 mixed.out_tensor)
    dg = dgn.DeviceGraph.from_coo(mixed, validate=True)
    csr = {n: v.cpu().numpy() for n, v in dg.csr().items()}
    for name in ("in_rowptr", "in_idx", "out_rowptr", "out_idx", "prod_rowptr", "prod_idx"):
        assert np.array_equal(csr[name], getattr(adj, name)), f"{which}: {name}"
    _, _, out = gpu_prune(dgn, mixed, tg)
    assert_same(out, oracle.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx), which)


@pytest.mark.parametrize("offset", [1, 3, 4])
def test_flag_bytes_at_unaligned_addresses_and_ragged_sizes(dgn, oracle, offset):
    """The flag bytes leave the count pass eight at a time when they can; a flag buffer that is not 8-byte
    aligned and an operator count that is not a multiple of 8 (or of the tile) must give the same bytes."""
    import torch
    g, tg = gg.config(1, 0.3)
    keep_in, keep_out = g.in_op < g.num_ops - 3, g.out_op < g.num_ops - 3        # drop three operators: ragged count
    g = gg.Graph(g.num_ops - 3, g.num_tensors, g.in_op[keep_in].copy(), g.in_tensor[keep_in].copy(),
                 g.out_op[keep_out].copy(), g.out_tensor[keep_out].copy(), name="ragged")
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.PruneBuffers(dg, tg.num_sets)
    big = torch.full((g.num_ops + 16,), 77, dtype=torch.uint8, device="cuda")
    flags = big[offset:offset + g.num_ops]
    rc = dgn.dgn_prune(dg.handle, tg.num_sets, int(tg.tgt_idx.shape[0]), torch.from_numpy(tg.tgt_rowptr).cuda(),
                       torch.from_numpy(tg.tgt_idx).cuda(), buf.tensor_mask, buf.op_mask, flags, buf.kept_ops,
                       buf.kept_masks, buf.kept_count, buf.per_query_count, buf.scratch, buf.scratch_bytes)
    assert rc == 0
    torch.cuda.synchronize()
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    ref = oracle.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx)
    assert np.array_equal(flags.cpu().numpy(), ref.op_flag)
    assert (big[:offset] == 77).all().item() and (big[offset + g.num_ops:] == 77).all().item()   # nothing written outside
    out = buf.to_host()
    assert np.array_equal(out["op_mask"], ref.op_mask) and np.array_equal(out["kept_ops"], ref.kept_ops)


def test_csr_builder_with_long_runs_of_empty_rows(dgn, oracle):
    """Operators without edges and tensors nobody writes leave long runs of empty rows; ordered input takes
    the single-pass path, which hands such runs to a separate row-pointer pass."""
    P, T = 5000, 20000
    ops = [([], []) for _ in range(P)]
    ops[10] = ([3, 15000], [16000])
    ops[3000] = ([16000, 7], [16001, 19999])
    ops[4999] = ([19999], [200])                    # writes a low-numbered tensor: producer lists need their sort
    g = graph_from_ops(ops, T)
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    for variant in ("ordered", "shuffled"):
        gv = g if variant == "ordered" else gg.shuffle_coo(g, 9)
        ref = oracle.build_adjacency(gv.num_ops, gv.num_tensors, gv.in_op, gv.in_tensor, gv.out_op, gv.out_tensor)
        dg = dgn.DeviceGraph.from_coo(gv)
        csr = {n: v.cpu().numpy() for n, v in dg.csr().items()}
        for name in ("in_rowptr", "in_idx", "out_rowptr", "out_idx", "prod_rowptr", "prod_idx"):
            assert np.array_equal(csr[name], getattr(ref, name)), f"{variant}: {name}"
    tg = targets_from_sets([[200], [16001]])
    _, _, out = gpu_prune(dgn, g, tg)
    assert_same(out, oracle.forward_prune(adj, 2, tg.tgt_rowptr, tg.tgt_idx), "sparse rows")


def test_edges_and_targets_that_cross_packed_graphs_are_reported(dgn):
    """In a packed batch every edge of an operator and every target of a set must stay inside its graph."""
    import torch
    parts = []
    rng = np.random.default_rng(3)
    for i in range(70):
        gi, _ = random_small_graph(rng, 40, num_inputs=3)
        parts.append((gi, [[0], [1]]))
    g, tg = _pack(parts, 2)
    bad = gg.Graph(g.num_ops, g.num_tensors, g.in_op.copy(), g.in_tensor.copy(), g.out_op.copy(), g.out_tensor.copy(),
                   g.num_graphs, g.graph_op_offsets, g.graph_tensor_offsets, "crossing")
    e = int(np.flatnonzero(bad.in_op >= g.graph_op_offsets[5])[0])          # an input edge of graph 5 ...
    bad.in_tensor[e] = int(g.graph_tensor_offsets[9])                        # ... reads a tensor of graph 9
    with pytest.raises(dgn.DgnError) as err:
        dgn.DeviceGraph.from_coo(bad, validate=True)
    assert err.value.code == dgn.DGN_ERR_ID_OUT_OF_RANGE
    # a target of graph 0's first set that lies in graph 3
    dg = dgn.DeviceGraph.from_coo(g, validate=True)
    buf = dgn.PruneBuffers(dg, 2)
    idx = tg.tgt_idx.copy()
    idx[0] = int(g.graph_tensor_offsets[3])
    rc = buf.prune(torch.from_numpy(tg.tgt_rowptr).cuda(), torch.from_numpy(idx).cuda())
    assert rc == dgn.DGN_ERR_ID_OUT_OF_RANGE


def test_depth_stress_unrolled_rnn_with_every_recurrent_edge(dgn, oracle):
    """The unrolled-RNN family with a recurrent edge on EVERY operator and the final loss as the only target: the
    dependence chain runs through all time steps, so the traversal needs at least as many levels as there are
    steps (2 000 here, 50 operators each; the workload's own recurrent probability of 0.1 dies out after a few)."""
    steps = 2000
    g = gg.rnn(steps, 50, gg.BASE_SEED + 2000, rec_prob=1.0, name="rnn-depth-stress")
    tg = targets_from_sets([[g.num_tensors - 1]])
    st = dgn.dgn_stats()
    _, _, out = gpu_prune(dgn, g, tg, stats=st)
    _, r = oracle_prune(oracle, g, tg)
    assert_same(out, r, "depth stress")
    assert st.levels >= steps
    kept_steps = np.unique(r.kept_ops // 50)
    assert len(kept_steps) == steps            # every time step keeps an operator
    _, _, out = gpu_prune(dgn, g, tg, traversal=2, defer_percent=70)
    assert_same(out, r, "depth stress, deferral on")


def test_borrowed_csr_with_bad_row_pointers_is_reported(dgn, oracle):
    """dgn_graph_from_csr checks the borrowed row pointers on the device before any kernel trusts them."""
    import torch
    g, _ = gg.config(0, 0.5)
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    c = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    good = dict(in_rowptr=adj.in_rowptr.copy(), in_idx=adj.in_idx.copy(), out_rowptr=adj.out_rowptr.copy(),
                out_idx=adj.out_idx.copy())

    def build(**changed):
        a = dict(good, **changed)
        dev = [c(a[n]) for n in ("in_rowptr", "in_idx", "out_rowptr", "out_idx")]     # alive until the build returns
        desc = dgn.make_csr_desc(g.num_ops, g.num_tensors, *dev)
        rc, gb, sb = dgn.dgn_graph_from_csr_workspace(desc)
        assert rc == 0
        mem = torch.empty(gb, dtype=torch.uint8, device="cuda")
        scr = torch.empty(sb, dtype=torch.uint8, device="cuda")
        rc, h = dgn.dgn_graph_from_csr(desc, mem, gb, scr, sb)
        if h:
            dgn.dgn_graph_destroy(h)
        return rc

    assert build() == 0
    rp = good["in_rowptr"].copy()
    rp[5], rp[6] = rp[6] + 1, rp[5]                      # decreasing somewhere in the middle
    assert build(in_rowptr=rp) == dgn.DGN_ERR_BAD_CSR
    rp = good["out_rowptr"].copy()
    rp[-1] -= 1                                          # does not end at nnz
    assert build(out_rowptr=rp) == dgn.DGN_ERR_BAD_CSR
    rp = good["out_rowptr"].copy()
    rp[0] = 1                                            # does not start at zero
    assert build(out_rowptr=rp) == dgn.DGN_ERR_BAD_CSR
    ix = good["in_idx"].copy()
    ix[3] = g.num_tensors                                # a tensor id out of range
    assert build(in_idx=ix) == dgn.DGN_ERR_ID_OUT_OF_RANGE
