"""Pins for the CPU oracle: things the paper and the mathematics fix, none of them computed by the
oracle itself.  A dropped term, a wrong direction, a transposed adjacency or an off-by-one in the
oracle fails at least one of these."""
import numpy as np
import pytest

import graphgen as gg
from helpers import (brute_force_masks, graph_from_ops, load_worked_example, naive_forward_marks,
                     random_small_graph, targets_from_sets)


def run(orc, g, tg):
    adj = orc.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    return adj, orc.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx, g.num_graphs,
                                  g.graph_op_offsets)


# ---- the paper's worked example (Sec. 2.2) ----------------------------------------------------
def test_worked_example_values(oracle):
    g, tid, cases = load_worked_example()
    for c in cases:
        _, r = run(oracle, g, c["targets"])
        assert np.array_equal(r.tensor_mask, c["M"]), c["name"]
        assert np.array_equal(r.op_mask, c["K"]), c["name"]
        assert np.array_equal(r.kept_ops, c["kept"]), c["name"]
        assert np.array_equal(r.per_query_count[: len(c["pq"])], c["pq"]), c["name"]
        assert r.kept_count[0] == len(c["kept"])
        assert np.array_equal(r.op_flag, (c["K"] != 0).astype(np.uint8))


def test_worked_example_b_not_marked_but_naive_marks_it(oracle):
    g, tid, cases = load_worked_example()
    _, r = run(oracle, g, cases[0]["targets"])          # solve y = a*x only
    assert r.tensor_mask[tid["b"]] == 0
    ops = [([0, 1], [3]), ([3, 2], [4]), ([4], [5]), ([1, 5], [6])]
    assert tid["b"] in naive_forward_marks(ops, 7)       # the strawman traversal does mark b


# ---- brute force over the definition on tiny graphs --------------------------------------------
@pytest.mark.parametrize("multi", [False, True])
def test_brute_force_tiny_graphs(oracle, multi):
    rng = np.random.default_rng(1234 + multi)
    for trial in range(60):
        P = int(rng.integers(1, 40))
        g, ops = random_small_graph(rng, P, num_inputs=int(rng.integers(1, 5)), multi_producer=multi)
        Q = int(rng.integers(1, 6))
        sets = [[int(rng.integers(0, g.num_tensors)) for _ in range(int(rng.integers(0, 4)))]
                for _ in range(Q)]
        tg = targets_from_sets(sets)
        _, r = run(oracle, g, tg)
        M, K = brute_force_masks(ops, g.num_tensors, sets, Q)
        assert np.array_equal(r.tensor_mask, M), (trial, ops, sets)
        assert np.array_equal(r.op_mask, K), (trial, ops, sets)
        assert np.array_equal(r.kept_ops, np.nonzero(K)[0].astype(np.int32))


# ---- closed forms ---------------------------------------------------------------------------
def test_chain(oracle):
    n = 50
    g = graph_from_ops([([i], [i + 1]) for i in range(n)], n + 1)
    for k in (0, 1, 17, n):
        _, r = run(oracle, g, targets_from_sets([[k]]))
        assert np.array_equal(r.tensor_mask, (np.arange(n + 1) <= k).astype(np.uint64))
        assert np.array_equal(r.kept_ops, np.arange(k, dtype=np.int32))


def test_deep_chain_needs_no_call_stack(oracle):
    n = 300_000
    ops = np.arange(n, dtype=np.int32)
    g = gg.Graph(n, n + 1, ops, ops, ops, ops + 1)
    _, r = run(oracle, g, targets_from_sets([[n]]))
    assert int(r.kept_count[0]) == n and r.tensor_mask.all()
    assert r.parent_edges[0] == n


def test_binary_reduction_tree(oracle):
    # leaves 0..2^d-1; node at height h combines two nodes of height h-1
    d = 6
    ops, level, nxt = [], list(range(2 ** d)), 2 ** d
    heights = {t: 0 for t in level}
    while len(level) > 1:
        new = []
        for i in range(0, len(level), 2):
            ops.append(([level[i], level[i + 1]], [nxt]))
            heights[nxt] = heights[level[i]] + 1
            new.append(nxt)
            nxt += 1
        level = new
    g = graph_from_ops(ops, nxt)
    for t in (0, 2 ** d, 2 ** d + 5, nxt - 3, nxt - 1):
        _, r = run(oracle, g, targets_from_sets([[t]]))
        h = heights[t]
        assert int((r.tensor_mask != 0).sum()) == 2 ** (h + 1) - 1
        assert int(r.kept_count[0]) == 2 ** h - 1


def test_disconnected_component_stays_zero(oracle):
    a = [([0], [2]), ([2], [3])]
    b = [([1], [4]), ([4], [5])]
    g = graph_from_ops([a[0], b[0], a[1], b[1]], 6)
    _, r = run(oracle, g, targets_from_sets([[3]]))
    assert list(r.tensor_mask) == [1, 0, 1, 1, 0, 0]
    assert list(r.kept_ops) == [0, 2]


def test_all_sinks_keep_everything_empty_keeps_nothing(oracle):
    g, tg = gg.config(0)
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    consumed = np.zeros(g.num_tensors, bool)
    consumed[g.in_tensor] = True
    produced = np.zeros(g.num_tensors, bool)
    produced[g.out_tensor] = True
    sinks = np.nonzero(~consumed)[0]
    r = oracle.forward_prune(adj, 1, np.array([0, len(sinks)], np.int32), sinks.astype(np.int32))
    # every operator has an output, and every tensor reaches a sink: all ops kept; every tensor that
    # is read or produced (or is itself a sink) is coloured
    assert int(r.kept_count[0]) == g.num_ops
    assert r.tensor_mask.all()
    r0 = oracle.forward_prune(adj, 3, np.zeros(4, np.int32), np.zeros(0, np.int32))
    assert not r0.tensor_mask.any() and not r0.op_mask.any() and r0.kept_count[0] == 0
    assert not r0.per_query_count.any()


def test_zero_output_operator_removed_and_partial_outputs_kept(oracle):
    # op0: x -> (u, v); op1: u -> (nothing); op2: u -> w.  target w.
    g = graph_from_ops([([0], [1, 2]), ([1], []), ([1], [3])], 4)
    _, r = run(oracle, g, targets_from_sets([[3]]))
    assert list(r.tensor_mask) == [1, 1, 0, 1]      # v stays un-coloured although op0 is kept
    assert list(r.kept_ops) == [0, 2]               # the zero-output op1 is removed


def test_duplicate_edges_and_duplicate_targets(oracle):
    g = graph_from_ops([([0, 0], [1]), ([1, 1, 0], [2])], 3)    # Mul(x, x) style duplicates
    _, r = run(oracle, g, targets_from_sets([[2, 2, 2], [1, 2]]))
    assert list(r.tensor_mask) == [3, 3, 3]
    assert list(r.op_mask) == [3, 3]


# ---- a second algorithm and the fixed-point certificate, on the five workload families ---------
SMALL = [(0, 1.0), (1, 0.1), (2, 0.004), (3, 0.002), (4, 0.002)]


@pytest.mark.parametrize("k,scale", SMALL)
def test_reverse_sweep_and_certificate_agree(oracle, k, scale):
    g, tg = gg.config(k, scale)
    adj, r = run(oracle, g, tg)
    S = oracle.seed_masks(g.num_tensors, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx)
    M2, K2 = oracle.reverse_sweep(adj, S)
    assert np.array_equal(M2, r.tensor_mask)
    assert np.array_equal(K2, r.op_mask)
    assert oracle.certificate(adj, S, r.tensor_mask, r.op_mask) == 0
    # the certificate is not vacuous: any single wrong bit is caught
    rng = np.random.default_rng(k)
    for _ in range(5):
        Mb = r.tensor_mask.copy()
        t = int(rng.integers(0, g.num_tensors))
        Mb[t] ^= np.uint64(1 << int(rng.integers(0, tg.num_sets)))
        assert oracle.certificate(adj, S, Mb, r.op_mask) > 0
    # the result is non-trivial (something kept, something removed) on every family
    assert 0 < r.kept_count[0] < g.num_ops
    # O(n) claim of Sec. 2.2: a set never examines more Parent() entries than the graph holds
    fan_in = np.diff(adj.in_rowptr).astype(np.int64)
    n_out = np.diff(adj.out_rowptr).astype(np.int64)
    assert r.parent_edges.max() <= int((fan_in * n_out).sum())


@pytest.mark.parametrize("k,scale", SMALL[:4])
def test_batch_semantics(oracle, k, scale):
    g, tg = gg.config(k, scale)
    adj, r = run(oracle, g, tg)
    Q = tg.num_sets
    for q in sorted({0, Q // 2, Q - 1}):
        a, b = tg.tgt_rowptr[q], tg.tgt_rowptr[q + 1]
        single = oracle.forward_prune(adj, 1, np.array([0, b - a], np.int32), tg.tgt_idx[a:b])
        bit = (r.tensor_mask >> np.uint64(q)) & np.uint64(1)
        assert np.array_equal(bit, single.tensor_mask)
        assert np.array_equal((r.op_mask >> np.uint64(q)) & np.uint64(1), single.op_mask)
        assert r.per_query_count[q] == single.kept_count[0]
    # union of two sets = OR of the results; adding targets never clears a bit
    if Q >= 2:
        a0, a1, a2 = tg.tgt_rowptr[0], tg.tgt_rowptr[1], tg.tgt_rowptr[2]
        both = oracle.forward_prune(adj, 1, np.array([0, a2 - a0], np.int32), tg.tgt_idx[a0:a2])
        u = ((r.tensor_mask | (r.tensor_mask >> np.uint64(1))) & np.uint64(1))
        assert np.array_equal(both.tensor_mask, u)
    # bits at or above Q are never set
    if Q < 64:
        assert not (r.tensor_mask >> np.uint64(Q)).any() and not (r.op_mask >> np.uint64(Q)).any()


@pytest.mark.parametrize("k,scale", SMALL)
def test_keep_and_compaction_properties(oracle, k, scale):
    g, tg = gg.config(k, scale)
    adj, r = run(oracle, g, tg)
    assert np.all(np.diff(r.kept_ops) > 0)                                  # creation order kept
    assert r.kept_count[0] == int(r.op_flag.sum()) == len(r.kept_ops)
    assert np.array_equal(r.kept_masks, r.op_mask[r.kept_ops])
    bits = ((r.op_mask[:, None] >> np.arange(64, dtype=np.uint64)[None, :]) & np.uint64(1))
    if g.num_graphs == 1:
        assert np.array_equal(bits.sum(0).astype(np.int64), r.per_query_count)
    else:
        for gi in range(g.num_graphs):
            a, b = g.graph_op_offsets[gi], g.graph_op_offsets[gi + 1]
            assert np.array_equal(bits[a:b].sum(0).astype(np.int64), r.per_query_count[gi * 64:(gi + 1) * 64])
            assert r.kept_count[1 + gi] == int((r.kept_ops < a).sum())
        assert r.kept_count[1 + g.num_graphs] == r.kept_count[0]
    # closure: each input of a kept operator is a graph input or produced by an operator kept for
    # the same sets
    prod_of = np.full(g.num_tensors, -1, np.int64)
    prod_of[g.out_tensor] = g.out_op
    src = prod_of[g.in_tensor]
    need = r.op_mask[g.in_op]
    have = np.where(src >= 0, r.op_mask[np.maximum(src, 0)], np.uint64(0xFFFFFFFFFFFFFFFF))
    assert not (need & ~have).any()
    # idempotence: pruning the compacted graph with the same targets removes nothing
    keep_e_in = r.op_flag[g.in_op] != 0
    keep_e_out = r.op_flag[g.out_op] != 0
    new_id = np.cumsum(r.op_flag, dtype=np.int64) - 1
    g2 = gg.Graph(int(r.kept_count[0]), g.num_tensors, new_id[g.in_op[keep_e_in]].astype(np.int32),
                  g.in_tensor[keep_e_in], new_id[g.out_op[keep_e_out]].astype(np.int32),
                  g.out_tensor[keep_e_out])
    adj2 = oracle.build_adjacency(g2.num_ops, g2.num_tensors, g2.in_op, g2.in_tensor, g2.out_op, g2.out_tensor)
    r2 = oracle.forward_prune(adj2, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx)
    assert r2.kept_count[0] == g2.num_ops
    assert np.array_equal(r2.tensor_mask, r.tensor_mask)


def test_relabelling_tensors_permutes_M_only(oracle):
    g, tg = gg.config(1, 0.05)
    _, r = run(oracle, g, tg)
    g2, tg2, perm = gg.relabel_tensors(g, tg, 99)
    _, r2 = run(oracle, g2, tg2)
    assert np.array_equal(r2.tensor_mask[perm], r.tensor_mask)
    assert np.array_equal(r2.op_mask, r.op_mask)
    assert np.array_equal(r2.kept_ops, r.kept_ops)


def test_packed_batch_equals_graph_by_graph(oracle):
    g, tg = gg.config(4, 0.001)     # 4 graphs of 20 000 operators
    assert g.num_graphs == 4
    _, r = run(oracle, g, tg)
    Q = tg.num_sets
    for gi in range(g.num_graphs):
        one = gg.layered(20000, gg.BASE_SEED + 4000 + gi)
        t1 = gg.targets_tail(one, gg.BASE_SEED + 4000 + gi, Q, 4, 4, 0.10)
        _, r1 = run(oracle, one, t1)
        ta, tb = g.graph_tensor_offsets[gi], g.graph_tensor_offsets[gi + 1]
        oa, ob = g.graph_op_offsets[gi], g.graph_op_offsets[gi + 1]
        assert np.array_equal(r.tensor_mask[ta:tb], r1.tensor_mask)
        assert np.array_equal(r.op_mask[oa:ob], r1.op_mask)
        sel = (r.kept_ops >= oa) & (r.kept_ops < ob)
        assert np.array_equal(r.kept_ops[sel] - oa, r1.kept_ops)


# ---- the adjacency builder --------------------------------------------------------------------
def test_csr_builder_is_a_stable_sort(oracle):
    g, _ = gg.config(1, 0.05)
    gs = gg.shuffle_coo(g, 7)
    adj = oracle.build_adjacency(gs.num_ops, gs.num_tensors, gs.in_op, gs.in_tensor, gs.out_op, gs.out_tensor)
    o = np.argsort(gs.in_op, kind="stable")
    assert np.array_equal(adj.in_idx, gs.in_tensor[o])
    assert np.array_equal(adj.in_rowptr, np.searchsorted(gs.in_op[o], np.arange(gs.num_ops + 1)).astype(np.int32))
    o2 = np.argsort(gs.out_op, kind="stable")
    assert np.array_equal(adj.out_idx, gs.out_tensor[o2])
    # producers: sorted by (tensor, operator)
    o3 = np.lexsort((gs.out_op, gs.out_tensor))
    assert np.array_equal(adj.prod_idx, gs.out_op[o3])
    assert np.array_equal(adj.prod_rowptr,
                          np.searchsorted(gs.out_tensor[o3], np.arange(gs.num_tensors + 1)).astype(np.int32))
    assert adj.in_rowptr[-1] == gs.nnz_in and adj.prod_rowptr[-1] == gs.nnz_out
    with pytest.raises(ValueError):
        oracle.build_csr(3, np.array([0, 3], np.int32), np.array([0, 0], np.int32))


def test_generators_are_topological_and_seeded():
    for k, scale in SMALL:
        g, tg = gg.config(k, scale)
        g_again, tg_again = gg.config(k, scale)
        assert np.array_equal(g.in_tensor, g_again.in_tensor) and np.array_equal(tg.tgt_idx, tg_again.tgt_idx)
        prod_of = np.full(g.num_tensors, -1, np.int64)
        prod_of[g.out_tensor] = g.out_op
        assert np.all(prod_of[g.in_tensor] < g.in_op)            # producer created before consumer
        assert np.all(np.diff(g.in_op) >= 0) and np.all(np.diff(g.out_op) >= 0)   # op-major COO
        assert np.unique(g.out_tensor).size == g.nnz_out          # single producer per tensor
        assert tg.tgt_idx.min() >= 0 and tg.tgt_idx.max() < g.num_tensors
        if g.num_graphs > 1:                                      # no edges across packed graphs
            gi_in = np.searchsorted(g.graph_tensor_offsets, g.in_tensor, side="right") - 1
            go_in = np.searchsorted(g.graph_op_offsets, g.in_op, side="right") - 1
            assert np.array_equal(gi_in, go_in)


def test_generators_follow_the_stated_recipes():
    """Sizes, fan-in and fan-out distributions, edge spans and target draws of the five workloads, as their
    recipes state them (checked on the small config at full size and on scaled-down copies of the others)."""
    def fan(g):
        return np.bincount(g.in_op, minlength=g.num_ops), np.bincount(g.out_op, minlength=g.num_ops)

    # config 0: 2 000 operators, fan-in uniform 1..3 from the last 64 produced tensors + 16 inputs, 1..2 outputs
    g, tg = gg.config(0, 1.0)
    fi, fo = fan(g)
    assert g.num_ops == 2000 and tg.num_sets == 1 and np.diff(tg.tgt_rowptr).tolist() == [4]
    assert set(np.unique(fi)) == {1, 2, 3} and set(np.unique(fo)) == {1, 2}
    assert abs(fi.mean() - 2.0) < 0.1 and abs(fo.mean() - 1.5) < 0.05
    first_out = np.full(g.num_ops, g.num_tensors, np.int64)
    np.minimum.at(first_out, g.out_op, g.out_tensor)
    reach = first_out[g.in_op] - g.in_tensor                  # how far back an input lies, in tensor ids
    from_inputs = g.in_tensor < 16
    assert np.all(reach[~from_inputs] >= 1) and np.all(reach[~from_inputs] <= 64)
    assert 0.1 < from_inputs.mean() < 0.3                    # 16 of 80 pool entries are graph inputs
    assert tg.tgt_idx.min() >= int(0.9 * g.num_tensors) - 1   # targets from the last 10 % of the tensors

    # config 1: layers of 400 operators, fan-in 1..3, a fifth of the inputs are skips of 2..32 layers, 64 sets of 1..8
    g, tg = gg.config(1, 0.2)
    fi, fo = fan(g)
    assert g.num_ops % 400 == 0 and tg.num_sets == 64
    assert set(np.unique(fi)) == {1, 2, 3} and set(np.unique(fo)) == {1, 2}
    n_t = np.diff(tg.tgt_rowptr)
    assert n_t.min() >= 1 and n_t.max() <= 8
    prod_of = np.full(g.num_tensors, -400, np.int64)          # graph inputs: "layer -1"
    prod_of[g.out_tensor] = g.out_op
    span = g.in_op // 400 - prod_of[g.in_tensor] // 400       # layers between consumer and producer
    inner = g.in_op // 400 >= 33                              # (near the bottom, skips are clamped to layer -1)
    assert span[inner].min() == 1 and span[inner].max() <= 32
    assert abs((span[inner] > 1).mean() - 0.2) < 0.02

    # config 2: 1 000 operators per step, one output each, intra-step fan-in 1..3 plus a recurrent edge with prob. 0.1
    g, tg = gg.config(2, 0.02)
    fi, fo = fan(g)
    assert g.num_ops % 1000 == 0 and np.all(fo == 1) and tg.num_sets == 1
    assert np.diff(tg.tgt_rowptr).tolist() == [33]            # the loss tensor and 32 others
    later = g.in_op >= 1000                                   # from the second step on
    assert set(np.unique(fi[1000:])) <= {1, 2, 3, 4}
    prod_of = np.full(g.num_tensors, -1, np.int64)
    prod_of[g.out_tensor] = g.out_op
    p = prod_of[g.in_tensor]
    recurrent = later & (p >= 0) & (p == g.in_op - 1000)
    assert abs(recurrent.sum() / (g.num_ops - 1000) - 0.1) < 0.01

    # config 3: fan-in ~ k^-2.1 on 1..64 (truncated: P(1) = 0.645, mean 2.57), sources uniform over everything
    # earlier, 1..3 outputs, 64 sets of 1..16 tensors from the last 5 %
    g, tg = gg.config(3, 0.01)
    fi, fo = fan(g)
    w = np.arange(1, 65, dtype=np.float64) ** -2.1
    w /= w.sum()
    assert fi.min() == 1 and fi.max() <= 64 and set(np.unique(fo)) == {1, 2, 3}
    assert abs((fi == 1).mean() - w[0]) < 0.01 and abs(fi.mean() - (w * np.arange(1, 65)).sum()) < 0.05
    assert abs((fi == 2).mean() - w[1]) < 0.01 and abs(fo.mean() - 2.0) < 0.02
    first_out = np.full(g.num_ops, g.num_tensors, np.int64)
    np.minimum.at(first_out, g.out_op, g.out_tensor)
    rel = g.in_tensor / np.maximum(first_out[g.in_op], 1)     # uniform over [0, first own output): mean one half
    big = g.in_op > g.num_ops // 10
    assert np.all(g.in_tensor < first_out[g.in_op]) and abs(rel[big].mean() - 0.5) < 0.01
    n_t = np.diff(tg.tgt_rowptr)
    assert tg.num_sets == 64 and n_t.min() >= 1 and n_t.max() <= 16
    assert tg.tgt_idx.min() >= int(0.95 * g.num_tensors) - 1

    # config 4: independent graphs of 20 000 operators, each as config 0, 64 sets of 4 targets per graph
    g, tg = gg.config(4, 0.002)
    assert g.num_graphs >= 2 and np.all(np.diff(g.graph_op_offsets) == 20000) and tg.num_sets == 64
    assert np.all(np.diff(tg.tgt_rowptr) == 4) and len(tg.tgt_rowptr) == 64 * g.num_graphs + 1
    fi, fo = fan(g)
    assert set(np.unique(fi)) == {1, 2, 3} and set(np.unique(fo)) == {1, 2}
    g0 = slice(int(g.graph_op_offsets[0]), int(g.graph_op_offsets[1]))
    g1 = slice(int(g.graph_op_offsets[1]), int(g.graph_op_offsets[2]))
    assert not np.array_equal(fi[g0], fi[g1])                 # every graph has its own seed


@pytest.mark.parametrize("cfg,scale", [(0, 1.0), (1, 0.2), (3, 0.002)])
def test_adding_targets_to_finished_marks_is_incremental(oracle, cfg, scale):
    """Algorithm 1 skips what is already marked ("if not m_x"), so running it for more targets on top of
    finished marks gives the marks of all targets together: what an incremental prune relies on."""
    g, tg = gg.config(cfg, scale)
    adj = oracle.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
    Q = tg.num_sets
    cnt = np.diff(tg.tgt_rowptr)
    first = cnt.copy()
    first[1::2] = 0
    if len(cnt) == 1:
        first[0] = cnt[0] // 2
    rp1 = np.concatenate([[0], np.cumsum(first)]).astype(np.int32)
    idx1 = np.concatenate([tg.tgt_idx[tg.tgt_rowptr[s]:tg.tgt_rowptr[s] + first[s]] for s in range(len(cnt))]).astype(np.int32)
    M1, _ = oracle.mark(adj, Q, rp1, idx1)
    M2, _ = oracle.mark(adj, Q, tg.tgt_rowptr, tg.tgt_idx, M=M1.copy())
    Mfull, _ = oracle.mark(adj, Q, tg.tgt_rowptr, tg.tgt_idx)
    assert np.array_equal(M2, Mfull)
    assert not np.any(M1 & ~Mfull) and np.any(M1 != Mfull)
