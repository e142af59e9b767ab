"""GPU parity of the in-place pass (Algorithm 3 on the pruned graph): the rename dictionary computed by
the HIP path, through the C ABI binding, against the CPU oracle, element by element (integer ids:
the bar is exact equality)."""
import numpy as np
import pytest

import graphgen as gg
from helpers import graph_from_ops, load_inplace_examples, random_small_graph, targets_from_sets

pytestmark = pytest.mark.gpu

ALL = 2**64 - 1


@pytest.fixture(scope="module")
def dgn():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1707_08265_amd as d
    return d


def _adj(orc, g):
    return orc.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)


def gpu_inplace(d, dg, K, select=ALL, buf=None):
    """K: numpy uint64 [P] or a device int64 tensor. Returns (rename, renamed_count, rounds)."""
    import torch
    if isinstance(K, np.ndarray):
        K = torch.from_numpy(K.view(np.int64).copy()).cuda()
    buf = buf or d.InplaceBuffers(dg)
    rc = buf.run(K, select)
    assert rc == 0, d.dgn_strerror(rc)
    torch.cuda.synchronize()
    out = buf.rename.cpu().numpy(), int(buf.renamed_count.item()), buf.rounds
    # the same from the list of kept operators (ascending ids of the operators with K != 0, as a prune leaves it):
    # the two entry points must agree
    kept = torch.nonzero(K != 0).flatten().to(torch.int32)
    spare = torch.full((5,), -7, dtype=torch.int32, device=kept.device)        # entries beyond the count are not read
    kept_ops = torch.cat([kept, spare])
    kept_count = torch.tensor([kept.numel()], dtype=torch.int64, device=kept.device)
    buf.rename.fill_(-99)
    rc = buf.run(K, select, kept_ops=kept_ops, kept_count=kept_count)
    assert rc == 0, d.dgn_strerror(rc)
    torch.cuda.synchronize()
    assert np.array_equal(buf.rename.cpu().numpy(), out[0]), "dgn_inplace_kept differs from dgn_inplace"
    assert int(buf.renamed_count.item()) == out[1]
    return out


def check(rd, count, ref, what):
    assert np.array_equal(rd, ref), f"{what}: rename dictionaries differ"
    assert count == int(((ref >= 0) & (ref != np.arange(ref.shape[0]))).sum()), f"{what}: renamed count"


@pytest.mark.parametrize("case", load_inplace_examples(), ids=lambda c: c["name"][:40])
def test_hand_worked_cases(dgn, case):
    g = case["graph"]
    dg = dgn.DeviceGraph.from_coo(g)
    rd, count, _ = gpu_inplace(dgn, dg, case["K"], case["select"])
    check(rd, count, case["rename"], case["name"])


@pytest.mark.parametrize("seed", range(12))
def test_random_small_graphs(dgn, oracle, seed):
    rng = np.random.default_rng(7000 + seed)
    g, _ = random_small_graph(rng, int(rng.integers(1, 400)), multi_producer=bool(seed % 3 == 0))
    if seed % 2:
        g, _, _ = gg.relabel_tensors(g, targets_from_sets([[0]]), seed)
    K = rng.integers(0, 4, g.num_ops).astype(np.uint64)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.InplaceBuffers(dg)
    adj = _adj(oracle, g)
    for select in (1, 2, 3, ALL):
        rd, count, _ = gpu_inplace(dgn, dg, K, select, buf)       # buffers reused across calls
        check(rd, count, oracle.inplace(adj, K, select), f"seed {seed} select {select}")


@pytest.mark.parametrize("k,scale", [(0, 1.0), (1, 1.0), (2, 0.02), (3, 0.02), (4, 0.002)])
def test_after_prune_on_configs(dgn, oracle, k, scale):
    import torch
    g, tg = gg.config(k, scale)
    print(f"config {k} scale {scale}: P={g.num_ops} T={g.num_tensors}", flush=True)
    dg = dgn.DeviceGraph.from_coo(g)
    pb = dgn.PruneBuffers(dg, tg.num_sets)
    rc = pb.prune(torch.from_numpy(tg.tgt_rowptr).cuda(), torch.from_numpy(tg.tgt_idx).cuda())
    assert rc == 0
    adj = _adj(oracle, g)
    ref = oracle.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx, g.num_graphs, g.graph_op_offsets)
    buf = dgn.InplaceBuffers(dg)
    selects = [ALL] + ([1, 1 << 5, 1 << (tg.num_sets - 1)] if tg.num_sets > 1 else [])
    for select in selects:
        rd, count, rounds = gpu_inplace(dgn, dg, pb.op_mask, select, buf)
        check(rd, count, oracle.inplace(adj, ref.op_mask, select), f"cfg{k} select {select:#x}")
        assert 1 <= rounds <= 32


def test_long_chain_needs_logarithmic_rounds(dgn, oracle):
    n = 300_000                                   # 2^18 < n < 2^19: 19 doubling rounds, run in batches of four
    ops = [([i], [i + 1]) for i in range(n)]
    g = graph_from_ops(ops, n + 1)
    dg = dgn.DeviceGraph.from_coo(g)
    rd, count, rounds = gpu_inplace(dgn, dg, np.ones(n, np.uint64))
    assert (rd == 0).all() and count == n
    assert rounds == 20
    K = np.ones(n, np.uint64)
    K[[5, 77_777, 250_000]] = 0                   # three operators pruned away: four chains
    rd, count, _ = gpu_inplace(dgn, dg, K)
    check(rd, count, oracle.inplace(_adj(oracle, g), K), "cut chain")
    # a chain whose ids run against the walk: every node keeps its own name except ... none
    g2 = graph_from_ops([([n - i], [n - i - 1]) for i in range(n)], n + 1)
    dg2 = dgn.DeviceGraph.from_coo(g2)
    rd, count, _ = gpu_inplace(dgn, dg2, np.ones(n, np.uint64))
    check(rd, count, oracle.inplace(_adj(oracle, g2), np.ones(n, np.uint64)), "descending chain")
    assert count == 0


def test_nothing_kept_and_empty_graph(dgn):
    g, _ = gg.config(0, 1.0)
    dg = dgn.DeviceGraph.from_coo(g)
    rd, count, _ = gpu_inplace(dgn, dg, np.zeros(g.num_ops, np.uint64))
    assert (rd == -1).all() and count == 0
    rd, count, _ = gpu_inplace(dgn, dg, np.ones(g.num_ops, np.uint64), select=2)   # no operator has bit 1
    assert (rd == -1).all() and count == 0


def test_argument_errors(dgn):
    import torch
    g, _ = gg.config(0, 1.0)
    dg = dgn.DeviceGraph.from_coo(g)
    buf = dgn.InplaceBuffers(dg)
    K = torch.zeros(g.num_ops, dtype=torch.int64, device="cuda")
    rc, _ = dgn.dgn_inplace(dg.handle, K, ALL, buf.rename, buf.renamed_count, buf.scratch, buf.scratch_bytes - 1)
    assert rc == dgn.DGN_ERR_WORKSPACE_TOO_SMALL
    rc, _ = dgn.dgn_inplace(dg.handle, None, ALL, buf.rename, buf.renamed_count, buf.scratch, buf.scratch_bytes)
    assert rc == dgn.DGN_ERR_NULL_PTR
    rc, _ = dgn.dgn_inplace(dg.handle, K, ALL, None, buf.renamed_count, buf.scratch, buf.scratch_bytes)
    assert rc == dgn.DGN_ERR_NULL_PTR
    rc, _ = dgn.dgn_inplace(dg.handle, K, ALL, buf.rename, None, buf.scratch, buf.scratch_bytes)
    assert rc == 0


@pytest.mark.parametrize("k", [1, 3])
def test_full_size(dgn, oracle, k):
    import torch
    g, tg = gg.config(k, 1.0)
    print(f"config {k} full size: P={g.num_ops} T={g.num_tensors}", flush=True)
    dg = dgn.DeviceGraph.from_coo(g)
    pb = dgn.PruneBuffers(dg, tg.num_sets)
    rc = pb.prune(torch.from_numpy(tg.tgt_rowptr).cuda(), torch.from_numpy(tg.tgt_idx).cuda())
    assert rc == 0
    K = pb.op_mask.cpu().numpy().view(np.uint64)          # parity of K itself is covered by the prune tests
    buf = dgn.InplaceBuffers(dg)
    rd, count, rounds = gpu_inplace(dgn, dg, pb.op_mask, ALL, buf)
    print(f"renamed {count} tensors in {rounds} rounds", flush=True)
    check(rd, count, oracle.inplace(_adj(oracle, g), K, ALL), f"cfg{k} full")
