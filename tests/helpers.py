"""Helpers shared by the CPU and GPU test modules (graph builders and slow reference checkers).

Nothing here touches the GPU library or the C oracle: the checkers below are independent
re-statements of the *definition* (forward reachability over consumers), written as tiny Python
loops, used to pin the oracle.
"""
from __future__ import annotations

import json
import os

import numpy as np

import graphgen as gg

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def graph_from_ops(ops, num_tensors, name="handmade") -> gg.Graph:
    """ops: list of (inputs, outputs) with integer tensor ids, in creation order."""
    in_op, in_t, out_op, out_t = [], [], [], []
    for o, (ins, outs) in enumerate(ops):
        for t in ins:
            in_op.append(o)
            in_t.append(t)
        for t in outs:
            out_op.append(o)
            out_t.append(t)
    a = lambda x: np.asarray(x, dtype=np.int32)
    return gg.Graph(len(ops), num_tensors, a(in_op), a(in_t), a(out_op), a(out_t), name=name)


def targets_from_sets(sets, num_sets=None) -> gg.Targets:
    """sets: list (over graphs*sets) of lists of tensor ids."""
    rowptr = np.zeros(len(sets) + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum([len(s) for s in sets])
    idx = np.asarray([t for s in sets for t in s], dtype=np.int32)
    return gg.Targets(num_sets if num_sets is not None else len(sets), rowptr, idx)


def load_worked_example():
    with open(os.path.join(GOLDEN, "worked_example.json")) as f:
        ex = json.load(f)
    names = ex["tensors"]
    tid = {n: i for i, n in enumerate(names)}
    ops = [([tid[t] for t in op["in"]], [tid[t] for t in op["out"]]) for op in ex["ops"]]
    g = graph_from_ops(ops, len(names), "worked-example")
    cases = []
    for c in ex["cases"]:
        tg = targets_from_sets([[tid[t] for t in s] for s in c["target_sets"]])
        M = np.asarray([c["tensor_mask"][n] for n in names], dtype=np.uint64)
        cases.append(dict(name=c["name"], targets=tg, M=M, K=np.asarray(c["op_mask"], np.uint64),
                          kept=np.asarray(c["kept_ops"], np.int32),
                          pq=np.asarray(c["per_query_count"], np.int64)))
    return g, tid, cases


def random_small_graph(rng: np.random.Generator, num_ops: int, num_inputs: int = 3,
                       multi_producer: bool = False, topological: bool = True):
    """Tiny random operator list with the awkward cases the library must accept: zero-input and
    zero-output operators, duplicate edges, optionally several producers for one tensor."""
    ops = []
    n_t = num_inputs
    for o in range(num_ops):
        n_in = int(rng.integers(0, 4))
        n_out = int(rng.integers(0, 3))
        ins = [int(rng.integers(0, n_t)) for _ in range(n_in)] if n_t else []
        outs = []
        for _ in range(n_out):
            if multi_producer and n_t > num_inputs and rng.random() < 0.25:
                # write again to an existing non-input tensor that is newer than every input read
                lo = max([num_inputs] + [i + 1 for i in ins])
                if lo < n_t:
                    outs.append(int(rng.integers(lo, n_t)))
                    continue
            outs.append(n_t)
            n_t += 1
        ops.append((ins, outs))
    return graph_from_ops(ops, max(n_t, 1), "random-small"), ops


def brute_force_masks(ops, num_tensors, sets, Q):
    """Definition, not algorithm: bit q of M[t] iff t is in set q or t reaches a member of set q by
    following tensor->consumer-operator->output edges forwards.  One search per (tensor, set)."""
    consumers = [[] for _ in range(num_tensors)]
    for o, (ins, _) in enumerate(ops):
        for t in ins:
            consumers[t].append(o)
    M = np.zeros(num_tensors, dtype=np.uint64)
    for s, members in enumerate(sets):
        q = s % Q
        goal = set(members)
        for t in range(num_tensors):
            seen, stack, hit = {t}, [t], False
            while stack and not hit:
                x = stack.pop()
                if x in goal:
                    hit = True
                    break
                for o in consumers[x]:
                    for y in ops[o][1]:
                        if y not in seen:
                            seen.add(y)
                            stack.append(y)
            if hit:
                M[t] |= np.uint64(1 << q)
    K = np.zeros(len(ops), dtype=np.uint64)
    for o, (_, outs) in enumerate(ops):
        for y in outs:
            K[o] |= M[y]
    return M, K


def naive_forward_marks(ops, num_tensors):
    """The strawman of Sec. 2.2: start from tensors of in-degree zero and mark everything connected."""
    produced = set(y for _, outs in ops for y in outs)
    marked = set(t for t in range(num_tensors) if t not in produced)
    changed = True
    while changed:
        changed = False
        for ins, outs in ops:
            if any(t in marked for t in ins):
                for y in outs:
                    if y not in marked:
                        marked.add(y)
                        changed = True
    return marked


def load_inplace_examples():
    """Hand-worked cases for Algorithm 3: list of dicts with graph, op_mask, select, expected RD."""
    with open(os.path.join(GOLDEN, "inplace_examples.json")) as f:
        ex = json.load(f)
    out = []
    for c in ex["cases"]:
        names = c["tensors"]
        tid = {n: i for i, n in enumerate(names)}
        ops = [([tid[t] for t in op["in"]], [tid[t] for t in op["out"]]) for op in c["ops"]]
        g = graph_from_ops(ops, len(names), c["name"])
        rd = np.asarray([-1 if c["rename"][n] is None else tid[c["rename"][n]] for n in names], np.int32)
        out.append(dict(name=c["name"], graph=g, K=np.asarray(c["op_mask"], np.uint64), select=int(c["select"]),
                        rename=rd))
    return out


def single_child_links(g: gg.Graph, kept):
    """(in_graph, link) of the pruned graph, from the definition: link[x] = c when the surviving
    operators that read x write exactly one distinct tensor c, else -1."""
    children = [set() for _ in range(g.num_tensors)]
    in_graph = np.zeros(g.num_tensors, bool)
    outs = [[] for _ in range(g.num_ops)]
    for o, t in zip(g.out_op.tolist(), g.out_tensor.tolist()):
        outs[o].append(t)
    for o, t in zip(g.out_op.tolist(), g.out_tensor.tolist()):
        if kept[o]:
            in_graph[t] = True
    for o, t in zip(g.in_op.tolist(), g.in_tensor.tolist()):
        if kept[o]:
            in_graph[t] = True
            children[t].update(outs[o])
    link = np.asarray([next(iter(c)) if len(c) == 1 else -1 for c in children], np.int64)
    return in_graph, link


def rename_by_reachability(g: gg.Graph, kept):
    """What Algorithm 3 must produce on an acyclic graph, stated without walking in node order: the
    ancestor of v is the smallest id among the nodes from which v is reached over single-child links
    (v included).  Proof idea: that node is not entered by any earlier walk (an earlier start that
    reached it would also reach v), so it starts its own walk, and nothing on its way to v has been
    entered before, for the same reason."""
    in_graph, link = single_child_links(g, kept)
    rd = np.full(g.num_tensors, -1, np.int64)
    for u in range(g.num_tensors):          # walk down from every node, keep the minimum start per node
        if not in_graph[u]:
            continue
        v, steps = u, 0
        while v != -1 and steps <= g.num_tensors:
            if rd[v] == -1 or u < rd[v]:
                rd[v] = u
            v = link[v]
            steps += 1
    return rd.astype(np.int32)


def load_backward_examples():
    """Hand-worked cases for Algorithm 2: graph, pairs, expected marked masks and kept operators."""
    with open(os.path.join(GOLDEN, "backward_examples.json")) as f:
        ex = json.load(f)
    out = []
    for c in ex["cases"]:
        names = c["tensors"]
        tid = {n: i for i, n in enumerate(names)}
        ops = [([tid[t] for t in op["in"]], [tid[t] for t in op["out"]]) for op in c["ops"]]
        g = graph_from_ops(ops, len(names), c["name"])
        obj = np.asarray([tid[p[0]] for p in c["pairs"]], np.int32)
        wrt = np.asarray([tid[p[1]] for p in c["pairs"]], np.int32)
        M = np.zeros(len(names), np.uint64)
        for i, marked in enumerate(c["marked"]):
            for n in marked:
                M[tid[n]] |= np.uint64(1 << i)
        out.append(dict(name=c["name"], graph=g, ops=ops, obj=obj, wrt=wrt, M=M,
                        kept=np.asarray(c["kept_ops"], np.int32)))
    return out


def marks_by_route_enumeration(ops, num_tensors, obj, wrt):
    """Definition, not algorithm: bit i of M[x] iff x lies on some route x_obj -> ... -> x_wrt of at
    least one edge; every route is enumerated explicitly (tiny graphs only)."""
    children = [set() for _ in range(num_tensors)]
    for ins, outs in ops:
        for x in ins:
            children[x].update(outs)
    M = np.zeros(num_tensors, dtype=np.uint64)
    for i, (a, b) in enumerate(zip(obj.tolist(), wrt.tolist())):
        path = [a]

        def walk(x):
            for c in children[x]:
                path.append(c)
                if c == b:
                    for n in path:
                        M[n] |= np.uint64(1 << i)
                else:
                    walk(c)
                path.pop()
        walk(a)
    return M


def marks_by_closure(ops, num_tensors, obj, wrt):
    """Second statement of the same set: x is marked for pair (a, b), a != b, iff a reaches x and x
    reaches b, reachability being the reflexive-transitive closure of the child relation (boolean
    matrix powers)."""
    R = np.eye(num_tensors, dtype=bool)
    for ins, outs in ops:
        for x in ins:
            for y in outs:
                R[x, y] = True
    for _ in range(max(1, int(np.ceil(np.log2(max(2, num_tensors)))))):
        R = R | ((R.astype(np.int64) @ R.astype(np.int64)) > 0)
    M = np.zeros(num_tensors, dtype=np.uint64)
    for i, (a, b) in enumerate(zip(obj.tolist(), wrt.tolist())):
        if a == b:
            continue
        on = R[a, :] & R[:, b]
        M[on] |= np.uint64(1 << i)
    return M
