/*
 * CPU oracle for the in-place optimisation -- TEST INFRASTRUCTURE, not part of the product path.
 *
 * Plain, slow, single-threaded C written from Sec. 2.4 and Algorithm 3 ("Forward Traversing for
 * Available In-place Structures") of the paper (Dragon, arXiv 1707.08265):
 *   - the graph G is the graph left after pruning (the section says renaming must follow the prune);
 *     its nodes are the tensors that a surviving operator reads or writes, and Child(x) is the set of
 *     tensors written by surviving operators that read x (graph model of Sec. 2.2);
 *   - every node is visited in node order; a node not yet in the rename dictionary RD becomes its
 *     own ancestor, and the search then walks on while the current node has exactly one child,
 *     giving every node it enters the same ancestor and stopping at a node already in RD.
 *
 * Readings where the paper is silent: node order is ascending tensor id; Child(x) is a set (an
 * operator that lists x twice, or two operators that write the same tensor, give one child);
 * an operator survives when (K[o] & select) != 0, K being the per-operator mask of the prune and
 * `select` the target sets whose pruned graph is meant; tensors outside G get -1.
 *
 * It shares no source with the GPU library.  Parity status: pinned (see tests/).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int32_t x, child; } pair_t;

static int cmp_pair(const void *a, const void *b)
{
    const pair_t *p = (const pair_t *)a, *q = (const pair_t *)b;
    if (p->x != q->x) return p->x < q->x ? -1 : 1;
    if (p->child != q->child) return p->child < q->child ? -1 : 1;
    return 0;
}

/* Child sets of the pruned graph as a CSR over tensors: child_rowptr[T+1], child_idx[<= nnz]
 * (distinct children, ascending), in_graph[T] (1 when a surviving operator touches the tensor).
 * Returns the number of (x, child) entries, or -1 on a failed allocation. */
int64_t orc_child_sets(int64_t num_ops, int64_t num_tensors, const int32_t *in_rowptr, const int32_t *in_idx,
                       const int32_t *out_rowptr, const int32_t *out_idx, const uint64_t *K, uint64_t select,
                       int32_t *child_rowptr, int32_t *child_idx, int64_t child_cap, uint8_t *in_graph)
{
    int64_t n = 0;
    for (int64_t o = 0; o < num_ops; ++o)
        if (K[o] & select)
            n += (int64_t)(in_rowptr[o + 1] - in_rowptr[o]) * (out_rowptr[o + 1] - out_rowptr[o]);
    pair_t *pairs = (pair_t *)malloc((size_t)(n ? n : 1) * sizeof(pair_t));
    if (!pairs) return -1;
    memset(in_graph, 0, (size_t)num_tensors);
    int64_t m = 0;
    for (int64_t o = 0; o < num_ops; ++o) {
        if (!(K[o] & select)) continue;
        for (int32_t i = in_rowptr[o]; i < in_rowptr[o + 1]; ++i) in_graph[in_idx[i]] = 1;
        for (int32_t j = out_rowptr[o]; j < out_rowptr[o + 1]; ++j) in_graph[out_idx[j]] = 1;
        for (int32_t i = in_rowptr[o]; i < in_rowptr[o + 1]; ++i)
            for (int32_t j = out_rowptr[o]; j < out_rowptr[o + 1]; ++j) {
                pairs[m].x = in_idx[i];
                pairs[m].child = out_idx[j];
                ++m;
            }
    }
    qsort(pairs, (size_t)m, sizeof(pair_t), cmp_pair);
    int64_t w = 0;
    memset(child_rowptr, 0, (size_t)(num_tensors + 1) * sizeof(int32_t));
    for (int64_t e = 0; e < m; ++e) {
        if (e > 0 && pairs[e].x == pairs[e - 1].x && pairs[e].child == pairs[e - 1].child) continue;
        if (w >= child_cap) { free(pairs); return -1; }
        child_idx[w++] = pairs[e].child;
        child_rowptr[pairs[e].x + 1]++;
    }
    for (int64_t x = 0; x < num_tensors; ++x) child_rowptr[x + 1] += child_rowptr[x];
    free(pairs);
    return w;
}

/* Algorithm 3.  RD[x] = ancestor for every node of G, -1 for tensors outside G. */
void orc_inplace(int64_t num_tensors, const int32_t *child_rowptr, const int32_t *child_idx,
                 const uint8_t *in_graph, int32_t *RD)
{
    for (int64_t x = 0; x < num_tensors; ++x) RD[x] = -1;             /* RD = {} */
    for (int64_t start = 0; start < num_tensors; ++start) {           /* for x^ in G */
        if (!in_graph[start]) continue;
        int32_t x = (int32_t)start;
        const int32_t ancestor = (int32_t)start;
        for (;;) {                                                    /* DepthFirstSearch(x, ancestor) */
            if (RD[x] != -1) break;                                   /* x in RD: return */
            RD[x] = ancestor;
            if (child_rowptr[x + 1] - child_rowptr[x] != 1) break;    /* len(Child(x)) is 1 */
            x = child_idx[child_rowptr[x]];
        }
    }
}
