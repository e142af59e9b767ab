/*
 * CPU oracle for Forward Prune -- TEST INFRASTRUCTURE, not part of the product path.
 *
 * Plain, slow, single-threaded C written from the paper (Dragon, arXiv 1707.08265):
 *   - graph model: nodes are tensors; x_i -> x_j is an edge iff some operator takes x_i as an
 *     input and x_j as an output (Sec. 2.2, first paragraph);
 *   - Algorithm 1 "Backward Traversing for Forward-Pass": from every solving target, a depth-first
 *     search over Parent(x) that sets m_x and skips parents already marked;
 *   - removal rule: an operator whose outputs are all un-coloured is removed (Sec. 2.1);
 *   - surviving operators keep their creation order (Sec. 3.2).
 *
 * Batching reading: target set s = g*Q + q (graph g of a packed batch, q < Q <= 64) is an
 * independent run of Algorithm 1 whose flag m_x is bit q of M[x].
 *
 * It shares no source with the GPU library and must only be used by tests, the smoke check and
 * the bench's cpu_baseline leg.  Parity status of every function below: pinned (see tests/).
 * Performance claims: parity unpinned (the paper prints no timing for this path).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- adjacency -------------------------------------------------------------------------- */

/* Stable counting sort of (row[e], col[e]) by row: rowptr[n_rows+1], idx[nnz] keep COO order
 * inside a row.  Returns 0, or -1 when an id is out of range / allocation fails. */
int orc_build_csr(int64_t n_rows, int64_t nnz, const int32_t *row, const int32_t *col,
                  int32_t *rowptr, int32_t *idx)
{
    int64_t *cursor = (int64_t *)calloc((size_t)n_rows + 1, sizeof(int64_t));
    if (!cursor) return -1;
    for (int64_t e = 0; e < nnz; ++e) {
        if (row[e] < 0 || row[e] >= n_rows) { free(cursor); return -1; }
        cursor[row[e] + 1]++;
    }
    for (int64_t r = 0; r < n_rows; ++r) cursor[r + 1] += cursor[r];
    for (int64_t r = 0; r <= n_rows; ++r) rowptr[r] = (int32_t)cursor[r];
    for (int64_t e = 0; e < nnz; ++e) idx[cursor[row[e]]++] = col[e];
    free(cursor);
    return 0;
}

/* tensor -> producing operators, each row ascending in operator id (ties = duplicate edges).
 * Input is the operator->output CSR, walked in operator order, so the counting sort by tensor
 * yields (tensor, operator) order. */
int orc_build_producers(int64_t num_ops, int64_t num_tensors, const int32_t *out_rowptr,
                        const int32_t *out_idx, int32_t *prod_rowptr, int32_t *prod_idx)
{
    int64_t *cursor = (int64_t *)calloc((size_t)num_tensors + 1, sizeof(int64_t));
    if (!cursor) return -1;
    int64_t nnz = out_rowptr[num_ops];
    for (int64_t e = 0; e < nnz; ++e) {
        if (out_idx[e] < 0 || out_idx[e] >= num_tensors) { free(cursor); return -1; }
        cursor[out_idx[e] + 1]++;
    }
    for (int64_t t = 0; t < num_tensors; ++t) cursor[t + 1] += cursor[t];
    for (int64_t t = 0; t <= num_tensors; ++t) prod_rowptr[t] = (int32_t)cursor[t];
    for (int64_t o = 0; o < num_ops; ++o)
        for (int32_t e = out_rowptr[o]; e < out_rowptr[o + 1]; ++e)
            prod_idx[cursor[out_idx[e]]++] = (int32_t)o;
    free(cursor);
    return 0;
}

/* ---- Algorithm 1 ------------------------------------------------------------------------- */

typedef struct {
    int32_t x;      /* tensor being expanded                                   */
    int32_t p;      /* cursor over the producers of x (position in prod_idx)   */
    int32_t e;      /* cursor over the inputs of the current producer, or -1   */
    int32_t e_end;
} frame_t;

/* DepthFirstSearch(x) of Algorithm 1 with an explicit stack in place of recursion (deep graphs
 * would overflow the call stack).  Parent(x) is enumerated in the order "producers of x by
 * ascending id, inputs of each producer in their stored order".  The parent loop resumes where
 * it stopped after each recursive call returns, exactly as the recursion would. */
static int dfs(int32_t start, uint64_t bit, const int32_t *in_rowptr, const int32_t *in_idx,
               const int32_t *prod_rowptr, const int32_t *prod_idx, uint64_t *M,
               frame_t **stack, int64_t *cap, int64_t *parent_edges)
{
    int64_t top = 0;
    frame_t *st = *stack;
    M[start] |= bit;                                   /* m_x <- True */
    st[top].x = start; st[top].p = prod_rowptr[start]; st[top].e = -1; st[top].e_end = -1;
    ++top;
    while (top > 0) {
        frame_t *f = &st[top - 1];
        if (f->e < 0) {                                /* open next producer of x, or return */
            if (f->p == prod_rowptr[f->x + 1]) { --top; continue; }
            int32_t o = prod_idx[f->p];
            f->e = in_rowptr[o];
            f->e_end = in_rowptr[o + 1];
        }
        if (f->e == f->e_end) { f->p++; f->e = -1; continue; }
        int32_t parent = in_idx[f->e++];               /* for x_parent in Parent(x) */
        ++*parent_edges;
        if (!(M[parent] & bit)) {                      /* if not m_parent: DFS(parent) */
            if (top == *cap) {
                int64_t ncap = *cap * 2;
                frame_t *ns = (frame_t *)realloc(st, (size_t)ncap * sizeof(frame_t));
                if (!ns) return -1;
                st = ns; *stack = ns; *cap = ncap;
            }
            M[parent] |= bit;
            st[top].x = parent; st[top].p = prod_rowptr[parent]; st[top].e = -1; st[top].e_end = -1;
            ++top;
        }
    }
    return 0;
}

/* M[num_tensors] must be zero on entry (or hold flags to start from).  num_sets_total = G*Q sets;
 * set s marks bit (s % Q).  parent_edges (may be NULL) receives, per set, the number of Parent()
 * entries examined -- the O(n) sanity counter.  Returns 0 on success, -1 on bad ids / no memory. */
int orc_forward_prune(int64_t num_ops, int64_t num_tensors, const int32_t *in_rowptr,
                      const int32_t *in_idx, const int32_t *prod_rowptr, const int32_t *prod_idx,
                      int64_t num_sets_total, int32_t Q, const int32_t *tgt_rowptr,
                      const int32_t *tgt_idx, uint64_t *M, int64_t *parent_edges)
{
    (void)num_ops;
    if (Q < 1 || Q > 64) return -1;
    int64_t cap = 1024;
    frame_t *stack = (frame_t *)malloc((size_t)cap * sizeof(frame_t));
    if (!stack) return -1;
    int rc = 0;
    for (int64_t s = 0; s < num_sets_total && rc == 0; ++s) {
        uint64_t bit = (uint64_t)1 << (s % Q);
        int64_t edges = 0;
        for (int32_t j = tgt_rowptr[s]; j < tgt_rowptr[s + 1]; ++j) {   /* for t in T */
            int32_t x = tgt_idx[j];
            if (x < 0 || x >= num_tensors) { rc = -1; break; }
            if (!(M[x] & bit))                                          /* if not m_x */
                rc = dfs(x, bit, in_rowptr, in_idx, prod_rowptr, prod_idx, M, &stack, &cap, &edges);
            if (rc) break;
        }
        if (parent_edges) parent_edges[s] = edges;
    }
    free(stack);
    return rc;
}

/* ---- removal rule and ordered compaction --------------------------------------------------- */

/* K[o] = OR of M over the outputs of o; flag[o] = (K[o] != 0).  An operator with no outputs has
 * K = 0 and is removed (all of its zero outputs are un-coloured). */
void orc_keep(int64_t num_ops, const int32_t *out_rowptr, const int32_t *out_idx, const uint64_t *M,
              uint64_t *K, uint8_t *flag)
{
    for (int64_t o = 0; o < num_ops; ++o) {
        uint64_t k = 0;
        for (int32_t e = out_rowptr[o]; e < out_rowptr[o + 1]; ++e) k |= M[out_idx[e]];
        K[o] = k;
        if (flag) flag[o] = (uint8_t)(k != 0);
    }
}

/* Kept operators in creation order.  kept_count[0] = number kept; when num_graphs > 1,
 * kept_count[1 + g] = number of kept operators with id < graph_op_offsets[g] (g = 0..G).
 * per_query_count[g*64 + q] = operators of graph g whose K has bit q. */
void orc_compact(int64_t num_ops, const uint64_t *K, int32_t num_graphs,
                 const int64_t *graph_op_offsets, int32_t *kept_ops, uint64_t *kept_masks,
                 int64_t *kept_count, int64_t *per_query_count)
{
    int64_t n = 0;
    int32_t g = 0;
    int batched = num_graphs > 1 && graph_op_offsets;
    if (per_query_count) memset(per_query_count, 0, sizeof(int64_t) * 64 * (size_t)(batched ? num_graphs : 1));
    for (int64_t o = 0; o < num_ops; ++o) {
        if (batched) {
            while (g < num_graphs && o >= graph_op_offsets[g]) { kept_count[1 + g] = n; ++g; }
        }
        if (K[o]) {
            kept_ops[n] = (int32_t)o;
            if (kept_masks) kept_masks[n] = K[o];
            ++n;
            if (per_query_count) {
                int64_t *row = per_query_count + (batched ? 64 * (int64_t)(g - 1) : 0);
                for (int q = 0; q < 64; ++q) row[q] += (K[o] >> q) & 1;
            }
        }
    }
    if (batched) while (g <= num_graphs) { kept_count[1 + g] = n; ++g; }
    kept_count[0] = n;
}

/* ---- independent cross-checks (used only to pin the functions above) ---------------------- */

/* Seed masks: S[t] has bit (s % Q) for every target t of set s. */
int orc_seed_masks(int64_t num_tensors, int64_t num_sets_total, int32_t Q, const int32_t *tgt_rowptr,
                   const int32_t *tgt_idx, uint64_t *S)
{
    for (int64_t s = 0; s < num_sets_total; ++s)
        for (int32_t j = tgt_rowptr[s]; j < tgt_rowptr[s + 1]; ++j) {
            if (tgt_idx[j] < 0 || tgt_idx[j] >= num_tensors) return -1;
            S[tgt_idx[j]] |= (uint64_t)1 << (s % Q);
        }
    return 0;
}

/* A second algorithm for the same fixed point: one sweep over operators in descending id
 * (valid only when operator ids are a topological order).  M must hold the seed masks on entry. */
void orc_reverse_sweep(int64_t num_ops, const int32_t *in_rowptr, const int32_t *in_idx,
                       const int32_t *out_rowptr, const int32_t *out_idx, uint64_t *M, uint64_t *K)
{
    for (int64_t o = num_ops - 1; o >= 0; --o) {
        uint64_t k = 0;
        for (int32_t e = out_rowptr[o]; e < out_rowptr[o + 1]; ++e) k |= M[out_idx[e]];
        K[o] = k;
        for (int32_t e = in_rowptr[o]; e < in_rowptr[o + 1]; ++e) M[in_idx[e]] |= k;
    }
}

/* Fixed-point certificate: counts violations of
 *     K[o] == OR M[out(o)]      and      M[t] == S[t] | OR_{o reads t} K[o].
 * On a DAG these equations have exactly one solution, so 0 violations proves (M, K) correct.
 * R is caller-provided scratch of num_tensors words holding S on entry. */
int64_t orc_certificate(int64_t num_ops, int64_t num_tensors, const int32_t *in_rowptr,
                        const int32_t *in_idx, const int32_t *out_rowptr, const int32_t *out_idx,
                        const uint64_t *M, const uint64_t *K, uint64_t *R)
{
    int64_t bad = 0;
    for (int64_t o = 0; o < num_ops; ++o) {
        uint64_t k = 0;
        for (int32_t e = out_rowptr[o]; e < out_rowptr[o + 1]; ++e) k |= M[out_idx[e]];
        if (k != K[o]) ++bad;
        for (int32_t e = in_rowptr[o]; e < in_rowptr[o + 1]; ++e) R[in_idx[e]] |= K[o];
    }
    for (int64_t t = 0; t < num_tensors; ++t) if (R[t] != M[t]) ++bad;
    return bad;
}
