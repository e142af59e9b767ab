/*
 * CPU oracle for Backward Prune -- TEST INFRASTRUCTURE, not part of the product path.
 *
 * Plain, slow, single-threaded C written from Sec. 2.3 and Algorithm 2 ("Forward Traversing for
 * Backward-Pass") of the paper (Dragon, arXiv 1707.08265): for every pair (x_obj, x_wrt) the
 * visited flags V are cleared and a memorised depth-first search runs forwards (over Child(x)) from
 * x_obj; v = 1 means "entered", v = 2 means "known to lead to x_wrt"; whenever the search meets
 * x_wrt among the children, or re-enters a node with v = 2, every node of the current path gets
 * v = 2 and m = True.  Nodes are tensors; Child(x) = tensors written by operators that read x
 * (edge definition at the start of Sec. 2.2).
 *
 * Readings where the printed algorithm is garbled or at odds with the text (the section's stated
 * aim is to eliminate every node that is not on a route from an objective to a derivative target):
 *   (a) after marking the path on re-entering a node with v = 2 the search returns (the printed
 *       block falls through to "v <- 1" and would search that node again);
 *   (b) after finding x_wrt among the children the search goes on with the remaining children
 *       (the printed early exit would skip routes through the node's other children and make the
 *       result depend on the order of the children);
 *   (c) Child(x) is enumerated as "consumers of x in ascending operator id, outputs of each in their
 *       stored order"; with (a) and (b) the result does not depend on that order;
 *   (d) pair i owns bit i of M[x]; a pair with x_obj = x_wrt marks nothing (only children are ever
 *       compared with x_wrt, and a DAG has no route back).
 * Marking the path costs its length each time; because a marked node on the stack implies that
 * every node below it is marked too, marking stops at the first node that already has v = 2.
 *
 * It shares no source with the GPU library.  Parity status: pinned (see tests/).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t x;      /* node being expanded                                        */
    int32_t c;      /* cursor over the consumers of x (position in cons_idx)      */
    int32_t e;      /* cursor over the outputs of the current consumer, or -1     */
    int32_t e_end;
} bframe_t;

static void mark_path(const bframe_t *st, int64_t top, uint8_t *V, uint64_t *M, uint64_t bit)
{
    for (int64_t i = top - 1; i >= 0; --i) {            /* for x^ in Path */
        if (V[st[i].x] == 2) break;                     /* everything below is marked already */
        V[st[i].x] = 2;
        M[st[i].x] |= bit;
    }
}

/* M[num_tensors] must be zero on entry.  V: scratch of num_tensors bytes.  Returns 0, or -1 on a
 * bad id / failed allocation. */
int orc_backward_prune(int64_t num_tensors, const int32_t *cons_rowptr, const int32_t *cons_idx,
                       const int32_t *out_rowptr, const int32_t *out_idx, int32_t num_pairs,
                       const int32_t *obj, const int32_t *wrt, uint64_t *M, uint8_t *V)
{
    if (num_pairs < 0 || num_pairs > 64) return -1;
    int64_t cap = 1024;
    bframe_t *st = (bframe_t *)malloc((size_t)cap * sizeof(bframe_t));
    if (!st) return -1;
    for (int32_t i = 0; i < num_pairs; ++i) {                           /* for (x_obj, x_wrt) in P */
        const uint64_t bit = (uint64_t)1 << i;
        const int32_t x_obj = obj[i], x_wrt = wrt[i];
        if (x_obj < 0 || x_obj >= num_tensors || x_wrt < 0 || x_wrt >= num_tensors) { free(st); return -1; }
        memset(V, 0, (size_t)num_tensors);                              /* Clear(V) */
        int64_t top = 0;
        V[x_obj] = 1;                                                   /* DFS(x_obj, x_wrt, {x_obj}) */
        st[top].x = x_obj; st[top].c = cons_rowptr[x_obj]; st[top].e = -1; st[top].e_end = -1;
        ++top;
        while (top > 0) {
            bframe_t *f = &st[top - 1];
            if (f->e < 0) {                                             /* open the next consumer, or return */
                if (f->c == cons_rowptr[f->x + 1]) { --top; continue; }
                const int32_t o = cons_idx[f->c];
                f->e = out_rowptr[o];
                f->e_end = out_rowptr[o + 1];
            }
            if (f->e == f->e_end) { f->c++; f->e = -1; continue; }
            const int32_t child = out_idx[f->e++];                      /* for x_child in Child(x) */
            if (child == x_wrt) {                                       /* route found: mark NewPath */
                mark_path(st, top, V, M, bit);
                V[child] = 2;
                M[child] |= bit;
                continue;                                               /* reading (b) */
            }
            if (V[child] > 0) {                                         /* visited already */
                if (V[child] == 2) mark_path(st, top, V, M, bit);       /* it leads to x_wrt: so does the path */
                continue;                                               /* reading (a) */
            }
            if (top == cap) {
                const int64_t ncap = cap * 2;
                bframe_t *ns = (bframe_t *)realloc(st, (size_t)ncap * sizeof(bframe_t));
                if (!ns) { free(st); return -1; }
                st = ns; cap = ncap;
            }
            V[child] = 1;                                               /* v_x <- 1 */
            st[top].x = child; st[top].c = cons_rowptr[child]; st[top].e = -1; st[top].e_end = -1;
            ++top;
        }
    }
    free(st);
    return 0;
}
