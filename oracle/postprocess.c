/*
 * CPU oracle for what a graph runtime reads off a prune result -- TEST INFRASTRUCTURE.
 *
 * Written from Sec. 3.2 of the paper (Dragon, arXiv 1707.08265): removed operators disappear, but
 * tensors stay for the completeness of the graph, and the tensors that are no longer used are
 * renamed "ignore"; every function (target set) executes its own surviving operators in creation
 * order.
 *   - ignore[t], bit q: t is written by an operator that survives for set q, but t itself is not
 *     coloured for q (nothing the targets of q depend on reads it);
 *   - list of set q: the operators whose K has bit q, in ascending (creation) order.
 * Both are definitions written out; nothing here is an algorithm of the paper.
 * It shares no source with the GPU library.  Parity status: pinned (see tests/).
 */
#include <stdint.h>
#include <string.h>

void orc_ignore_mask(int64_t num_ops, int64_t num_tensors, const int32_t *out_rowptr, const int32_t *out_idx,
                     const uint64_t *K, const uint64_t *M, uint64_t *ignore)
{
    memset(ignore, 0, (size_t)num_tensors * sizeof(uint64_t));
    for (int64_t o = 0; o < num_ops; ++o)
        for (int32_t e = out_rowptr[o]; e < out_rowptr[o + 1]; ++e)
            ignore[out_idx[e]] |= K[o] & ~M[out_idx[e]];
}

/* set_rowptr[65]; set_ops must hold sum over q of popcount of bit q over K.  Returns the total. */
int64_t orc_per_set_lists(int64_t num_ops, const uint64_t *K, int64_t *set_rowptr, int32_t *set_ops)
{
    int64_t n = 0;
    for (int q = 0; q < 64; ++q) {
        set_rowptr[q] = n;
        for (int64_t o = 0; o < num_ops; ++o)
            if ((K[o] >> q) & 1) set_ops[n++] = (int32_t)o;
    }
    set_rowptr[64] = n;
    return n;
}
