// In-place structures on the pruned graph (Sec. 2.4, Algorithm 3 of the paper).
//
// Algorithm 3 walks the nodes in order; a node not yet renamed becomes its own ancestor and hands that
// ancestor down while the current node has exactly one child.  On an acyclic graph the outcome does
// not depend on doing this one walk after the other: the nodes with exactly one child and their child
// form a forest of links p -> c, and the ancestor of v is the smallest id among the nodes from which v
// is reached over links, v included (that node cannot have been entered by an earlier walk, and
// neither can anything on its way to v).  That minimum is computed here by pointer doubling:
//   round k:  rename[J_k[u]] = min(rename[J_k[u]], rename[u]),  J_{k+1}[u] = J_k[J_k[u]]
// with J_0 = the link.  After round k every node has seen all nodes fewer than 2^(k+1) links upstream.
// rename[] is lowered in place with atomicMin (any value a round reads is an id that reaches the node,
// and at least as small as the value the round started with); the jump pointers are double buffered.
//
// Nodes are tensors; Child(x) = distinct tensors written by surviving operators that read x, where an
// operator survives when (K[o] & select) != 0.  "Exactly one child" is decided without building the
// sets: the smallest and the largest child id of x are kept with atomicMin / atomicMax and compared.
#include "common.h"

namespace dgn {

constexpr int kIpThreads = 256;
constexpr int kNoChildLo = 0x7fffffff;

__global__ __launch_bounds__(kIpThreads) void k_inplace_init(int32_t *rename, int2 *child_range, int64_t T,
                                                              int32_t *counters, int num_counters,
                                                              int64_t *renamed_count)
{
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < T; x += gsize) {
        rename[x] = -1;
        child_range[x] = make_int2(kNoChildLo, -1);
    }
    if (blockIdx.x == 0) {
        if ((int)threadIdx.x < num_counters) counters[threadIdx.x] = 0;
        if (threadIdx.x == 0 && renamed_count) *renamed_count = 0;
    }
}

// Every surviving operator marks the tensors it touches as nodes of the graph (rename[x] = x) and
// offers its smallest / largest output as child of each of its inputs.
__global__ __launch_bounds__(kIpThreads) void k_inplace_children(GraphView g, const u64 *K, u64 select,
                                                                  int32_t *rename, int2 *child_range)
{
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < g.num_ops; o += gsize) {
        if ((K[o] & select) == 0) continue;
        int lo = kNoChildLo, hi = -1;
        for (int32_t e = g.out_rowptr[o]; e < g.out_rowptr[o + 1]; ++e) {
            const int32_t u = g.out_idx[e];
            rename[u] = u;
            lo = min(lo, u);
            hi = max(hi, u);
        }
        for (int32_t e = g.in_rowptr[o]; e < g.in_rowptr[o + 1]; ++e) {
            const int32_t x = g.in_idx[e];
            rename[x] = x;
            if (hi >= 0) {
                atomicMin(&child_range[x].x, lo);
                atomicMax(&child_range[x].y, hi);
            }
        }
    }
}

// link[x] = the only child of x, or -1; nodes with a link are listed.  Both jump buffers are set for
// every node, so that a later round may read the pointer of a node that has no link.
__global__ __launch_bounds__(kIpThreads) void k_inplace_links(const int32_t *rename, const int2 *child_range,
                                                               int64_t T, int32_t *J0, int32_t *J1,
                                                               int32_t *linkers, int32_t *num_linkers)
{
    const int lane = lane_id();
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    const int64_t rounds = (T + gsize - 1) / gsize;
    for (int64_t r = 0; r < rounds; ++r) {                  // whole waves stay in the loop (ballot below)
        const int64_t x = r * gsize + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
        int32_t link = -1;
        if (x < T && rename[x] >= 0) {
            const int2 c = child_range[x];
            if (c.x == c.y) link = c.x;
            J0[x] = link;
            J1[x] = -1;
        }
        const u64 has = ballot64(link >= 0);
        if (has) {
            int base = 0;
            if (lane == 0) base = atomicAdd(num_linkers, __popcll(has));
            base = __shfl(base, 0, kWave);
            if (link >= 0) linkers[base + __popcll(has & lanemask_lt())] = (int32_t)x;
        }
    }
}

__global__ __launch_bounds__(kIpThreads) void k_inplace_round(const int32_t *linkers, const int32_t *num_linkers,
                                                               const int32_t *Jcur, int32_t *Jnext, int32_t *rename,
                                                               int32_t *active, int64_t *renamed_count)
{
    const int n = *num_linkers;
    const int gsize = gridDim.x * blockDim.x;
    bool more = false;
    int newly = 0;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gsize) {
        const int32_t u = linkers[i];
        const int32_t v = Jcur[u];
        int32_t next = -1;
        if (v >= 0) {
            const int32_t a = rename[u];
            const int32_t old = atomicMin(&rename[v], a);
            if (old == v && a < v) ++newly;                 // v carried its own name until now
            next = Jcur[v];
        }
        Jnext[u] = next;
        more |= next >= 0;
    }
    if (ballot64(more) && lane_id() == 0) *active = 1;
    const int wnew = wave_sum(newly);
    if (wnew && lane_id() == 0 && renamed_count) atomicAdd((u64 *)renamed_count, (u64)wnew);
}

size_t inplace_scratch_bytes(int64_t T)
{
    const size_t t = (size_t)(T > 0 ? T : 1);
    return ((t * 8 + 255) & ~(size_t)255) + 3 * ((t * 4 + 255) & ~(size_t)255) + 256;
}

InplaceBuffers inplace_buffers(void *scratch, int64_t T)
{
    const size_t t = (size_t)(T > 0 ? T : 1);
    char *p = static_cast<char *>(scratch);
    InplaceBuffers b;
    b.child_range = reinterpret_cast<int2 *>(p); p += (t * 8 + 255) & ~(size_t)255;
    b.J[0] = reinterpret_cast<int32_t *>(p); p += (t * 4 + 255) & ~(size_t)255;
    b.J[1] = reinterpret_cast<int32_t *>(p); p += (t * 4 + 255) & ~(size_t)255;
    b.linkers = reinterpret_cast<int32_t *>(p); p += (t * 4 + 255) & ~(size_t)255;
    b.counters = reinterpret_cast<int32_t *>(p);
    return b;
}

hipError_t launch_inplace_setup(const GraphView &g, const u64 *K, u64 select, int32_t *rename, int64_t *renamed_count,
                                const InplaceBuffers &b, int grid_blocks, hipStream_t s)
{
    const int64_t T = g.num_tensors, P = g.num_ops;
    auto blocks_for = [&](int64_t n) {
        int64_t nb = (n + kIpThreads - 1) / kIpThreads;
        if (nb > (int64_t)grid_blocks * 4) nb = (int64_t)grid_blocks * 4;
        return dim3((unsigned)(nb > 0 ? nb : 1));
    };
    hipLaunchKernelGGL(k_inplace_init, blocks_for(T), dim3(kIpThreads), 0, s, rename, b.child_range, T, b.counters,
                       kInplaceMaxRounds + 1, renamed_count);
    if (P > 0) hipLaunchKernelGGL(k_inplace_children, blocks_for(P), dim3(kIpThreads), 0, s, g, K, select, rename, b.child_range);
    if (T > 0)
        hipLaunchKernelGGL(k_inplace_links, blocks_for(T), dim3(kIpThreads), 0, s, rename, b.child_range, T, b.J[0], b.J[1],
                           b.linkers, b.counters);
    return hipGetLastError();
}

hipError_t launch_inplace_round(int round, int32_t *rename, int64_t *renamed_count, const InplaceBuffers &b,
                                int grid_blocks, hipStream_t s)
{
    hipLaunchKernelGGL(k_inplace_round, dim3((unsigned)grid_blocks), dim3(kIpThreads), 0, s, b.linkers, b.counters,
                       b.J[round & 1], b.J[(round & 1) ^ 1], rename, b.counters + 1 + round, renamed_count);
    return hipGetLastError();
}

}  // namespace dgn
