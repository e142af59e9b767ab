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
// sets: child[x] holds the only child seen so far and is set to "many" by whoever brings a second one.
#include "common.h"

namespace dgn {

constexpr int kIpThreads = 256;
constexpr int kManyChildren = -2;                   // child[x]: -1 none yet, >= 0 the only child so far

// p[0..n) = -1, with 16-byte stores over the aligned bulk
__device__ __forceinline__ void fill_minus_one(int32_t *p, int64_t n, int64_t gtid, int64_t gsize)
{
    int64_t head = (int64_t)(((16 - ((uintptr_t)p & 15)) & 15) >> 2);
    if (head > n) head = n;
    if (gtid < head) p[gtid] = -1;
    int4 *bulk = reinterpret_cast<int4 *>(p + head);
    const int64_t quads = (n - head) >> 2;
    const int4 m = make_int4(-1, -1, -1, -1);
    for (int64_t i = gtid; i < quads; i += gsize) bulk[i] = m;
    const int64_t done = head + (quads << 2);
    if (gtid < n - done) p[done + gtid] = -1;
}

__global__ __launch_bounds__(kIpThreads) void k_inplace_init(int32_t *rename, int32_t *child, int64_t T,
                                                              int32_t *counters, int num_counters,
                                                              int64_t *renamed_count)
{
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    fill_minus_one(rename, T, gtid, gsize);
    fill_minus_one(child, T, gtid, gsize);
    if (blockIdx.x == 0) {
        if ((int)threadIdx.x < num_counters) counters[threadIdx.x] = 0;
        if (threadIdx.x == 0 && renamed_count) *renamed_count = 0;
    }
}

// One surviving operator: the tensors it touches become nodes of the graph (rename[x] = x), and each
// input learns the operator's output(s) as child.  child[x] only moves -1 -> id -> kManyChildren.
__device__ __forceinline__ void offer_children(const GraphView &g, int64_t o, int32_t *rename, int32_t *child)
{
    int lo = 0x7fffffff, hi = -1;
    for (int32_t e = g.out_rowptr[o]; e < g.out_rowptr[o + 1]; ++e) {
        const int32_t u = g.out_idx[e];
        rename[u] = u;
        lo = min(lo, u);
        hi = max(hi, u);
    }
    // An input learns the child on offer.  `seen`: what its child word held a moment ago (a stale value only
    // costs an atomic).
    auto offer = [&](int32_t x, int32_t seen) {
        rename[x] = x;
        if (hi < 0) return;                                 // an operator without outputs offers nothing
        if (lo != hi) {                                     // two distinct children at once
            __hip_atomic_store(&child[x], kManyChildren, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (seen == lo || seen == kManyChildren) return;
        const int32_t old = atomicCAS(&child[x], -1, lo);
        if (old != -1 && old != lo && old != kManyChildren)
            __hip_atomic_store(&child[x], kManyChildren, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    const bool look = hi >= 0 && lo == hi;                  // exactly one child on offer: the words are worth a look
    const int32_t ib = g.in_rowptr[o], ie = g.in_rowptr[o + 1];
    if (ie - ib <= 4) {
        for (int32_t e = ib; e < ie; ++e) {
            const int32_t x = g.in_idx[e];
            offer(x, look ? child[x] : 0);
        }
        return;
    }
    // Many inputs: four at a time, their ids and then their child words fetched together (past the end the last
    // input is read again) -- one after the other, an operator with dozens of inputs holds its wave for three
    // dependent accesses per input.
    for (int32_t e0 = ib; e0 < ie; e0 += 4) {
        int32_t x[4], seen[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = g.in_idx[min(e0 + j, ie - 1)];
#pragma unroll
        for (int j = 0; j < 4; ++j) seen[j] = look ? child[x[j]] : 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (e0 + j < ie) offer(x[j], seen[j]);
    }
}

// Surviving operators can be a few percent of all: a wave reads 512 masks, packs the ids of the
// survivors into LDS and works on them 64 at a time, so that the dependent loads of the expansion
// run with all lanes busy.
constexpr int kIpWaves = kIpThreads / kWave;
constexpr int kMaskRounds = 8;                      // masks per lane and step

__global__ __launch_bounds__(kIpThreads) void k_inplace_children(GraphView g, const u64 *K, u64 select,
                                                                  int32_t *rename, int32_t *child)
{
    __shared__ int32_t s_ops[kIpWaves][kWave * (kMaskRounds + 1)];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    int32_t *ops = s_ops[wave];
    int count = 0;                                          // wave-uniform
    const int64_t step = (int64_t)kWave * kMaskRounds;
    const int64_t steps = ((int64_t)g.num_ops + step - 1) / step;
    const int64_t wave_id = (int64_t)blockIdx.x * kIpWaves + wave, num_waves = (int64_t)gridDim.x * kIpWaves;
    for (int64_t st = wave_id; st < steps; st += num_waves) {
        u64 k[kMaskRounds];
#pragma unroll
        for (int r = 0; r < kMaskRounds; ++r) {
            const int64_t o = st * step + r * kWave + lane;
            k[r] = o < g.num_ops ? K[o] : 0;
        }
#pragma unroll
        for (int r = 0; r < kMaskRounds; ++r) {
            const bool kept = (k[r] & select) != 0;
            const u64 m = ballot64(kept);
            if (kept) ops[count + __popcll(m & lanemask_lt())] = (int32_t)(st * step + r * kWave + lane);
            count += __popcll(m);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        while (count >= kWave) {
            count -= kWave;
            offer_children(g, ops[count + lane], rename, child);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    if (lane < count) offer_children(g, ops[lane], rename, child);
}

// The same from the list of kept operators that the prune wrote (ascending ids of the operators with K != 0):
// a pruned graph is a few percent of the recorded one, and the list spares the pass over all of K.  An entry
// whose mask misses `select` is skipped.
__global__ __launch_bounds__(kIpThreads) void k_inplace_children_list(GraphView g, const u64 *K, u64 select,
                                                                       const int32_t *kept_ops, const int64_t *kept_count,
                                                                       int32_t *rename, int32_t *child)
{
    const int64_t kept = kept_count[0];
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < kept; i += gsize) {
        const int32_t o = kept_ops[i];
        if ((K[o] & select) != 0) offer_children(g, o, rename, child);
    }
}

// link[x] = the only child of x, or -1; nodes with a link are listed (gathered per workgroup in LDS, so
// that the list's counter is bumped once per thousand entries, not once per wave).  Both jump buffers
// are set for every node, so that a later round may read the pointer of a node that has no link.
constexpr int kLinkItems = 4;                       // independent loads per thread and step
constexpr int kLinkTile = kIpThreads * kLinkItems;

__global__ __launch_bounds__(kIpThreads) void k_inplace_links(const int32_t *rename, const int32_t *child,
                                                               int64_t T, int32_t *J0, int32_t *J1,
                                                               int32_t *linkers, int32_t *num_linkers)
{
    __shared__ int32_t s_list[2 * kLinkTile];
    __shared__ int s_count, s_base;
    const int lane = lane_id();
    if (threadIdx.x == 0) s_count = 0;
    __syncthreads();
    const int64_t tiles = (T + kLinkTile - 1) / kLinkTile;
    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {          // whole workgroups stay in the loop
        int32_t r[kLinkItems];
#pragma unroll
        for (int k = 0; k < kLinkItems; ++k) {
            const int64_t x = t * kLinkTile + k * kIpThreads + threadIdx.x;
            r[k] = x < T ? rename[x] : -1;
        }
#pragma unroll
        for (int k = 0; k < kLinkItems; ++k) {
            const int64_t x = t * kLinkTile + k * kIpThreads + threadIdx.x;
            int32_t link = -1;
            if (r[k] >= 0) {
                const int32_t c = child[x];
                if (c >= 0) link = c;
                J0[x] = link;
                J1[x] = -1;
            }
            const u64 has = ballot64(link >= 0);
            if (has) {
                int base = 0;
                if (lane == 0) base = atomicAdd(&s_count, __popcll(has));
                base = __shfl(base, 0, kWave);
                if (link >= 0) s_list[base + __popcll(has & lanemask_lt())] = (int32_t)x;
            }
        }
        __syncthreads();                                    // this tile's entries are in the list
        const int n = s_count;                              // at most one tile's worth is added per step
        __syncthreads();                                    // everyone has read the count before it changes again
        if (n >= kLinkTile || t + gridDim.x >= tiles) {     // flush: the next tile needs the room, or this was the last
            if (threadIdx.x == 0) {
                s_base = n ? atomicAdd(num_linkers, n) : 0;
                s_count = 0;
            }
            __syncthreads();
            for (int i = threadIdx.x; i < n; i += kIpThreads) linkers[s_base + i] = s_list[i];
            __syncthreads();
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
    return 4 * ((t * 4 + 255) & ~(size_t)255) + 256;
}

InplaceBuffers inplace_buffers(void *scratch, int64_t T)
{
    const size_t t = (size_t)(T > 0 ? T : 1);
    char *p = static_cast<char *>(scratch);
    InplaceBuffers b;
    b.child = reinterpret_cast<int32_t *>(p); p += (t * 4 + 255) & ~(size_t)255;
    b.J[0] = reinterpret_cast<int32_t *>(p); p += (t * 4 + 255) & ~(size_t)255;
    b.J[1] = reinterpret_cast<int32_t *>(p); p += (t * 4 + 255) & ~(size_t)255;
    b.linkers = reinterpret_cast<int32_t *>(p); p += (t * 4 + 255) & ~(size_t)255;
    b.counters = reinterpret_cast<int32_t *>(p);
    return b;
}

hipError_t launch_inplace_setup(const GraphView &g, const u64 *K, u64 select, const int32_t *kept_ops,
                                const int64_t *kept_count, int32_t *rename, int64_t *renamed_count,
                                const InplaceBuffers &b, int grid_blocks, hipStream_t s)
{
    const int64_t T = g.num_tensors, P = g.num_ops;
    auto blocks_for = [&](int64_t n) {
        int64_t nb = (n + kIpThreads - 1) / kIpThreads;
        if (nb > (int64_t)grid_blocks) nb = (int64_t)grid_blocks;
        return dim3((unsigned)(nb > 0 ? nb : 1));
    };
    hipLaunchKernelGGL(k_inplace_init, blocks_for(T), dim3(kIpThreads), 0, s, rename, b.child, T, b.counters,
                       kInplaceMaxRounds + 1, renamed_count);
    if (P > 0 && kept_ops)
        hipLaunchKernelGGL(k_inplace_children_list, dim3((unsigned)grid_blocks), dim3(kIpThreads), 0, s, g, K, select,
                           kept_ops, kept_count, rename, b.child);
    else if (P > 0)
        hipLaunchKernelGGL(k_inplace_children, blocks_for(P), dim3(kIpThreads), 0, s, g, K, select, rename, b.child);
    if (T > 0)
        hipLaunchKernelGGL(k_inplace_links, blocks_for(T), dim3(kIpThreads), 0, s, rename, b.child, T, b.J[0], b.J[1],
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
