// Backward Prune (Sec. 2.3, Algorithm 2 of the paper): for every pair (x_obj, x_wrt) the nodes on a
// route from x_obj to x_wrt are marked; everything else can be eliminated.
//
// A node is on such a route iff x_obj reaches it and it reaches x_wrt.  The second half is what the
// forward prune computes when x_wrt is the only target of set i (its coloured set: everything x_wrt
// depends on), so pair i owns bit i and the first stage is one ordinary 64-set prune with targets
// x_wrt.  The second stage runs forwards from x_obj, but only *inside* that coloured set: every node
// between x_obj and a marked node reaches x_wrt as well, and every operator between two such nodes was
// kept by the first stage.  So the forward stage never leaves the (usually small) kept operator list
// of the first stage and needs no tensor -> consumer adjacency:
//     for every kept operator o:   F[y] |= (OR_{x in in(o)} F[x]) & B[y]    for y in out(o)
// repeated over the list, which is in creation order, until nothing changes.  F is the marked set.
#include "common.h"

namespace dgn {

// rowptr[i] = i, i = 0..n: target set i holds exactly entry i
__global__ __launch_bounds__(64) void k_iota(int32_t *rowptr, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= n) rowptr[i] = i;
}

// flags[0] collects error bits; pair i seeds bit i at x_obj when x_obj leads to x_wrt (bit i of B) and
// the two differ (only children are ever compared with x_wrt: a node is not a route to itself).
__global__ __launch_bounds__(64) void k_seed_pairs(int64_t T, int num_pairs, const int32_t *obj, const int32_t *wrt,
                                                   const u64 *B, u64 *F, int32_t *flags)
{
    const int i = threadIdx.x;
    if (i >= num_pairs) return;
    const int32_t a = obj[i], b = wrt[i];
    if (a < 0 || a >= T || b < 0 || b >= T) {
        atomicOr(&flags[0], kErrIdRange);
        return;
    }
    const u64 bit = (u64)1 << i;
    if (a != b && (B[a] & bit)) atomicOr(&F[a], bit);
}

constexpr int kFwThreads = 256;

// One pass over the kept operators of the first stage, 64 consecutive ones per wave and step.  A group
// is repeated until it adds nothing (operators of one group usually feed each other); *changed is set
// when the pass added anything at all.  Values of F read here may be stale: F only grows, and the host
// repeats the pass until one of them changes nothing.
// A lane's operator comes as its 16-byte record (one access instead of four row pointers), which also names the
// outputs when they are numbered consecutively: the marks of the first two outputs are then asked for together with
// the inputs', not behind them.
__global__ __launch_bounds__(kFwThreads) void k_forward_within(GraphView g, const int32_t *kept, const int64_t *kept_count,
                                                                const u64 *B, u64 *F, int32_t *changed)
{
    const int lane = lane_id();
    const int64_t n = *kept_count;
    const int64_t wave_id = (int64_t)blockIdx.x * (kFwThreads / kWave) + (threadIdx.x >> 6);
    const int64_t num_waves = (int64_t)gridDim.x * (kFwThreads / kWave);
    bool added = false;
    for (int64_t base = wave_id * kWave; base < n; base += num_waves * kWave) {
        const bool valid = base + lane < n;
        int4 r = make_int4(0, 0, 0, 0);
        if (valid) r = g.orec[kept[base + lane]];
        const int ib = r.x, ie = r.x + r.y;
        const int n_out = r.w >= 0 ? r.w : -r.w;
        // the first two outputs and what of them may be marked at all (B does not change during these passes)
        int32_t y0 = -1, y1 = -1;
        if (n_out > 0) y0 = r.w >= 0 ? r.z : g.out_idx[r.z];
        if (n_out > 1) y1 = r.w >= 0 ? r.z + 1 : g.out_idx[r.z + 1];
        const u64 b0 = y0 >= 0 ? B[y0] : 0, b1 = y1 >= 0 ? B[y1] : 0;
        for (int iter = 0; iter < kWave; ++iter) {          // a chain inside the group is at most 64 long
            const u64 fy0 = y0 >= 0 ? load_coherent(&F[y0]) : 0, fy1 = y1 >= 0 ? load_coherent(&F[y1]) : 0;
            // four inputs at a time, their ids and then their marks in flight together (past the row's end the last
            // input is read again): an operator with dozens of inputs would otherwise hold its wave for two dependent
            // accesses per input
            u64 fin = 0;
            for (int e = ib; e < ie; e += 4) {
                const int last = ie - 1;
                const int32_t x0 = g.in_idx[e], x1 = g.in_idx[min(e + 1, last)], x2 = g.in_idx[min(e + 2, last)],
                              x3 = g.in_idx[min(e + 3, last)];
                const u64 f0 = load_coherent(&F[x0]), f1 = load_coherent(&F[x1]), f2 = load_coherent(&F[x2]),
                          f3 = load_coherent(&F[x3]);
                fin |= (f0 | f1) | (f2 | f3);
            }
            bool any_new = false;
            if (fin) {
                if ((fin & b0) & ~fy0) {
                    atomicOr(&F[y0], fin & b0);
                    any_new = true;
                }
                if ((fin & b1) & ~fy1) {
                    atomicOr(&F[y1], fin & b1);
                    any_new = true;
                }
                for (int j = 2; j < n_out; ++j) {
                    const int32_t y = r.w >= 0 ? r.z + j : g.out_idx[r.z + j];
                    const u64 add = fin & B[y];
                    if (add & ~load_coherent(&F[y])) {
                        atomicOr(&F[y], add);
                        any_new = true;
                    }
                }
            }
            if (ballot64(any_new) == 0) break;
            added = true;
        }
    }
    if (ballot64(added) && lane == 0) *changed = 1;         // same value from every writer
}

// K[o] = OR of F over the outputs of o (removal rule of Sec. 2.1), for the operators of a kept list only; flags
// (or NULL): a byte per operator that is 1 exactly for the operators of the list on entry, 1 where K != 0 on return
__global__ __launch_bounds__(kFwThreads) void k_keep_from_list(GraphView g, const int32_t *kept, const int64_t *kept_count,
                                                                const u64 *F, u64 *K, uint8_t *flags)
{
    const int64_t n = *kept_count;
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gsize) {
        const int32_t o = kept[i];
        u64 k = 0;
        for (int32_t e = g.out_rowptr[o]; e < g.out_rowptr[o + 1]; ++e) k |= F[g.out_idx[e]];
        K[o] = k;
        if (flags && k == 0) flags[o] = 0;
    }
}

hipError_t launch_keep_from_list(const GraphView &g, const int32_t *kept, const int64_t *kept_count, const u64 *F, u64 *K,
                                 uint8_t *flags, int grid_blocks, hipStream_t s)
{
    hipLaunchKernelGGL(k_keep_from_list, dim3((unsigned)grid_blocks), dim3(kFwThreads), 0, s, g, kept, kept_count, F, K,
                       flags);
    return hipGetLastError();
}

hipError_t launch_backward_seed(int64_t T, int num_pairs, const int32_t *obj, const int32_t *wrt, int32_t *tgt_rowptr,
                                const u64 *B, u64 *F, int32_t *flags, bool rowptr_only, hipStream_t s)
{
    if (rowptr_only) {
        hipLaunchKernelGGL(k_iota, dim3(2), dim3(64), 0, s, tgt_rowptr, num_pairs);
    } else {
        hipLaunchKernelGGL(k_seed_pairs, dim3(1), dim3(64), 0, s, T, num_pairs, obj, wrt, B, F, flags);
    }
    return hipGetLastError();
}

hipError_t launch_forward_within(const GraphView &g, const int32_t *kept, const int64_t *kept_count, const u64 *B, u64 *F,
                                 int32_t *changed, int grid_blocks, hipStream_t s)
{
    hipLaunchKernelGGL(k_forward_within, dim3((unsigned)grid_blocks), dim3(kFwThreads), 0, s, g, kept, kept_count, B, F,
                       changed);
    return hipGetLastError();
}

}  // namespace dgn
