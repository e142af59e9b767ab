// CSR builder support: row-degree histograms with id range checks, and the validation passes.
// The adjacency follows the edge definition of Sec. 2.2 of the paper: an operator with the tensors it
// reads and the tensors it writes; Parent(x) of Algorithm 1 = inputs of every operator that writes x.
#include "common.h"

namespace dgn {

// deg[key] += 1.  Ids outside their range are reported and skipped, so later passes never index
// out of bounds with them (the sort itself only ever uses masked digits of the keys).
//
// The same pass notes whether the keys ever decrease (*unsorted = 1): recorded graphs are usually handed
// over operator by operator, and edges that are already in row order need no sort at all.
__global__ __launch_bounds__(256) void k_degree_hist(const int32_t *keys, const int32_t *vals, int64_t nnz,
                                                      int32_t n_rows, int32_t n_vals, int32_t *deg, int32_t *error,
                                                      int32_t *unsorted)
{
    // Runs of equal keys inside a wave (operator-major COO is one long sequence of such runs) are added
    // with ONE atomic by the run's first lane: atomics on one address serialise, and an operator with
    // fan-in 64 would otherwise be 64 of them.
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    const int lane = lane_id();
    bool bad = false, descends = false;
    for (int64_t base = (int64_t)blockIdx.x * blockDim.x + (threadIdx.x & ~(kWave - 1)); base < nnz; base += gsize) {
        const int64_t e = base + lane;                      // wave-uniform loop, lanes past the end idle
        const bool valid = e < nnz;
        const int32_t k = valid ? keys[e] : -1;
        const int32_t v = (valid && vals) ? vals[e] : 0;
        const bool good = valid && k >= 0 && k < n_rows;
        if (valid && (!good || v < 0 || v >= n_vals)) bad = true;
        int32_t prev = __shfl_up(k, 1, kWave);
        if (lane == 0) prev = base > 0 ? keys[base - 1] : k;    // the key just before this wave's first one
        if (valid && prev > k) descends = true;
        const u64 gmask = ballot64(good);
        const bool leader = good && (lane == 0 || !((gmask >> (lane - 1)) & 1) || prev != k);
        const u64 boundaries = ballot64(leader) | ~gmask;   // a run ends at the next leader or the next bad lane
        if (leader) {
            const u64 above = lane == kWave - 1 ? 0 : boundaries >> (lane + 1);
            const int run = above ? __builtin_ctzll(above) + 1 : kWave - lane;
            atomicAdd(&deg[k], run);
        }
    }
    if (ballot64(bad) != 0 && lane == 0) atomicOr(error, kErrIdRange);
    // shuffled input would have every wave report: look first, and store (same value from everyone) only if needed
    if (ballot64(descends) != 0 && lane == 0 && load_coherent(unsorted) == 0) store_coherent(unsorted, 1);
}

hipError_t launch_degree_hist(const int32_t *keys, const int32_t *vals, int64_t nnz, int32_t n_rows,
                              int32_t n_vals, int32_t *deg, int32_t *error, int32_t *unsorted, hipStream_t s)
{
    if (nnz == 0) return hipSuccess;
    int64_t blocks = (nnz + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_degree_hist, dim3((unsigned)blocks), dim3(256), 0, s, keys, vals, nnz, n_rows, n_vals,
                       deg, error, unsorted);
    return hipGetLastError();
}

// One pass over an edge list in the order it was handed over: range check of both ids, whether the keys
// ever decrease (*unsorted = 1), and -- on the assumption that they do not, which holds for a graph
// recorded operator by operator -- the finished row: idx_out = the values as they stand, rowptr = first
// position of every key.  If the keys do decrease somewhere, what was written is simply overwritten by the
// sort that follows.  No atomic in the common case.
__device__ __forceinline__ void write_rows(int32_t *rowptr, int lo, int hi, int32_t val)
{
    // rows lo..hi get val; gaps longer than a few rows are filled by the whole wave (call wave-uniformly)
    constexpr int kShort = 4;
    for (int r = lo; r <= hi && r < lo + kShort; ++r) rowptr[r] = val;
    u64 longer = ballot64(hi - lo >= kShort);
    while (longer) {
        const int src = __builtin_ctzll(longer);
        longer &= longer - 1;
        const int s_lo = __shfl(lo, src, kWave) + kShort, s_hi = __shfl(hi, src, kWave);
        const int32_t s_val = __shfl(val, src, kWave);
        for (int r = s_lo + lane_id(); r <= s_hi; r += kWave) rowptr[r] = s_val;
    }
}

constexpr int kMaxGapHere = 64;

__global__ __launch_bounds__(256) void k_scan_edges(const int32_t *keys, const int32_t *vals, int64_t nnz,
                                                     int32_t n_rows, int32_t n_vals, int32_t *idx_out, int32_t *rowptr,
                                                     int32_t *error, int32_t *unsorted, int32_t *wide_gap)
{
    // a thread takes four neighbouring positions per step, in 16-byte loads and stores where the arrays are aligned
    // for them: with a single position per thread the pass waits for memory most of its time
    constexpr int kPer = 4;
    const bool wide = ((reinterpret_cast<uintptr_t>(keys) | reinterpret_cast<uintptr_t>(vals) |
                        reinterpret_cast<uintptr_t>(idx_out)) & 15) == 0;
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x * kPer;
    const int64_t steps = (nnz + 1 + gsize - 1) / gsize;                // position nnz closes the last rows
    bool bad = false, descends = false, gap = false;
    for (int64_t st = 0; st < steps; ++st) {                            // whole waves stay in the loop
        const int64_t e0 = st * gsize + ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * kPer;
        int32_t k[kPer + 1], v[kPer];                                   // k[j] = key before position e0 + j
        k[0] = e0 > 0 && e0 <= nnz ? keys[e0 - 1] : -1;
        if (wide && e0 + kPer <= nnz) {
            const int4 kk = *reinterpret_cast<const int4 *>(keys + e0);
            const int4 vv = *reinterpret_cast<const int4 *>(vals + e0);
            k[1] = kk.x; k[2] = kk.y; k[3] = kk.z; k[4] = kk.w;
            v[0] = vv.x; v[1] = vv.y; v[2] = vv.z; v[3] = vv.w;
            *reinterpret_cast<int4 *>(idx_out + e0) = vv;
        } else {
#pragma unroll
            for (int j = 0; j < kPer; ++j) {
                const bool edge = e0 + j < nnz;
                k[j + 1] = edge ? keys[e0 + j] : n_rows;
                v[j] = edge ? vals[e0 + j] : 0;
                if (edge) idx_out[e0 + j] = v[j];
            }
        }
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int64_t e = e0 + j;
            int lo = 0, hi = -1;
            if (e <= nnz) {
                const int32_t prev = k[j], cur = k[j + 1];
                if (e < nnz) {
                    if (cur < 0 || cur >= n_rows || v[j] < 0 || v[j] >= n_vals) bad = true;
                    if (prev > cur) descends = true;
                }
                // rows (prev, cur]; keys outside their range write nothing (the call fails anyway)
                if (prev >= -1 && prev < n_rows && cur >= 0 && cur <= n_rows) {
                    lo = prev + 1;
                    hi = cur;
                }
                // A long run of empty rows is left to a pass of its own (*wide_gap): keys in random order jump far
                // at nearly every position, and filling those jumps here would cost more than the sort that follows.
                if (hi - lo >= kMaxGapHere) {
                    gap = true;
                    hi = lo - 1;
                }
            }
            write_rows(rowptr, lo, hi, (int32_t)e);
        }
    }
    if (ballot64(gap) != 0 && lane_id() == 0 && load_coherent(wide_gap) == 0) store_coherent(wide_gap, 1);
    if (ballot64(bad) != 0 && lane_id() == 0) atomicOr(error, kErrIdRange);
    // shuffled input would have every wave report: look first, and store (same value from everyone) only if needed
    if (ballot64(descends) != 0 && lane_id() == 0 && load_coherent(unsorted) == 0) store_coherent(unsorted, 1);
}

hipError_t launch_scan_edges(const int32_t *keys, const int32_t *vals, int64_t nnz, int32_t n_rows, int32_t n_vals,
                             int32_t *idx_out, int32_t *rowptr, int32_t *error, int32_t *unsorted, int32_t *wide_gap,
                             hipStream_t s)
{
    int64_t blocks = (nnz + 1 + 1023) / 1024;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_scan_edges, dim3((unsigned)blocks), dim3(256), 0, s, keys, vals, nnz, n_rows, n_vals, idx_out,
                       rowptr, error, unsorted, wide_gap);
    return hipGetLastError();
}

// Row pointers from keys in row order: rowptr[r] = first position whose key is >= r, rowptr[n_rows] = nnz.
// Position i writes the rows (keys[i-1], keys[i]]; gaps longer than a few rows are filled by the whole wave.
__global__ __launch_bounds__(256) void k_row_bounds(const int32_t *keys, int64_t nnz, int32_t n_rows, int32_t *rowptr)
{
    // a thread takes four neighbouring positions per step (one 16-byte load when the keys are aligned for it): with a
    // single position per thread the pass waits for memory most of its time
    constexpr int kPer = 4;
    const bool wide = (reinterpret_cast<uintptr_t>(keys) & 15) == 0;
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x * kPer;
    const int64_t steps = (nnz + 1 + gsize - 1) / gsize;                // position nnz closes the last rows
    for (int64_t st = 0; st < steps; ++st) {                            // whole waves stay in the loop
        const int64_t i0 = st * gsize + ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * kPer;
        int32_t k[kPer + 1];                                            // k[j] = key before position i0 + j
        if (i0 <= nnz) k[0] = i0 == 0 ? -1 : keys[i0 - 1];
        if (wide && i0 + kPer <= nnz) {
            const int4 v = *reinterpret_cast<const int4 *>(keys + i0);
            k[1] = v.x; k[2] = v.y; k[3] = v.z; k[4] = v.w;
        } else {
#pragma unroll
            for (int j = 0; j < kPer; ++j) k[j + 1] = i0 + j < nnz ? keys[i0 + j] : n_rows;
        }
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            int lo = 0, hi = -1;                                        // rows lo..hi get the value i0 + j
            if (i0 + j <= nnz) {
                lo = k[j] + 1;
                hi = k[j + 1];
            }
            write_rows(rowptr, lo, hi, (int32_t)(i0 + j));
        }
    }
}

hipError_t launch_row_bounds(const int32_t *keys, int64_t nnz, int32_t n_rows, int32_t *rowptr, hipStream_t s)
{
    int64_t blocks = (nnz + 1 + 1023) / 1024;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_row_bounds, dim3((unsigned)blocks), dim3(256), 0, s, keys, nnz, n_rows, rowptr);
    return hipGetLastError();
}

// Borrowed CSR: rowptr[0] == 0, monotone, rowptr[n_rows] == nnz, every idx in [0, n_vals).
__global__ __launch_bounds__(256) void k_check_csr(const int32_t *rowptr, const int32_t *idx, int32_t n_rows,
                                                    int32_t nnz, int32_t n_vals, int32_t *error)
{
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int bad = 0;
    for (int64_t r = gtid; r <= n_rows; r += gsize) {
        const int32_t a = rowptr[r];
        if (a < 0 || a > nnz) bad |= kErrCsr;
        if (r == 0 && a != 0) bad |= kErrCsr;
        if (r == n_rows && a != nnz) bad |= kErrCsr;
        if (r < n_rows && rowptr[r + 1] < a) bad |= kErrCsr;
    }
    for (int64_t e = gtid; e < nnz; e += gsize) {
        const int32_t v = idx[e];
        if (v < 0 || v >= n_vals) bad |= kErrIdRange;
    }
    if (bad) atomicOr(error, bad);
}

hipError_t launch_check_csr(const int32_t *rowptr, const int32_t *idx, int32_t n_rows, int32_t nnz,
                            int32_t n_vals, int32_t *error, hipStream_t s)
{
    int64_t work = (int64_t)n_rows + 1 > nnz ? (int64_t)n_rows + 1 : nnz;
    int64_t blocks = (work + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_check_csr, dim3((unsigned)blocks), dim3(256), 0, s, rowptr, idx, n_rows, nnz, n_vals, error);
    return hipGetLastError();
}

// row_of[e] = r for every entry e of row r (operator id of every entry of a borrowed out CSR)
__global__ __launch_bounds__(256) void k_expand_rows(const int32_t *rowptr, int32_t n_rows, int32_t *row_of)
{
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n_rows; r += gsize)
        for (int32_t e = rowptr[r]; e < rowptr[r + 1]; ++e) row_of[e] = (int32_t)r;
}

hipError_t launch_expand_rows(const int32_t *rowptr, int32_t n_rows, int32_t *row_of, hipStream_t s)
{
    if (n_rows == 0) return hipSuccess;
    int64_t blocks = ((int64_t)n_rows + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_expand_rows, dim3((unsigned)blocks), dim3(256), 0, s, rowptr, n_rows, row_of);
    return hipGetLastError();
}

// Topological precondition (Sec. 3.2: operators run in creation order): every producer of an
// operator's input was created before the operator.
__global__ __launch_bounds__(256) void k_check_topological(GraphView g, int32_t *error)
{
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < g.num_ops; o += gsize) {
        for (int32_t e = g.in_rowptr[o]; e < g.in_rowptr[o + 1]; ++e) {
            const int32_t t = g.in_idx[e];
            if (t < 0 || t >= g.num_tensors) continue;      // reported by the range check
            const int32_t pr = g.prod1[t];                  // one word instead of two CSR hops
            if (pr >= 0) {
                if (pr >= o) bad = true;
            } else if (pr == kMulti) {
                for (int32_t p = g.prod_rowptr[t]; p < g.prod_rowptr[t + 1]; ++p)
                    if (g.prod_idx[p] >= o) bad = true;
            }
        }
    }
    if (bad) atomicOr(error, kErrTopo);
}

hipError_t launch_check_topological(const GraphView &g, int32_t *error, hipStream_t s)
{
    if (g.num_ops == 0) return hipSuccess;
    int64_t blocks = ((int64_t)g.num_ops + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_check_topological, dim3((unsigned)blocks), dim3(256), 0, s, g, error);
    return hipGetLastError();
}

// Packed batch: every edge of an operator of graph g must touch a tensor of graph g.
__device__ __forceinline__ int find_graph(const int64_t *off, int num_graphs, int64_t id)
{
    int lo = 0, hi = num_graphs;          // largest g with off[g] <= id
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= id) lo = mid; else hi = mid;
    }
    return lo;
}

// also_topological: the topological precondition is checked in the same walk (see k_check_topological), which
// spares a packed batch a second pass over its input edges.
__global__ __launch_bounds__(256) void k_check_graph_ranges(GraphView g, int32_t *error, bool also_topological)
{
    // a wave walks a contiguous stretch of operators 64 at a time, so a lane's graph index only ever steps
    // forward: one binary search per lane, not one per operator
    const int64_t waves = (int64_t)gridDim.x * (blockDim.x / kWave);
    const int64_t wave_id = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6);
    const int64_t per = (((int64_t)g.num_ops + waves - 1) / waves + kWave - 1) / kWave * kWave;
    const int64_t first = wave_id * per, last = min(first + per, (int64_t)g.num_ops);
    bool bad = false, late = false;
    int gi = -1;
    for (int64_t o = first + lane_id(); o < last; o += kWave) {
        if (gi < 0) gi = find_graph(g.op_off, g.num_graphs, o);
        while (o >= g.op_off[gi + 1]) ++gi;                 // op_off[num_graphs] == num_ops > o: stops in range
        const int64_t lo = g.t_off[gi], hi = g.t_off[gi + 1];
        for (int32_t e = g.in_rowptr[o]; e < g.in_rowptr[o + 1]; ++e) {
            const int32_t t = g.in_idx[e];
            if (t < lo || t >= hi) bad = true;
            if (also_topological && t >= 0 && t < g.num_tensors) {
                const int32_t pr = g.prod1[t];
                if (pr >= 0) {
                    if (pr >= o) late = true;
                } else if (pr == kMulti) {
                    for (int32_t p = g.prod_rowptr[t]; p < g.prod_rowptr[t + 1]; ++p)
                        if (g.prod_idx[p] >= o) late = true;
                }
            }
        }
        for (int32_t e = g.out_rowptr[o]; e < g.out_rowptr[o + 1]; ++e)
            if (g.out_idx[e] < lo || g.out_idx[e] >= hi) bad = true;
    }
    if (bad || late) atomicOr(error, (bad ? kErrCrossGraph : 0) | (late ? kErrTopo : 0));
}

hipError_t launch_check_graph_ranges(const GraphView &g, int32_t *error, bool also_topological, hipStream_t s)
{
    if (g.num_ops == 0 || g.num_graphs <= 1) return hipSuccess;
    int64_t blocks = ((int64_t)g.num_ops + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_check_graph_ranges, dim3((unsigned)blocks), dim3(256), 0, s, g, error, also_topological);
    return hipGetLastError();
}

}  // namespace dgn
