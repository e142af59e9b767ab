// What a graph runtime reads off a prune result (Sec. 3.2 of the paper): the tensors to rename
// "ignore" (written by a surviving operator, used by nothing the targets need) and, per target set,
// the surviving operators in creation order.  Both work on the compacted kept list, so their cost
// follows the pruned graph, not the recorded one (apart from clearing the ignore mask).
#include "common.h"

namespace dgn {

constexpr int kPpThreads = 256;

// ignore[y] |= K[o] & ~M[y] for every output y of every kept operator o; tensors with a new non-zero
// mask are counted (a tensor with several producers is counted once: by the add that found it zero).
__global__ __launch_bounds__(kPpThreads) void k_ignore_mask(GraphView g, const int32_t *kept_ops, const u64 *kept_masks,
                                                             const int64_t *kept_count, const u64 *M, u64 *ignore,
                                                             int64_t *ignore_count)
{
    const int64_t n = *kept_count;
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    int found = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gsize) {
        const int32_t o = kept_ops[i];
        const u64 k = kept_masks[i];
        for (int32_t e = g.out_rowptr[o]; e < g.out_rowptr[o + 1]; ++e) {
            const int32_t y = g.out_idx[e];
            const u64 ig = k & ~M[y];
            if (ig) found += atomicOr(&ignore[y], ig) == 0;
        }
    }
    const int wfound = wave_sum(found);
    if (wfound && lane_id() == 0 && ignore_count) atomicAdd((u64 *)ignore_count, (u64)wfound);
}

// Per-set lists.  The kept list is cut into tiles of 64 entries; a 64x64 bit-matrix transpose gives
// lane q the entries of the tile that belong to set q.  Counts go into a set-major table
// (table[q * tiles + tile]), so that ONE exclusive scan over the table yields, for every set and tile,
// the first slot of that tile's entries in the set's list -- lists laid out set after set.
__global__ __launch_bounds__(kPpThreads) void k_set_count(const u64 *kept_masks, int64_t n, int64_t tiles, int32_t *table)
{
    const int lane = lane_id();
    const int64_t wave_id = (int64_t)blockIdx.x * (kPpThreads / kWave) + (threadIdx.x >> 6);
    const int64_t num_waves = (int64_t)gridDim.x * (kPpThreads / kWave);
    for (int64_t tile = wave_id; tile < tiles; tile += num_waves) {
        const int64_t i = tile * kWave + lane;
        const u64 k = i < n ? kept_masks[i] : 0;
        table[(int64_t)lane * tiles + tile] = __popcll(wave_transpose64(k));
    }
}

__global__ __launch_bounds__(kPpThreads) void k_set_scatter(const int32_t *kept_ops, const u64 *kept_masks, int64_t n,
                                                             int64_t tiles, const int32_t *table, int32_t *set_ops,
                                                             int64_t capacity)
{
    __shared__ int32_t s_ops[kPpThreads / kWave][kWave];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t wave_id = (int64_t)blockIdx.x * (kPpThreads / kWave) + wave;
    const int64_t num_waves = (int64_t)gridDim.x * (kPpThreads / kWave);
    for (int64_t tile = wave_id; tile < tiles; tile += num_waves) {
        const int64_t i = tile * kWave + lane;
        const u64 k = i < n ? kept_masks[i] : 0;
        s_ops[wave][lane] = i < n ? kept_ops[i] : -1;
        u64 col = wave_transpose64(k);                      // lane q: bit j set iff entry j of the tile is in set q
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        int64_t pos = table[(int64_t)lane * tiles + tile];
        while (col) {                                       // ascending entries: the list stays in creation order
            const int j = __builtin_ctzll(col);
            col &= col - 1;
            if (pos < capacity) set_ops[pos] = s_ops[wave][j];
            ++pos;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

__global__ __launch_bounds__(128) void k_set_rowptr(const int32_t *table, int64_t tiles, int64_t *set_rowptr)
{
    const int q = threadIdx.x;
    if (q <= 64) set_rowptr[q] = tiles > 0 ? table[(int64_t)q * tiles] : 0;    // entry 64*tiles holds the total
}

size_t set_lists_scratch_bytes(int64_t num_kept)
{
    const int64_t tiles = (num_kept + kWave - 1) / kWave;
    const size_t table = ((size_t)(64 * tiles + 1) * 4 + 255) & ~(size_t)255;
    return table + scan_tmp_bytes(64 * tiles) + 256;
}

hipError_t launch_ignore_mask(const GraphView &g, const int32_t *kept_ops, const u64 *kept_masks, const int64_t *kept_count,
                              const u64 *M, u64 *ignore, int64_t *ignore_count, int grid_blocks, hipStream_t s)
{
    FillRegion clr[2] = {{ignore, (size_t)g.num_tensors * 8}, {ignore_count, ignore_count ? sizeof(int64_t) : 0}};
    hipError_t e = launch_clear(clr, 2, s);
    if (e != hipSuccess) return e;
    if (g.num_ops > 0)
        hipLaunchKernelGGL(k_ignore_mask, dim3((unsigned)grid_blocks), dim3(kPpThreads), 0, s, g, kept_ops, kept_masks,
                           kept_count, M, ignore, ignore_count);
    return hipGetLastError();
}

hipError_t launch_set_lists(const int32_t *kept_ops, const u64 *kept_masks, int64_t num_kept, int64_t *set_rowptr,
                            int32_t *set_ops, int64_t capacity, void *scratch, int grid_blocks, hipStream_t s)
{
    const int64_t tiles = (num_kept + kWave - 1) / kWave;
    int32_t *table = static_cast<int32_t *>(scratch);
    void *scan_tmp = static_cast<char *>(scratch) + (((size_t)(64 * tiles + 1) * 4 + 255) & ~(size_t)255);
    if (tiles > 0) {
        int64_t blocks = (tiles + (kPpThreads / kWave) - 1) / (kPpThreads / kWave);
        if (blocks > grid_blocks) blocks = grid_blocks;
        hipLaunchKernelGGL(k_set_count, dim3((unsigned)blocks), dim3(kPpThreads), 0, s, kept_masks, num_kept, tiles, table);
        hipError_t e = launch_exclusive_scan(table, table, 64 * tiles, scan_tmp, s);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_set_scatter, dim3((unsigned)blocks), dim3(kPpThreads), 0, s, kept_ops, kept_masks, num_kept,
                           tiles, table, set_ops, capacity);
    }
    hipLaunchKernelGGL(k_set_rowptr, dim3(1), dim3(128), 0, s, table, tiles, set_rowptr);
    return hipGetLastError();
}

}  // namespace dgn
