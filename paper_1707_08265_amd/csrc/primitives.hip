// Streaming primitives: multi-region clear and device-wide exclusive prefix sum.
// Both are pure HBM streams; the scan reads its input twice (reduce, then scan-with-offset) so that
// no workgroup ever waits on another.
#include "common.h"

namespace dgn {

// ------------------------------------------------------------------------------------------------
// clear: the output masks must start at zero before the seeds are scattered (main loop of
// Algorithm 1 starts from "nothing marked").  16-byte stores, grid-stride, up to 8 regions per launch.
// ------------------------------------------------------------------------------------------------
constexpr int kMaxClearRegions = 8;
struct ClearArgs {
    u64 *ptr[kMaxClearRegions];
    size_t words[kMaxClearRegions];
    int n;
};

__device__ __forceinline__ void clear_regions(const ClearArgs &a)
{
    const size_t gtid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t gsize = (size_t)gridDim.x * blockDim.x;
    for (int r = 0; r < a.n; ++r) {
        u64 *p = a.ptr[r];
        size_t w = a.words[r];
        if (w == 0) continue;
        if (((uintptr_t)p & 8) != 0) {          // make the bulk 16-byte aligned
            if (gtid == 0) p[0] = 0;
            ++p; --w;
        }
        ulonglong2 *p2 = reinterpret_cast<ulonglong2 *>(p);
        const size_t pairs = w >> 1;
        const ulonglong2 z = make_ulonglong2(0, 0);
        for (size_t i = gtid; i < pairs; i += gsize) p2[i] = z;
        if ((w & 1) && gtid == 0) p[w - 1] = 0;
    }
}

__global__ __launch_bounds__(256) void k_clear(ClearArgs a) { clear_regions(a); }

// The same, unless the scratch buffer says that the output buffers still hold the result of the previous
// prune of this graph, unchanged: then only the words that prune set are zeroed -- M of the tensors in its
// log, K, the deferral marker and the keep flag of its kept operators -- a few MB of scattered stores instead of 8(T + P)
// bytes of streaming ones.
__global__ __launch_bounds__(256) void k_clear_or_reset(ClearArgs a, const RecycleHeader *hdr, RecycleHeader want,
                                                        u64 *found_out, ColourLog log, const int32_t *kept_ops,
                                                        const int64_t *kept_count, u64 *M, u64 *K, uint8_t *DB,
                                                        uint8_t *flags)
{
    __shared__ int s_pref[kMaxSeg + 1];
    u64 *also_M = static_cast<u64 *>(const_cast<void *>(want.also_M));
    u64 *also_K = static_cast<u64 *>(const_cast<void *>(want.also_K));
    const RecycleHeader have = *hdr;
    const bool found = same_header(have, want);             // the same answer in every block
    if (blockIdx.x == 0 && threadIdx.x == 0) found_out[0] = found ? 1 : 0;
    if (!found) {
        clear_regions(a);
        return;
    }
    if (threadIdx.x < kWave) {
        const int lane = lane_id();
        const int incl = wave_incl_scan(min(log.cnt[lane].v, log.seg_cap));
        if (lane == 0) s_pref[0] = 0;
        s_pref[lane + 1] = incl;
    }
    __syncthreads();
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    const int total = s_pref[kMaxSeg];
    for (int64_t i = gtid; i < total; i += gsize) {
        int lo = 0, hi = kMaxSeg - 1;           // segment holding entry i: last s with s_pref[s] <= i
#pragma unroll
        for (int it = 0; it < 6; ++it) {
            const int mid = (lo + hi + 1) >> 1;
            if (s_pref[mid] <= (int)i) lo = mid; else hi = mid - 1;
        }
        const int32_t t = log.entries[(int64_t)lo * log.seg_cap + ((int)i - s_pref[lo])];
        M[t] = 0;
        if (also_M) also_M[t] = 0;
    }
    const int64_t kept = kept_count[0];
    for (int64_t i = gtid; i < kept; i += gsize) {
        const int32_t o = kept_ops[i];
        K[o] = 0;
        DB[o] = 0;
        flags[o] = 0;
        if (also_K) also_K[o] = 0;
    }
}

hipError_t launch_clear(const FillRegion *regions, int num_regions, hipStream_t s)
{
    for (int base = 0; base < num_regions; base += kMaxClearRegions) {
        ClearArgs a{};
        size_t total = 0;
        a.n = 0;
        for (int r = base; r < num_regions && a.n < kMaxClearRegions; ++r) {
            if (regions[r].bytes == 0 || regions[r].ptr == nullptr) continue;
            a.ptr[a.n] = static_cast<u64 *>(regions[r].ptr);
            a.words[a.n] = regions[r].bytes / 8;
            total += a.words[a.n];
            ++a.n;
        }
        if (a.n == 0) continue;
        size_t blocks = (total / 2 + 255) / 256;
        if (blocks < 1) blocks = 1;
        if (blocks > 4096) blocks = 4096;     // 16 workgroups per CU, then grid-stride
        hipLaunchKernelGGL(k_clear, dim3((unsigned)blocks), dim3(256), 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_clear_or_reset(const FillRegion *regions, int num_regions, const RecycleHeader *hdr,
                                 const RecycleHeader &want, u64 *found_out, const ColourLog &log, const int32_t *kept_ops,
                                 const int64_t *kept_count, u64 *M, u64 *K, uint8_t *DB, uint8_t *flags, hipStream_t s)
{
    if (num_regions > kMaxClearRegions) return hipErrorInvalidValue;
    ClearArgs a{};
    size_t total = 0;
    for (int r = 0; r < num_regions; ++r) {
        if (regions[r].bytes == 0 || regions[r].ptr == nullptr) continue;
        a.ptr[a.n] = static_cast<u64 *>(regions[r].ptr);
        a.words[a.n] = regions[r].bytes / 8;
        total += a.words[a.n];
        ++a.n;
    }
    size_t blocks = (total / 2 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_clear_or_reset, dim3((unsigned)blocks), dim3(256), 0, s, a, hdr, want, found_out, log, kept_ops,
                       kept_count, M, K, DB, flags);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// exclusive scan (int32), n+1 outputs
// ------------------------------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;

__device__ __forceinline__ int block_excl_scan_256(int v, int *total, int *lds /* >= 5 ints */)
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    int incl = wave_incl_scan(v);
    if (lane == kWave - 1) lds[wave] = incl;
    __syncthreads();
    int woff = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / kWave; ++w) {
        int c = lds[w];
        if (w < wave) woff += c;
        tot += c;
    }
    __syncthreads();
    *total = tot;
    return woff + incl - v;
}

__global__ __launch_bounds__(kScanThreads) void k_scan_reduce(const int32_t *in, int64_t n, int32_t *sums)
{
    __shared__ int lds[8];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    int acc = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k)
        if (base + k < n) acc += in[base + k];
    acc = wave_sum(acc);
    if (lane_id() == 0) lds[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sums[blockIdx.x] = lds[0] + lds[1] + lds[2] + lds[3];
}

// One workgroup scans m entries in place (exclusive) and writes the total to v[m].
__global__ __launch_bounds__(1024) void k_scan_single(int32_t *v, int64_t m)
{
    __shared__ int wtot[16];
    __shared__ int carry_s;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < m; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const int x = i < m ? v[i] : 0;
        const int incl = wave_incl_scan(x);
        if (lane == kWave - 1) wtot[wave] = incl;
        __syncthreads();
        int woff = 0, tot = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int c = wtot[w];
            if (w < wave) woff += c;
            tot += c;
        }
        const int carry = carry_s;
        if (i < m) v[i] = carry + woff + incl - x;
        __syncthreads();
        if (threadIdx.x == 0) carry_s = carry + tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) v[m] = carry_s;
}

__global__ __launch_bounds__(kScanThreads) void k_scan_apply(const int32_t *in, int32_t *out, int64_t n,
                                                              const int32_t *offsets)
{
    __shared__ int lds[8];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    int x[kScanItems];
    int tsum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        x[k] = (base + k < n) ? in[base + k] : 0;
        tsum += x[k];
    }
    int tot;
    int run = offsets[blockIdx.x] + block_excl_scan_256(tsum, &tot, lds);   // barriers inside: all loads done
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        if (base + k <= n) out[base + k] = run;     // position n receives the grand total
        run += x[k];
    }
}

static inline int64_t scan_blocks(int64_t n) { return (n + 1 + kScanTile - 1) / kScanTile; }

size_t scan_tmp_bytes(int64_t n) { return (size_t)(scan_blocks(n) + 1) * sizeof(int32_t); }

hipError_t launch_exclusive_scan(const int32_t *in, int32_t *out, int64_t n, void *tmp, hipStream_t s)
{
    const int64_t nb = scan_blocks(n);
    int32_t *sums = static_cast<int32_t *>(tmp);
    hipLaunchKernelGGL(k_scan_reduce, dim3((unsigned)nb), dim3(kScanThreads), 0, s, in, n, sums);
    hipLaunchKernelGGL(k_scan_single, dim3(1), dim3(1024), 0, s, sums, nb);
    hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)nb), dim3(kScanThreads), 0, s, in, out, n, sums);
    return hipGetLastError();
}

}  // namespace dgn
