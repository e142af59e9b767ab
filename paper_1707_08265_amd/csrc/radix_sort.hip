// Stable LSD radix sort of (int32 key, int32 value) pairs, 9 bits per pass, for the CSR builder.
//
// Per pass: (1) per-tile digit histogram, stored digit-major so that one exclusive scan over the
// whole table yields, for every (digit, tile), the first output slot of that tile's keys with that
// digit; (2) the scan; (3) a scatter in which every wave ranks its keys with ballot "match" masks:
// keys of one tile are visited in their stored order, so equal keys keep their relative order.
// Only the significant key bits are sorted (ceil(log2(rows)) of them), so 50M operators (26 bits) or 100M
// tensors (27 bits) cost three passes.  (Eight bits per pass and four passes: 9 % slower on that graph; a pass
// with 512 digits costs more than one with 256, because a tile of 4 096 keys then leaves in runs of 8 keys per
// digit instead of 16, but not a third more.)
#include "common.h"

namespace dgn {

constexpr int kRadixBits = 9;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortThreads = kRadix;                    // one thread per digit in the per-tile bookkeeping
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kSortRounds = 8;                          // keys per lane
constexpr int kSortTile = kSortThreads * kSortRounds;   // keys per workgroup

__device__ __forceinline__ int digit_of(int32_t key, int shift) { return ((uint32_t)key >> shift) & (kRadix - 1); }

__global__ __launch_bounds__(kSortThreads) void k_sort_hist(const int32_t *keys, int64_t n, int shift,
                                                             int32_t *table, int64_t num_tiles)
{
    __shared__ int hist[kRadix];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll 4
    for (int r = 0; r < kSortRounds; ++r) {
        const int64_t i = base + r * kSortThreads + threadIdx.x;
        if (i < n) atomicAdd(&hist[digit_of(keys[i], shift)], 1);
    }
    __syncthreads();
    table[(int64_t)threadIdx.x * num_tiles + blockIdx.x] = hist[threadIdx.x];
}

template <bool kWriteKeys>
__global__ __launch_bounds__(kSortThreads) void k_sort_scatter(const int32_t *keys, const int32_t *vals,
                                                                int32_t *keys_out, int32_t *vals_out,
                                                                int64_t n, int shift, const int32_t *table,
                                                                int64_t num_tiles)
{
    __shared__ int wcount[kSortWaves][kRadix];
    __shared__ int s_delta[kRadix];          // global slot of a key = its slot in the locally sorted tile + this
    __shared__ int s_wtot[kSortWaves];
    __shared__ int32_t s_keys[kSortTile], s_vals[kSortTile];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < kSortWaves * kRadix; i += kSortThreads) (&wcount[0][0])[i] = 0;
    __syncthreads();

    // wave w owns kSortRounds * 64 consecutive keys of the tile, visited 64 at a time
    const int64_t tbase = (int64_t)blockIdx.x * kSortTile;
    const int64_t wbase = tbase + (int64_t)wave * (kSortRounds * kWave);
    int32_t key[kSortRounds], val[kSortRounds];
    int rank[kSortRounds];
    const u64 lt = lanemask_lt();
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int64_t i = wbase + r * kWave + lane;
        const bool valid = i < n;
        key[r] = valid ? keys[i] : 0;
        val[r] = valid ? vals[i] : 0;
        const int d = digit_of(key[r], shift);
        u64 peers = ballot64(valid);
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            const u64 m = ballot64((d >> b) & 1);
            peers &= ((d >> b) & 1) ? m : ~m;
        }
        // lanes with the same digit read the running count, then their first lane bumps it
        const int c = wcount[wave][d];
        const int before = __popcll(peers & lt);
        __builtin_amdgcn_wave_barrier();
        if (valid && before == 0) wcount[wave][d] = c + __popcll(peers);
        __builtin_amdgcn_wave_barrier();
        rank[r] = c + before;
    }
    __syncthreads();
    {   // digit d (one per thread): per-wave counts -> first slot of each wave's keys in the locally sorted tile
        const int d = threadIdx.x;
        int cnt = 0;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) cnt += wcount[w][d];
        const int incl = wave_incl_scan(cnt);
        if (lane == kWave - 1) s_wtot[wave] = incl;
        __syncthreads();
        int lbase = incl - cnt;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w)
            if (w < wave) lbase += s_wtot[w];
        s_delta[d] = table[(int64_t)d * num_tiles + blockIdx.x] - lbase;
        int run = lbase;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) {
            const int c = wcount[w][d];
            wcount[w][d] = run;
            run += c;
        }
    }
    __syncthreads();
    // sort the tile inside LDS, so that the global writes below go out in long contiguous runs per digit
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int64_t i = wbase + r * kWave + lane;
        if (i < n) {
            const int li = wcount[wave][digit_of(key[r], shift)] + rank[r];
            s_keys[li] = key[r];
            s_vals[li] = val[r];
        }
    }
    __syncthreads();
    const int count = (int)min((int64_t)kSortTile, n - tbase);
    for (int li = threadIdx.x; li < count; li += kSortThreads) {
        const int32_t k = s_keys[li];
        const int pos = li + s_delta[digit_of(k, shift)];
        if (kWriteKeys) keys_out[pos] = k;
        vals_out[pos] = s_vals[li];
    }
}

static inline int64_t sort_tiles(int64_t n) { return (n + kSortTile - 1) / kSortTile; }

// layout of tmp: keyA[n] valA[n] keyB[n] valB[n] table[kRadix*tiles + 1] scan_tmp
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t sort_tmp_bytes(int64_t n)
{
    const int64_t tiles = sort_tiles(n);
    return 4 * align256((size_t)n * 4) + align256((size_t)(kRadix * tiles + 1) * 4) +
           align256(scan_tmp_bytes(kRadix * tiles));
}

hipError_t launch_sort_pairs(const int32_t *keys_in, const int32_t *vals_in, int32_t *keys_out,
                             int32_t *vals_out, int64_t n, int key_bits, void *tmp, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const int64_t tiles = sort_tiles(n);
    char *p = static_cast<char *>(tmp);
    int32_t *kbuf[2], *vbuf[2];
    kbuf[0] = reinterpret_cast<int32_t *>(p); p += align256((size_t)n * 4);
    vbuf[0] = reinterpret_cast<int32_t *>(p); p += align256((size_t)n * 4);
    kbuf[1] = reinterpret_cast<int32_t *>(p); p += align256((size_t)n * 4);
    vbuf[1] = reinterpret_cast<int32_t *>(p); p += align256((size_t)n * 4);
    int32_t *table = reinterpret_cast<int32_t *>(p); p += align256((size_t)(kRadix * tiles + 1) * 4);
    void *scan_tmp = p;

    if (key_bits < 1) key_bits = 1;
    const int passes = (key_bits + kRadixBits - 1) / kRadixBits;
    const int32_t *ksrc = keys_in, *vsrc = vals_in;
    for (int pass = 0; pass < passes; ++pass) {
        const bool last = pass == passes - 1;
        const int shift = pass * kRadixBits;
        int32_t *kdst = last ? keys_out : kbuf[pass & 1];
        int32_t *vdst = last ? vals_out : vbuf[pass & 1];
        hipLaunchKernelGGL(k_sort_hist, dim3((unsigned)tiles), dim3(kSortThreads), 0, s, ksrc, n, shift, table, tiles);
        hipError_t e = launch_exclusive_scan(table, table, kRadix * tiles, scan_tmp, s);
        if (e != hipSuccess) return e;
        if (kdst)
            hipLaunchKernelGGL(k_sort_scatter<true>, dim3((unsigned)tiles), dim3(kSortThreads), 0, s, ksrc, vsrc,
                               kdst, vdst, n, shift, table, tiles);
        else
            hipLaunchKernelGGL(k_sort_scatter<false>, dim3((unsigned)tiles), dim3(kSortThreads), 0, s, ksrc, vsrc,
                               kdst, vdst, n, shift, table, tiles);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        ksrc = kdst;
        vsrc = vdst;
    }
    return hipSuccess;
}

}  // namespace dgn
