// Stable LSD radix sort of (int32 key, int32 value) pairs, 9 bits per pass, for the CSR builder.
//
// Per pass: (1) digit counts per tile of 8 192 keys, already summed inside groups of 16 tiles, and each group's totals;
// (2) a small scan over the groups' totals; (3) a scatter in which every wave ranks its keys against the keys of its
// lower lanes and earlier rounds (ballot "match" masks): keys of one tile are visited in their stored order, so
// equal keys keep their relative order.  The tile is sorted inside LDS first, so that it leaves in one run per digit.
// Only the significant key bits are sorted (ceil(log2(rows)) of them), so 50M operators (26 bits) or 100M
// tensors (27 bits) cost three passes.  (Eight bits per pass and four passes: 9 % slower on that graph; a pass
// with 512 digits costs more than one with 256, because a tile then leaves in runs half as long, but not a third more.)
//
// What a pass costs, per 110 M pairs on the 50 M-operator graph: counting 0.10 ms (the keys once, at the rate of a
// copy), the scan 0.015 ms, the scatter 0.51 ms = 3.4 TB/s of 16 bytes per pair.  The scatter's time went, in turn, to
// the write-back of half-written cache lines (fixed by giving each die a contiguous range of tiles), to one cache
// line per digit and tile for the slot table (fixed by the tile-major tables), and to the vector instructions of the
// ranking (halved by the three-input bit operation and longer tiles).
#include "common.h"

namespace dgn {

constexpr int kRadixBits = 9;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortThreads = 1024;                      // threads of a scattering workgroup; the first kRadix of them
                                                        // also keep the books of one digit each
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kDigitWaves = kRadix / kWave;
constexpr int kSortRounds = 8;                          // keys per lane
constexpr int kSortTile = kSortThreads * kSortRounds;   // keys per workgroup

__device__ __forceinline__ int digit_of(int32_t key, int shift) { return ((uint32_t)key >> shift) & (kRadix - 1); }

// The first output slot of a tile's keys with digit d is the number of keys that sort before them: all keys with a
// smaller digit, and the keys with digit d of earlier tiles.  It is kept in two tables, both tile-major (a row of
// kRadix words per tile or per group of tiles), so that the workgroup that counts a tile and the one that scatters it
// both touch one contiguous row -- a digit-major table costs the scatter one cache line per digit and tile, a fifth of
// all the cache lines it asks for:
//   table[tile][d]   keys with digit d in the earlier tiles of the tile's group of kHistTiles consecutive tiles,
//   totals[group][d] first the group's keys with digit d, then (k_col_*) the keys with a smaller digit anywhere plus
//                    those with digit d in earlier groups.
constexpr int kHistTiles = 16;
constexpr int kColChunks = 64;              // the groups are scanned in up to this many chunks of consecutive groups

__global__ __launch_bounds__(kRadix) void k_sort_hist(const int32_t *keys, int64_t n, int shift,
                                                             int32_t *table, int32_t *totals)
{
    __shared__ int hist[kHistTiles][kRadix];
#pragma unroll
    for (int t = 0; t < kHistTiles; ++t) hist[t][threadIdx.x] = 0;
    __syncthreads();
    const int64_t tile0 = (int64_t)blockIdx.x * kHistTiles;
    const bool wide = (reinterpret_cast<uintptr_t>(keys) & 15) == 0;
    constexpr int kPerThread = kSortTile / kRadix;           // keys of a tile that one thread counts
    static_assert(kPerThread % 4 == 0, "a thread counts whole 16-byte groups of keys");
    for (int t = 0; t < kHistTiles; ++t) {
        // the order inside a tile does not matter for its counts: a thread takes neighbouring keys
        const int64_t i = (tile0 + t) * kSortTile + (int64_t)threadIdx.x * kPerThread;
        if (i >= n) break;
        if (wide && i + kPerThread <= n) {
            int4 a[kPerThread / 4];
#pragma unroll
            for (int q = 0; q < kPerThread / 4; ++q) a[q] = *reinterpret_cast<const int4 *>(keys + i + 4 * q);
#pragma unroll
            for (int q = 0; q < kPerThread / 4; ++q) {
                atomicAdd(&hist[t][digit_of(a[q].x, shift)], 1);
                atomicAdd(&hist[t][digit_of(a[q].y, shift)], 1);
                atomicAdd(&hist[t][digit_of(a[q].z, shift)], 1);
                atomicAdd(&hist[t][digit_of(a[q].w, shift)], 1);
            }
        } else {
            for (int r = 0; r < kPerThread; ++r)
                if (i + r < n) atomicAdd(&hist[t][digit_of(keys[i + r], shift)], 1);
        }
    }
    __syncthreads();
    // the table has a row for each of the group's kHistTiles tiles, also past the last tile
    int32_t *row = table + tile0 * kRadix + threadIdx.x;
    int run = 0;
#pragma unroll
    for (int t = 0; t < kHistTiles; ++t) {
        row[t * kRadix] = run;
        run += hist[t][threadIdx.x];
    }
    totals[(int64_t)blockIdx.x * kRadix + threadIdx.x] = run;
}

// Exclusive scan of totals[group][d] in the order (d, group), in three small steps: per chunk of consecutive groups
// the sum of every column; one workgroup turns those into each chunk's start per column (the columns' totals scanned
// across the digits, plus the earlier chunks of the column); every chunk then walks down its rows.
// (every walk down a column asks for kColBatch rows at a time: one row per round trip would leave these small
// kernels waiting for memory most of their time)
constexpr int kColBatch = 8;

__global__ __launch_bounds__(kRadix) void k_col_sums(const int32_t *totals, int64_t groups, int per_chunk,
                                                            int32_t *chunk_sums)
{
    const int64_t g0 = (int64_t)blockIdx.x * per_chunk;
    const int rows = (int)min((int64_t)per_chunk, groups - g0);
    const int32_t *col = totals + g0 * kRadix + threadIdx.x;
    int sum = 0;
    for (int r = 0; r < rows; r += kColBatch) {
        int v[kColBatch];
#pragma unroll
        for (int j = 0; j < kColBatch; ++j) v[j] = r + j < rows ? col[(r + j) * kRadix] : 0;
#pragma unroll
        for (int j = 0; j < kColBatch; ++j) sum += v[j];
    }
    chunk_sums[blockIdx.x * kRadix + threadIdx.x] = sum;
}

__global__ __launch_bounds__(kRadix) void k_col_bases(int32_t *chunk_sums, int chunks)
{
    __shared__ int s_wtot[kDigitWaves];
    const int d = threadIdx.x, lane = lane_id(), wave = threadIdx.x >> 6;
    int v[kColChunks];                                       // the whole column, in registers
#pragma unroll
    for (int c = 0; c < kColChunks; ++c) v[c] = c < chunks ? chunk_sums[c * kRadix + d] : 0;
    int col = 0;
#pragma unroll
    for (int c = 0; c < kColChunks; ++c) col += v[c];
    const int incl = wave_incl_scan(col);
    if (lane == kWave - 1) s_wtot[wave] = incl;
    __syncthreads();
    int run = incl - col;                                    // keys with a smaller digit
#pragma unroll
    for (int w = 0; w < kDigitWaves; ++w)
        if (w < wave) run += s_wtot[w];
#pragma unroll
    for (int c = 0; c < kColChunks; ++c) {
        if (c < chunks) chunk_sums[c * kRadix + d] = run;
        run += v[c];
    }
}

__global__ __launch_bounds__(kRadix) void k_col_apply(int32_t *totals, int64_t groups, int per_chunk,
                                                             const int32_t *chunk_sums)
{
    const int64_t g0 = (int64_t)blockIdx.x * per_chunk;
    const int rows = (int)min((int64_t)per_chunk, groups - g0);
    int32_t *col = totals + g0 * kRadix + threadIdx.x;
    int run = chunk_sums[blockIdx.x * kRadix + threadIdx.x];
    for (int r = 0; r < rows; r += kColBatch) {
        int v[kColBatch];
#pragma unroll
        for (int j = 0; j < kColBatch; ++j) v[j] = r + j < rows ? col[(r + j) * kRadix] : 0;
#pragma unroll
        for (int j = 0; j < kColBatch; ++j) {
            if (r + j < rows) col[(r + j) * kRadix] = run;
            run += v[j];
        }
    }
}

// (eight waves per SIMD: two workgroups of 1 024 threads per CU, which caps the kernel at 64 vector registers)
template <bool kWriteKeys>
__global__ __launch_bounds__(kSortThreads) __attribute__((amdgpu_waves_per_eu(8, 8)))
void k_sort_scatter(const int32_t *keys, const int32_t *vals, int32_t *keys_out, int32_t *vals_out, int64_t n, int shift,
                    const int32_t *table, const int32_t *totals, int64_t num_tiles)
{
    // Workgroups go to the chip's eight dies in turn, each with a second-level cache of its own.  Neighbouring tiles
    // write neighbouring runs of the output (a run is shorter than a cache line), so a die takes a contiguous eighth
    // of the tiles and the two halves of a line meet in one cache.
    const int64_t per_die = (num_tiles + 7) >> 3;
    const int64_t tile = (int64_t)(blockIdx.x & 7) * per_die + (blockIdx.x >> 3);
    if (tile >= num_tiles) return;
    // first output slot of this tile's keys with digit threadIdx.x: asked for now, needed after the ranking
    const bool keeps_digit = threadIdx.x < kRadix;
    int32_t first_slot = 0;
    if (keeps_digit) first_slot = table[tile * kRadix + threadIdx.x] + totals[tile / kHistTiles * kRadix + threadIdx.x];
    // the per-wave digit counts are dead once every key knows its slot in the sorted tile: the tile takes their place
    __shared__ int32_t s_raw[2 * kSortTile];
    static_assert(kSortWaves * kRadix <= 2 * kSortTile, "the counts fit into the tile's storage");
    int (*wcount)[kRadix] = reinterpret_cast<int (*)[kRadix]>(s_raw);
    int32_t *s_keys = s_raw, *s_vals = s_raw + kSortTile;
    __shared__ int s_delta[kRadix];          // global slot of a key = its slot in the locally sorted tile + this
    __shared__ int s_wtot[kDigitWaves];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < kSortWaves * kRadix; i += kSortThreads) (&wcount[0][0])[i] = 0;
    __syncthreads();

    // wave w owns kSortRounds * 64 consecutive keys of the tile, visited 64 at a time
    const int64_t tbase = tile * kSortTile;
    const int count = (int)min((int64_t)kSortTile, n - tbase);          // keys of this tile
    const int32_t *tile_keys = keys + tbase, *tile_vals = vals + tbase;
    const int wofs = wave * (kSortRounds * kWave) + lane;
    int32_t key[kSortRounds], val[kSortRounds];
    int rank[kSortRounds];
    const u64 lt = lanemask_lt();
    const uint32_t lt_lo = (uint32_t)lt, lt_hi = (uint32_t)(lt >> 32);
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int i = wofs + r * kWave;
        const bool valid = i < count;
        key[r] = valid ? tile_keys[i] : 0;
        val[r] = valid ? tile_vals[i] : 0;
        const int d = digit_of(key[r], shift);
        // others = the lanes whose digit differs from this lane's in some bit (or that hold no key).  For bit b, m =
        // the lanes that have it set and e = this lane's own bit spread over a word: m ^ e marks the lanes that
        // differ in b.  Kept as two 32-bit halves and as the complement of the usual "peers" mask, this is four
        // vector instructions per bit; the kernel's time is mostly vector instructions, and most of them are these.
        const u64 held = ballot64(valid);
        uint32_t others_lo = ~(uint32_t)held, others_hi = ~(uint32_t)(held >> 32);
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            int32_t e = __builtin_amdgcn_sbfe(d, b, 1);                 // -1 if bit b of d is set, else 0
            asm("" : "+v"(e));                                          // (compare e itself, not d shifted once more)
            const u64 m = ballot64(e != 0);
            others_lo = or_of_xor(others_lo, (uint32_t)m, (uint32_t)e);
            others_hi = or_of_xor(others_hi, (uint32_t)(m >> 32), (uint32_t)e);
        }
        // lanes with the same digit read the running count, then their first lane bumps it
        const int c = wcount[wave][d];
        const int before = lane - (__popc(others_lo & lt_lo) + __popc(others_hi & lt_hi));
        const int same = kWave - (__popc(others_lo) + __popc(others_hi));
        __builtin_amdgcn_wave_barrier();
        if (valid && before == 0) wcount[wave][d] = c + same;
        __builtin_amdgcn_wave_barrier();
        rank[r] = c + before;
    }
    __syncthreads();
    {   // digit d (one per thread): per-wave counts -> first slot of each wave's keys in the locally sorted tile
        const int d = threadIdx.x;
        int cnt = 0, incl = 0;
        if (keeps_digit) {
#pragma unroll
            for (int w = 0; w < kSortWaves; ++w) cnt += wcount[w][d];
            incl = wave_incl_scan(cnt);
            if (lane == kWave - 1) s_wtot[wave] = incl;
        }
        __syncthreads();
        if (keeps_digit) {
            int lbase = incl - cnt;
#pragma unroll
            for (int w = 0; w < kDigitWaves; ++w)
                if (w < wave) lbase += s_wtot[w];
            s_delta[d] = first_slot - lbase;
            int run = lbase;
#pragma unroll
            for (int w = 0; w < kSortWaves; ++w) {
                const int c = wcount[w][d];
                wcount[w][d] = run;
                run += c;
            }
        }
    }
    __syncthreads();
    // sort the tile inside LDS, so that the global writes below go out in long contiguous runs per digit
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) rank[r] += wcount[wave][digit_of(key[r], shift)];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        if (wofs + r * kWave < count) {
            s_keys[rank[r]] = key[r];
            s_vals[rank[r]] = val[r];
        }
    }
    __syncthreads();
    for (int li = threadIdx.x; li < count; li += kSortThreads) {
        const int32_t k = s_keys[li];
        const int pos = li + s_delta[digit_of(k, shift)];
        if (kWriteKeys) keys_out[pos] = k;
        vals_out[pos] = s_vals[li];
    }
}

static inline int64_t sort_tiles(int64_t n) { return (n + kSortTile - 1) / kSortTile; }
static inline int64_t sort_groups(int64_t tiles) { return (tiles + kHistTiles - 1) / kHistTiles; }

// layout of tmp: keyA[n] valA[n] keyB[n] valB[n] table[groups*kHistTiles][kRadix] totals[groups][kRadix]
// chunk_sums[kColChunks][kRadix]
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t sort_tmp_bytes(int64_t n)
{
    const int64_t groups = sort_groups(sort_tiles(n));
    return 4 * align256((size_t)n * 4) + align256((size_t)(groups * kHistTiles * kRadix) * 4) +
           align256((size_t)(groups * kRadix) * 4) + align256((size_t)kColChunks * kRadix * 4);
}

hipError_t launch_sort_pairs(const int32_t *keys_in, const int32_t *vals_in, int32_t *keys_out,
                             int32_t *vals_out, int64_t n, int key_bits, void *tmp, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const int64_t tiles = sort_tiles(n), groups = sort_groups(tiles);
    const int per_chunk = (int)((groups + kColChunks - 1) / kColChunks);
    const int chunks = (int)((groups + per_chunk - 1) / per_chunk);
    const unsigned scatter_grid = (unsigned)(((tiles + 7) >> 3) << 3);
    char *p = static_cast<char *>(tmp);
    int32_t *kbuf[2], *vbuf[2];
    kbuf[0] = reinterpret_cast<int32_t *>(p); p += align256((size_t)n * 4);
    vbuf[0] = reinterpret_cast<int32_t *>(p); p += align256((size_t)n * 4);
    kbuf[1] = reinterpret_cast<int32_t *>(p); p += align256((size_t)n * 4);
    vbuf[1] = reinterpret_cast<int32_t *>(p); p += align256((size_t)n * 4);
    int32_t *table = reinterpret_cast<int32_t *>(p); p += align256((size_t)(groups * kHistTiles * kRadix) * 4);
    int32_t *totals = reinterpret_cast<int32_t *>(p); p += align256((size_t)(groups * kRadix) * 4);
    int32_t *chunk_sums = reinterpret_cast<int32_t *>(p);

    if (key_bits < 1) key_bits = 1;
    const int passes = (key_bits + kRadixBits - 1) / kRadixBits;
    const int32_t *ksrc = keys_in, *vsrc = vals_in;
    for (int pass = 0; pass < passes; ++pass) {
        const bool last = pass == passes - 1;
        const int shift = pass * kRadixBits;
        int32_t *kdst = last ? keys_out : kbuf[pass & 1];
        int32_t *vdst = last ? vals_out : vbuf[pass & 1];
        hipLaunchKernelGGL(k_sort_hist, dim3((unsigned)groups), dim3(kRadix), 0, s, ksrc, n, shift, table, totals);
        hipLaunchKernelGGL(k_col_sums, dim3(chunks), dim3(kRadix), 0, s, totals, groups, per_chunk, chunk_sums);
        hipLaunchKernelGGL(k_col_bases, dim3(1), dim3(kRadix), 0, s, chunk_sums, chunks);
        hipLaunchKernelGGL(k_col_apply, dim3(chunks), dim3(kRadix), 0, s, totals, groups, per_chunk, chunk_sums);
        if (kdst)
            hipLaunchKernelGGL(k_sort_scatter<true>, dim3(scatter_grid), dim3(kSortThreads), 0, s, ksrc, vsrc,
                               kdst, vdst, n, shift, table, totals, tiles);
        else
            hipLaunchKernelGGL(k_sort_scatter<false>, dim3(scatter_grid), dim3(kSortThreads), 0, s, ksrc, vsrc,
                               kdst, vdst, n, shift, table, totals, tiles);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        ksrc = kdst;
        vsrc = vdst;
    }
    return hipSuccess;
}

}  // namespace dgn
