// Removal rule and ordered compaction.
//   - Sec. 2.1 of the paper: an operator whose outputs are all un-coloured is removed, i.e. operator o
//     is kept for set q iff bit q of K[o] = OR_{u in out(o)} M[u] is set;
//   - Sec. 3.2: surviving operators keep their creation order, so the kept list is the ascending
//     list of operator ids with K != 0.
// Three streaming passes, none of which waits on another workgroup:
//   count   : K (read, or computed from M and written), flags, one bit per operator into `opbits`,
//             per-tile kept counts, per-set counts;
//   scan    : exclusive prefix of the tile counts (one workgroup), total -> kept_count[0];
//   scatter : ranks from `opbits` by popcount, K gathered only for kept operators.
#include "common.h"

namespace dgn {

constexpr int kCThreads = 256;
constexpr int kCWaves = kCThreads / kWave;
constexpr int kCRounds = kCompactTile / kCThreads;   // 8 operators per lane
constexpr int kCWords = kCompactTile / kWave;        // 32 bitmap words per tile

__device__ __forceinline__ int graph_of(const int64_t *off, int num_graphs, int64_t id)
{
    int lo = 0, hi = num_graphs;          // largest g with off[g] <= id
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= id) lo = mid; else hi = mid;
    }
    return lo;
}

template <bool kFromM>
__global__ __launch_bounds__(kCThreads) void k_keep_count(CompactArgs a)
{
    __shared__ int s_wcount[kCWaves];
    const GraphView &g = a.g;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t tile_base = (int64_t)blockIdx.x * kCompactTile;
    const bool batched = g.num_graphs > 1;

    // Per-set counters are hot words (every wave of the grid adds to the same 64 of them when there is
    // one graph), so waves add into one of pq_replicas private copies that a tiny kernel sums up later.
    int64_t *pq = a.per_query_count;
    int pqs = 1;                  // replica counters sit 64 bytes apart (no two hot words in one line half)
    if (pq && a.pq_part) {
        pqs = kPqStride;
        pq = a.pq_part + (int64_t)((blockIdx.x * kCWaves + wave) & (a.pq_replicas - 1)) * 64 * g.num_graphs * kPqStride;
    }

    int kept = 0;                 // wave-uniform
    u64 qcount = 0;               // lane q: operators of the current graph whose K has bit q
    int cur_graph = 0;
    int64_t g_lo = 0, g_hi = g.num_ops;
    if (batched) {
        cur_graph = graph_of(g.op_off, g.num_graphs, tile_base < g.num_ops ? tile_base : g.num_ops - 1);
        g_lo = g.op_off[cur_graph];
        g_hi = g.op_off[cur_graph + 1];
    }

    // all loads of the tile are issued before anything is consumed (8 independent loads per lane)
    u64 kk[kCRounds];
#pragma unroll
    for (int r = 0; r < kCRounds; ++r) {
        const int64_t o = tile_base + (int64_t)r * kCThreads + threadIdx.x;
        kk[r] = 0;
        if (o < g.num_ops) {
            if (kFromM) {
                const int32_t b = g.out_rowptr[o], e = g.out_rowptr[o + 1];
                u64 k = 0;
                for (int32_t j = b; j < e; ++j) k |= a.M[g.out_idx[j]];
                kk[r] = k;
            } else {
                kk[r] = a.K[o];
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kCRounds; ++r) {
        const int64_t o0 = tile_base + (int64_t)r * kCThreads + wave * kWave;   // first operator of this wave-round
        const int64_t o = o0 + lane;
        const bool valid = o < g.num_ops;
        const u64 k = kk[r];
        if (valid) {
            if (kFromM) a.K[o] = k;
            if (a.op_flag) a.op_flag[o] = (uint8_t)(k != 0);
        }
        const u64 word = ballot64(k != 0);
        if (lane == 0 && o0 < g.num_ops) a.opbits[o0 >> 6] = word;
        kept += __popcll(word);

        if (pq && word) {
            const int64_t o_last = min(o0 + kWave, (int64_t)g.num_ops) - 1;
            if (batched && (o0 < g_lo || o_last >= g_hi)) {
                // this wave-round leaves the current graph: flush, then either move on or go lane by lane
                if (qcount) atomicAdd((u64 *)&pq[((int64_t)cur_graph * 64 + lane) * pqs], qcount);
                qcount = 0;
                const int ga = graph_of(g.op_off, g.num_graphs, o0);
                const int gb = graph_of(g.op_off, g.num_graphs, o_last);
                if (ga == gb) {
                    cur_graph = ga;
                    g_lo = g.op_off[ga];
                    g_hi = g.op_off[ga + 1];
                } else {
                    if (valid && k) {
                        const int gi = graph_of(g.op_off, g.num_graphs, o);
                        u64 kk = k;
                        while (kk) {
                            const int q = __builtin_ctzll(kk);
                            kk &= kk - 1;
                            atomicAdd((u64 *)&pq[((int64_t)gi * 64 + q) * pqs], (u64)1);
                        }
                    }
                    continue;      // wave-uniform: every lane of the round takes this path
                }
            }
            u64 any = wave_or(k);
            if (__popcll(any) > 6) {
                // many sets present: transpose the 64x64 bit matrix, lane q then holds column q
                qcount += (u64)__popcll(wave_transpose64(k));
            } else {
                while (any) {                               // wave-uniform loop over the few sets present
                    const int q = __builtin_ctzll(any);
                    any &= any - 1;
                    const int c = __popcll(ballot64((k >> q) & 1));
                    if (lane == q) qcount += (u64)c;
                }
            }
        }
    }
    if (pq && qcount) atomicAdd((u64 *)&pq[((int64_t)cur_graph * 64 + lane) * pqs], qcount);

    if (lane == 0) s_wcount[wave] = kept;
    __syncthreads();
    if (threadIdx.x == 0) {
        int tot = 0;
#pragma unroll
        for (int w = 0; w < kCWaves; ++w) tot += s_wcount[w];
        a.block_counts[blockIdx.x] = tot;
    }
}

// per_query_count[i] = sum over the replicas of pq_part[r][i]: one wave per output, one lane per replica
__global__ __launch_bounds__(256) void k_reduce_pq(CompactArgs a)
{
    const int n = 64 * a.g.num_graphs;
    const int i = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6);
    if (i >= n) return;
    const int lane = lane_id();
    long long v = 0;
    if (lane < a.pq_replicas) v = a.pq_part[((int64_t)lane * n + i) * kPqStride];
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    if (lane == 0) a.per_query_count[i] = v;
}

// Single workgroup: exclusive scan of the tile counts in place, total -> counts[m] and kept_count[0].
// 4096 entries per round (four consecutive ones per thread).
__global__ __launch_bounds__(1024) void k_scan_tiles(int32_t *counts, int64_t m, int64_t *kept_count)
{
    __shared__ int wtot[2][16];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    int carry = 0, buf = 0;
    for (int64_t base = 0; base < m; base += 4096, buf ^= 1) {
        const int64_t i = base + (int64_t)threadIdx.x * 4;
        int x[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) x[c] = i + c < m ? counts[i + c] : 0;
        const int sum = x[0] + x[1] + x[2] + x[3];
        const int incl = wave_incl_scan(sum);
        if (lane == kWave - 1) wtot[buf][wave] = incl;
        __syncthreads();                      // double-buffered totals: one barrier per round is enough
        int woff = 0, tot = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int c = wtot[buf][w];
            if (w < wave) woff += c;
            tot += c;
        }
        int run = carry + woff + incl - sum;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (i + c < m) counts[i + c] = run;
            run += x[c];
        }
        carry += tot;
    }
    if (threadIdx.x == 0) {
        counts[m] = carry;
        kept_count[0] = carry;
    }
}

__global__ __launch_bounds__(kCThreads) void k_scatter(CompactArgs a)
{
    __shared__ int s_off[kCWords];
    const GraphView &g = a.g;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t tile_base = (int64_t)blockIdx.x * kCompactTile;
    const int64_t n_words = ((int64_t)g.num_ops + 63) >> 6;
    const int64_t word_base = tile_base >> 6;
    const int base = a.block_counts[blockIdx.x];
    if (a.block_counts[blockIdx.x + 1] == base) return;     // nothing kept in this tile (uniform)

    // exclusive prefix of the popcounts of this tile's 32 bitmap words (wave 0)
    if (wave == 0) {
        u64 w = 0;
        if (lane < kCWords && word_base + lane < n_words) w = a.opbits[word_base + lane];
        const int c = __popcll(w);
        const int incl = wave_incl_scan(c);
        if (lane < kCWords) s_off[lane] = incl - c;
    }
    __syncthreads();
    for (int r = 0; r < kCRounds; ++r) {
        const int wi = r * kCWaves + wave;                  // word index inside the tile
        if (word_base + wi >= n_words) break;               // wave-uniform
        const u64 word = a.opbits[word_base + wi];
        if ((word >> lane) & 1) {
            const int64_t o = tile_base + (int64_t)wi * kWave + lane;
            const int pos = base + s_off[wi] + __popcll(word & lanemask_lt());
            a.kept_ops[pos] = (int32_t)o;
            if (a.kept_masks) a.kept_masks[pos] = a.K[o];
        }
    }
}

// kept_count[1 + g] = number of kept operators with id < op_off[g], g = 0..G
__global__ __launch_bounds__(256) void k_graph_offsets(CompactArgs a)
{
    const GraphView &g = a.g;
    const int gi = blockIdx.x * blockDim.x + threadIdx.x;
    if (gi > g.num_graphs) return;
    const int64_t o = g.op_off[gi];
    if (o >= g.num_ops) { a.kept_count[1 + gi] = a.block_counts[((int64_t)g.num_ops + kCompactTile - 1) / kCompactTile]; return; }
    const int64_t tile = o / kCompactTile;
    int64_t c = a.block_counts[tile];
    const int64_t w0 = tile * kCWords, w1 = o >> 6;
    for (int64_t w = w0; w < w1; ++w) c += __popcll(a.opbits[w]);
    if (o & 63) c += __popcll(a.opbits[w1] & (((u64)1 << (o & 63)) - 1));
    a.kept_count[1 + gi] = c;
}

hipError_t launch_keep_compact(const CompactArgs &a, hipStream_t s, hipEvent_t *ev)
{
    const int64_t P = a.g.num_ops;
    const int64_t tiles = (P + kCompactTile - 1) / kCompactTile;
    if (tiles > 0) {
        if (a.from_tensor_mask)
            hipLaunchKernelGGL(k_keep_count<true>, dim3((unsigned)tiles), dim3(kCThreads), 0, s, a);
        else
            hipLaunchKernelGGL(k_keep_count<false>, dim3((unsigned)tiles), dim3(kCThreads), 0, s, a);
    }
    if (a.per_query_count && a.pq_part)
        hipLaunchKernelGGL(k_reduce_pq, dim3((unsigned)((64 * a.g.num_graphs + 3) / 4)), dim3(256), 0, s, a);
    if (ev) (void)hipEventRecord(ev[0], s);
    hipLaunchKernelGGL(k_scan_tiles, dim3(1), dim3(1024), 0, s, a.block_counts, tiles, a.kept_count);
    if (ev) (void)hipEventRecord(ev[1], s);
    if (tiles > 0) hipLaunchKernelGGL(k_scatter, dim3((unsigned)tiles), dim3(kCThreads), 0, s, a);
    if (a.g.num_graphs > 1)
        hipLaunchKernelGGL(k_graph_offsets, dim3((unsigned)((a.g.num_graphs + 1 + 255) / 256)), dim3(256), 0, s, a);
    if (ev) (void)hipEventRecord(ev[2], s);
    return hipGetLastError();
}

}  // namespace dgn
