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
constexpr int kCountGrid = 2048;                      // workgroups of the count pass (8 per compute unit)
constexpr int kTransposeAbove = 16;                  // kept operators per 64 above which per-set counting transposes

__device__ __forceinline__ int graph_of(const int64_t *off, int num_graphs, int64_t id)
{
    int lo = 0, hi = num_graphs;          // largest g with off[g] <= id
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= id) lo = mid; else hi = mid;
    }
    return lo;
}

// kFromM: K is computed from M and written.  Otherwise K is read: all of it, or (kFlags) only where the byte the
// traversal sets when an operator first receives bits says that it is not zero -- P bytes instead of 8P.
template <bool kFromM, bool kFlags>
__global__ __launch_bounds__(kCThreads) void k_keep_count(CompactArgs a)
{
    __shared__ int s_wcount[2][kCWaves];
    __shared__ uint32_t s_q[kCWaves][kWave];
    const GraphView &g = a.g;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const bool batched = g.num_graphs > 1;
    const int64_t tiles = ((int64_t)g.num_ops + kCompactTile - 1) / kCompactTile;

    // Per-set counters are hot words, so a workgroup walks over many tiles with the counts in
    // registers and adds them, once, into one of pq_replicas private copies that a tiny kernel sums up.
    int64_t *pq = a.per_query_count;
    int pqs = 1;                  // replica counters sit 64 bytes apart (no two hot words in one line half)
    if (pq && a.pq_part) {
        pqs = kPqStride;
        const int user = batched ? blockIdx.x * kCWaves + wave : blockIdx.x;    // who adds: a wave, or the workgroup
        pq = a.pq_part + (int64_t)(user & (a.pq_replicas - 1)) * 64 * g.num_graphs * kPqStride;
    }

    uint32_t qcount = 0;          // lane q: operators of the current graph whose K has bit q
    int cur_graph = 0;
    int64_t g_lo = 0, g_hi = g.num_ops;
    if (batched) {
        const int64_t tile_base = (int64_t)blockIdx.x * kCompactTile;
        cur_graph = graph_of(g.op_off, g.num_graphs, tile_base < g.num_ops ? tile_base : g.num_ops - 1);
        g_lo = g.op_off[cur_graph];
        g_hi = g.op_off[cur_graph + 1];
    }

    int buf = 0;
    for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x, buf ^= 1) {
        // a wave owns 512 consecutive operators, 64 per round; all loads of the tile are issued before
        // anything is consumed (8 independent loads per lane)
        const int64_t wave_base = tile * kCompactTile + (int64_t)wave * (kCRounds * kWave);
        int kept = 0;                 // wave-uniform
        u64 kk[kCRounds];
        uint8_t fl[kCRounds] = {};
        if (kFlags) {
#pragma unroll
            for (int r = 0; r < kCRounds; ++r) {
                const int64_t o = wave_base + r * kWave + lane;
                fl[r] = o < g.num_ops ? a.flag_in[o] : 0;
            }
        }
#pragma unroll
        for (int r = 0; r < kCRounds; ++r) {
            const int64_t o = wave_base + r * kWave + lane;
            kk[r] = 0;
            if (kFlags) {
                if (fl[r]) kk[r] = a.K[o];
            } else if (o < g.num_ops) {
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
        u64 bword = 0;                // lane r < 8: bitmap word of round r
        u64 fword = 0;                // lane l: bitmap word of round l / 8, the one holding operators 8l .. 8l+7
#pragma unroll
        for (int r = 0; r < kCRounds; ++r) {
            const int64_t o0 = wave_base + r * kWave;            // first operator of this wave-round
            const int64_t o = o0 + lane;
            const bool valid = o < g.num_ops;
            const u64 k = kk[r];
            if (kFromM && valid) a.K[o] = k;
            const u64 word = ballot64(k != 0);
            if (lane == r) bword = word;
            if ((lane >> 3) == r) fword = word;
            kept += __popcll(word);

            if (pq && word) {
                const int64_t o_last = min(o0 + kWave, (int64_t)g.num_ops) - 1;
                if (batched && (o0 < g_lo || o_last >= g_hi)) {
                    // this wave-round leaves the current graph: flush, then either move on or go lane by lane
                    if (qcount) atomicAdd((u64 *)&pq[((int64_t)cur_graph * 64 + lane) * pqs], (u64)qcount);
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
                            u64 rest = k;
                            while (rest) {
                                const int q = __builtin_ctzll(rest);
                                rest &= rest - 1;
                                atomicAdd((u64 *)&pq[((int64_t)gi * 64 + q) * pqs], (u64)1);
                            }
                        }
                        continue;      // wave-uniform: every lane of the round takes this path
                    }
                }
                if (__popcll(word) > kTransposeAbove) {
                    // many operators kept: transpose the 64x64 bit matrix, lane q then holds column q
                    qcount += (uint32_t)__popcll(wave_transpose64(k));
                } else {
                    // few kept: broadcast each kept operator's mask, lane q picks its bit out of it
                    u64 rest = word;
                    while (rest) {                              // wave-uniform
                        const int l = __builtin_ctzll(rest);
                        rest &= rest - 1;
                        const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)k, l);
                        const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(k >> 32), l);
                        qcount += (uint32_t)(((((u64)hi << 32) | lo) >> lane) & 1);
                    }
                }
            }
        }
        if (lane < kCRounds && wave_base + lane * kWave < g.num_ops) a.opbits[(wave_base >> 6) + lane] = bword;
        if (a.op_flag && !(kFlags && a.op_flag == a.flag_in)) {
            // bits 8(l%8) .. 8(l%8)+7 of fword -> eight 0/1 bytes, one 8-byte store per lane
            const u64 b = (fword >> ((lane & 7) * 8)) & 0xff;
            u64 bytes = (b * 0x0101010101010101ull) & 0x8040201008040201ull;
            bytes = ((bytes + 0x7f7f7f7f7f7f7f7full) >> 7) & 0x0101010101010101ull;
            const int64_t o = wave_base + 8 * lane;
            uint8_t *dst = a.op_flag + o;
            if (o + 8 <= g.num_ops && ((uintptr_t)a.op_flag & 7) == 0) {
                *reinterpret_cast<u64 *>(dst) = bytes;
            } else {
                for (int i = 0; i < 8; ++i)
                    if (o + i < g.num_ops) dst[i] = (uint8_t)(bytes >> (8 * i));
            }
        }

        // tile total; the totals are double-buffered, so one barrier per tile is enough
        if (lane == 0) s_wcount[buf][wave] = kept;
        __syncthreads();
        if (threadIdx.x == 0) {
            int tot = 0;
#pragma unroll
            for (int w = 0; w < kCWaves; ++w) tot += s_wcount[buf][w];
            a.block_counts[tile] = tot;
        }
    }

    if (!pq) return;
    if (batched) {                // waves may be in different graphs
        if (qcount) atomicAdd((u64 *)&pq[((int64_t)cur_graph * 64 + lane) * pqs], (u64)qcount);
        return;
    }
    s_q[wave][lane] = qcount;
    __syncthreads();
    if (wave == 0) {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < kCWaves; ++w) c += s_q[w][lane];
        if (c) atomicAdd((u64 *)&pq[(int64_t)lane * pqs], (u64)c);
    }
}

// Count pass of a single graph whose keep flags the traversal has already written (a byte per operator, 1 where
// K != 0; they are the caller's op_flag or stand in for it).  A wave takes a whole tile: 2048 flag bytes in four
// 8-byte loads per lane, squeezed to the tile's 32 bitmap words and its kept count without touching K.  The ids
// of the kept operators go through a small list in LDS, and K is read for 64 of them at a time for the per-set
// counts -- about P/8 + 8 P_kept bytes of traffic instead of 9P, and no barrier anywhere.
constexpr int kPendCap = 128;
constexpr int64_t kFlagsCountGrid = 8192;
// Below this many operators all of K is a few microseconds of reading, and the kernel that reads it is the
// faster one where most operators are kept (it needs no list of kept ids).
constexpr int64_t kFlagsCountMinOps = (int64_t)1 << 22;

__device__ __forceinline__ uint32_t count_pending(const CompactArgs &a, const int32_t *ids, int n)
{
    const int lane = lane_id();
    const u64 k = lane < n ? a.K[ids[lane]] : 0;
    if (n > kTransposeAbove) return (uint32_t)__popcll(wave_transpose64(k));   // lane q: column q of the bit matrix
    uint32_t c = 0;
    for (int l = 0; l < n; ++l) {                                               // wave-uniform
        const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)k, l);
        const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(k >> 32), l);
        c += (uint32_t)(((((u64)hi << 32) | lo) >> lane) & 1);
    }
    return c;
}

__global__ __launch_bounds__(kCThreads) void k_keep_count_flags(CompactArgs a)
{
    __shared__ int32_t s_ids[kCWaves][kPendCap];
    __shared__ uint32_t s_q[kCWaves][kWave];
    const GraphView &g = a.g;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t tiles = ((int64_t)g.num_ops + kCompactTile - 1) / kCompactTile;
    const int64_t n_words = ((int64_t)g.num_ops + 63) >> 6;
    const bool want_pq = a.per_query_count != nullptr;
    int32_t *ids = &s_ids[wave][0];
    int npend = 0;                // wave-uniform
    uint32_t qcount = 0;          // lane q: kept operators whose K has bit q
    for (int64_t tile = (int64_t)blockIdx.x * kCWaves + wave; tile < tiles; tile += (int64_t)gridDim.x * kCWaves) {
        const int64_t base = tile * kCompactTile;
        u64 f[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t o = base + j * 512 + lane * 8;      // this lane's eight operators of stretch j
            f[j] = o < g.num_ops ? *reinterpret_cast<const u64 *>(a.flag_in + o) : 0;
        }
        int kept = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // bytes are 0 or 1: bit 0 of each into one byte
            const uint32_t b = (uint32_t)(((f[j] & 0x0101010101010101ull) * 0x0102040810204080ull) >> 56);
            kept += __popc(b);
            // eight neighbouring lanes hold one bitmap word
            u64 w = (u64)b << (8 * (lane & 7));
            w |= shfl_xor64(w, 1);
            w |= shfl_xor64(w, 2);
            w |= shfl_xor64(w, 4);
            const int64_t wi = (base >> 6) + j * 8 + (lane >> 3);
            if ((lane & 7) == 0 && wi < n_words) a.opbits[wi] = w;
            if (want_pq && ballot64(b != 0)) {
                const int32_t o0 = (int32_t)(base + j * 512 + lane * 8);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const bool has = (b >> i) & 1;
                    const u64 m = ballot64(has);
                    if (!m) continue;                           // wave-uniform
                    if (has) ids[npend + __popcll(m & lanemask_lt())] = o0 + i;
                    npend += __popcll(m);
                    if (npend >= kWave) {
                        __builtin_amdgcn_wave_barrier();
                        qcount += count_pending(a, ids, kWave);
                        const int32_t rest = lane + kWave < npend ? ids[lane + kWave] : 0;
                        __builtin_amdgcn_wave_barrier();
                        ids[lane] = rest;
                        npend -= kWave;
                    }
                }
            }
        }
        kept = wave_sum(kept);
        if (lane == 0) a.block_counts[tile] = kept;
    }
    if (!want_pq) return;
    __builtin_amdgcn_wave_barrier();
    if (npend > 0) qcount += count_pending(a, ids, npend);
    // one add per workgroup and set into one of the replicated counters
    int64_t *pq = a.per_query_count;
    int pqs = 1;
    if (a.pq_part) {
        pqs = kPqStride;
        pq = a.pq_part + (int64_t)(blockIdx.x & (a.pq_replicas - 1)) * 64 * kPqStride;
    }
    s_q[wave][lane] = qcount;
    __syncthreads();
    if (wave == 0) {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < kCWaves; ++w) c += s_q[w][lane];
        if (c) atomicAdd((u64 *)&pq[(int64_t)lane * pqs], (u64)c);
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

constexpr int kScanVecs = 16;             // int4 per thread that the tile scan keeps in registers
constexpr int kFoldPqOutputs = 256;      // up to this many per-set counters are summed by the scan kernel itself

// Single workgroup: exclusive scan of the tile counts in place, total -> counts[m] and kept_count[0].
// Every thread owns one contiguous run of counts: it sums the run, the block scans the 1024 sums, the thread
// walks its run again and writes the prefixes -- two rounds of independent loads whatever m is.  With few
// per-set counters the kernel also sums their replicas (one wave per counter), which saves a launch.
__global__ __launch_bounds__(1024) void k_scan_tiles(int32_t *counts, int64_t m, int64_t *kept_count, CompactArgs a,
                                                     bool fold_pq)
{
    __shared__ int wtot[16];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    if (fold_pq) {
        const int n = 64 * a.g.num_graphs;
        for (int i0 = wave; i0 < n; i0 += 64) {          // four counters per wave and step, their loads in flight together
            long long v[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int i = i0 + 16 * c;
                v[c] = (i < n && lane < a.pq_replicas) ? a.pq_part[((int64_t)lane * n + i) * kPqStride] : 0;
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
#pragma unroll
                for (int d = kWave / 2; d >= 1; d >>= 1) v[c] += __shfl_xor(v[c], d, kWave);
                if (lane == 0 && i0 + 16 * c < n) a.per_query_count[i0 + 16 * c] = v[c];
            }
        }
    }
    // runs are a multiple of four counts long and start 16-byte aligned.  Up to kScanVecs int4 per thread (tile
    // counts of 134 million operators) stay in registers between the two passes: all loads in flight at once, one
    // trip to memory in all; longer runs are read twice.
    const int64_t per = (((m + 1023) / 1024) + 3) & ~(int64_t)3;
    const int64_t lo = (int64_t)threadIdx.x * per;
    const int64_t hi = lo + per < m ? lo + per : m;
    const bool in_regs = per <= 4 * kScanVecs;
    int4 v[kScanVecs];
    int sum = 0;
    if (in_regs) {
#pragma unroll
        for (int j = 0; j < kScanVecs; ++j) {
            const int64_t i = lo + 4 * j;
            v[j] = make_int4(0, 0, 0, 0);
            if (i + 4 <= hi) {
                v[j] = *reinterpret_cast<const int4 *>(counts + i);
            } else if (i < hi) {                         // the ragged end of the array: one by one
                v[j].x = counts[i];
                if (i + 1 < hi) v[j].y = counts[i + 1];
                if (i + 2 < hi) v[j].z = counts[i + 2];
            }
        }
#pragma unroll
        for (int j = 0; j < kScanVecs; ++j) sum += v[j].x + v[j].y + v[j].z + v[j].w;
    } else {
        for (int64_t i = lo; i < hi; ++i) sum += counts[i];
    }
    const int incl = wave_incl_scan(sum);
    if (lane == kWave - 1) wtot[wave] = incl;
    __syncthreads();
    int woff = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const int c = wtot[w];
        if (w < wave) woff += c;
        tot += c;
    }
    int run = woff + incl - sum;
    if (in_regs) {
#pragma unroll
        for (int j = 0; j < kScanVecs; ++j) {
            const int64_t i = lo + 4 * j;
            const int4 o = make_int4(run, run + v[j].x, run + v[j].x + v[j].y, run + v[j].x + v[j].y + v[j].z);
            run += v[j].x + v[j].y + v[j].z + v[j].w;
            if (i + 4 <= hi) {
                *reinterpret_cast<int4 *>(counts + i) = o;
            } else if (i < hi) {
                counts[i] = o.x;
                if (i + 1 < hi) counts[i + 1] = o.y;
                if (i + 2 < hi) counts[i + 2] = o.z;
            }
        }
    } else {
        for (int64_t i = lo; i < hi; ++i) {
            const int c = counts[i];
            counts[i] = run;
            run += c;
        }
    }
    if (threadIdx.x == 0) {
        counts[m] = tot;
        kept_count[0] = tot;
    }
}

// A wave takes a tile.  With few kept operators in it (the usual case on a large pruned graph: a few dozen of
// 2 048) lane w < 32 walks the set bits of bitmap word w; with many, the 64 lanes take one word at a time, lane =
// bit.  No shared memory, no barrier; a tile with nothing kept costs two loads.
constexpr int kScatterByBitsBelow = 192;
constexpr int64_t kScatterByWaveAboveTiles = 16384;     // 33 million operators

__global__ __launch_bounds__(kCThreads) void k_scatter(CompactArgs a)
{
    const GraphView &g = a.g;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    // last pass of a prune: say in the scratch buffer which buffers now hold a result with a complete log
    if (a.hdr && blockIdx.x == 0 && threadIdx.x == 0 && *a.error == 0) *a.hdr = a.want;
    const int64_t tiles = ((int64_t)g.num_ops + kCompactTile - 1) / kCompactTile;
    const int64_t tile = (int64_t)blockIdx.x * kCWaves + wave;
    if (tile >= tiles) return;
    const int64_t tile_base = tile * kCompactTile;
    const int64_t n_words = ((int64_t)g.num_ops + 63) >> 6;
    const int64_t word_base = tile_base >> 6;
    const int base = a.block_counts[tile];
    const int kept = a.block_counts[tile + 1] - base;
    if (kept == 0) return;                                  // wave-uniform

    // exclusive prefix of the popcounts of the tile's 32 bitmap words
    u64 w = 0;
    if (lane < kCWords && word_base + lane < n_words) w = a.opbits[word_base + lane];
    const int c = __popcll(w);
    const int off = wave_incl_scan(c) - c;
    if (kept < kScatterByBitsBelow) {
        int pos = base + off;
        while (w) {
            const int b = __builtin_ctzll(w);
            w &= w - 1;
            const int64_t o = tile_base + (int64_t)lane * kWave + b;
            a.kept_ops[pos] = (int32_t)o;
            if (a.kept_masks) a.kept_masks[pos] = a.K[o];
            ++pos;
        }
    } else {
        for (int wi = 0; wi < kCWords; ++wi) {
            const u64 word = shfl64(w, wi);
            const int woff = __shfl(off, wi, kWave);
            if ((word >> lane) & 1) {
                const int64_t o = tile_base + (int64_t)wi * kWave + lane;
                const int pos = base + woff + __popcll(word & lanemask_lt());
                a.kept_ops[pos] = (int32_t)o;
                if (a.kept_masks) a.kept_masks[pos] = a.K[o];
            }
        }
    }
}

// The same with a workgroup per tile, four bitmap words in flight per step: for graphs of so few tiles that a wave
// per tile would leave most of the chip idle.
__global__ __launch_bounds__(kCThreads) void k_scatter_block(CompactArgs a)
{
    __shared__ int s_off[kCWords];
    const GraphView &g = a.g;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t tile_base = (int64_t)blockIdx.x * kCompactTile;
    const int64_t n_words = ((int64_t)g.num_ops + 63) >> 6;
    const int64_t word_base = tile_base >> 6;
    const int base = a.block_counts[blockIdx.x];
    if (a.hdr && blockIdx.x == 0 && threadIdx.x == 0 && *a.error == 0) *a.hdr = a.want;
    if (a.block_counts[blockIdx.x + 1] == base) return;     // nothing kept in this tile (uniform)
    if (wave == 0) {                                        // exclusive prefix of the popcounts of the tile's words
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
    const int64_t count_grid = tiles < kCountGrid ? tiles : kCountGrid;
    if (tiles > 0) {
        if (a.from_tensor_mask)
            hipLaunchKernelGGL((k_keep_count<true, false>), dim3((unsigned)count_grid), dim3(kCThreads), 0, s, a);
        else if (a.flag_in && a.g.num_graphs == 1 && (a.op_flag == nullptr || a.op_flag == a.flag_in) &&
                 P >= kFlagsCountMinOps)
        {
            // a wave takes whole tiles: up to kFlagsCountGrid workgroups, so that most waves have one tile only
            const int64_t wg = (tiles + kCWaves - 1) / kCWaves;
            const int64_t flags_grid = wg < kFlagsCountGrid ? wg : kFlagsCountGrid;
            hipLaunchKernelGGL(k_keep_count_flags, dim3((unsigned)flags_grid), dim3(kCThreads), 0, s, a);
        }
        else if (a.flag_in)
            hipLaunchKernelGGL((k_keep_count<false, true>), dim3((unsigned)count_grid), dim3(kCThreads), 0, s, a);
        else
            hipLaunchKernelGGL((k_keep_count<false, false>), dim3((unsigned)count_grid), dim3(kCThreads), 0, s, a);
    }
    const bool reduce_pq = a.per_query_count && a.pq_part;
    const bool fold_pq = reduce_pq && 64 * a.g.num_graphs <= kFoldPqOutputs;
    if (reduce_pq && !fold_pq)
        hipLaunchKernelGGL(k_reduce_pq, dim3((unsigned)((64 * a.g.num_graphs + 3) / 4)), dim3(256), 0, s, a);
    if (ev) (void)hipEventRecord(ev[0], s);
    hipLaunchKernelGGL(k_scan_tiles, dim3(1), dim3(1024), 0, s, a.block_counts, tiles, a.kept_count, a, fold_pq);
    if (ev) (void)hipEventRecord(ev[1], s);
    if (tiles > kScatterByWaveAboveTiles)
        hipLaunchKernelGGL(k_scatter, dim3((unsigned)((tiles + kCWaves - 1) / kCWaves)), dim3(kCThreads), 0, s, a);
    else if (tiles > 0)
        hipLaunchKernelGGL(k_scatter_block, dim3((unsigned)tiles), dim3(kCThreads), 0, s, a);
    if (a.g.num_graphs > 1)
        hipLaunchKernelGGL(k_graph_offsets, dim3((unsigned)((a.g.num_graphs + 1 + 255) / 256)), dim3(256), 0, s, a);
    if (ev) (void)hipEventRecord(ev[2], s);
    return hipGetLastError();
}

}  // namespace dgn
