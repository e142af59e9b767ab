// Backward traversal of Algorithm 1 (Dragon paper, Sec. 2.2), run for up to 64 target sets at once
// as level-synchronous, bit-parallel reverse reachability.
//
// The DFS of Algorithm 1 computes, per target set, the set of tensors with a directed path to a
// target.  Marking is monotone (flags are only ever set), so the marked set is the least fixed point
// of "a marked tensor marks all of its parents" and does not depend on visiting order: here the
// frontier is processed level by level in parallel instead of depth first.
//
// Invariants maintained by every kernel in this file (u64 masks, bit q = flag of set q):
//   (I1)  K[o] only receives bits that some output of o holds in M;
//   (I2)  whenever K[o] gains bits n, the same launch ORs n into M[i] of every input i of o;
//   (I3)  whenever M[t] gains bits, t is in the next frontier (once: a per-level bitmap dedupes);
//   (I4)  processing frontier entry t ORs the *whole* current M[t] into K of every producer of t.
// At an empty frontier: K[o] = OR M[out(o)] and M[t] = S[t] | OR_{o reads t} K[o].
#include "common.h"

namespace dgn {

// ------------------------------------------------------------------------------------------------
// seed: main loop of Algorithm 1 ("for t in T: if not m_t: ...") -- scatter the target bits
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_seed(GraphView g, int32_t Q, int64_t num_targets, int64_t num_sets_total,
                                               const int32_t *tgt_rowptr, const int32_t *tgt_idx, u64 *M,
                                               TravState *st, int32_t *q0, u64 *bm0)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool push = false, bad = false, cross = false;
    int32_t t = 0;
    if (j < num_targets) {
        // set s owns entries [tgt_rowptr[s], tgt_rowptr[s+1]): largest s with tgt_rowptr[s] <= j
        int64_t lo = 0, hi = num_sets_total;
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (tgt_rowptr[mid] <= j) lo = mid; else hi = mid;
        }
        const bool owned = tgt_rowptr[lo] <= j && j < tgt_rowptr[lo + 1];
        t = tgt_idx[j];
        if (owned) {
            if (t < 0 || t >= g.num_tensors) {
                bad = true;
            } else {
                if (g.num_graphs > 1) {
                    const int64_t gi = lo / Q;
                    if (t < g.t_off[gi] || t >= g.t_off[gi + 1]) cross = true;
                }
                const u64 bit = (u64)1 << (lo % Q);
                atomicOr(&M[t], bit);
                const u64 tb = (u64)1 << (t & 63);
                const u64 was = atomicOr(&bm0[t >> 6], tb);
                push = (was & tb) == 0;
            }
        }
    }
    // wave-aggregated slot reservation: one counter update per wave
    const u64 pm = ballot64(push);
    if (pm) {
        int base = 0;
        if (lane_id() == 0) base = atomicAdd(&st->slot[0].n, __popcll(pm));
        base = __builtin_amdgcn_readfirstlane(base);
        if (push) q0[base + __popcll(pm & lanemask_lt())] = t;
    }
    const int err = (bad ? kErrIdRange : 0) | (cross ? kErrCrossGraph : 0);
    if (err) atomicOr(&st->error, err);
}

hipError_t launch_seed(const GraphView &g, int32_t Q, int64_t num_targets, const int32_t *tgt_rowptr,
                       const int32_t *tgt_idx, u64 *M, TravState *st, int32_t *q0, u64 *bm0, hipStream_t s)
{
    if (num_targets == 0) return hipSuccess;
    const int64_t blocks = (num_targets + 255) / 256;
    hipLaunchKernelGGL(k_seed, dim3((unsigned)blocks), dim3(256), 0, s, g, Q, num_targets,
                       (int64_t)g.num_graphs * Q, tgt_rowptr, tgt_idx, M, st, q0, bm0);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// one frontier level per launch
// ------------------------------------------------------------------------------------------------
constexpr int kLevelThreads = 256;
constexpr int kLevelWaves = kLevelThreads / kWave;
constexpr int kStageCap = 512;     // staged pushes per wave before a flush (ints)

// Per-wave staging of next-frontier entries in LDS: slots are reserved with ballot + popcount, the
// global counter is touched once per flush instead of once per push.
struct WaveStage {
    int32_t *buf;     // this wave's kStageCap ints in LDS
    int cnt;          // wave-uniform
};

__device__ __forceinline__ void stage_flush(WaveStage &ws, int32_t *qout, int32_t *n_out)
{
    if (ws.cnt > 0) {
        int base = 0;
        if (lane_id() == 0) base = atomicAdd(n_out, ws.cnt);
        base = __builtin_amdgcn_readfirstlane(base);
        for (int k = lane_id(); k < ws.cnt; k += kWave) qout[base + k] = ws.buf[k];
        ws.cnt = 0;
    }
}

__device__ __forceinline__ void stage_push(WaveStage &ws, bool push, int32_t v, int32_t *qout, int32_t *n_out)
{
    const u64 pm = ballot64(push);
    if (pm) {                                   // wave-uniform branch
        const int np = __popcll(pm);
        if (ws.cnt + np > kStageCap) stage_flush(ws, qout, n_out);
        if (push) ws.buf[ws.cnt + __popcll(pm & lanemask_lt())] = v;
        ws.cnt += np;
    }
}

// Expand 64 frontier entries held one per lane (valid lanes only).  All loops have wave-uniform trip
// counts, so ballots and shuffles always see the whole wave.
__device__ __forceinline__ void expand_wave(const GraphView &g, bool valid, int32_t t, u64 *bm_in, u64 *bm_out,
                                            u64 *M, u64 *K, int *s_incl /* this wave's 64 ints in LDS */,
                                            WaveStage &ws, int32_t *qout, int32_t *n_out)
{
    const int lane = lane_id();
    u64 m = 0;
    int pb = 0, pe = 0;
    if (valid) {
        atomicAnd(&bm_in[t >> 6], ~((u64)1 << (t & 63)));   // leave the bitmap clean for its next use
        m = load_coherent(&M[t]);                           // (I4): everything t holds right now
        pb = g.prod_rowptr[t];
        pe = g.prod_rowptr[t + 1];
    }
    const int max_prod = wave_max(pe - pb);                 // 0 or 1 unless tensors have several producers
    for (int r = 0; r < max_prod; ++r) {
        u64 nb = 0;
        int eb = 0, deg = 0;
        if (pb + r < pe) {
            const int32_t o = g.prod_idx[pb + r];
            const u64 old = atomicOr(&K[o], m);             // (I1)
            nb = m & ~old;                                  // bits o did not have yet
            if (nb) {
                eb = g.in_rowptr[o];
                deg = g.in_rowptr[o + 1] - eb;
            }
        }
        // spread the input edges of all 64 operators evenly over the lanes
        const int incl = wave_incl_scan(deg);
        const int excl = incl - deg;
        const int total = __shfl(incl, kWave - 1, kWave);
        s_incl[lane] = incl;
        __builtin_amdgcn_wave_barrier();
        for (int e0 = 0; e0 < total; e0 += kWave) {
            const int e = e0 + lane;
            const bool ev = e < total;
            int lo = 0, hi = kWave - 1;                     // first lane whose inclusive sum exceeds e
#pragma unroll
            for (int it = 0; it < 6; ++it) {
                const int mid = (lo + hi) >> 1;
                if (s_incl[mid] > e) hi = mid; else lo = mid + 1;
            }
            const int owner = lo;
            const int o_eb = __shfl(eb, owner, kWave);
            const int o_excl = __shfl(excl, owner, kWave);
            const u64 bits = shfl64(nb, owner);
            bool push = false;
            int32_t u = 0;
            if (ev) {
                u = g.in_idx[o_eb + (e - o_excl)];
                const u64 old2 = atomicOr(&M[u], bits);     // (I2)
                if (bits & ~old2) {                         // (I3)
                    const u64 ub = (u64)1 << (u & 63);
                    const u64 was = atomicOr(&bm_out[u >> 6], ub);
                    push = (was & ub) == 0;
                }
            }
            stage_push(ws, push, u, qout, n_out);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

__global__ __launch_bounds__(kLevelThreads) void k_level(GraphView g, TravState *st, int launch_no, int32_t *q0,
                                                          int32_t *q1, u64 *bm0, u64 *bm1, u64 *M, u64 *K)
{
    __shared__ int32_t s_stage[kLevelWaves][kStageCap];
    __shared__ int s_incl[kLevelWaves][kWave];

    const LevelSlot in = st->slot[launch_no & 1];
    LevelSlot *out = &st->slot[(launch_no + 1) & 1];
    const int n = in.n;
    if (n == 0) {                                           // traversal already finished: carry the state on
        if (blockIdx.x == 0 && threadIdx.x == 0) { out->level = in.level; out->n = 0; }
        return;
    }
    const int nwork = min((int)gridDim.x, (n + kLevelThreads - 1) / kLevelThreads);
    if ((int)blockIdx.x >= nwork) return;

    const int cur = in.level & 1;
    const int32_t *qin = cur ? q1 : q0;
    int32_t *qout = cur ? q0 : q1;
    u64 *bm_in = cur ? bm1 : bm0;
    u64 *bm_out = cur ? bm0 : bm1;

    const int wave = threadIdx.x >> 6;
    WaveStage ws{&s_stage[wave][0], 0};
    for (int base = blockIdx.x * kLevelThreads; base < n; base += nwork * kLevelThreads) {
        const int i = base + threadIdx.x;
        const bool valid = i < n;
        const int32_t t = valid ? qin[i] : 0;
        expand_wave(g, valid, t, bm_in, bm_out, M, K, &s_incl[wave][0], ws, qout, &out->n);
    }
    stage_flush(ws, qout, &out->n);

    // the last working block to finish publishes the next level
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        const int tk = atomicAdd(&st->ticket, 1);
        if (tk == nwork - 1) {
            st->ticket = 0;
            st->slot[launch_no & 1].n = 0;                  // becomes the push counter of the next launch
            out->level = in.level + 1;
            st->tensor_visits += (u64)n;
            if ((u64)n > st->max_frontier) st->max_frontier = (u64)n;
        }
    }
}

hipError_t launch_level(const GraphView &g, TravState *st, int launch_no, int32_t *q0, int32_t *q1, u64 *bm0,
                        u64 *bm1, u64 *M, u64 *K, int grid_blocks, hipStream_t s)
{
    hipLaunchKernelGGL(k_level, dim3((unsigned)grid_blocks), dim3(kLevelThreads), 0, s, g, st, launch_no, q0, q1,
                       bm0, bm1, M, K);
    return hipGetLastError();
}

}  // namespace dgn
