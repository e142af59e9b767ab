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
//   (I2)  whenever K[o] gains bits n, the same thread ORs n into M[i] of every input i of o;
//   (I3)  whenever M[t] gains bits, t is in a later frontier (once per level: a bitmap dedupes);
//   (I4)  processing frontier entry t ORs the *whole* current M[t] into K of every producer of t;
//   (I5)  an entry that is deferred stays in the frontier until it is processed.
// At an empty frontier: K[o] = OR M[out(o)] and M[t] = S[t] | OR_{o reads t} K[o].
//
// Deferral (I5) is only a schedule: operator ids are a topological order, so an entry whose producer
// id is still below the level's threshold is likely to receive more bits from operators with higher
// ids; it waits (re-queued, 16 sequential bytes) while the threshold decays geometrically, and is
// then expanded once with all of its bits instead of once per arrival.
#include "common.h"

namespace dgn {

// Frontier entry: tensor id plus its producer record once that has been looked up.
//   o >= 0 : single producer o with inputs in_idx[eb .. eb+deg)
//   o == kFresh : not looked up yet         o == kMulti : several producers, prod_idx[eb .. eb+deg)
//   o == kNoProducer : graph input (never queued again)
struct __align__(16) Entry { int32_t t, o, eb, deg; };

__device__ __forceinline__ Entry load_entry(const Entry *q, int i)
{
    // two 8-byte loads that bypass the per-CU cache: a persistent workgroup re-reads queue slots that
    // it wrote itself two levels earlier
    const u64 *p = reinterpret_cast<const u64 *>(q + i);
    const u64 a = load_coherent(p), b = load_coherent(p + 1);
    Entry e;
    e.t = (int32_t)(a & 0xffffffffu);
    e.o = (int32_t)(a >> 32);
    e.eb = (int32_t)(b & 0xffffffffu);
    e.deg = (int32_t)(b >> 32);
    return e;
}

// ------------------------------------------------------------------------------------------------
// producer records, built once per graph
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_build_pinfo(GraphView g, int4 *pinfo)
{
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < g.num_tensors; t += gsize) {
        const int32_t pb = g.prod_rowptr[t], pe = g.prod_rowptr[t + 1];
        int4 r;
        if (pe == pb) {
            r = make_int4(kNoProducer, 0, 0, 0);
        } else if (pe - pb == 1) {
            const int32_t o = g.prod_idx[pb];
            const int32_t eb = g.in_rowptr[o];
            r = make_int4(o, eb, g.in_rowptr[o + 1] - eb, 0);
        } else {
            r = make_int4(kMulti, pb, pe - pb, 0);
        }
        pinfo[t] = r;
    }
}

hipError_t launch_build_pinfo(const GraphView &g, int4 *pinfo, hipStream_t s)
{
    if (g.num_tensors == 0) return hipSuccess;
    int64_t blocks = ((int64_t)g.num_tensors + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_build_pinfo, dim3((unsigned)blocks), dim3(256), 0, s, g, pinfo);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// seed: main loop of Algorithm 1 ("for t in T: if not m_t: ...") -- scatter the target bits
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_seed(GraphView g, int32_t Q, int64_t num_targets, int64_t num_sets_total,
                                               const int32_t *tgt_rowptr, const int32_t *tgt_idx, u64 *M,
                                               TravState *st, Entry *q0, u64 *bm0, int32_t theta0)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j == 0) st->slot[0].theta = theta0;
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
        if (push) q0[base + __popcll(pm & lanemask_lt())] = Entry{t, kFresh, 0, 0};
    }
    const int err = (bad ? kErrIdRange : 0) | (cross ? kErrCrossGraph : 0);
    if (err) atomicOr(&st->error, err);
}

hipError_t launch_seed(const GraphView &g, int32_t Q, int64_t num_targets, const int32_t *tgt_rowptr,
                       const int32_t *tgt_idx, u64 *M, TravState *st, void *q0, u64 *bm0, int32_t theta0,
                       hipStream_t s)
{
    const int64_t blocks = num_targets > 0 ? (num_targets + 255) / 256 : 1;
    hipLaunchKernelGGL(k_seed, dim3((unsigned)blocks), dim3(256), 0, s, g, Q, num_targets,
                       (int64_t)g.num_graphs * Q, tgt_rowptr, tgt_idx, M, st, static_cast<Entry *>(q0), bm0, theta0);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// frontier expansion shared by the level kernels
// ------------------------------------------------------------------------------------------------
constexpr int kStageCap = 192;     // staged pushes per wave before a flush (16-byte entries)

// Per-wave staging of next-frontier entries in LDS: slots are reserved with ballot + popcount, the
// queue counter is touched once per flush instead of once per push.
struct WaveStage {
    Entry *buf;       // this wave's kStageCap entries in LDS
    int cnt;          // wave-uniform
};

struct Frontier {     // one level's output side
    Entry *qout;
    int32_t *n_out;   // global or LDS counter
    u64 *bm_out;
};

__device__ __forceinline__ void stage_flush(WaveStage &ws, const Frontier &f)
{
    if (ws.cnt > 0) {
        int base = 0;
        if (lane_id() == 0) base = atomicAdd(f.n_out, ws.cnt);
        base = __builtin_amdgcn_readfirstlane(base);
        for (int k = lane_id(); k < ws.cnt; k += kWave) f.qout[base + k] = ws.buf[k];
        ws.cnt = 0;
    }
}

__device__ __forceinline__ void stage_push(WaveStage &ws, bool push, const Entry &v, const Frontier &f)
{
    const u64 pm = ballot64(push);
    if (pm) {                                   // wave-uniform branch
        const int np = __popcll(pm);
        if (ws.cnt + np > kStageCap) stage_flush(ws, f);
        if (push) ws.buf[ws.cnt + __popcll(pm & lanemask_lt())] = v;
        ws.cnt += np;
    }
}

// Lane l holds operator-side work (eb, deg, bits): OR `bits` into M of the deg inputs starting at
// in_idx[eb].  The edges of all 64 lanes are spread evenly over the wave (prefix sum + search), so a
// fan-in of 64 next to fan-ins of 1 costs no idle lanes.  Wave-uniform control flow throughout.
__device__ __forceinline__ void expand_edges(const GraphView &g, int eb, int deg, u64 bits, u64 *M, int *s_incl,
                                             WaveStage &ws, const Frontier &f)
{
    const int lane = lane_id();
    const int incl = wave_incl_scan(deg);
    const int excl = incl - deg;
    const int total = __shfl(incl, kWave - 1, kWave);
    if (total == 0) return;
    s_incl[lane] = incl;
    __builtin_amdgcn_wave_barrier();
    for (int e0 = 0; e0 < total; e0 += kWave) {
        const int e = e0 + lane;
        const bool ev = e < total;
        int lo = 0, hi = kWave - 1;                         // first lane whose inclusive sum exceeds e
#pragma unroll
        for (int it = 0; it < 6; ++it) {
            const int mid = (lo + hi) >> 1;
            if (s_incl[mid] > e) hi = mid; else lo = mid + 1;
        }
        const int owner = lo;
        const int o_eb = __shfl(eb, owner, kWave);
        const int o_excl = __shfl(excl, owner, kWave);
        const u64 b = shfl64(bits, owner);
        bool push = false;
        int32_t u = 0;
        if (ev) {
            u = g.in_idx[o_eb + (e - o_excl)];
            const u64 old = atomicOr(&M[u], b);             // (I2)
            if (b & ~old) {                                 // (I3)
                const u64 ub = (u64)1 << (u & 63);
                const u64 was = atomicOr(&f.bm_out[u >> 6], ub);
                push = (was & ub) == 0;
            }
        }
        stage_push(ws, push, Entry{u, kFresh, 0, 0}, f);
    }
    __builtin_amdgcn_wave_barrier();
}

struct LevelCounters {   // per-lane tallies, reduced by the caller
    int processed;
    int max_deferred_key;
};

// Process 64 frontier entries held one per lane (valid lanes only).
__device__ __forceinline__ void process_wave(const GraphView &g, bool valid, Entry e, int32_t theta, u64 *bm_in,
                                             u64 *M, u64 *K, int *s_incl, WaveStage &ws, const Frontier &f,
                                             LevelCounters &lc)
{
    u64 m = 0;
    bool defer = false;
    if (valid) {
        atomicAnd(&bm_in[e.t >> 6], ~((u64)1 << (e.t & 63)));   // leave the bitmap clean for its next use
        if (e.o == kFresh) {
            const int4 pi = g.pinfo[e.t];
            e.o = pi.x; e.eb = pi.y; e.deg = pi.z;
        }
        defer = e.o >= 0 && e.o < theta;                    // (I5); multi-producer tensors are never deferred
        if (!defer && e.o != kNoProducer) m = load_coherent(&M[e.t]);   // (I4): everything t holds right now
    }
    // deferred entries go back into the frontier (unless a push of this level already put t there)
    {
        bool push = false;
        if (defer) {
            const u64 tb = (u64)1 << (e.t & 63);
            const u64 was = atomicOr(&f.bm_out[e.t >> 6], tb);
            push = (was & tb) == 0;
            lc.max_deferred_key = max(lc.max_deferred_key, e.o);
        }
        stage_push(ws, push, e, f);
    }
    const bool active = valid && !defer && e.o != kNoProducer;
    if (active) lc.processed++;
    // single-producer tensors (the common case)
    {
        u64 nb = 0;
        int deg = 0;
        if (active && e.o >= 0) {
            const u64 old = atomicOr(&K[e.o], m);           // (I1)
            nb = m & ~old;                                  // bits o did not have yet
            if (nb) deg = e.deg;
        }
        expand_edges(g, e.eb, deg, nb, M, s_incl, ws, f);
    }
    // tensors with several producers: one pass per producer rank
    const bool multi = active && e.o == kMulti;
    const int max_prod = wave_max(multi ? e.deg : 0);
    for (int r = 0; r < max_prod; ++r) {
        u64 nb = 0;
        int eb = 0, deg = 0;
        if (multi && r < e.deg) {
            const int32_t o = g.prod_idx[e.eb + r];
            const u64 old = atomicOr(&K[o], m);
            nb = m & ~old;
            if (nb) {
                eb = g.in_rowptr[o];
                deg = g.in_rowptr[o + 1] - eb;
            }
        }
        expand_edges(g, eb, deg, nb, M, s_incl, ws, f);
    }
}

__device__ __forceinline__ int32_t next_theta(int32_t theta, float decay, int processed, int max_deferred_key)
{
    if (theta <= 0) return 0;
    float base = (float)theta;
    if (processed == 0 && max_deferred_key >= 0) base = (float)max_deferred_key + 1.0f;   // jump to the work
    const int32_t t = (int32_t)(base * decay);
    return t < kThetaFloor ? 0 : t;
}

// ------------------------------------------------------------------------------------------------
// wide levels: one frontier level per launch, the whole chip
// ------------------------------------------------------------------------------------------------
constexpr int kLevelThreads = 256;
constexpr int kLevelWaves = kLevelThreads / kWave;

__global__ __launch_bounds__(kLevelThreads) void k_level(GraphView g, TravState *st, int launch_no, Entry *q0,
                                                          Entry *q1, u64 *bm0, u64 *bm1, u64 *M, u64 *K,
                                                          int narrow_cap, float decay)
{
    __shared__ Entry s_stage[kLevelWaves][kStageCap];
    __shared__ int s_incl[kLevelWaves][kWave];
    __shared__ int s_proc[kLevelWaves], s_maxkey[kLevelWaves];

    const LevelSlot in = st->slot[launch_no & 1];
    LevelSlot *out = &st->slot[(launch_no + 1) & 1];
    const int n = in.n;
    if (n <= narrow_cap) {       // finished, or small enough for the single-workgroup kernel: pass the state on
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            out->level = in.level;
            out->theta = in.theta;
            out->n = n;
            st->slot[launch_no & 1].n = 0;
        }
        return;
    }
    const int nwork = min((int)gridDim.x, (n + kLevelThreads - 1) / kLevelThreads);
    if ((int)blockIdx.x >= nwork) return;

    const int cur = in.level & 1;
    const Entry *qin = cur ? q1 : q0;
    u64 *bm_in = cur ? bm1 : bm0;
    const Frontier f{cur ? q0 : q1, &out->n, cur ? bm0 : bm1};

    const int wave = threadIdx.x >> 6;
    WaveStage ws{&s_stage[wave][0], 0};
    LevelCounters lc{0, -1};
    for (int base = blockIdx.x * kLevelThreads; base < n; base += nwork * kLevelThreads) {
        const int i = base + threadIdx.x;
        const bool valid = i < n;
        Entry e{0, kNoProducer, 0, 0};
        if (valid) e = load_entry(qin, i);
        process_wave(g, valid, e, in.theta, bm_in, M, K, &s_incl[wave][0], ws, f, lc);
    }
    stage_flush(ws, f);

    const int wproc = wave_sum(lc.processed), wkey = wave_max(lc.max_deferred_key);
    if (lane_id() == 0) { s_proc[wave] = wproc; s_maxkey[wave] = wkey; }
    // the last working block to finish publishes the next level
    __syncthreads();
    if (threadIdx.x == 0) {
        int proc = 0, mk = -1;
        for (int w = 0; w < kLevelWaves; ++w) { proc += s_proc[w]; mk = max(mk, s_maxkey[w]); }
        if (proc) atomicAdd(&st->processed, proc);
        if (mk >= 0) atomicMax(&st->max_deferred_key, mk);
        __threadfence();
        const int tk = atomicAdd(&st->ticket, 1);
        if (tk == nwork - 1) {
            __threadfence();
            const int tot_proc = load_coherent(&st->processed);
            const int tot_key = load_coherent(&st->max_deferred_key);
            st->ticket = 0;
            st->processed = 0;
            st->max_deferred_key = -1;
            st->slot[launch_no & 1].n = 0;                  // becomes the push counter of the next launch
            out->level = in.level + 1;
            out->theta = next_theta(in.theta, decay, tot_proc, tot_key);
            st->tensor_visits += (u64)tot_proc;
            if ((u64)n > st->max_frontier) st->max_frontier = (u64)n;
        }
    }
}

hipError_t launch_level(const GraphView &g, TravState *st, int launch_no, void *q0, void *q1, u64 *bm0, u64 *bm1,
                        u64 *M, u64 *K, int grid_blocks, int narrow_cap, float decay, hipStream_t s)
{
    hipLaunchKernelGGL(k_level, dim3((unsigned)grid_blocks), dim3(kLevelThreads), 0, s, g, st, launch_no,
                       static_cast<Entry *>(q0), static_cast<Entry *>(q1), bm0, bm1, M, K, narrow_cap, decay);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// narrow levels: one workgroup walks level after level while the frontier is small, with workgroup
// barriers instead of kernel launches (deep graphs have hundreds of small levels)
// ------------------------------------------------------------------------------------------------
constexpr int kNarrowThreads = 1024;
constexpr int kNarrowWaves = kNarrowThreads / kWave;

__global__ __launch_bounds__(kNarrowThreads) void k_narrow(GraphView g, TravState *st, int launch_no, Entry *q0,
                                                            Entry *q1, u64 *bm0, u64 *bm1, u64 *M, u64 *K,
                                                            int narrow_cap)
{
    __shared__ Entry s_stage[kNarrowWaves][kStageCap];
    __shared__ int s_incl[kNarrowWaves][kWave];
    __shared__ int s_nout;

    const LevelSlot in = st->slot[launch_no & 1];
    int level = in.level, n = in.n;
    const int wave = threadIdx.x >> 6;
    WaveStage ws{&s_stage[wave][0], 0};
    LevelCounters lc{0, -1};
    u64 visits = 0, maxf = 0;
    while (n > 0 && n <= narrow_cap) {
        if (threadIdx.x == 0) s_nout = 0;
        __syncthreads();
        const int cur = level & 1;
        const Entry *qin = cur ? q1 : q0;
        u64 *bm_in = cur ? bm1 : bm0;
        const Frontier f{cur ? q0 : q1, &s_nout, cur ? bm0 : bm1};
        for (int base = 0; base < n; base += kNarrowThreads) {
            const int i = base + threadIdx.x;
            const bool valid = i < n;
            Entry e{0, kNoProducer, 0, 0};
            if (valid) e = load_entry(qin, i);
            // threshold 0: a small frontier is latency bound, so nothing is gained by deferring
            process_wave(g, valid, e, 0, bm_in, M, K, &s_incl[wave][0], ws, f, lc);
        }
        stage_flush(ws, f);
        __threadfence();          // queue entries and bitmap updates reach the device-coherent level
        __syncthreads();
        visits += (u64)n;
        if ((u64)n > maxf) maxf = (u64)n;
        n = s_nout;
        ++level;
        __syncthreads();          // everyone has read s_nout before it is reset
    }
    if (threadIdx.x == 0) {
        LevelSlot *out = &st->slot[(launch_no + 1) & 1];
        out->level = level;
        out->theta = in.theta;
        out->n = n;
        st->slot[launch_no & 1].n = 0;
        st->tensor_visits += visits;
        if (maxf > st->max_frontier) st->max_frontier = maxf;
    }
}

hipError_t launch_narrow(const GraphView &g, TravState *st, int launch_no, void *q0, void *q1, u64 *bm0, u64 *bm1,
                         u64 *M, u64 *K, int narrow_cap, hipStream_t s)
{
    hipLaunchKernelGGL(k_narrow, dim3(1), dim3(kNarrowThreads), 0, s, g, st, launch_no, static_cast<Entry *>(q0),
                       static_cast<Entry *>(q1), bm0, bm1, M, K, narrow_cap);
    return hipGetLastError();
}

}  // namespace dgn
