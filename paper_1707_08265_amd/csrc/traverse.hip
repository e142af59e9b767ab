// Backward traversal of Algorithm 1 (Dragon paper, Sec. 2.2), run for up to 64 target sets at once
// as level-synchronous, bit-parallel reverse reachability.
//
// The DFS of Algorithm 1 computes, per target set, the set of tensors with a directed path to a
// target.  Marking is monotone (flags are only ever set), so the marked set is the least fixed point
// of "a marked tensor marks all of its parents" and does not depend on visiting order: here the
// work is processed level by level in parallel instead of depth first.
//
// The unit of work is an OPERATOR whose outputs have gained bits: processing o reads M of its outputs,
// k = OR M[out(o)], and ORs the bits K[o] did not have yet into M of every input; an input u that gains
// bits hands its producer on as new work.  Invariants (u64 masks, bit q = flag of set q):
//   (I1)  K[o] only receives bits that some output of o holds in M;
//   (I2)  whenever K[o] gains bits n, the same lane ORs n into M[u] of every input u of o;
//   (I3)  whenever M[u] gains bits (the atomic's return value says so, to exactly one lane), every producer
//         of u is noted for a LATER step: queued for the next level, or -- when its id is below the level's
//         threshold -- stamped in a byte map that is read when the threshold has passed it; if a queue is
//         full an overflow flag is raised and fix-up sweeps restore the fixed point afterwards;
//   (I4)  a noted operator is processed in a launch (or, in the single-workgroup kernel, a barrier-separated
//         level) after the one that noted it, so it sees the bits it was noted for.
// With no work left: K[o] = OR M[out(o)] and M[t] = S[t] | OR_{o reads t} K[o].
//
// K is read and written without atomics.  Several lanes may process one operator in the same launch (the queue
// is not deduplicated) and the last store may then lack bits another lane had seen; but such bits arrived during
// this launch, so by (I3)/(I4) the operator is processed again later, and in the last launch that processes it
// nothing arrives any more: every lane reads the same masks and stores the same, final, value.  A bit is pushed
// to the inputs by the first lane that stores it (it was not in the K that lane had read).  Launches in which a
// wave expands its own pushes at once (see run_level) break (I4) and use atomic ORs on K instead.
//
// Why thresholds: 64-bit atomics retire at roughly 20 G/s on this chip whatever their locality, so the
// traversal is bound by the number of atomics -- one per input edge of a processed operator.  Operator ids are a
// topological order, hence a low-numbered producer keeps receiving bits from higher-numbered operators for many
// levels; processing it once, after the geometrically decaying threshold has passed it, replaces several
// expansions by one.  It is a schedule only: the fixed point is the same for any order.
#include "common.h"

namespace dgn {

// ------------------------------------------------------------------------------------------------
// operator records and producer words, built once per graph
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_build_records(GraphView g, int4 *orec, int32_t *prod1, int32_t *multi)
{
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x, gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t t = gtid; t < g.num_tensors; t += gsize) {
        const int32_t pb = g.prod_rowptr[t], pe = g.prod_rowptr[t + 1];
        int32_t r = kNoProducer;
        if (pe - pb == 1) {
            r = g.prod_idx[pb];
        } else if (pe - pb > 1) {
            r = kMulti;
            *multi = 1;                                      // (the same value from every writer)
        }
        prod1[t] = r;
    }
    for (int64_t o = gtid; o < g.num_ops; o += gsize) {
        const int32_t ib = g.in_rowptr[o], ie = g.in_rowptr[o + 1];
        const int32_t ob = g.out_rowptr[o], oe = g.out_rowptr[o + 1];
        const int32_t first = oe > ob ? g.out_idx[ob] : 0;
        bool consecutive = true;
        for (int32_t e = ob + 1; e < oe; ++e) consecutive &= g.out_idx[e] == first + (e - ob);
        orec[o] = consecutive ? make_int4(ib, ie - ib, first, oe - ob) : make_int4(ib, ie - ib, ob, -(oe - ob));
    }
}

hipError_t launch_build_records(const GraphView &g, int4 *orec, int32_t *prod1, int32_t *multi, hipStream_t s)
{
    const int64_t n = g.num_tensors > g.num_ops ? g.num_tensors : g.num_ops;
    if (n == 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_build_records, dim3((unsigned)blocks), dim3(256), 0, s, g, orec, prod1, multi);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// segmented work queues
//
// A queue holds operator ids.  It is split into S segments with one push counter each (64 bytes apart):
// atomics on ONE address retire at about 11 ns each on this chip, so a single counter bumped by every
// wave of a wide level would cost more than the level's real work.
// ------------------------------------------------------------------------------------------------
constexpr int kStageCap = 256;     // staged pushes per wave before a flush (a power of two: the buffer is a ring)
constexpr int kLogStageCap = 128;  // staged log entries per wave

// Per-wave staging in LDS.  Queue entries sit in a ring: slots are reserved with ballot + popcount, a
// segment counter in memory is touched once per flush instead of once per push, and a wave may take entries
// back out of the ring to process them itself before they ever reach memory (see run_level).  Tensors coloured
// for the first time are noted in a second, small buffer that is written to the log when it fills up and when
// the kernel ends.
struct WaveStage {
    int32_t *buf;     // this wave's kStageCap ints
    int head, tail;   // wave-uniform, ever growing; the pending entries are buf[head & mask .. tail & mask)
    int32_t *lbuf;    // this wave's kLogStageCap ints, or NULL: no log is kept
    int lcnt;         // wave-uniform
};

struct Frontier {     // where one wave pushes
    int32_t *seg;     // start of the wave's segment in the output queue
    int32_t *cnt;     // that segment's push counter, global or LDS (may run past seg_cap: readers clamp)
    int32_t seg_cap;
    int32_t *error;   // sticky error word of the traversal state
    int32_t *log;     // start of the wave's segment of the log of coloured tensors, or NULL: no log
    int32_t *log_cnt; // that segment's counter
    int32_t log_cap;
    int32_t *mirror;  // NULL, or an array in LDS that receives a copy of the first mirror_cap entries of the segment
    int32_t mirror_cap;   // (the single-workgroup kernel reads its next frontier from there, not from memory)
};

// Write the pending entries out to the wave's queue segment.
__device__ __forceinline__ void flush_entries(WaveStage &ws, const Frontier &f)
{
    const int n = ws.tail - ws.head;
    if (n > 0) {
        int base = 0;
        if (lane_id() == 0) {
            base = atomicAdd(f.cnt, n);
            if (base + n > f.seg_cap) atomicOr(f.error, kErrOverflow);   // (I3): fix-up sweeps will follow
        }
        base = __builtin_amdgcn_readfirstlane(base);
        for (int k = lane_id(); k < n; k += kWave) {
            const int32_t v = ws.buf[(ws.head + k) & (kStageCap - 1)];
            if (base + k < f.seg_cap) store_coherent(&f.seg[base + k], v);   // read by other blocks
            if (base + k < f.mirror_cap) f.mirror[base + k] = v;
        }
        ws.head = ws.tail;
    }
}

// Write the waiting log entries out to the wave's log segment.
__device__ __forceinline__ void flush_log(WaveStage &ws, const Frontier &f)
{
    if (ws.lcnt > 0) {
        int base = 0;
        if (lane_id() == 0) {
            base = atomicAdd(f.log_cnt, ws.lcnt);
            if (base + ws.lcnt > f.log_cap) atomicOr(f.error, kErrLogFull);
        }
        base = __builtin_amdgcn_readfirstlane(base);
        for (int k = lane_id(); k < ws.lcnt; k += kWave)
            if (base + k < f.log_cap) f.log[base + k] = ws.lbuf[k];
        ws.lcnt = 0;
    }
}

// Both at once, at the end of a launch: the two counter updates are in flight together, so the wave waits for one
// trip to memory, not two.
__device__ __forceinline__ void flush_both(WaveStage &ws, const Frontier &f)
{
    const int n = ws.tail - ws.head, nl = ws.lcnt;
    if (n <= 0 && nl <= 0) return;                          // wave-uniform
    int base = 0, lbase = 0;
    if (lane_id() == 0) {
        if (n > 0) base = atomicAdd(f.cnt, n);
        if (nl > 0) lbase = atomicAdd(f.log_cnt, nl);
        if (n > 0 && base + n > f.seg_cap) atomicOr(f.error, kErrOverflow);      // (I3): fix-up sweeps will follow
        if (nl > 0 && lbase + nl > f.log_cap) atomicOr(f.error, kErrLogFull);
    }
    base = __builtin_amdgcn_readfirstlane(base);
    lbase = __builtin_amdgcn_readfirstlane(lbase);
    for (int k = lane_id(); k < n; k += kWave) {
        const int32_t v = ws.buf[(ws.head + k) & (kStageCap - 1)];
        if (base + k < f.seg_cap) store_coherent(&f.seg[base + k], v);           // read by other blocks
        if (base + k < f.mirror_cap) f.mirror[base + k] = v;
    }
    for (int k = lane_id(); k < nl; k += kWave)
        if (lbase + k < f.log_cap) f.log[lbase + k] = ws.lbuf[k];
    ws.head = ws.tail;
    ws.lcnt = 0;
}

// Lanes with `push` queue operator `op`; lanes with `first` note tensor `t` as coloured by this prune (its
// mask was zero before, which the atomic tells exactly one lane).  Wave-uniform control flow.
__device__ __forceinline__ void stage_push(WaveStage &ws, bool push, int32_t op, bool first, int32_t t, const Frontier &f)
{
    const u64 pm = ballot64(push);
    if (pm) {
        const int np = __popcll(pm);
        if (ws.tail - ws.head + np > kStageCap) flush_entries(ws, f);
        if (push) ws.buf[(ws.tail + __popcll(pm & lanemask_lt())) & (kStageCap - 1)] = op;
        ws.tail += np;
    }
    if (ws.lbuf) {
        const u64 fm = ballot64(first);
        if (fm) {
            const int nf = __popcll(fm);
            if (ws.lcnt + nf > kLogStageCap) flush_log(ws, f);
            if (first) ws.lbuf[ws.lcnt + __popcll(fm & lanemask_lt())] = t;
            ws.lcnt += nf;
        }
    }
}

// Reader side: item i of a queue whose segment counts have the prefix sums s_pref[0..S].
__device__ __forceinline__ int32_t load_item(const int32_t *q, const QueueGeom &qg, const int *s_pref, int i)
{
    int lo = 0, hi = kMaxSeg - 1;               // segment holding item i: last s with s_pref[s] <= i
#pragma unroll
    for (int it = 0; it < 6; ++it) {
        const int mid = (lo + hi + 1) >> 1;
        if (s_pref[mid] <= i) lo = mid; else hi = mid - 1;
    }
    // bypass the per-CU cache: the single-workgroup kernel re-reads queue slots it wrote two levels earlier
    return load_coherent(&q[(int64_t)lo * qg.seg_cap + (i - s_pref[lo])]);
}

// ------------------------------------------------------------------------------------------------
// seed: main loop of Algorithm 1 ("for t in T: if not m_t: ...") -- scatter the target bits; the producers of
// the targets are the first work
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_seed(GraphView g, int32_t Q, int64_t num_targets, int64_t num_sets_total,
                                               const int32_t *tgt_rowptr, const int32_t *tgt_idx, u64 *M,
                                               TravState *st, TravCounters *ctr, int32_t *q0, QueueGeom qg,
                                               int32_t theta0, ColourLog log)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j == 0) {                                           // the record "before launch 0": nothing done yet
        st->slot[1].theta = theta0;
        st->slot[1].theta_hi = g.num_ops;
    }
    bool fresh = false, first = false, bad = false, cross = false;
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
                const u64 old = atomicOr(&M[t], bit);
                fresh = (old & bit) == 0;                   // a duplicate target adds nothing new
                first = old == 0;                           // this thread coloured t
            }
        }
    }
    // The producers of the tensors that gained a bit are queued (all of them, whatever the threshold: there are
    // few).  Wave-aggregated slot reservation: one counter update per wave and round, counters spread over
    // segments.  (No queue in the per-graph sweep mode: the bits in M are all it needs.)
    bool overflow = false;
    if (q0) {
        int32_t pr = kNoProducer, pb = 0, np = 0;
        if (fresh) {
            pr = g.prod1[t];
            if (pr >= 0) np = 1;
            else if (pr == kMulti) { pb = g.prod_rowptr[t]; np = g.prod_rowptr[t + 1] - pb; }
        }
        const int rounds = wave_max(np);
        const int seg = (int)((j >> 6) & (qg.S - 1));
        for (int r = 0; r < rounds; ++r) {
            const bool push = r < np;
            const u64 pm = ballot64(push);
            int base = 0;
            if (lane_id() == 0) base = atomicAdd(&ctr->cnt[2][seg].v, __popcll(pm));   // tallies "of launch -1"
            base = __builtin_amdgcn_readfirstlane(base);
            const int pos = base + __popcll(pm & lanemask_lt());
            if (push) {
                const int32_t op = pr >= 0 ? pr : g.prod_idx[pb + r];
                if (pos < qg.seg_cap) q0[(int64_t)seg * qg.seg_cap + pos] = op;
                else overflow = true;
            }
        }
    }
    bool log_full = false;
    const u64 fm = (q0 && log.entries) ? ballot64(first) : 0;
    if (fm) {
        const int lseg = (int)((j >> 6) & (kMaxSeg - 1));
        int base = 0;
        if (lane_id() == 0) base = atomicAdd(&log.cnt[lseg].v, __popcll(fm));
        base = __builtin_amdgcn_readfirstlane(base);
        const int pos = base + __popcll(fm & lanemask_lt());
        if (first) {
            if (pos < log.seg_cap) log.entries[(int64_t)lseg * log.seg_cap + pos] = t;
            else log_full = true;
        }
    }
    const int err = (bad ? kErrIdRange : 0) | (cross ? kErrCrossGraph : 0) | (overflow ? kErrOverflow : 0) |
                    (log_full ? kErrLogFull : 0);
    if (err) atomicOr(&st->error, err);
}

hipError_t launch_seed(const GraphView &g, int32_t Q, int64_t num_targets, const int32_t *tgt_rowptr,
                       const int32_t *tgt_idx, u64 *M, TravState *st, TravCounters *ctr, int32_t *q0,
                       const QueueGeom &qg, int32_t theta0, const ColourLog &log, hipStream_t s)
{
    const int64_t blocks = num_targets > 0 ? (num_targets + 255) / 256 : 1;
    hipLaunchKernelGGL(k_seed, dim3((unsigned)blocks), dim3(256), 0, s, g, Q, num_targets,
                       (int64_t)g.num_graphs * Q, tgt_rowptr, tgt_idx, M, st, ctr, q0, qg, theta0, log);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// operator processing shared by the level kernels
// ------------------------------------------------------------------------------------------------
struct LevelCounters {   // per-lane tallies, reduced by the caller
    int processed;
    int max_deferred_key;
    int atomics;         // atomic ORs issued (statistics only)
};

struct Masks {           // what a prune writes
    u64 *M, *K;
    uint8_t *DB;         // a byte per operator: "has gained bits and waits for the threshold to pass it"
    uint8_t *flags;      // a byte per operator: K != 0 (read by the count pass instead of all of K)
};

// A tensor has gained bits: note one of its producers for a later step (I3).  Returns whether to queue it.
__device__ __forceinline__ bool note_producer(int32_t op, int32_t theta, uint8_t *DB, LevelCounters &lc)
{
    if (op >= theta) return true;
    DB[op] = 1;                 // a plain byte store, no atomic: read by a later launch, when theta has passed op
    lc.max_deferred_key = max(lc.max_deferred_key, op);
    return false;
}

// Lane l holds (eb, deg, bits): OR `bits` into M of the deg inputs starting at in_idx[eb].  The edges of
// all 64 lanes are spread evenly over the wave (prefix sum + search), so a fan-in of 64 next to fan-ins
// of 1 costs no idle lanes.  A wave with more than 64 edges takes kEdgeRounds rounds of 64 at a time: their
// targets are fetched together, then their atomics sent together, so that a wave that met an operator with many
// inputs pays the two dependent accesses once, not once per round.  Wave-uniform control flow throughout.
constexpr int kEdgeRounds = 1;          // (two and four were measured: no gain, more registers)

__device__ __forceinline__ void expand_edges(const GraphView &g, int eb, int deg, u64 bits, int32_t theta, const Masks &mk,
                                             int *s_incl, WaveStage &ws, const Frontier &f, LevelCounters &lc)
{
    const int lane = lane_id();
    const int incl = wave_incl_scan(deg);
    const int excl = incl - deg;
    const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
    if (total == 0) return;
    for (int e0 = 0; e0 < total; e0 += kWave * kEdgeRounds) {
        int32_t u[kEdgeRounds], pr[kEdgeRounds];
        u64 b[kEdgeRounds], old[kEdgeRounds];
        bool ev[kEdgeRounds];
#pragma unroll
        for (int r = 0; r < kEdgeRounds; ++r) {
            const int e = e0 + r * kWave + lane, w0 = e0 + r * kWave;
            ev[r] = e < total;
            // Whose edge is edge e?  Every lane whose edges reach into this window of 64 marks the window position
            // where they begin (0: they began before it); the owners ascend with the position, so a running maximum
            // over the marks gives each position its owner.
            s_incl[lane] = 0;
            __builtin_amdgcn_wave_barrier();
            if (deg > 0 && incl > w0 && excl < w0 + kWave) s_incl[max(excl - w0, 0)] = lane + 1;
            __builtin_amdgcn_wave_barrier();
            const int owner = max(wave_incl_max(s_incl[lane]) - 1, 0);
            __builtin_amdgcn_wave_barrier();
            const int o_eb = __shfl(eb, owner, kWave);
            const int o_excl = __shfl(excl, owner, kWave);
            b[r] = shfl64(bits, owner);
            u[r] = ev[r] ? g.in_idx[o_eb + (e - o_excl)] : 0;
        }
#pragma unroll
        for (int r = 0; r < kEdgeRounds; ++r) {
            pr[r] = kNoProducer;
            old[r] = ~(u64)0;
            if (ev[r]) {
                old[r] = atomicOr(&mk.M[u[r]], b[r]);       // (I2)
                pr[r] = g.prod1[u[r]];                      // in flight together with the atomic (which goes first: the earlier it lands, the fewer pushes come late)
                lc.atomics++;
            }
        }
#pragma unroll
        for (int r = 0; r < kEdgeRounds; ++r) {
            if (e0 + r * kWave >= total) break;             // wave-uniform
            bool push = false, many = false;
            const bool first = ev[r] && old[r] == 0;
            if (ev[r] && (b[r] & ~old[r]) != 0) {           // (I3): u gained bits
                if (pr[r] >= 0) push = note_producer(pr[r], theta, mk.DB, lc);
                else many = pr[r] == kMulti;
            }
            stage_push(ws, push, pr[r], first, u[r], f);
            if (ballot64(many)) {                           // tensors with several producers: one round per producer rank
                int pb = 0, np = 0;
                if (many) { pb = g.prod_rowptr[u[r]]; np = g.prod_rowptr[u[r] + 1] - pb; }
                const int rounds = wave_max(np);
                for (int k = 0; k < rounds; ++k) {
                    int32_t op = 0;
                    bool p2 = false;
                    if (k < np) {
                        op = g.prod_idx[pb + k];
                        p2 = note_producer(op, theta, mk.DB, lc);
                    }
                    stage_push(ws, p2, op, false, 0, f);
                }
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// 64 operators held one per lane (valid lanes only): k = OR of M over the outputs of o; the bits K[o] did not
// have go to the inputs.  atomic_k: OR into K atomically (launches that process an operator in the launch that
// noted it, and the fix-up sweep); else K is read and written plainly (see the header).  Returns whether this
// lane's operator gained bits.
__device__ __forceinline__ bool process_ops(const GraphView &g, bool valid, int32_t o, int32_t theta, bool atomic_k,
                                            const Masks &mk, int *s_incl, WaveStage &ws, const Frontier &f,
                                            LevelCounters &lc)
{
    int4 r = make_int4(0, 0, 0, 0);
    u64 kold = 0, k = 0;
    if (valid) {
        r = g.orec[o];
        kold = load_coherent(&mk.K[o]);
        const int n_out = r.w >= 0 ? r.w : -r.w;
        // the masks of the first four outputs are fetched together
        u64 m0 = 0, m1 = 0, m2 = 0, m3 = 0;
        if (r.w >= 0) {
            if (n_out > 0) m0 = load_coherent(&mk.M[r.z]);
            if (n_out > 1) m1 = load_coherent(&mk.M[r.z + 1]);
            if (n_out > 2) m2 = load_coherent(&mk.M[r.z + 2]);
            if (n_out > 3) m3 = load_coherent(&mk.M[r.z + 3]);
            for (int j = 4; j < n_out; ++j) k |= load_coherent(&mk.M[r.z + j]);
        } else {
            const int32_t t0 = n_out > 0 ? g.out_idx[r.z] : 0, t1 = n_out > 1 ? g.out_idx[r.z + 1] : 0;
            const int32_t t2 = n_out > 2 ? g.out_idx[r.z + 2] : 0, t3 = n_out > 3 ? g.out_idx[r.z + 3] : 0;
            if (n_out > 0) m0 = load_coherent(&mk.M[t0]);
            if (n_out > 1) m1 = load_coherent(&mk.M[t1]);
            if (n_out > 2) m2 = load_coherent(&mk.M[t2]);
            if (n_out > 3) m3 = load_coherent(&mk.M[t3]);
            for (int j = 4; j < n_out; ++j) k |= load_coherent(&mk.M[g.out_idx[r.z + j]]);
        }
        k |= m0 | m1 | m2 | m3;
        lc.processed++;
    }
    const u64 nb = k & ~kold;                               // bits o did not have yet
    if (nb) {
        if (atomic_k) { atomicOr(&mk.K[o], k); lc.atomics++; }   // (I1)
        else store_coherent(&mk.K[o], kold | k);
        if (kold == 0) mk.flags[o] = 1;                     // o is kept
    }
    expand_edges(g, r.x, nb ? r.y : 0, nb, theta, mk, s_incl, ws, f, lc);
    return nb != 0;
}

// A level that expanded little is latency bound, not atomics bound: the threshold then takes two or
// four decay steps at once, trading a few repeated expansions for fewer such levels.
__device__ __forceinline__ int32_t next_theta(int32_t theta, const Schedule &sch, int expanded, int n_next,
                                              int max_deferred_key)
{
    if (theta <= 0) return 0;
    float base = (float)theta;
    if (expanded == 0 && n_next == 0 && max_deferred_key >= 0 && max_deferred_key + 1 < theta)
        base = (float)max_deferred_key + 1.0f;               // nothing to do above the highest deferred operator
    float d = sch.decay;
    if (expanded < sch.small_level) d *= d;
    if (expanded < sch.small_level / 8) d *= d;
    const int32_t t = (int32_t)(base * d);
    return t < sch.theta_floor ? 0 : t;
}

// ------------------------------------------------------------------------------------------------
// wide levels: one level per launch, the whole chip
//
// No block waits for another and nobody "closes" a level.  A launch leaves behind (a) a record: the
// state it started from, and whether it ran a level from there; (b) its tallies, spread over 64 words:
// pushes per queue segment, operators processed, largest deferred id.  Every block of the NEXT launch folds the
// two into the state it starts from -- a few dozen loads and a wave reduction, the same arithmetic in
// every block, so all blocks agree without talking to each other.  Records alternate between two slots
// and tallies between three buffers (written by launch e, read by e + 1, zeroed by e + 2), so nothing a
// launch reads is written during that launch.
// ------------------------------------------------------------------------------------------------
constexpr int kLevelThreads = 256;
constexpr int kLevelWaves = kLevelThreads / kWave;
constexpr int kThinPerWave = 8;                    // queue entries dealt to a wave, when the grid has the waves for it
constexpr int kMinChunkLog = 3;                    // a wave scans between 8 ...
constexpr int kMaxChunkLog = 12;                   // ... and 4096 marker bytes per step (64 per lane)
constexpr int kListCap = 16 * kWave;               // marked operators listed per wave before they are processed
constexpr int kChaseHops = 1;                      // hops a wave adds on its own in a launch ...
constexpr int kTailHops = 32;                      // ... and once the threshold has reached zero

struct LevelShared {
    int32_t stage[kLevelWaves][kStageCap];
    int32_t lstage[kLevelWaves][kLogStageCap];
    int incl[kLevelWaves][kWave];
    int32_t ops[kLevelWaves][kListCap];
    int pref[kMaxSeg + 1];
    int derived[3];         // operators processed, 1 + largest deferred id and atomics of the previous launch
    int tally[kLevelWaves][3];
};

// How one level's work is dealt to `grid` blocks.  Queue entries and range chunks go to different blocks, so that
// the two dependent-access chains of a level overlap and no wave does one after the other.
struct LevelPlan {
    int band_lo, band_hi;  // marker bytes of the operators [band_lo, band_hi) are read: the range [theta, theta_hi) that
                           // opens at this level, its lower end rounded down to a whole load
    int cs, lw_log, chunks;// the range is dealt to the waves in chunks of cs operators (8..4096), a lane reading
                           // 1 << lw_log marker bytes (cs <= 512: 1, 2, 4 or 8 and only cs >> lw_log lanes read; above: cs / 64):
                           // as small as the number of waves allows -- a range far down the graph is dense with marked
                           // operators, and a wave that finds 64 of them works through several hundred input edges while
                           // the rest of the chip idles -- and large enough that a wide, sparse range needs one step per wave
    int nb_e, nb_s;        // blocks that take the queue entries / the range chunks
    int nwork;             // blocks that have something to do
    int per_wave;          // the entries are dealt thinly, per_wave (8..64) to a wave: all the waves that the range leaves
                           // idle share them.  0: more entries than that; every wave then takes 64 at a time
    bool chase;            // (per_wave > 0) a wave then processes what it has just pushed itself, a second hop within the
                           // same launch
};

__device__ __forceinline__ LevelPlan plan_level(const LevelSlot &in, int n, bool ranges_left, int grid)
{
    LevelPlan p;
    p.band_lo = p.band_hi = p.chunks = 0;
    p.cs = 1 << kMinChunkLog;
    p.lw_log = 0;
    const int waves = grid * kLevelWaves;
    // no operator above the largest id noted so far is marked
    const int top = min(in.theta_hi, in.max_key1);
    if (ranges_left && top > in.theta) {
        // the waves that the queue entries leave over, but at least half of them
        const int reserve = (n + kThinPerWave - 1) / kThinPerWave;
        const int avail = max(waves - reserve, waves / 2);
        const int span = top - in.theta;
        int cs = max((span + avail) / avail, 1 << kMinChunkLog);            // > span / avail
        if (cs <= 512) {
            while ((kWave << p.lw_log) < cs) ++p.lw_log;
            cs = (cs + (1 << p.lw_log) - 1) & ~((1 << p.lw_log) - 1);
        } else {
            int lg = 10;
            while (lg < kMaxChunkLog && (1 << lg) < cs) ++lg;
            cs = 1 << lg;
            p.lw_log = lg - 6;
        }
        p.cs = cs;
        p.band_lo = in.theta & ~((1 << min(p.lw_log, 4)) - 1);
        p.band_hi = top;
        p.chunks = (p.band_hi - p.band_lo + cs - 1) / cs;
    }
    // (more chunks than waves: the waves loop.  The grid has at least two blocks: one is left for the entries)
    p.nb_s = min((p.chunks + kLevelWaves - 1) / kLevelWaves, grid - (n > 0 ? 1 : 0));
    const int room = (grid - p.nb_s) * kLevelWaves;                        // waves for the entries
    p.per_wave = 0;
    p.nb_e = 0;
    p.chase = false;
    if (n > 0) {
        const int per = max((n + room - 1) / room, kThinPerWave);
        if (per <= kWave) {
            p.per_wave = per;
            p.nb_e = (n + per * kLevelWaves - 1) / (per * kLevelWaves);
            p.chase = true;
        } else {
            p.nb_e = grid - p.nb_s;
        }
    }
    p.nwork = max(1, p.nb_e + p.nb_s);
    return p;
}

// bit j of the result = bit 0 of byte j of x (marker bytes are 0 or 1)
__device__ __forceinline__ uint32_t gather4(uint32_t x) { return ((x & 0x01010101u) * 0x01020408u) >> 24; }

// The work of block `blk` (< p.nwork) in one level: its share of the queue entries and of the newly opened
// operator range.  Adds the block's tallies to `tally`.
__device__ __forceinline__ void run_level(const GraphView &g, const LevelSlot &in, int n, const LevelPlan &p, int blk,
                                          const int32_t *qin, const QueueGeom &qg, const Frontier &f, const Masks &mk,
                                          LevelShared &sh, SegCounter *tally)
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const bool do_entries = blk < p.nb_e;
    const bool do_scan = !do_entries;
    const int e_blocks = p.nb_e, e_first = blk;
    const int s_blocks = p.nb_s, s_first = blk - p.nb_e;
    const bool atomic_k = p.chase;                          // the same in every block of the launch

    WaveStage ws{&sh.stage[wave][0], 0, 0, f.log ? &sh.lstage[wave][0] : nullptr, 0};
    LevelCounters lc{0, -1, 0};
    if (p.per_wave > 0) {
        if (do_entries) {
            const int i = (e_first * kLevelWaves + wave) * p.per_wave + lane;
            const bool valid = lane < p.per_wave && i < n;
            const int32_t o = valid ? load_item(qin, qg, sh.pref, i) : 0;
            process_ops(g, valid, o, in.theta, atomic_k, mk, &sh.incl[wave][0], ws, f, lc);
        }
    } else {
        for (int base = e_first * kLevelThreads; do_entries && base < n; base += e_blocks * kLevelThreads) {
            const int i = base + threadIdx.x;
            const bool valid = i < n;
            const int32_t o = valid ? load_item(qin, qg, sh.pref, i) : 0;
            process_ops(g, valid, o, in.theta, atomic_k, mk, &sh.incl[wave][0], ws, f, lc);
        }
    }
    // the marker bytes of the newly opened range, a chunk per step: every lane fetches its 1..64 bytes at once and
    // squeezes them into a bit mask; the marked operators are listed in LDS, sixteen bytes per lane at a time, and
    // processed 64 per step
    const int lw_log = p.lw_log, lw = 1 << lw_log;                          // marker bytes per lane
    const int lanes_on = min(p.cs >> lw_log, kWave);
    const int parts = max(lw >> 4, 1);                                      // 16-byte pieces per lane (1..4)
    const int64_t limit = ((int64_t)p.band_hi + 63) & ~(int64_t)63;         // the byte map is padded to whole 64s
    for (int c = s_first * kLevelWaves + wave; do_scan && c < p.chunks; c += s_blocks * kLevelWaves) {
        const int64_t c_lo = (int64_t)p.band_lo + (int64_t)c * p.cs;
        // Up to 8 bytes per lane: lane l looks at the lw operators from c_lo + l * lw on.  More: the chunk is taken in
        // pieces of 1024 operators, lane l looking at 16 of each, so that every load of the wave is one contiguous KiB.
        const int64_t op0 = lw >= 16 ? c_lo + lane * 16 : c_lo + ((int64_t)lane << lw_log);
        u64 bits = 0;                                       // piece p in bits [16 p, 16 p + 16)
        if (lw >= 16) {
            uint4 x[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                x[q] = make_uint4(0, 0, 0, 0);
                if (q < parts && op0 + q * 1024 < limit) x[q] = *reinterpret_cast<const uint4 *>(mk.DB + op0 + q * 1024);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (q >= parts) break;
                uint32_t b16 = gather4(x[q].x) | (gather4(x[q].y) << 4) | (gather4(x[q].z) << 8) | (gather4(x[q].w) << 12);
                // keep only ids in [theta, theta_hi)
                const int64_t lo_cut = in.theta - (op0 + q * 1024), hi_cut = in.theta_hi - (op0 + q * 1024);
                if (lo_cut > 0) b16 &= lo_cut >= 16 ? 0u : ~((1u << lo_cut) - 1u);
                if (hi_cut < 16) b16 &= hi_cut <= 0 ? 0u : (1u << hi_cut) - 1u;
                bits |= (u64)b16 << (16 * q);
            }
        } else if (lane < lanes_on && op0 < limit) {
            uint32_t b16;
            if (lw == 8) {
                const uint2 x = *reinterpret_cast<const uint2 *>(mk.DB + op0);
                b16 = gather4(x.x) | (gather4(x.y) << 4);
            } else if (lw == 4) {
                b16 = gather4(*reinterpret_cast<const uint32_t *>(mk.DB + op0));
            } else if (lw == 2) {
                b16 = gather4(*reinterpret_cast<const uint16_t *>(mk.DB + op0));
            } else {
                b16 = mk.DB[op0] & 1u;
            }
            const int64_t lo_cut = in.theta - op0, hi_cut = in.theta_hi - op0;
            if (lo_cut > 0) b16 &= lo_cut >= 16 ? 0u : ~((1u << lo_cut) - 1u);
            if (hi_cut < lw) b16 &= hi_cut <= 0 ? 0u : (1u << hi_cut) - 1u;
            bits = b16;
        }
        for (int part = 0; part < parts; ++part) {
            uint32_t bits16 = (uint32_t)(bits >> (16 * part)) & 0xffffu;
            const int cnt = __popc(bits16);
            const int incl = wave_incl_scan(cnt);
            const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
            if (total == 0) continue;                       // wave-uniform
            int pos = incl - cnt;
            const int32_t op_base = (int32_t)op0 + 1024 * part;
            while (bits16) {
                const int b = __builtin_ctz(bits16);
                bits16 &= bits16 - 1;
                sh.ops[wave][pos++] = op_base + b;
            }
            __builtin_amdgcn_wave_barrier();
            for (int i0 = 0; i0 < total; i0 += kWave) {
                const bool valid = i0 + lane < total;
                const int32_t o = valid ? sh.ops[wave][i0 + lane] : 0;
                process_ops(g, valid, o, in.theta, atomic_k, mk, &sh.incl[wave][0], ws, f, lc);
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    // A level is a chain of dependent accesses plus the fixed cost of a launch: the wave then processes what it has
    // just pushed itself, one more hop within this launch, and only what that hop pushes goes to memory (any order
    // reaches the same fixed point).  While the threshold comes down this keeps the late pushes -- producers inside
    // ranges that are open already -- from trailing through the following levels; once it is zero a hop done here
    // is a launch saved.
    if (p.chase) {
        const int hops = in.theta > 0 ? kChaseHops : kTailHops;
        for (int hop = 0; hop < hops; ++hop) {
            int gen_end = ws.tail;                          // the entries pushed so far: the next hop of this launch
            if (gen_end - ws.head <= 0) break;              // wave-uniform
            while (gen_end - ws.head > 0) {                 // wave-uniform (a flush empties the ring: head = tail)
                const int take = min(gen_end - ws.head, kWave);
                const bool valid = lane < take;
                const int32_t o = valid ? ws.buf[(ws.head + lane) & (kStageCap - 1)] : 0;
                ws.head += take;
                __builtin_amdgcn_wave_barrier();
                process_ops(g, valid, o, in.theta, atomic_k, mk, &sh.incl[wave][0], ws, f, lc);
                if (ws.head > gen_end) gen_end = ws.head;   // the ring was flushed under us: nothing of this hop is left
            }
        }
    }
    flush_both(ws, f);
    // the block's tallies go to one of 64 spread words; nobody waits for them
    const int wproc = wave_sum(lc.processed), wkey = wave_max(lc.max_deferred_key), wat = wave_sum(lc.atomics);
    if (lane == 0) {
        sh.tally[wave][0] = wproc;
        sh.tally[wave][1] = wkey;
        sh.tally[wave][2] = wat;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int bproc = 0, bkey = -1, bat = 0;
#pragma unroll
        for (int w = 0; w < kLevelWaves; ++w) {
            bproc += sh.tally[w][0];
            bkey = max(bkey, sh.tally[w][1]);
            bat += sh.tally[w][2];
        }
        const int word = blk & (kMaxSeg - 1);
        if (bproc | bat)
            atomicAdd(reinterpret_cast<unsigned long long *>(&tally[word].proc), (u64)(uint32_t)bproc | ((u64)(uint32_t)bat << 32));
        if (bkey >= 0) atomicMax(&tally[word].key1, bkey + 1);
    }
}

// The state a launch starts from, derived by every block on its own from the record of the previous
// launch and, if that launch ran a level, from its tallies.  Whole block; fills s_pref (prefix sums of
// the queue's segment counts).  prev = tallies buffer of the previous launch.
__device__ __forceinline__ LevelSlot derive_state(const TravState *st, const TravCounters *ctr, int launch_no,
                                                  const QueueGeom &qg, const Schedule &sch, int *s_pref, int *s_derived,
                                                  int *tot_proc_out)
{
    const int prev = (launch_no + 2) % 3;
    const LevelSlot rec = st->slot[(launch_no + 1) & 1];
    if (threadIdx.x < kWave) {
        const int lane = lane_id();
        const SegCounter *tally = &ctr->cnt[prev][lane];     // written by the previous launch: plain loads will do
        int c = 0;
        if (lane < qg.S) c = min(tally->v, qg.seg_cap);
        const int pr = tally->proc;
        const int mk = tally->key1;
        const int at = tally->atomics;
        const int incl = wave_incl_scan(c);
        if (lane == 0) s_pref[0] = 0;
        s_pref[lane + 1] = incl;
        const int tot = wave_sum(pr), key1 = wave_max(mk), tat = wave_sum(at);
        if (lane == 0) { s_derived[0] = tot; s_derived[1] = key1; s_derived[2] = tat; }
    }
    __syncthreads();
    LevelSlot s = rec;
    s.worked = 0;
    s.n = s_pref[kMaxSeg];
    *tot_proc_out = 0;
    if (rec.worked) {                                       // fold the level the previous launch ran into the state
        const int tot_proc = s_derived[0];
        const int key1 = max(rec.max_key1, s_derived[1]);
        const bool ranges_left = rec.deferred_seen && rec.theta_hi > 0;
        s.level = rec.level + 1;
        s.max_key1 = key1;
        s.deferred_seen = key1 > 0;
        s.theta_hi = ranges_left ? rec.theta : rec.theta_hi;               // [theta, theta_hi) has been scanned
        s.theta = (ranges_left || key1 > 0) ? next_theta(rec.theta, sch, tot_proc, s.n, key1 - 1) : rec.theta;
        *tot_proc_out = tot_proc;
    }
    return s;
}

// One thread per launch keeps the books: the record of this launch, running totals, the level trace; one
// wave clears the tallies buffer of the NEXT launch (last read by the previous one).  works: this launch
// runs a wide level; small: the state it starts from is one the single-workgroup kernel takes (or final).
__device__ __forceinline__ void keep_books(TravState *st, TravCounters *ctr, int launch_no, const LevelSlot &prev_rec,
                                           const LevelSlot &now, bool works, bool small, int tot_proc, int tot_atomics, int4 *trace)
{
    const int lane = lane_id();
    const int nxt = (launch_no + 1) % 3;
    ctr->cnt[nxt][lane].v = 0;
    ctr->cnt[nxt][lane].proc = 0;
    ctr->cnt[nxt][lane].key1 = 0;
    ctr->cnt[nxt][lane].atomics = 0;
    if (lane == 0) {
        LevelSlot rec = now;
        rec.worked = works ? 1 : 0;
        st->slot[launch_no & 1] = rec;
        if (prev_rec.worked) {
            st->tensor_visits += (u64)tot_proc;
            st->atomic_updates += (u64)tot_atomics;
            if ((u64)prev_rec.n > st->max_frontier) st->max_frontier = (u64)prev_rec.n;
            if (trace && prev_rec.level < kTraceLevels)
                trace[prev_rec.level] = make_int4(prev_rec.n, tot_proc, prev_rec.theta, (int)(uint32_t)wall_clock64());
        }
        // lengths of the stretches of wide levels, for the host to lay out the launches of the next prune
        if (works) {
            st->run_len++;
        } else if (small && st->run_len > 0) {
            if (st->n_runs < kMaxRuns) st->wide_runs[st->n_runs] = st->run_len;
            st->n_runs++;
            st->run_len = 0;
        }
    }
}

// The queue is handed to the next launch untouched: its segment counts move into this launch's tallies.
__device__ __forceinline__ void hand_on_frontier(TravCounters *ctr, int launch_no, const int *s_pref)
{
    const int lane = lane_id();
    ctr->cnt[launch_no % 3][lane].v = s_pref[lane + 1] - s_pref[lane];
}

__global__ __launch_bounds__(kLevelThreads) void k_level(GraphView g, TravState *st, TravCounters *ctr, int launch_no,
                                                          int32_t *q0, int32_t *q1, QueueGeom qg, Masks mk,
                                                          int narrow_cap, Schedule sch, ColourLog log, int4 *trace)
{
    __shared__ LevelShared sh;
    const int wave = threadIdx.x >> 6;
    const LevelSlot prev_rec = st->slot[(launch_no + 1) & 1];
    int tot_proc = 0;
    const LevelSlot in = derive_state(st, ctr, launch_no, qg, sch, sh.pref, sh.derived, &tot_proc);
    const int n = in.n;
    const bool ranges_left = in.deferred_seen && in.theta_hi > 0;
    // finished, or small enough for the single-workgroup kernel: nothing to do but to pass things on
    const bool works = !(n <= narrow_cap && !ranges_left);
    if (blockIdx.x == 0 && threadIdx.x < kWave) {
        keep_books(st, ctr, launch_no, prev_rec, in, works, !works, tot_proc, sh.derived[2], trace);
        if (!works) hand_on_frontier(ctr, launch_no, sh.pref);
    }
    if (!works) return;
    const LevelPlan p = plan_level(in, n, ranges_left, (int)gridDim.x);
    if ((int)blockIdx.x >= p.nwork) return;

    const int cur = in.level & 1;
    const int32_t *qin = cur ? q1 : q0;
    int32_t *qout = cur ? q0 : q1;
    const int mine = launch_no % 3;
    const int seg = (blockIdx.x * kLevelWaves + wave) & (qg.S - 1);
    const int lseg = (blockIdx.x * kLevelWaves + wave) & (kMaxSeg - 1);
    const Frontier f{qout + (int64_t)seg * qg.seg_cap, &ctr->cnt[mine][seg].v, qg.seg_cap, &st->error,
                     log.entries ? log.entries + (int64_t)lseg * log.seg_cap : nullptr, &log.cnt[lseg].v, log.seg_cap,
                     nullptr, 0};
    run_level(g, in, n, p, (int)blockIdx.x, qin, qg, f, mk, sh, ctr->cnt[mine]);
}

hipError_t launch_level(const GraphView &g, TravState *st, TravCounters *ctr, int launch_no, int32_t *q0, int32_t *q1,
                        const QueueGeom &qg, uint8_t *DB, uint8_t *flags, u64 *M, u64 *K, int grid_blocks, int narrow_cap,
                        const Schedule &sch, const ColourLog &log, int4 *trace, hipStream_t s)
{
    if (grid_blocks < 2) grid_blocks = 2;                   // entries and range chunks go to different blocks
    hipLaunchKernelGGL(k_level, dim3((unsigned)grid_blocks), dim3(kLevelThreads), 0, s, g, st, ctr, launch_no, q0, q1,
                       qg, Masks{M, K, DB, flags}, narrow_cap, sch, log, trace);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// narrow levels: one workgroup walks level after level while the queue is small, with workgroup
// barriers instead of kernel launches (deep graphs have hundreds of small levels)
// ------------------------------------------------------------------------------------------------
constexpr int kNarrowThreads = 1024;
constexpr int kNarrowWaves = kNarrowThreads / kWave;
constexpr int kNarrowFront = 1024;      // entries of a queue that the kernel also keeps in LDS

__global__ __launch_bounds__(kNarrowThreads) void k_narrow(GraphView g, TravState *st, TravCounters *ctr, int launch_no,
                                                            int32_t *q0, int32_t *q1, QueueGeom qg, Masks mk,
                                                            int narrow_cap, Schedule sch, ColourLog log, int4 *trace)
{
    __shared__ int32_t s_stage[kNarrowWaves][kStageCap];
    __shared__ int32_t s_lstage[kNarrowWaves][kLogStageCap];
    __shared__ int s_incl[kNarrowWaves][kWave];
    __shared__ int s_pref[kMaxSeg + 1];
    __shared__ int s_derived[3];
    __shared__ int s_nout;
    // The queue a level builds is also kept here: the next level -- at most kNarrowFront entries, or this
    // kernel does not run it -- takes it from LDS and need not wait for its own queue stores to reach memory.
    __shared__ int32_t s_front[2][kNarrowFront];

    const LevelSlot prev_rec = st->slot[(launch_no + 1) & 1];
    int tot_proc = 0;
    LevelSlot in = derive_state(st, ctr, launch_no, qg, sch, s_pref, s_derived, &tot_proc);
    const bool use_mirror = narrow_cap <= kNarrowFront;
    bool from_lds = false;
    int level = in.level;
    int n = in.n;
    const bool ranges_left = in.deferred_seen && in.theta_hi > 0;   // then the wide kernel must go on
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    WaveStage ws{&s_stage[wave][0], 0, 0, log.entries ? &s_lstage[wave][0] : nullptr, 0};
    LevelCounters lc{0, -1, 0};
    u64 visits = 0, maxf = 0;
    while (n > 0 && n <= narrow_cap && !ranges_left) {
        if (threadIdx.x == 0) s_nout = 0;
        __syncthreads();
        const int cur = level & 1;
        const int32_t *qin = cur ? q1 : q0;
        const Frontier f{cur ? q0 : q1, &s_nout, qg.seg_cap, &st->error,    // everything goes to segment 0
                         log.entries ? log.entries + (int64_t)wave * log.seg_cap : nullptr, &log.cnt[wave].v,
                         log.seg_cap, use_mirror ? &s_front[cur ^ 1][0] : nullptr, use_mirror ? kNarrowFront : 0};
        for (int base = 0; base < n; base += kNarrowThreads) {
            const int i = base + threadIdx.x;
            const bool valid = i < n;
            const int32_t o = !valid ? 0 : from_lds ? s_front[cur][i] : load_item(qin, qg, s_pref, i);
            // threshold 0: a small queue is latency bound, so nothing is gained by deferring.  What a level notes
            // is processed by the next one, behind a barrier: plain reads and writes of K will do (see the header)
            process_ops(g, valid, o, 0, false, mk, &s_incl[wave][0], ws, f, lc);
        }
        flush_entries(ws, f);
        // the block's stores (K, and without the copy in LDS the queue) must have completed before other waves of this
        // same block read them; no other block reads them before the kernel ends
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        visits += (u64)n;
        if ((u64)n > maxf) maxf = (u64)n;
        if (trace && threadIdx.x == 0 && level < kTraceLevels) trace[level] = make_int4(n, n, -1, (int)(uint32_t)wall_clock64());
        n = min(s_nout, qg.seg_cap);
        ++level;
        from_lds = use_mirror;
        // the next queue lives in segment 0 only
        if (threadIdx.x <= kMaxSeg) s_pref[threadIdx.x] = threadIdx.x == 0 ? 0 : n;
        __syncthreads();          // everyone has read s_nout before it is reset; s_pref is in place
    }
    if (log.entries) {
        const Frontier lf{nullptr, nullptr, 0, &st->error, log.entries + (int64_t)wave * log.seg_cap, &log.cnt[wave].v,
                          log.seg_cap, nullptr, 0};
        flush_log(ws, lf);
    }
    {
        const int wat = wave_sum(lc.atomics);
        if (lane == 0 && wat) atomicAdd(&st->atomic_updates, (u64)wat);
    }
    // This launch leaves no tallies to fold: its record IS the state after it.  The queue it ends with
    // (untouched, or the one it built in segment 0) goes to the next launch through this launch's counters.
    if (threadIdx.x < kWave) {
        keep_books(st, ctr, launch_no, prev_rec, in, false, in.n <= narrow_cap && !ranges_left, tot_proc, s_derived[2], trace);
        hand_on_frontier(ctr, launch_no, s_pref);
        if (lane == 0) {
            LevelSlot *rec = &st->slot[launch_no & 1];
            rec->level = level;
            rec->n = n;
            st->tensor_visits += visits;
            if (maxf > st->max_frontier) st->max_frontier = maxf;
        }
    }
}

hipError_t launch_narrow(const GraphView &g, TravState *st, TravCounters *ctr, int launch_no, int32_t *q0, int32_t *q1,
                         const QueueGeom &qg, uint8_t *DB, uint8_t *flags, u64 *M, u64 *K, int narrow_cap, const Schedule &sch,
                         const ColourLog &log, int4 *trace, hipStream_t s)
{
    hipLaunchKernelGGL(k_narrow, dim3(1), dim3(kNarrowThreads), 0, s, g, st, ctr, launch_no, q0, q1, qg,
                       Masks{M, K, DB, flags}, narrow_cap, sch, log, trace);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// fix-up sweep (only after a queue overflowed): every operator re-derives K from its outputs
// and pushes what is new to its inputs; repeated by the host until a sweep changes nothing
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kLevelThreads) void k_fix_sweep(GraphView g, Masks mk, int32_t *changed)
{
    __shared__ int32_t s_stage[kLevelWaves][kStageCap];
    __shared__ int s_incl[kLevelWaves][kWave];
    __shared__ int32_t s_sink, s_err;
    const int wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) { s_sink = 0; s_err = 0; }
    __syncthreads();
    WaveStage ws{&s_stage[wave][0], 0, 0, nullptr, 0};
    const Frontier f{nullptr, &s_sink, 0, &s_err, nullptr, nullptr, 0, nullptr, 0};   // capacity 0: pushes are counted and dropped
    LevelCounters lc{0, -1, 0};
    bool any = false;
    // descending ids: most of a sweep then sees its consumers' results (ids are a topological order).  Operators
    // are processed while their consumers still push, in no order between blocks: K by atomic ORs, threshold 0.
    const int64_t tiles = ((int64_t)g.num_ops + kLevelThreads - 1) / kLevelThreads;
    for (int64_t tile = tiles - 1 - blockIdx.x; tile >= 0; tile -= gridDim.x) {
        const int64_t o = tile * kLevelThreads + threadIdx.x;
        const bool valid = o < g.num_ops;
        any |= process_ops(g, valid, valid ? (int32_t)o : 0, 0, true, mk, &s_incl[wave][0], ws, f, lc);
        ws.head = ws.tail;
    }
    if (ballot64(any) != 0 && lane_id() == 0) atomicOr(changed, 1);
}

hipError_t launch_fix_sweep(const GraphView &g, u64 *M, u64 *K, uint8_t *flags, int32_t *changed, int grid_blocks, hipStream_t s)
{
    if (g.num_ops == 0) return hipSuccess;
    hipLaunchKernelGGL(k_fix_sweep, dim3((unsigned)grid_blocks), dim3(kLevelThreads), 0, s, g, Masks{M, K, nullptr, flags}, changed);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// per-graph descending sweep (packed batches of small graphs, operator ids topological)
//
// A tensor's consumers all have larger operator ids than its producer.  One wave walks one graph's
// operators from the highest id down, 64 at a time, so when a group is reached every consumer outside
// the group has already been handled.  Nothing of the graph's M is shared with another wave, which
// allows a scheme without a single global atomic (the atomic version ran at the chip's atomic rate:
// 75 M pushes at about 20 G/s):
//   - what consumers push to a tensor whose producer has not been reached yet is gathered in a hash table
//     in LDS ("pending"); the producer's group takes it from there, ORs it with the tensor's word in
//     memory (its seed bits), and WRITES the tensor's final M with a plain store;
//   - dependencies inside the group are resolved in LDS and registers: the group's output tensors go
//     into a second small table; an input edge that finds its tensor there registers its lane with the
//     producer's lane, the masks are then relaxed (every lane ORs in the masks of the lanes that read its
//     outputs, all lanes at once, until nothing changes), and the pushes to in-group tensors go to that
//     table's accumulators;
//   - when the pending table fills up it is written to memory (plain read-modify-write: its keys are
//     distinct) and emptied; a later producer finds those bits in the tensor's word.
// Loads and stores of M are ordinary cached ones: only this wave touches these words during the kernel.
// Row bounds and edge targets do not depend on M and are fetched one and two groups ahead, and M of a
// group's first two outputs at the end of the group before it (behind that group's flush of the pending
// table), so a group's critical path is: resolve, store.  The stores need no waiting for while every
// tensor has one producer; the graph build says whether some tensor of the batch has several.
// Each operator is expanded once with all 64 sets' bits (a level-synchronous traversal revisits the
// operators of such deep, thin graphs tens of times) and nothing is queued.  A group with too many
// edges for the tables, or with a tensor written twice inside the group, is walked one operator at a time.
// ------------------------------------------------------------------------------------------------
constexpr int kSweepThreads = 256;
constexpr int kOutSlots = 256;                      // table of the group's output tensors
constexpr int kOutMax = kOutSlots * 3 / 4;
constexpr int kPendSlots = 512;                     // pending pushes, kept across groups
constexpr int kPendMax = kPendSlots / 2;
constexpr int kInMax = 256;                         // input edges of a group handled through the tables
constexpr int kSweepDeps = 8;                       // in-group consumers per operator handled by the relaxation
static_assert(kSweepDeps == 8, "a lane's consumers are read as one 64-bit word");

struct SweepShared {
    int32_t okey[kOutSlots];                        // tensor id, -1 = empty
    u64 oacc[kOutSlots];                            // M of that tensor as far as known
    uint8_t oowner[kOutSlots];                      // lane of the operator that writes the tensor
    int32_t pkey[kPendSlots];
    u64 pval[kPendSlots];
    int ndep[kWave];                                // per lane: in-group consumers of its operator's outputs ...
    alignas(8) uint8_t dep[kWave][kSweepDeps];      // ... and the first few of them (their lanes)
};

__device__ __forceinline__ int out_slot_of(int32_t t) { return (int)(((uint32_t)t * 0x9E3779B1u) >> 24); }
__device__ __forceinline__ int pend_slot_of(int32_t t) { return (int)(((uint32_t)t * 0x9E3779B1u) >> 23); }

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// every earlier store of this wave has reached the cache that its later loads read
__device__ __forceinline__ void wave_stores_done()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__device__ __forceinline__ u64 readlane64(u64 v, int l)     // l wave-uniform
{
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((u64)hi << 32) | lo;
}

// position of tensor t in the table of output tensors, or -1.  span > 0: the group's outputs are the `span`
// consecutive tensors from `first` on (operators that number their outputs as they create them), and the table is
// indexed by t - first: nothing to look up.
__device__ __forceinline__ int find_out(const SweepShared &sh, int32_t t, int32_t first, int span)
{
    if (span > 0) return (uint32_t)(t - first) < (uint32_t)span ? t - first : -1;      // wave-uniform branch
    for (int slot = out_slot_of(t);; slot = (slot + 1) & (kOutSlots - 1)) {
        const int32_t key = sh.okey[slot];
        if (key == t) return slot;
        if (key == -1) return -1;
    }
}

// writes the pending pushes to memory and empties the table (keys are distinct: plain read-modify-write)
__device__ __forceinline__ void flush_pending(SweepShared &sh, u64 *M)
{
    wave_lds_sync();
    for (int i = lane_id(); i < kPendSlots; i += kWave) {
        const int32_t key = sh.pkey[i];
        if (key != -1) {
            const u64 v = sh.pval[i];
            if (v) M[key] |= v;
            sh.pkey[i] = -1;
            sh.pval[i] = 0;
        }
    }
    wave_lds_sync();
    wave_stores_done();
}

// Row bounds and the first few edge targets of one lane's operator.  The bounds are kept as loaded (no
// arithmetic on them where they are fetched, and no branch around the loads: lanes past the graph's first
// operator read its row instead), so that nothing waits for them before the group that uses them.
struct SweepRow {
    int ob, oe, ib, ie;
    int32_t to[2], ti[4];
};

__device__ __forceinline__ SweepRow sweep_row_bounds(const GraphView &g, int64_t o, int64_t o_lo)
{
    const int64_t oc = o >= o_lo ? o : o_lo;
    SweepRow r{};
    r.ob = g.out_rowptr[oc];
    r.oe = g.out_rowptr[oc + 1];
    r.ib = g.in_rowptr[oc];
    r.ie = g.in_rowptr[oc + 1];
    return r;
}

__device__ __forceinline__ void sweep_row_targets(const GraphView &g, SweepRow &r, bool valid)
{
    const int n_out = valid ? r.oe - r.ob : 0, n_in = valid ? r.ie - r.ib : 0;
#pragma unroll
    for (int j = 0; j < 2; ++j) r.to[j] = j < n_out ? g.out_idx[r.ob + j] : -1;
#pragma unroll
    for (int j = 0; j < 4; ++j) r.ti[j] = j < n_in ? g.in_idx[r.ib + j] : -1;
}

__device__ __forceinline__ int32_t sweep_out(const GraphView &g, const SweepRow &r, int j)
{
    return j == 0 ? r.to[0] : j == 1 ? r.to[1] : g.out_idx[r.ob + j];
}

__device__ __forceinline__ int32_t sweep_in(const GraphView &g, const SweepRow &r, int j)
{
    return j == 0 ? r.ti[0] : j == 1 ? r.ti[1] : j == 2 ? r.ti[2] : j == 3 ? r.ti[3] : g.in_idx[r.ib + j];
}

// Per-set counts of one graph without a transpose per group: every lane counts, for its own
// operators, how often each of the 64 bits was set, in bit-sliced form (plane i holds bit i of all
// 64 counters).  Four masks are folded at a time with full adders; only the resulting carry of
// weight 4 ripples through the higher planes.
constexpr int kCountPlanes = 13;                    // counters up to 2^13 - 1 groups of one graph

struct SlicedCount {
    u64 plane[kCountPlanes];
    u64 x0, x1, x2;                                 // masks waiting for the fourth
};

__device__ __forceinline__ void full_add(u64 a, u64 b, u64 c, u64 &sum, u64 &carry)
{
    const u64 ab = a ^ b;
    sum = ab ^ c;
    carry = (ab & c) | (a & b);
}

__device__ __forceinline__ void sliced_fold(SlicedCount &c, u64 x3, int planes_used)
{
    u64 s, ca, cb, cc;
    full_add(c.plane[0], c.x0, c.x1, s, ca);
    full_add(s, c.x2, x3, c.plane[0], cb);
    full_add(c.plane[1], ca, cb, c.plane[1], cc);
#pragma unroll
    for (int i = 2; i < kCountPlanes; ++i) {
        if (i < planes_used) {                      // wave-uniform
            const u64 t = c.plane[i] & cc;
            c.plane[i] ^= cc;
            cc = t;
        }
    }
}

__global__ __launch_bounds__(kSweepThreads) void k_sweep_graphs(GraphView g, u64 *M, u64 *K, int64_t *pq, int multi_producer)
{
    __shared__ SweepShared s_all[kSweepThreads / kWave];
    SweepShared &sh = s_all[threadIdx.x >> 6];
    const int lane = lane_id();
    const int gi = blockIdx.x * (kSweepThreads / kWave) + (threadIdx.x >> 6);
    if (gi >= g.num_graphs) return;                          // wave-uniform
    const int64_t o_lo = g.op_off[gi], o_hi = g.op_off[gi + 1];
    if (o_hi <= o_lo) {                                      // a graph without operators
        if (pq) pq[(int64_t)gi * 64 + lane] = 0;
        return;
    }
    const int n_groups = (int)((o_hi - o_lo + kWave - 1) / kWave);
    const int planes_used = 33 - __builtin_clz((unsigned)n_groups | 1u);   // bit length of n_groups, plus one
    SlicedCount cnt;
#pragma unroll
    for (int i = 0; i < kCountPlanes; ++i) cnt.plane[i] = 0;
    cnt.x0 = cnt.x1 = cnt.x2 = 0;
    for (int i = lane; i < kPendSlots; i += kWave) {
        sh.pkey[i] = -1;
        sh.pval[i] = 0;
    }
    int pending = 0;                                         // occupied slots of the pending table (wave-uniform)
    int group = 0;
    SweepRow cur = sweep_row_bounds(g, o_hi - 1 - lane, o_lo);
    sweep_row_targets(g, cur, o_hi - 1 - lane >= o_lo);
    SweepRow nxt = sweep_row_bounds(g, o_hi - kWave - 1 - lane, o_lo);
    // M of a group's first two outputs is fetched while the group before it is worked on
    u64 m_ahead0 = 0, m_ahead1 = 0;
    if (o_hi - 1 - lane >= o_lo) {
        if (cur.oe - cur.ob > 0) m_ahead0 = M[cur.to[0]];
        if (cur.oe - cur.ob > 1) m_ahead1 = M[cur.to[1]];
    }
    for (int64_t top = o_hi; top > o_lo; top -= kWave, ++group) {
        const int64_t o = top - 1 - lane;                    // lane 0 holds the highest id of the group
        const bool valid = o >= o_lo;
        const SweepRow row = cur;
        const u64 m_row0 = m_ahead0, m_row1 = m_ahead1;
        const int n_out = valid ? row.oe - row.ob : 0, n_in = valid ? row.ie - row.ib : 0;
        const int max_out = wave_max(n_out), max_in = wave_max(n_in);
        const int total_in = wave_sum(n_in);
        const int total_out = wave_sum(n_out);
        bool tables = total_out <= kOutMax && total_in <= kInMax;
        // Are the group's outputs one run of consecutive tensors, each written once?  (No tensor of the batch has two
        // producers, and the smallest and the largest id are as far apart as there are outputs.)
        int32_t first_out = 0;
        int span = 0;
        if (tables && !multi_producer && total_out > 0) {
            int32_t lo_t = 0x7fffffff, hi_t = -1;
            for (int r = 0; r < max_out; ++r) {
                if (r < n_out) {
                    const int32_t t = sweep_out(g, row, r);
                    lo_t = min(lo_t, t);
                    hi_t = max(hi_t, t);
                }
            }
            const int32_t glo = -wave_max(-lo_t), ghi = wave_max(hi_t);
            if (ghi - glo + 1 == total_out) { first_out = glo; span = total_out; }
        }
        if (tables && span > 0) {                            // the table is indexed by tensor: only the owners to note
            sh.ndep[lane] = 0;
            for (int r = 0; r < max_out; ++r)
                if (r < n_out) sh.oowner[sweep_out(g, row, r) - first_out] = (uint8_t)lane;
        } else if (tables) {                                 // the group's output tensors and who writes them
            for (int i = lane; i < kOutSlots; i += kWave) sh.okey[i] = -1;
            sh.ndep[lane] = 0;
            wave_lds_sync();
            bool twice = false;
            for (int r = 0; r < max_out; ++r) {
                if (r < n_out) {
                    const int32_t t = sweep_out(g, row, r);
                    for (int slot = out_slot_of(t);; slot = (slot + 1) & (kOutSlots - 1)) {
                        const int32_t old = atomicCAS(&sh.okey[slot], -1, t);
                        if (old == -1) { sh.oowner[slot] = (uint8_t)lane; break; }
                        if (old == t) { twice = true; break; }
                    }
                }
            }
            if (ballot64(twice) != 0) tables = false;        // a tensor written twice inside the group
        }
        // Fetch ahead, here where the wait for this group's own targets is over: targets of the next group (its
        // row bounds arrived with them), row bounds of the one after.
        sweep_row_targets(g, nxt, o - kWave >= o_lo);
        const SweepRow nxt2 = sweep_row_bounds(g, o - 2 * kWave, o_lo);
        u64 k = 0;
        if (tables) {
            wave_lds_sync();
            // the tensor's word in memory (seed bits, flushed pushes: fetched at the end of the previous
            // group, behind its flush) plus what is pending for it
            for (int r = 0; r < max_out; ++r) {
                if (r < n_out) {
                    const int32_t t = sweep_out(g, row, r);
                    u64 m = r == 0 ? m_row0 : r == 1 ? m_row1 : M[t];
                    for (int slot = pend_slot_of(t);; slot = (slot + 1) & (kPendSlots - 1)) {
                        const int32_t key = sh.pkey[slot];
                        if (key == -1) break;
                        if (key == t) {
                            m |= sh.pval[slot];
                            sh.pval[slot] = 0;               // taken: a later flush has nothing to write for it
                            break;
                        }
                    }
                    sh.oacc[find_out(sh, t, first_out, span)] = m;
                    k |= m;
                }
            }
            // in-group consumers register with the lane that writes the tensor they read
            u64 feeds = 0;
            for (int r = 0; r < max_in; ++r) {
                if (r < n_in) {
                    const int slot = find_out(sh, sweep_in(g, row, r), first_out, span);
                    if (slot >= 0) {
                        const int b = sh.oowner[slot];
                        if (b > lane && !((feeds >> b) & 1)) {       // first time this lane meets producer b
                            feeds |= (u64)1 << b;
                            const int at = atomicAdd(&sh.ndep[b], 1);
                            if (at < kSweepDeps) sh.dep[b][at] = (uint8_t)lane;
                        }
                    }
                }
            }
            wave_lds_sync();
            const int nd = sh.ndep[lane];
            const int max_nd = wave_max(nd);
            if (max_nd <= kSweepDeps) {
                // Relaxation: as many steps as the longest dependency chain inside the group.
                int d[kSweepDeps];
                const u64 row_of_deps = *reinterpret_cast<const u64 *>(&sh.dep[lane][0]);     // all eight in one read
#pragma unroll
                for (int j = 0; j < kSweepDeps; ++j) d[j] = j < nd ? (int)((row_of_deps >> (8 * j)) & 0xFF) : lane;
                for (int it = 0; it < kWave; ++it) {
                    u64 add = 0;
#pragma unroll
                    for (int j = 0; j < kSweepDeps; ++j)
                        if (j < max_nd) add |= shfl64(k, d[j]);      // wave-uniform bound; own lane when unused
                    const bool grew = (add & ~k) != 0;
                    k |= add;
                    if (ballot64(grew) == 0) break;
                }
            } else {
                u64 live = ballot64(feeds != 0);
                while (live) {                               // ascending lanes = descending operator ids
                    const int src = __builtin_ctzll(live);
                    live &= live - 1;
                    const u64 ks = readlane64(k, src);       // final: every lane that feeds lane src came earlier
                    if (ks == 0) continue;
                    if (__builtin_amdgcn_inverse_ballot_w64(readlane64(feeds, src))) k |= ks;
                }
            }
            // pushes: to the group's own tensors in their accumulators, to all others in the pending table
            int fresh_keys = 0;
            for (int r = 0; r < max_in; ++r) {
                if (r < n_in && k) {
                    const int32_t t = sweep_in(g, row, r);
                    const int os = find_out(sh, t, first_out, span);
                    if (os >= 0) {
                        atomicOr(&sh.oacc[os], k);
                    } else {
                        int slot = pend_slot_of(t);
                        for (;; slot = (slot + 1) & (kPendSlots - 1)) {
                            const int32_t old = atomicCAS(&sh.pkey[slot], -1, t);
                            if (old == -1) { ++fresh_keys; break; }
                            if (old == t) break;
                        }
                        atomicOr(&sh.pval[slot], k);
                    }
                }
            }
            pending += wave_sum(fresh_keys);
            wave_lds_sync();
            for (int r = 0; r < max_out; ++r)                // the group's tensors are final
                if (r < n_out) {
                    const int32_t t = sweep_out(g, row, r);
                    M[t] = sh.oacc[find_out(sh, t, first_out, span)];
                }
            wave_lds_sync();
        } else {
            // One operator at a time, its edges spread over the lanes.  Pushes go straight to memory with
            // plain read-modify-writes: lanes that meet the same tensor write the same value.
            if (pending) {
                flush_pending(sh, M);
                pending = 0;
            }
            const int n_valid = (int)min((int64_t)kWave, top - o_lo);
            for (int src = 0; src < n_valid; ++src) {
                wave_stores_done();
                const int s_ob = __shfl(row.ob, src, kWave), s_no = __shfl(n_out, src, kWave);
                const int s_ib = __shfl(row.ib, src, kWave), s_ni = __shfl(n_in, src, kWave);
                u64 part = 0;
                for (int e = lane; e < s_no; e += kWave) part |= M[g.out_idx[s_ob + e]];
                const u64 ks = wave_or(part);
                if (lane == src) k = ks;
                if (ks)
                    for (int e = lane; e < s_ni; e += kWave) M[g.in_idx[s_ib + e]] |= ks;
            }
            wave_stores_done();
        }
        if (valid) K[o] = k;
        cur = nxt;
        nxt = nxt2;
        // Room in the pending table for everything the next group may push.  The words of M that the next
        // group reads are fetched behind this flush, so they hold what it wrote; the stores of finished
        // groups need no waiting for, because a tensor with one producer is never read again -- with
        // several producers somewhere in the batch every group waits for them.
        const bool valid_next = o - kWave >= o_lo;
        if (pending + wave_sum(valid_next ? cur.ie - cur.ib : 0) > kPendMax) {
            flush_pending(sh, M);
            pending = 0;
        } else if (multi_producer) {
            wave_stores_done();
        }
        m_ahead0 = m_ahead1 = 0;
        if (valid_next) {
            if (cur.oe - cur.ob > 0) m_ahead0 = M[cur.to[0]];
            if (cur.oe - cur.ob > 1) m_ahead1 = M[cur.to[1]];
        }
        if (pq) {
            switch (group & 3) {                             // wave-uniform
            case 0: cnt.x0 = k; break;
            case 1: cnt.x1 = k; break;
            case 2: cnt.x2 = k; break;
            default: sliced_fold(cnt, k, planes_used); break;
            }
        }
    }
    flush_pending(sh, M);                                    // tensors no operator of the graph writes (its inputs)
    if (pq) {
        if (group & 3) {                                     // masks still waiting: fold them with zeros for the rest
            if ((group & 3) < 3) cnt.x2 = 0;
            if ((group & 3) < 2) cnt.x1 = 0;
            sliced_fold(cnt, 0, planes_used);
        }
        u64 total = 0;                                       // lane q: operators of this graph kept for set q
#pragma unroll
        for (int i = 0; i < kCountPlanes; ++i)
            if (i < planes_used)                             // wave-uniform
                total += (u64)__popcll(wave_transpose64(cnt.plane[i])) << i;
        pq[(int64_t)gi * 64 + lane] = (int64_t)total;
    }
}

hipError_t launch_sweep_graphs(const GraphView &g, u64 *M, u64 *K, int64_t *per_query_count, bool multi_producer,
                               hipStream_t s)
{
    if (g.num_graphs <= 0) return hipSuccess;
    const int per_block = kSweepThreads / kWave;
    hipLaunchKernelGGL(k_sweep_graphs, dim3((unsigned)((g.num_graphs + per_block - 1) / per_block)), dim3(kSweepThreads),
                       0, s, g, M, K, per_query_count, multi_producer ? 1 : 0);
    return hipGetLastError();
}

}  // namespace dgn
