// Internal declarations shared by the translation units of libdgn (gfx950, wave64 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dgn.h"

typedef unsigned long long u64;   // matches the operand type of HIP's 64-bit atomics
static_assert(sizeof(u64) == sizeof(uint64_t), "u64 must be 64 bits");

namespace dgn {

constexpr int kWave = 64;

// Sticky device-side error bits (TravState::error, BuildStatus::error).
enum : int32_t {
    kErrIdRange = 1,      // operator / tensor / target id out of range
    kErrTopo = 2,         // producer id >= consumer id
    kErrCsr = 4,          // row pointers not monotone / not ending at nnz
    kErrCrossGraph = 8,   // target or edge outside its own packed graph
    kErrOverflow = 16,    // internal: a frontier queue overflowed, the fix-up sweep must run
    kErrLogFull = 32,     // internal: the log of coloured tensors overflowed, the next prune clears everything
};

// Adjacency of a built graph as the kernels see it (device pointers).
struct GraphView {
    int32_t num_ops, num_tensors;
    int32_t nnz_in, nnz_out;
    int32_t num_graphs;
    const int32_t *in_rowptr, *in_idx;
    const int32_t *out_rowptr, *out_idx;
    const int32_t *prod_rowptr, *prod_idx;
    const int64_t *op_off, *t_off;    // [G+1] device copies, NULL when num_graphs == 1
    // What the traversal reads per operator and per pushed tensor, one access each (see traverse.hip):
    const int4 *orec;                 // [P] operator record (first input edge, fan-in, outputs)
    const int32_t *prod1;             // [T] the producer of a tensor, or kMulti / kNoProducer
};

// Operator record: x = first entry of the operator's row in in_idx, y = its fan-in, and the outputs: w >= 0
// says that the operator writes the w tensors z, z + 1, ... (consecutive ids in the order of its row, the usual
// case for a graph whose tensors are numbered as they are created), w < 0 that its -w outputs are
// out_idx[z], out_idx[z + 1], ...
// prod1 values below zero:
constexpr int32_t kMulti = -2;        // several producers: see prod_rowptr / prod_idx
constexpr int32_t kNoProducer = -3;   // graph input

// Record of one launch of the traversal: the state it started from and whether it ran a level.
// Launch e writes record e & 1 (one thread, at its start) and reads record (e - 1) & 1, which nobody
// writes while launch e runs.  No block ever waits for another: a launch leaves raw tallies behind
// (push counters, expansion counts, largest deferred operator id, all spread over 64 words), and EVERY
// block of the next launch derives the next state from the previous record and those tallies by itself.
struct LevelSlot {
    int32_t level;          // levels completed before this launch; queue parity = level & 1
    int32_t n;              // entries in the frontier this launch started from
    int32_t theta;          // entries whose producer id is below this are deferred at this level
    int32_t theta_hi;       // deferred operators with id in [theta, theta_hi) are expanded at this level
    int32_t deferred_seen;  // some operator has been deferred so far
    int32_t worked;         // the launch ran a level: its tallies still have to be folded into the state
    int32_t max_key1;       // 1 + largest operator id deferred so far (0: none)
    int32_t pad;
};

constexpr int kMaxRuns = 4;
struct TravState {            // header of the traversal state; the host reads these 128 bytes back
    LevelSlot slot[2];
    int32_t error;             // sticky kErr* bits
    int32_t pad0;
    u64 tensor_visits;         // expansions, summed over levels
    u64 max_frontier;
    int32_t changed;           // fix-up sweep: some operator gained bits
    int32_t run_len;           // wide levels run since the frontier was last small enough for one workgroup
    int32_t n_runs;            // such stretches completed so far; the first kMaxRuns lengths are kept
    int32_t wide_runs[kMaxRuns];
    int32_t pad;
    u64 atomic_updates;        // atomic ORs on M and K issued so far (one per input edge of an operator that gained bits)
};

// Contended words live 64 bytes apart, one per queue segment / block group.
constexpr int kMaxSeg = 64;
// Optional per-level trace (frontier size, expansions, threshold, range top), first kTraceLevels levels.
constexpr int kTraceLevels = 4096;
struct SegCounter {
    int32_t v;           // pushes into this segment of the frontier the launch produced (or handed on)
    int32_t key1;        // 1 + largest operator id deferred by the workgroups that tally here
    int32_t proc;        // entries / operators expanded by those workgroups ...
    int32_t atomics;     // ... and the atomic ORs on M and K they issued (the two are added as one 64-bit word)
    int32_t pad[12];
};
// Tallies of a launch, in buffer (launch number) % 3: written by launch e, read by launch e + 1, zeroed by
// launch e + 2 (one wave, at its start) for launch e + 3.
struct TravCounters { SegCounter cnt[3][kMaxSeg]; };
// Deferral schedule: the threshold starts at theta0, is multiplied by decay after every wide level and
// drops to 0 (nothing deferred any more) once it falls below theta_floor.
struct Schedule { float decay; int32_t theta0; int32_t theta_floor; int32_t small_level; };
// A frontier queue: S segments (power of two, <= kMaxSeg) of seg_cap entries each.
struct QueueGeom { int32_t S; int32_t seg_cap; };
static_assert(sizeof(TravState) == 128, "TravState is read back as 128 bytes");

// Log of the tensors a prune coloured (each exactly once, when its mask left zero), in kMaxSeg segments of
// seg_cap ids with one counter each.  entries == nullptr: no log is kept.
struct ColourLog { int32_t *entries; SegCounter *cnt; int32_t seg_cap; };
// What a prune that kept a complete log leaves in its scratch buffer: which buffers hold its result.  A later
// prune that finds exactly this there zeroes only what the log and the kept list name.
struct RecycleHeader {
    u64 magic, graph_serial;
    const void *M, *K, *kept_ops, *kept_count, *flags;
    const void *also_M, *also_K;   // two more arrays that hold non-zero words only where M / K do (or NULL)
    u64 pad[3];
};
__device__ __forceinline__ bool same_header(const RecycleHeader &a, const RecycleHeader &b)
{
    return a.magic == b.magic && a.graph_serial == b.graph_serial && a.M == b.M && a.K == b.K &&
           a.kept_ops == b.kept_ops && a.kept_count == b.kept_count && a.flags == b.flags && a.also_M == b.also_M &&
           a.also_K == b.also_K;
}

// ---- wave64 helpers ---------------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return (int)__lane_id(); }
__device__ __forceinline__ u64 lanemask_lt() { return ((u64)1 << lane_id()) - 1; }
__device__ __forceinline__ u64 ballot64(bool p) { return __ballot(p); }
// acc | (a ^ b) in one instruction (a three-input bit operation with the truth table 0xF0 | (0xCC ^ 0xAA))
__device__ __forceinline__ uint32_t or_of_xor(uint32_t acc, uint32_t a, uint32_t b)
{
    return __builtin_amdgcn_bitop3_b32(acc, a, b, 0xF6);
}

// Scans and reductions over the 64 lanes by data-parallel-primitive moves (shifts inside a row of 16 lanes, then a
// broadcast of lane 15 of a row to the next row and of lane 31 to the upper half): eight cheap vector instructions
// where a shuffle-based scan is six cross-lane permutes, each with the latency of an LDS access.
//   kRowShr + n: lane i of a row reads lane i - n of its row (lanes without a source keep `identity`);
//   kRowBcast15 / kRowBcast31 with row masks 0xa / 0xc: rows 1 and 3 read lane 15 of the row before, rows 2 and 3
//   read lane 31.
constexpr int kRowShr = 0x110, kRowBcast15 = 0x142, kRowBcast31 = 0x143;

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_move(int identity, int v)
{
    return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xf, false);
}

__device__ __forceinline__ int wave_incl_scan(int v)
{
    v += dpp_move<kRowShr + 1, 0xf>(0, v);
    v += dpp_move<kRowShr + 2, 0xf>(0, v);
    v += dpp_move<kRowShr + 4, 0xf>(0, v);
    v += dpp_move<kRowShr + 8, 0xf>(0, v);
    v += dpp_move<kRowBcast15, 0xa>(0, v);
    v += dpp_move<kRowBcast31, 0xc>(0, v);
    return v;
}
// inclusive running maximum
__device__ __forceinline__ int wave_incl_max(int v)
{
    constexpr int kLowest = -2147483647 - 1;
    v = max(v, dpp_move<kRowShr + 1, 0xf>(kLowest, v));
    v = max(v, dpp_move<kRowShr + 2, 0xf>(kLowest, v));
    v = max(v, dpp_move<kRowShr + 4, 0xf>(kLowest, v));
    v = max(v, dpp_move<kRowShr + 8, 0xf>(kLowest, v));
    v = max(v, dpp_move<kRowBcast15, 0xa>(kLowest, v));
    v = max(v, dpp_move<kRowBcast31, 0xc>(kLowest, v));
    return v;
}
__device__ __forceinline__ int wave_incl_or(int v)
{
    v |= dpp_move<kRowShr + 1, 0xf>(0, v);
    v |= dpp_move<kRowShr + 2, 0xf>(0, v);
    v |= dpp_move<kRowShr + 4, 0xf>(0, v);
    v |= dpp_move<kRowShr + 8, 0xf>(0, v);
    v |= dpp_move<kRowBcast15, 0xa>(0, v);
    v |= dpp_move<kRowBcast31, 0xc>(0, v);
    return v;
}
// reductions: the last lane of the scan holds the result (one scalar read)
__device__ __forceinline__ int wave_max(int v) { return __builtin_amdgcn_readlane(wave_incl_max(v), kWave - 1); }
__device__ __forceinline__ int wave_sum(int v) { return __builtin_amdgcn_readlane(wave_incl_scan(v), kWave - 1); }
__device__ __forceinline__ u64 wave_or(u64 v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane(wave_incl_or((int)(uint32_t)v), kWave - 1);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane(wave_incl_or((int)(uint32_t)(v >> 32)), kWave - 1);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 shfl64(u64 v, int src) { return (u64)__shfl((long long)v, src, kWave); }
__device__ __forceinline__ u64 shfl_xor64(u64 v, int mask) { return (u64)__shfl_xor((long long)v, mask, kWave); }

// Lanes hold 64-bit rows of a 64x64 bit matrix (row = lane); returns its transpose (lane q receives
// bit q of every lane's word, bit i coming from lane i).  Six butterfly steps.
template <int J>
__device__ __forceinline__ u64 transpose_step(u64 x, u64 lo_mask /* bit positions whose index has bit J clear */)
{
    const u64 other = (u64)__shfl_xor((long long)x, J, kWave);
    return (lane_id() & J) == 0 ? (x & lo_mask) | ((other & lo_mask) << J)
                                : (x & ~lo_mask) | ((other & ~lo_mask) >> J);
}
__device__ __forceinline__ u64 wave_transpose64(u64 x)
{
    x = transpose_step<32>(x, 0x00000000ffffffffull);
    x = transpose_step<16>(x, 0x0000ffff0000ffffull);
    x = transpose_step<8>(x, 0x00ff00ff00ff00ffull);
    x = transpose_step<4>(x, 0x0f0f0f0f0f0f0f0full);
    x = transpose_step<2>(x, 0x3333333333333333ull);
    x = transpose_step<1>(x, 0x5555555555555555ull);
    return x;
}

// Loads that must observe atomics performed by other workgroups / earlier levels: go to the
// device-coherent level instead of a possibly stale per-CU cache line.
__device__ __forceinline__ u64 load_coherent(const u64 *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t load_coherent(const int32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Stores that other workgroups read within the same kernel: written through to the device-coherent level.
__device__ __forceinline__ void store_coherent(int32_t *p, int32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_coherent(u64 *p, u64 v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_coherent(uint8_t *p, uint8_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t load_coherent(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- launch wrappers (each returns a hipError_t; nothing synchronises) -------------------------
struct FillRegion { void *ptr; size_t bytes; };   // ptr 8-byte aligned, bytes multiple of 8
hipError_t launch_clear(const FillRegion *regions, int num_regions, hipStream_t s);
// Zero `regions` (at most 8) -- unless *hdr equals `want`: then zero only M of the logged tensors and K and the
// deferral marker of the kept operators (the buffers are as the prune that wrote the header left them), and
// the same words of want.also_M / want.also_K where those are given.
// found_out[0] = 1 when the header was found, else 0.
hipError_t launch_clear_or_reset(const FillRegion *regions, int num_regions, const RecycleHeader *hdr,
                                 const RecycleHeader &want, u64 *found_out, const ColourLog &log, const int32_t *kept_ops,
                                 const int64_t *kept_count, u64 *M, u64 *K, uint8_t *DB, uint8_t *flags, hipStream_t s);

// out[i] = sum_{j<i} in[j], i = 0..n (n+1 outputs; out[n] = total).  in/out may alias when `in`
// holds n+1 entries.  tmp: scratch of scan_tmp_bytes(n) bytes.
size_t scan_tmp_bytes(int64_t n);
hipError_t launch_exclusive_scan(const int32_t *in, int32_t *out, int64_t n, void *tmp, hipStream_t s);

// Stable LSD radix sort of (key, val) pairs on the low `key_bits` bits of the keys.
// Result: vals_out (always) and keys_out (when not NULL).  keys_in / vals_in are not modified.
// tmp: scratch of sort_tmp_bytes(n) bytes.
size_t sort_tmp_bytes(int64_t n);
hipError_t launch_sort_pairs(const int32_t *keys_in, const int32_t *vals_in, int32_t *keys_out,
                             int32_t *vals_out, int64_t n, int key_bits, void *tmp, hipStream_t s);

// deg[key[e]] += 1 for keys in [0, n_rows); flags keys / vals outside their ranges in *error.
hipError_t launch_degree_hist(const int32_t *keys, const int32_t *vals, int64_t nnz, int32_t n_rows,
                              int32_t n_vals, int32_t *deg, int32_t *error, int32_t *unsorted, hipStream_t s);
// checks an edge list and, assuming its keys are in row order, writes the finished row (idx_out, rowptr)
hipError_t launch_scan_edges(const int32_t *keys, const int32_t *vals, int64_t nnz, int32_t n_rows, int32_t n_vals,
                             int32_t *idx_out, int32_t *rowptr, int32_t *error, int32_t *unsorted, int32_t *wide_gap,
                             hipStream_t s);
// rowptr[0..n_rows] from keys that are in row order (all in range)
hipError_t launch_row_bounds(const int32_t *keys, int64_t nnz, int32_t n_rows, int32_t *rowptr, hipStream_t s);
hipError_t launch_check_csr(const int32_t *rowptr, const int32_t *idx, int32_t n_rows, int32_t nnz,
                            int32_t n_vals, int32_t *error, hipStream_t s);
hipError_t launch_expand_rows(const int32_t *rowptr, int32_t n_rows, int32_t *row_of, hipStream_t s);
hipError_t launch_check_topological(const GraphView &g, int32_t *error, hipStream_t s);
hipError_t launch_check_graph_ranges(const GraphView &g, int32_t *error, bool also_topological, hipStream_t s);

// Traversal.
// operator records and producer words, once per graph; *multi = 1 when some tensor has several producers
hipError_t launch_build_records(const GraphView &g, int4 *orec, int32_t *prod1, int32_t *multi, hipStream_t s);
hipError_t launch_seed(const GraphView &g, int32_t Q, int64_t num_targets, const int32_t *tgt_rowptr,
                       const int32_t *tgt_idx, u64 *M, TravState *st, TravCounters *ctr, int32_t *q0,
                       const QueueGeom &qg, int32_t theta0, const ColourLog &log, hipStream_t s);
// One wide level (whole chip); a frontier of at most narrow_cap entries is left to launch_narrow unless
// deferred operators are waiting.  DB: deferred-operator markers, one byte per operator.
hipError_t launch_level(const GraphView &g, TravState *st, TravCounters *ctr, int launch_no, int32_t *q0, int32_t *q1,
                        const QueueGeom &qg, uint8_t *DB, uint8_t *flags, u64 *M, u64 *K, int grid_blocks, int narrow_cap,
                        const Schedule &sch, const ColourLog &log, int4 *trace, hipStream_t s);
// One workgroup runs level after level while 0 < frontier <= narrow_cap and nothing is deferred.  It leaves no
// tallies behind, so the record it writes is the state the host may read.
hipError_t launch_narrow(const GraphView &g, TravState *st, TravCounters *ctr, int launch_no, int32_t *q0, int32_t *q1,
                         const QueueGeom &qg, uint8_t *DB, uint8_t *flags, u64 *M, u64 *K, int narrow_cap, const Schedule &sch,
                         const ColourLog &log, int4 *trace, hipStream_t s);
// Packed batches of small graphs whose operator ids are a topological order: one wave per graph sweeps
// its operators once, highest ids first (no frontier at all); fills K and, when pq is not NULL, the
// per-graph per-set counts.
hipError_t launch_sweep_graphs(const GraphView &g, u64 *M, u64 *K, int64_t *per_query_count, bool multi_producer,
                               hipStream_t s);
// One sweep over all operators re-deriving K and pushing new bits to the inputs; *changed |= 1 if any.
hipError_t launch_fix_sweep(const GraphView &g, u64 *M, u64 *K, uint8_t *flags, int32_t *changed, int grid_blocks, hipStream_t s);

// Removal rule + compaction.
constexpr int kPqStride = 8;         // int64 words between two replicated per-set counters (64 bytes)
constexpr int kCompactTile = 2048;   // operators per workgroup in the count / scatter passes
struct CompactArgs {
    GraphView g;
    const u64 *M;            // used when from_tensor_mask
    u64 *K;
    uint8_t *op_flag;        // may be NULL
    int32_t *kept_ops;
    u64 *kept_masks;         // may be NULL
    int64_t *kept_count;
    int64_t *per_query_count;   // may be NULL
    int64_t *pq_part;           // [pq_replicas][G*64][kPqStride] zeroed scratch, or NULL: add straight into per_query_count
    int pq_replicas;            // power of two
    u64 *opbits;             // [ceil(P/64)] scratch
    int32_t *block_counts;   // [num_tiles + 1] scratch
    bool from_tensor_mask;   // K := OR M[out] (true) or read K as accumulated by the traversal
    const uint8_t *flag_in;  // when not NULL (and not from_tensor_mask): one byte per operator, 1 where K != 0, as the
                             // traversal left them; K is then read for those operators only
    RecycleHeader *hdr;      // when not NULL: the last pass writes `want` there if no error bit is set in *error
    RecycleHeader want;
    const int32_t *error;
};
// ev (may be NULL): three events recorded after the count, scan and scatter passes.
hipError_t launch_keep_compact(const CompactArgs &a, hipStream_t s, hipEvent_t *ev = nullptr);

// Read-outs of a prune result (Sec. 3.2): ignore mask from the kept list; per-set operator lists.
hipError_t launch_ignore_mask(const GraphView &g, const int32_t *kept_ops, const u64 *kept_masks, const int64_t *kept_count,
                              const u64 *M, u64 *ignore, int64_t *ignore_count, int grid_blocks, hipStream_t s);
size_t set_lists_scratch_bytes(int64_t num_kept);
hipError_t launch_set_lists(const int32_t *kept_ops, const u64 *kept_masks, int64_t num_kept, int64_t *set_rowptr,
                            int32_t *set_ops, int64_t capacity, void *scratch, int grid_blocks, hipStream_t s);

// Key of a transaction (Sec. 4.1): 128-bit digest of the target sets; *digest_dev points into `scratch`.
constexpr int kDigestMaxBlocks = 1024;
size_t digest_scratch_bytes();
hipError_t launch_target_digest(int32_t num_sets, int64_t n, const int32_t *tgt_rowptr, int64_t num_targets,
                                const int32_t *tgt_idx, void *scratch, u64 **digest_dev, hipStream_t s);

// Backward Prune (Algorithm 2): target row pointers 0..n (rowptr_only) or the seeds of the forward stage;
// one pass of the forward stage over the kept operators of the first stage.
hipError_t launch_backward_seed(int64_t T, int num_pairs, const int32_t *obj, const int32_t *wrt, int32_t *tgt_rowptr,
                                const u64 *B, u64 *F, int32_t *flags, bool rowptr_only, hipStream_t s);
hipError_t launch_keep_from_list(const GraphView &g, const int32_t *kept, const int64_t *kept_count, const u64 *F, u64 *K,
                                 uint8_t *flags, int grid_blocks, hipStream_t s);
hipError_t launch_forward_within(const GraphView &g, const int32_t *kept, const int64_t *kept_count, const u64 *B, u64 *F,
                                 int32_t *changed, int grid_blocks, hipStream_t s);

// In-place structures (Algorithm 3).  counters: [0] = number of nodes with exactly one child,
// [1 + r] = doubling round r left some jump pointer alive.
constexpr int kInplaceMaxRounds = 32;               // 2^32 links: longer than any chain of int32 ids
struct InplaceBuffers {
    int32_t *child;                                 // the only child of a tensor, -1 none, -2 several
    int32_t *J[2];                                  // jump pointers, double buffered
    int32_t *linkers;                               // nodes with exactly one child
    int32_t *counters;
};
size_t inplace_scratch_bytes(int64_t T);
InplaceBuffers inplace_buffers(void *scratch, int64_t T);
// init, children, links (the state before the first doubling round)
hipError_t launch_inplace_setup(const GraphView &g, const u64 *K, u64 select, const int32_t *kept_ops,
                                const int64_t *kept_count, int32_t *rename, int64_t *renamed_count,
                                const InplaceBuffers &b, int grid_blocks, hipStream_t s);
hipError_t launch_inplace_round(int round, int32_t *rename, int64_t *renamed_count, const InplaceBuffers &b,
                                int grid_blocks, hipStream_t s);

}  // namespace dgn
