/*
 * libdgn -- batched Forward Prune of tensor/operator DAGs on AMD CDNA4 (gfx950).
 *
 * What is computed (Dragon paper, arXiv 1707.08265):
 *   - graph model, Sec. 2.2: nodes are tensors; x_i -> x_j is an edge iff some operator takes x_i
 *     as an input and x_j as an output;
 *   - Algorithm 1 ("Backward Traversing for Forward-Pass"): starting from the solving targets,
 *     mark every tensor the targets depend on;
 *   - removal rule, Sec. 2.1: an operator whose outputs are all un-coloured is removed;
 *   - Sec. 3.2: surviving operators keep their creation (= topological) order.
 *
 * Here up to 64 target sets are solved at once: bit q of a 64-bit mask is the flag m_x of an
 * independent run of Algorithm 1 with target set q.  With
 *      K[o] = OR_{u in out(o)} M[u]                       (operator keep mask)
 *      M[t] = S[t] | OR_{o : t in in(o)} K[o]             (least fixed point; S = seed masks)
 * the library returns M, K, the flags K != 0 and the kept operators compacted in ascending id.
 *
 * General conventions
 *   - Plain C ABI.  Unless a parameter says HOST, every pointer is a DEVICE pointer owned by the
 *     caller; the library never allocates or frees device memory (sizes of the caller-provided
 *     graph storage and scratch come from the *_workspace queries).  Device buffers must be
 *     8-byte aligned (256-byte alignment is recommended for graph_mem and scratch).
 *   - dgn_stream is a hipStream_t (NULL = the default stream).  All kernels are enqueued on it.
 *   - Every function returns DGN_OK (0) or a negative DGN_ERR_* code; nothing throws or aborts.
 *   - All counts must be below 2^31 - 1 (ids and offsets are int32 on the device).
 *   - Operator ids must be a topological (creation) order: every producer of an operator's input
 *     has a smaller id than the operator.  M, K and the flags are correct for any DAG; the
 *     "ascending id = topological order" meaning of the kept list needs this precondition.
 *     Duplicate edges, tensors with several producers, and operators with no inputs or no
 *     outputs are legal.
 *   - Host threads: calls on one dgn_graph may run at the same time from several threads as long as each
 *     has output buffers, scratch and stream of its own (the handle only keeps launch-layout hints, which
 *     any call may overwrite); two calls that share a scratch or output buffer must not overlap.
 */
#ifndef DGN_H
#define DGN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DGN_VERSION 100 /* 0.1.0 */
#define DGN_MAX_SETS 64

typedef void *dgn_stream;             /* hipStream_t */
typedef struct dgn_graph dgn_graph;   /* opaque host handle; immutable after build */

enum {
    DGN_OK = 0,
    DGN_ERR_INVALID_ARG = -1,         /* negative size, inconsistent descriptor, bad option      */
    DGN_ERR_NULL_PTR = -2,            /* a required pointer is NULL                               */
    DGN_ERR_TOO_LARGE = -3,           /* a count is >= 2^31 - 1                                   */
    DGN_ERR_ID_OUT_OF_RANGE = -4,     /* an operator / tensor / target id is outside its range    */
    DGN_ERR_TOO_MANY_SETS = -5,       /* num_sets outside 1..64                                   */
    DGN_ERR_WORKSPACE_TOO_SMALL = -6, /* graph_bytes or scratch_bytes below the queried size      */
    DGN_ERR_NOT_TOPOLOGICAL = -7,     /* validation found a producer id >= its consumer id        */
    DGN_ERR_HIP = -8,                 /* a HIP call failed; see dgn_last_hip_error()              */
    DGN_ERR_BAD_CSR = -9              /* row pointers not monotone or not ending at nnz           */
};

/* Operators as two COO edge lists, in any order (Sec. 2.2: an operator with its inputs and its
 * outputs).  Edge e of the first list says "operator in_op[e] reads tensor in_tensor[e]", edge e
 * of the second "operator out_op[e] writes tensor out_tensor[e]".
 * A packed batch of independent graphs (num_graphs > 1) uses global ids; graph g owns operators
 * [graph_op_offsets[g], graph_op_offsets[g+1]) and tensors likewise; no edge may cross graphs. */
typedef struct dgn_coo_desc {
    int64_t num_ops, num_tensors;
    int64_t nnz_in, nnz_out;
    const int32_t *in_op, *in_tensor;       /* device [nnz_in]  */
    const int32_t *out_op, *out_tensor;     /* device [nnz_out] */
    int32_t num_graphs;                     /* 1, or G for a packed batch */
    const int64_t *graph_op_offsets;        /* HOST [G+1], or NULL when num_graphs == 1 */
    const int64_t *graph_tensor_offsets;    /* HOST [G+1], or NULL when num_graphs == 1 */
} dgn_coo_desc;

/* The same graph already in CSR form (operator -> inputs, operator -> outputs).  The four arrays
 * are BORROWED: they must stay valid and unchanged for the life of the handle. */
typedef struct dgn_csr_desc {
    int64_t num_ops, num_tensors;
    int64_t nnz_in, nnz_out;
    const int32_t *in_rowptr, *in_idx;      /* device [num_ops+1], [nnz_in]  */
    const int32_t *out_rowptr, *out_idx;    /* device [num_ops+1], [nnz_out] */
    int32_t num_graphs;
    const int64_t *graph_op_offsets;        /* HOST [G+1] or NULL */
    const int64_t *graph_tensor_offsets;    /* HOST [G+1] or NULL */
} dgn_csr_desc;

typedef struct dgn_options {
    int32_t validate;        /* build: also check the topological precondition (one extra pass)   */
    int32_t recompute_keep;  /* prune: recompute K from M with the stand-alone removal-rule pass
                                instead of using the K the traversal accumulated (same values)   */
    int32_t traversal;       /* 0 = automatic; 1 = one kernel launch per frontier level, nothing else;
                                2 = one launch per wide level plus the single-workgroup kernel for
                                small frontiers (what 0 chooses for a single graph)               */
    int32_t profile;         /* prune: 1 = bracket each phase with HIP events on `stream` and report
                                the elapsed times in dgn_stats.phase_ms (needs stats != NULL); an
                                event between two kernels leaves the stream idle for a few
                                microseconds, so 2 = only the two events around the traversal
                                (phase_ms[DGN_PHASE_TRAVERSE] alone is filled)                      */
    int32_t defer_percent;   /* prune: geometric decay (percent, 1..99) of the producer-id threshold
                                below which frontier entries wait for more bits; 100 = never defer,
                                0 = library default.  A schedule only: results do not depend on it */
    int32_t max_queue_entries; /* prune: cap on the frontier queues (0 = one entry per tensor).  A
                                smaller cap only forces the overflow fix-up path (testing aid);
                                results do not depend on it */
    int32_t defer_start_shift; /* prune: the threshold starts at num_ops >> this (0 = default)          */
    int32_t defer_floor_shift; /* prune: deferral stops once the threshold is below num_ops >> this
                                (0 = default).  Schedule knobs only: results do not depend on them   */
    int32_t incremental;     /* prune: tensor_mask and op_mask are IN/OUT.  On entry they hold the result of
                                an earlier prune of a graph that this one extends (the same graph, or a
                                prefix of its operators with the masks zero-extended by the caller) for
                                some of the target sets; the call colours what the given targets add and
                                leaves the fixed point for the union.  Nothing is cleared, only the new
                                bits are traversed; every other output is rewritten in full.  The masks
                                must be such a result: anything else gives unspecified masks             */
    int32_t recycle;         /* prune: the caller states that nothing but dgn_prune has written to `scratch`
                                since it last passed it to this library, and that, if the last such call
                                was a dgn_prune of this graph with this tensor_mask, op_mask, op_flag,
                                kept_ops and kept_count, those are still as that call left them.  The call then
                                zeroes only the words that call set (it finds them through a log the
                                earlier call kept in `scratch`, and checks on the device that graph and
                                buffers are the same) instead of all of tensor_mask and op_mask, and keeps
                                such a log itself.  Where no complete log is found (first call with this
                                flag, other buffers, a prune that coloured more than a quarter of the
                                tensors, packed batches swept per graph, after an incremental call)
                                everything is cleared as without the flag.  Outputs are the same either
                                way.  Do not set it on the first call with a scratch buffer whose contents
                                are undefined                                                          */
} dgn_options;

/* Indices into dgn_stats.phase_ms */
enum {
    DGN_PHASE_CLEAR = 0,     /* M, K, marker and flag bytes, state zeroed (all, or what the last call set) */
    DGN_PHASE_SEED = 1,      /* target bits scattered, first frontier built (one kernel)          */
    DGN_PHASE_TRAVERSE = 2,  /* all frontier levels                                               */
    DGN_PHASE_COUNT = 3,     /* removal rule / flags / per-tile and per-set counts (one kernel)   */
    DGN_PHASE_SCAN = 4,      /* prefix sum of the tile counts (one kernel)                        */
    DGN_PHASE_SCATTER = 5,   /* ordered scatter of the kept operators (+ per-graph offsets)       */
    DGN_PHASE_TOTAL = 6,     /* first kernel start to last kernel end                             */
    DGN_NUM_PHASES = 8
};

/* Schedule-dependent counters (not part of the result; excluded from parity). HOST struct. */
typedef struct dgn_stats {
    int64_t levels;          /* frontier levels processed                                        */
    int64_t tensor_visits;   /* frontier entries and deferred operators expanded, summed over levels */
    int64_t max_frontier;    /* largest frontier                                                 */
    int64_t launches;        /* kernels enqueued by the call                                     */
    int64_t level_launches;  /* of which frontier-level kernels                                  */
    int32_t *level_trace;    /* IN, optional HOST buffer: per level 4 ints (frontier size, entries and
                                operators expanded, deferral threshold or -1, low 32 bits of the device
                                wall clock in 10 ns ticks when the level was finished), for the first
                                level_trace_cap levels (at most 4096)                                    */
    int64_t level_trace_cap; /* IN: capacity of level_trace in levels                                     */
    int64_t reserved;        /* dgn_backward_prune: passes of its forward stage; 0 otherwise                */
    int64_t recycled;        /* 1 when options->recycle found the previous result in place and the call
                                zeroed only what that result had set                               */
    int64_t atomic_updates;  /* 64-bit atomic ORs the traversal issued (one per input edge of an operator that
                                gained bits, plus the seeds); 0 for a packed batch swept per graph      */
    float phase_ms[DGN_NUM_PHASES];   /* filled when options->profile is 1 (all) or 2 (traversal); zero otherwise */
} dgn_stats;

/* ---- graph construction -------------------------------------------------------------------- */

/* Bytes of caller-provided device storage for the graph (lives as long as the handle) and of
 * scratch (needed only during dgn_graph_build).  Validates the descriptor's sizes on the host. */
int dgn_graph_build_workspace(const dgn_coo_desc *desc, size_t *graph_bytes, size_t *scratch_bytes);

/* Build, on the device, the adjacency the traversal needs (Sec. 2.2 edge definition):
 *   operator -> input tensors   CSR, rows keep the COO order of their edges (stable);
 *   operator -> output tensors  CSR, likewise;
 *   tensor   -> producing operators CSR, rows ascending in operator id.
 * Stable LSD radix sort on the significant key bits plus prefix sums, all inside graph_mem /
 * scratch.  Every id is range-checked on the device (-> DGN_ERR_ID_OUT_OF_RANGE); with
 * options->validate the topological precondition is checked too (-> DGN_ERR_NOT_TOPOLOGICAL).
 * The call synchronises the stream once before returning to report those errors.  options may be
 * NULL.  On success *out receives a handle; scratch may be reused afterwards, graph_mem may not. */
int dgn_graph_build(const dgn_coo_desc *desc, void *graph_mem, size_t graph_bytes, void *scratch,
                    size_t scratch_bytes, const dgn_options *options, dgn_stream stream,
                    dgn_graph **out);

int dgn_graph_from_csr_workspace(const dgn_csr_desc *desc, size_t *graph_bytes, size_t *scratch_bytes);

/* As dgn_graph_build, for a caller that already holds the two operator CSRs: only the
 * tensor -> producer CSR is built (into graph_mem).  Row pointers are checked to be monotone and
 * to end at nnz (-> DGN_ERR_BAD_CSR), ids are range-checked. */
int dgn_graph_from_csr(const dgn_csr_desc *desc, void *graph_mem, size_t graph_bytes, void *scratch,
                       size_t scratch_bytes, const dgn_options *options, dgn_stream stream,
                       dgn_graph **out);

/* Device pointers of the built adjacency (any output pointer may be NULL).  For parity checks of
 * the builder; the arrays belong to the handle's graph_mem (or to the caller for borrowed CSRs). */
int dgn_graph_get_csr(const dgn_graph *g, const int32_t **in_rowptr, const int32_t **in_idx,
                      const int32_t **out_rowptr, const int32_t **out_idx,
                      const int32_t **prod_rowptr, const int32_t **prod_idx);

/* Sizes of a built graph (any output pointer may be NULL). */
int dgn_graph_get_sizes(const dgn_graph *g, int64_t *num_ops, int64_t *num_tensors, int64_t *nnz_in,
                        int64_t *nnz_out, int32_t *num_graphs);

/* Frees the host handle only (device storage belongs to the caller). NULL is accepted. */
void dgn_graph_destroy(dgn_graph *g);

/* ---- Forward Prune ----------------------------------------------------------------------- */

/* Scratch bytes dgn_prune / dgn_keep_compact need for this graph. */
int dgn_prune_workspace(const dgn_graph *g, int32_t num_sets, size_t *scratch_bytes);

/* Algorithm 1 for num_sets (= Q, 1..64) target sets per graph at once, then the removal rule of
 * Sec. 2.1 and the creation-order compaction of Sec. 3.2.
 *
 *   tgt_rowptr [G*Q+1], tgt_idx [num_targets]: CSR of the target sets; set s = g*Q + q belongs to
 *       graph g and owns bit q.  Ids are global tensor ids.  Empty sets, duplicate targets and a
 *       tensor in several sets are legal.  An id outside [0, num_tensors) is skipped and reported
 *       as DGN_ERR_ID_OUT_OF_RANGE.
 *   tensor_mask [num_tensors]  out: M.   op_mask [num_ops]  out: K.  Bits >= Q are zero.
 *   op_flag     [num_ops]      out: K != 0 as 0/1 bytes; may be NULL.
 *   kept_ops    [num_ops]      out: ascending ids of the operators with K != 0 (first kept_count).
 *   kept_masks  [num_ops]      out: K of each kept operator, parallel to kept_ops; may be NULL.
 *   kept_count  out int64: [0] = number kept; for a packed batch additionally [1+g], g = 0..G, =
 *       number of kept operators with id < graph_op_offsets[g]  (so [1 + G + 1] entries).
 *   per_query_count out int64 [64], or [G*64] for a packed batch: operators whose K has bit q;
 *       may be NULL.
 *   options, stats: HOST, may be NULL.
 *
 * All outputs are cleared (see options->recycle) and rewritten in full by the call; op_flag may already be
 * written while the traversal runs and is complete, like everything else, on return.  Kernels run on `stream`; the call
 * reads a few status words back and synchronises the stream before returning, because the number
 * of frontier levels depends on the data.  Calls on the same graph may run concurrently only with
 * distinct scratch and output buffers. */
int dgn_prune(const dgn_graph *g, int32_t num_sets, int64_t num_targets, const int32_t *tgt_rowptr,
              const int32_t *tgt_idx, uint64_t *tensor_mask, uint64_t *op_mask, uint8_t *op_flag,
              int32_t *kept_ops, uint64_t *kept_masks, int64_t *kept_count, int64_t *per_query_count,
              void *scratch, size_t scratch_bytes, const dgn_options *options, dgn_stats *stats,
              dgn_stream stream);

/* More than 64 target sets on one graph: dgn_prune once per word of 64 sets, one after the other.
 *   num_sets: any number >= 1; W = ceil(num_sets / 64) words; set s owns bit s % 64 of word s / 64.
 *   tgt_rowptr [num_sets+1], tgt_idx [num_targets]: as for dgn_prune.
 *   Outputs are word-major: tensor_mask [W][num_tensors], op_mask [W][num_ops], op_flag [W][num_ops],
 *   kept_ops [W][num_ops], kept_masks [W][num_ops], kept_count [W], per_query_count [W][64]
 *   (the same pointers may be NULL as for dgn_prune).  scratch: as for dgn_prune (reused by every word).
 *   stats: sums over the words (max_frontier: the maximum).
 * Single graphs only (DGN_ERR_INVALID_ARG for a packed batch).  The call synchronises the stream at
 * least once per word. */
int dgn_prune_words(const dgn_graph *g, int64_t num_sets, int64_t num_targets, const int32_t *tgt_rowptr,
                    const int32_t *tgt_idx, uint64_t *tensor_mask, uint64_t *op_mask, uint8_t *op_flag,
                    int32_t *kept_ops, uint64_t *kept_masks, int64_t *kept_count, int64_t *per_query_count,
                    void *scratch, size_t scratch_bytes, const dgn_options *options, dgn_stats *stats,
                    dgn_stream stream);

/* Removal rule + compaction only (Sec. 2.1, Sec. 3.2), for a caller that supplies the coloured
 * masks: K[o] = OR of tensor_mask_in over the outputs of o, then the same outputs as dgn_prune.
 * Asynchronous on `stream`: nothing is read back. */
int dgn_keep_compact(const dgn_graph *g, const uint64_t *tensor_mask_in, uint64_t *op_mask,
                     uint8_t *op_flag, int32_t *kept_ops, uint64_t *kept_masks, int64_t *kept_count,
                     int64_t *per_query_count, void *scratch, size_t scratch_bytes, dgn_stream stream);

/* For callers that cannot allocate device memory or size a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation): dgn_keep_compact with its scratch in a fixed array that is
 * part of the library's code object instead of a caller-provided buffer.  Same arguments otherwise, same outputs,
 * asynchronous on `stream`; the call allocates nothing, frees nothing and reads nothing back (the first call on
 * a device looks up the array's device address, which loads the code object if nothing has yet).
 *   Limits: num_ops <= 2^26 (DGN_ERR_TOO_LARGE beyond); the array takes about 8.4 MB of every device the
 *   library runs kernels on, until the process ends.  dgn_keep_compact_static_limits reports both numbers
 *   (either pointer may be NULL).
 *   The device that `stream` belongs to must be the current device.  Every call on a device shares that
 *   device's array: two calls that overlap on one device (different streams, or host threads) race on it
 *   and give unspecified outputs; calls on one stream, one after the other, are fine.  The array keeps
 *   the last call's contents; the call clears what it needs at zero itself. */
int dgn_keep_compact_static_limits(int64_t *max_ops, size_t *static_bytes);
int dgn_keep_compact_static(const dgn_graph *g, const uint64_t *tensor_mask_in, uint64_t *op_mask,
                            uint8_t *op_flag, int32_t *kept_ops, uint64_t *kept_masks, int64_t *kept_count,
                            int64_t *per_query_count, dgn_stream stream);

/* ---- Backward Prune ---------------------------------------------------------------------- */

/* Scratch bytes dgn_backward_prune needs for this graph. */
int dgn_backward_prune_workspace(const dgn_graph *g, size_t *scratch_bytes);

/* Algorithm 2 (Sec. 2.3) for num_pairs (1..64) pairs (x_obj, x_wrt) at once, then the removal rule
 * of Sec. 2.1 and the creation-order compaction of Sec. 3.2, exactly as dgn_prune applies them.
 *
 *   obj [num_pairs], wrt [num_pairs]: DEVICE int32 tensor ids; pair i owns bit i.
 *   tensor_mask [num_tensors] out: bit i set iff the tensor lies on a route from obj[i] to wrt[i]
 *       (Child(x) = tensors written by operators that read x); a pair with obj[i] == wrt[i], or
 *       whose target cannot be reached, marks nothing.
 *   op_mask, op_flag, kept_ops, kept_masks, kept_count, per_query_count: as for dgn_prune, derived
 *       from tensor_mask (an operator is kept for pair i iff one of its outputs is marked for i).
 *   options, stats: HOST, may be NULL; stats describes the first stage (the traversal from the
 *       derivative targets), stats->reserved = passes of the forward stage.  options->recycle: the
 *       caller states that the last call that used `scratch` was a dgn_backward_prune of this graph
 *       with this tensor_mask, op_mask and op_flag, and that nobody has written to them since: the call
 *       then zeroes only the words that call set (checked on the device, as for dgn_prune).
 *
 * Single graphs only (DGN_ERR_INVALID_ARG for a packed batch).  An id outside [0, num_tensors) is
 * reported as DGN_ERR_ID_OUT_OF_RANGE.  All outputs are rewritten in full; the call synchronises the
 * stream several times (the number of passes depends on the data). */
int dgn_backward_prune(const dgn_graph *g, int32_t num_pairs, const int32_t *obj, const int32_t *wrt,
                       uint64_t *tensor_mask, uint64_t *op_mask, uint8_t *op_flag, int32_t *kept_ops,
                       uint64_t *kept_masks, int64_t *kept_count, int64_t *per_query_count, void *scratch,
                       size_t scratch_bytes, const dgn_options *options, dgn_stats *stats, dgn_stream stream);

/* ---- Reading a prune result (Sec. 3.2) --------------------------------------------------- */

/* Tensors to rename "ignore": bit q of ignore_mask[t] is set iff t is written by an operator that
 * survives for set q (bit q of its K) while t itself is not coloured for q.  Works from the compacted
 * list, so it costs the pruned graph plus clearing the mask.
 *   tensor_mask [num_tensors] in (DEVICE): M.   kept_ops / kept_masks / kept_count in (DEVICE): as
 *       written by dgn_prune, dgn_keep_compact or dgn_backward_prune (kept_count[0] is read on the device).
 *   ignore_mask [num_tensors] out (DEVICE), rewritten in full.
 *   ignore_count out (DEVICE int64 [1]): tensors with a non-zero ignore mask; may be NULL.
 * Asynchronous on `stream`: nothing is read back. */
int dgn_ignore_mask(const dgn_graph *g, const uint64_t *tensor_mask, const int32_t *kept_ops,
                    const uint64_t *kept_masks, const int64_t *kept_count, uint64_t *ignore_mask,
                    int64_t *ignore_count, dgn_stream stream);

/* Key of a transaction (Sec. 4.1: a function -- the graph pruned for one choice of fetches and feeds -- is
 * bound to a hashing key generated from that choice, and asking for it again builds nothing new).  The paper
 * names no hash.  The key here: the graph handle, num_sets, and this 128-bit digest of the target sets exactly as
 * dgn_prune would receive them -- the sequence of 32-bit words
 *     w = [ num_sets, n, tgt_rowptr[0..n], tgt_idx[0..num_targets-1] ],   n = num_sets * number of graphs,
 *     digest_out[k] = sum over positions i of mix((i + 1) * G + w_i * C_k + S_k)  mod 2^64,
 * mix = the output function of SplitMix64 (z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; z ^= z >> 27;
 * z *= 0x94D049BB133111EB; z ^= z >> 31), G = 0x9E3779B97F4A7C15, w_i taken as unsigned,
 * C_0 = 0xC2B2AE3D27D4EB4F, S_0 = 0x165667B19E3779F9, C_1 = 0xD6E8FEB86659FD93, S_1 = 0x27D4EB2F165667C5.
 * Equal target sets give equal digests; the same targets in another order, or split differently over the sets,
 * give another one (a cache keyed by it may miss where it could have hit, it does not hit wrongly short of a
 * 128-bit collision).
 *   tgt_rowptr, tgt_idx: DEVICE, as for dgn_prune; digest_out: HOST, two words; scratch: DEVICE, 8-byte
 *   aligned, dgn_target_digest_workspace bytes.  Synchronises `stream`.  Ids are not validated. */
int dgn_target_digest_workspace(size_t *scratch_bytes);
int dgn_target_digest(const dgn_graph *g, int32_t num_sets, int64_t num_targets, const int32_t *tgt_rowptr,
                      const int32_t *tgt_idx, uint64_t *digest_out, void *scratch, size_t scratch_bytes,
                      dgn_stream stream);

/* Scratch bytes dgn_per_set_lists needs for a kept list of num_kept entries. */
int dgn_per_set_lists_workspace(int64_t num_kept, size_t *scratch_bytes);

/* For every bit q = 0..63 the operators of the kept list whose mask has bit q, in creation order
 * (what the function of target set q executes, Sec. 3.2), laid out set after set.
 *   kept_ops / kept_masks [num_kept] in (DEVICE); num_kept is a HOST value (kept_count[0] read back).
 *   set_rowptr out (DEVICE int64 [65]): list q is set_ops[set_rowptr[q] .. set_rowptr[q+1]);
 *       set_rowptr[64] is the total number of entries.
 *   set_ops out (DEVICE int32 [set_ops_capacity]): entries beyond the capacity are dropped, so the
 *       caller compares set_rowptr[64] with the capacity (the sum of per_query_count is enough).
 * num_kept above 2^31 / 64 is DGN_ERR_TOO_LARGE (slots are counted in int32).  For a packed batch bit
 * q mixes the graphs' q-th sets; kept_count[1 + g] cuts every list by graph.  Asynchronous. */
int dgn_per_set_lists(const int32_t *kept_ops, const uint64_t *kept_masks, int64_t num_kept,
                      int64_t *set_rowptr, int32_t *set_ops, int64_t set_ops_capacity, void *scratch,
                      size_t scratch_bytes, dgn_stream stream);

/* ---- In-place structures ----------------------------------------------------------------- */

/* Scratch bytes dgn_inplace needs for this graph. */
int dgn_inplace_workspace(const dgn_graph *g, size_t *scratch_bytes);

/* Algorithm 3 (Sec. 2.4) on the graph left by the prune: the rename dictionary.
 *
 * The nodes are the tensors that a surviving operator reads or writes; an operator survives when
 * (op_mask[o] & select) != 0, so select = 1 << q gives the graph pruned for target set q and
 * select = ~0 the union over all sets.  Child(x) = the distinct tensors written by surviving
 * operators that read x.  Nodes are taken in ascending id; a node not yet renamed becomes its own
 * ancestor and passes that ancestor on while the current node has exactly one child.
 *
 *   op_mask [num_ops]      in : K as written by dgn_prune / dgn_keep_compact (DEVICE).
 *   rename  [num_tensors]  out: ancestor id of every node, -1 for tensors outside the graph (DEVICE).
 *   renamed_count          out: int64 [1], nodes whose ancestor is another tensor (DEVICE); may be NULL.
 *   rounds_out             out: HOST int32, pointer-doubling rounds that were run; may be NULL.
 *
 * The pruned graph must be acyclic (tensor ids need not be topological); on a cyclic one the call
 * still ends, after 32 rounds, with unspecified ancestors for the nodes on the cycle.  Kernels run on
 * `stream`; the call reads one status word back every four rounds and has synchronised the stream
 * when it returns.  For a packed batch the graphs are handled together (ids are global). */
int dgn_inplace(const dgn_graph *g, const uint64_t *op_mask, uint64_t select, int32_t *rename,
                int64_t *renamed_count, void *scratch, size_t scratch_bytes, int32_t *rounds_out,
                dgn_stream stream);

/* The same for a caller that still has the kept list of the prune that wrote op_mask: kept_ops [>= kept_count[0]]
 * and kept_count [1] (DEVICE) as dgn_prune / dgn_keep_compact left them, i.e. the ascending ids of the operators
 * with op_mask != 0.  The pass then visits those operators instead of reading all of op_mask -- on a graph
 * pruned to a few percent of its operators that is most of its time.  Same outputs. */
int dgn_inplace_kept(const dgn_graph *g, const uint64_t *op_mask, uint64_t select, const int32_t *kept_ops,
                     const int64_t *kept_count, int32_t *rename, int64_t *renamed_count, void *scratch,
                     size_t scratch_bytes, int32_t *rounds_out, dgn_stream stream);

/* ---- machine rates --------------------------------------------------------------------------- */

/* The traversal of Algorithm 1 moves few bytes; it is made of random 8-byte reads, 64-bit atomic ORs, kernel
 * launches (one per wide frontier level) and chains of accesses that each wait for the one before.  None of
 * these has a published peak, so dgn_calibrate measures them on this GPU, with HIP events on `stream`:
 * they are the ceilings the traversal's own counts (atomics per prune, levels per prune) are priced against.
 * HOST struct. */
typedef struct dgn_machine_rates {
    float random_load_gps;         /* 10^9 independent 8-byte loads per second, addresses uniform over the buffer */
    float random_atomic_gps;       /* the same with returning 64-bit atomic ORs                                   */
    float random_store_gps;        /* the same with plain 8-byte stores                                           */
    float dependent_load_ns;       /* one step of a chain of loads whose address needs the value loaded before   */
    float dependent_atomic_ns;     /* the same with returning atomics                                             */
    float same_address_atomic_ns;  /* per atomic when 8 192 waves add to ONE word (a single shared counter)      */
    float launch_floor_us;         /* event-to-event time of one empty kernel of 2 048 workgroups                 */
    float launch_back_to_back_us;  /* per kernel in a run of 100 such kernels                                     */
    float copy_gbs;                /* streaming copy inside the buffer, bytes read + written, 10^9 per second     */
    float random_atomic_noreturn_gps;  /* random 64-bit atomic ORs whose old value is not asked for                */
    float random_load_and_atomic_gps;  /* pairs per second of one random load and one random atomic OR, unrelated
                                          addresses, issued together: do the two rates share a ceiling?            */
    float run_atomic_gps;              /* atomic ORs (old value not asked for) whose 64 lanes hit 64 consecutive words,
                                          the runs at random places: what an OR on K of neighbouring operators costs */
    float reserved[4];
    int64_t buffer_bytes;
} dgn_machine_rates;

/* buffer: DEVICE, 16-byte aligned, at least 1 MiB; its contents are destroyed.  Pass a buffer of the size of
 * the mask array of the workload (8 bytes per tensor) so that the random accesses see the workload's locality.
 * Creates and destroys two HIP events, synchronises `stream` repeatedly, takes a few milliseconds. */
int dgn_calibrate(void *buffer, size_t bytes, dgn_machine_rates *out, dgn_stream stream);

/* The kernels add up and compare values across the 64 lanes of a wave with data-parallel-primitive moves (row shifts,
 * row broadcasts) whose lane layout is a property of the GPU generation the library is built for.  This runs every such
 * scan and reduction on 64 waves of fixed test values and compares with the same sums computed on the host; and the
 * three-input bit operation of the sort's ranking (its truth table is an immediate operand) with the plain expression.
 * buffer: DEVICE, 16-byte aligned, at least 98 304 bytes (destroyed).  Returns the number of values that differ (0: all
 * well) or a negative DGN_ERR_*.  Synchronises `stream`; not thread safe (static host arrays). */
int dgn_selftest_wave_ops(void *buffer, size_t bytes, dgn_stream stream);

/* ---- misc ---------------------------------------------------------------------------------- */
const char *dgn_strerror(int code);
int dgn_version(void);
int dgn_last_hip_error(void);   /* hipError_t of the last failed HIP call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* DGN_H */
