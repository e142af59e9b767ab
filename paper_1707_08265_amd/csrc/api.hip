// C ABI of libdgn: argument checking, workspace layout and kernel sequencing (declared in dgn.h).
// Host code only decides *which* kernels run and where their buffers live; every step of the path
// itself (adjacency build, seeding, traversal, removal rule, compaction) is a device kernel.
#include <new>
#include <string.h>

#include "common.h"

#include <atomic>

using namespace dgn;

namespace {

thread_local int t_last_hip = 0;

inline int hip_fail(hipError_t e)
{
    t_last_hip = (int)e;
    return DGN_ERR_HIP;
}
#define DGN_HIP(expr)                                   \
    do {                                                \
        hipError_t e__ = (expr);                        \
        if (e__ != hipSuccess) return hip_fail(e__);    \
    } while (0)

constexpr int64_t kMaxCount = 2147483646;   // counts must stay below 2^31 - 1
constexpr int kLevelBlocksPerCU = 5;   // workgroups of a wide level per compute unit
constexpr int kNarrowCap = 1024;            // frontiers up to this size are walked by one workgroup (one round of its threads)
constexpr int kWidePerGroup = 12;           // wide level launches between two single-workgroup launches
constexpr int kWideGroupsFirst = 4;         // groups in the first batch (one state read-back per batch) ...
constexpr int kWideGroups = 6;              // ... and in the following ones
constexpr int kMaxBatch = 512;              // launches enqueued between two state read-backs, at most
constexpr int kTailLevels = 1;              // wide launches enqueued beyond the layout the previous prune needed ...
constexpr int kExactStreak = 3;             // ... until that layout has fitted exactly this many prunes in a row
constexpr int kStatusMulti = 16;            // word of the build's status block that says "a tensor has several producers"
constexpr int kBackwardMaxBatch = 60;       // forward passes of the backward prune between two read-backs, at most
constexpr int kSweepMinGraphs = 64;         // packed batches with at least this many graphs ...
constexpr int64_t kSweepMaxGraphOps = 1 << 18;   // ... none larger than this use the per-graph sweep
constexpr u64 kRecycleMagic = 0x44474e5f52435943ull;   // "DGN_RCYC"
constexpr int kSmallLevel = 16384;           // levels expanding fewer entries than this decay the threshold faster
constexpr int kDefaultDeferPercent = 74;
constexpr int kDefaultStartShift = 1;       // deferral threshold starts at P >> 1 ...
constexpr int kDefaultFloorShift = 10;      // ... and stops (drops to 0) below P >> 10

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// carve consecutive 256-byte aligned regions out of one buffer
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <typename T> T *take(size_t count)
    {
        T *r = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += align256(count * sizeof(T));
        return r;
    }
};

inline int key_bits_for(int64_t n)
{
    int b = 1;
    while (b < 31 && ((int64_t)1 << b) < n) ++b;
    return b;
}

int check_sizes(int64_t P, int64_t T, int64_t Ein, int64_t Eout, int32_t G, const int64_t *op_off,
                const int64_t *t_off)
{
    if (P < 0 || T < 0 || Ein < 0 || Eout < 0 || G < 1) return DGN_ERR_INVALID_ARG;
    if (P > kMaxCount || T > kMaxCount || Ein > kMaxCount || Eout > kMaxCount) return DGN_ERR_TOO_LARGE;
    if (G > 1) {
        if (!op_off || !t_off) return DGN_ERR_NULL_PTR;
        if (op_off[0] != 0 || t_off[0] != 0 || op_off[G] != P || t_off[G] != T) return DGN_ERR_INVALID_ARG;
        for (int32_t g = 0; g < G; ++g)
            if (op_off[g + 1] < op_off[g] || t_off[g + 1] < t_off[g]) return DGN_ERR_INVALID_ARG;
    }
    return DGN_OK;
}

struct GraphLayout {
    int32_t *in_rowptr, *in_idx, *out_rowptr, *out_idx, *prod_rowptr, *prod_idx;
    int4 *orec;
    int32_t *prod1;
    int64_t *op_off, *t_off;
    size_t bytes;
};

GraphLayout graph_layout(void *mem, int64_t P, int64_t T, int64_t Ein, int64_t Eout, int32_t G, bool own_op_csr)
{
    Carver c(mem);
    GraphLayout L{};
    if (own_op_csr) {
        L.in_rowptr = c.take<int32_t>(P + 1);
        L.in_idx = c.take<int32_t>(Ein);
        L.out_rowptr = c.take<int32_t>(P + 1);
        L.out_idx = c.take<int32_t>(Eout);
    }
    L.prod_rowptr = c.take<int32_t>(T + 1);
    L.prod_idx = c.take<int32_t>(Eout);
    L.orec = c.take<int4>(P);
    L.prod1 = c.take<int32_t>(T);
    if (G > 1) {
        L.op_off = c.take<int64_t>(G + 1);
        L.t_off = c.take<int64_t>(G + 1);
    }
    L.bytes = c.off > 0 ? c.off : 256;
    return L;
}

struct BuildScratch {
    int32_t *status;        // [64] ints; status[0] = error bits
    int32_t *sorted_ops;    // [Eout] operator id of every entry of out_idx
    int32_t *sorted_keys;   // [max(Ein, Eout)] keys of a sort in row order, for the row pointers
    void *sort_tmp;
    void *scan_tmp;
    size_t bytes;
};

BuildScratch build_scratch(void *mem, int64_t P, int64_t T, int64_t Ein, int64_t Eout)
{
    Carver c(mem);
    BuildScratch S{};
    S.status = c.take<int32_t>(64);
    S.sorted_ops = c.take<int32_t>(Eout);
    const int64_t emax = Ein > Eout ? Ein : Eout;
    S.sorted_keys = c.take<int32_t>(emax);
    S.sort_tmp = c.take<char>(sort_tmp_bytes(emax));
    S.scan_tmp = c.take<char>(scan_tmp_bytes((P > T ? P : T) + 1));
    S.bytes = c.off;
    return S;
}

struct PruneScratch {
    TravState *state;
    TravCounters *ctr;
    int32_t *q0, *q1;       // frontier queues: qg.S segments of qg.seg_cap tensor ids each
    QueueGeom qg;
    uint8_t *DB;            // deferred-operator markers, one byte per operator
    uint8_t *flagbuf;       // keep flags (a byte per operator) when the caller's op_flag cannot take them
    u64 *opbits;
    int32_t *block_counts;
    int4 *trace;            // per-level trace records (profiling only)
    int64_t *pq_part;       // replicated per-set counters (few graphs only), NULL otherwise
    int pq_replicas;
    size_t pq_part_bytes;
    size_t db_bytes, opbits_bytes;
    RecycleHeader *hdr;     // says which buffers hold the result of the last prune that kept a complete log
    ColourLog log;          // tensors that prune coloured
    size_t bytes;
};

// Segments: enough of them that no push counter sees more than a few hundred waves per level, few
// enough that tiny graphs do not pay for empty segments.  Total capacity 2T + slack: a level can hold
// more than T entries because the frontier is not deduplicated (beyond that, the overflow path runs).
QueueGeom queue_geometry(int64_t T, int64_t max_entries)
{
    int S = 1;
    while (S < kMaxSeg && (int64_t)S * 16384 < T) S *= 2;
    int64_t total = 2 * T + 1024;
    if (max_entries > 0 && max_entries < total) total = max_entries;
    int64_t seg = (total + S - 1) / S;
    if (seg < 1) seg = 1;
    return QueueGeom{S, (int32_t)seg};
}

PruneScratch prune_scratch(void *mem, int64_t P, int64_t T, int32_t G, int64_t max_entries)
{
    Carver c(mem);
    PruneScratch S{};
    // What one prune leaves for the next comes first, where no option moves it.  Log of coloured tensors: a
    // quarter of T in all.  Recycling only pays while a prune colours a small part of the graph; one that
    // overflows the log makes the next prune clear everything, as if there were no log.
    S.hdr = c.take<RecycleHeader>(4);
    S.log.cnt = c.take<SegCounter>(kMaxSeg);
    int64_t lcap = T / (4 * kMaxSeg);
    if (lcap < 4096) lcap = 4096;
    S.log.seg_cap = (int32_t)lcap;
    S.log.entries = c.take<int32_t>((size_t)kMaxSeg * (size_t)lcap);
    S.state = c.take<TravState>(2);
    S.ctr = c.take<TravCounters>(1);
    S.qg = queue_geometry(T, max_entries);
    const size_t qn = (size_t)S.qg.S * (size_t)S.qg.seg_cap;
    S.q0 = c.take<int32_t>(qn);
    S.q1 = c.take<int32_t>(qn);
    const size_t obw = (size_t)((P + 63) / 64);
    S.DB = c.take<uint8_t>(obw * 64);         // a whole number of 64-operator words, so chunk loads stay inside
    S.db_bytes = obw * 64;
    S.flagbuf = c.take<uint8_t>(obw * 64);
    S.opbits = c.take<u64>(obw);
    S.opbits_bytes = obw * 8;
    S.block_counts = c.take<int32_t>((P + kCompactTile - 1) / kCompactTile + 1);
    S.trace = c.take<int4>(kTraceLevels);
    // with fewer than 64 graphs the 64*G per-set counters would be hot words: replicate them
    S.pq_replicas = 1;
    while (S.pq_replicas * 2 * (int64_t)G <= 64) S.pq_replicas *= 2;
    S.pq_part_bytes = S.pq_replicas > 1 ? sizeof(int64_t) * 64 * (size_t)G * S.pq_replicas * kPqStride : 0;
    S.pq_part = c.take<int64_t>(S.pq_part_bytes / sizeof(int64_t));
    if (S.pq_replicas == 1) S.pq_part = nullptr;
    S.bytes = c.off;
    return S;
}

// One small pinned buffer per host thread for status read-backs (never freed: a few hundred bytes).
int pinned_buffer(void **out)
{
    thread_local void *buf = nullptr;
    if (!buf) DGN_HIP(hipHostMalloc(&buf, 256, hipHostMallocDefault));
    *out = buf;
    return DGN_OK;
}

// Events for options->profile, created once per host thread.
int profile_events(hipEvent_t **out)
{
    thread_local hipEvent_t ev[8];
    thread_local bool ready = false;
    if (!ready) {
        for (int i = 0; i < 8; ++i) DGN_HIP(hipEventCreate(&ev[i]));
        ready = true;
    }
    *out = ev;
    return DGN_OK;
}

int error_bits_to_code(int32_t bits)
{
    if (bits & kErrCsr) return DGN_ERR_BAD_CSR;
    if (bits & (kErrIdRange | kErrCrossGraph)) return DGN_ERR_ID_OUT_OF_RANGE;
    if (bits & kErrTopo) return DGN_ERR_NOT_TOPOLOGICAL;
    return DGN_OK;
}

int check_options(const dgn_options *o)
{
    if (!o) return DGN_OK;
    if (o->traversal < 0 || o->traversal > 2) return DGN_ERR_INVALID_ARG;
    if (o->defer_percent < 0 || o->defer_percent > 100) return DGN_ERR_INVALID_ARG;
    if (o->max_queue_entries < 0) return DGN_ERR_INVALID_ARG;
    if (o->recycle < 0 || o->recycle > 1) return DGN_ERR_INVALID_ARG;
    if (o->profile < 0 || o->profile > 2) return DGN_ERR_INVALID_ARG;
    if (o->defer_start_shift < 0 || o->defer_start_shift > 30) return DGN_ERR_INVALID_ARG;
    if (o->defer_floor_shift < 0 || o->defer_floor_shift > 30) return DGN_ERR_INVALID_ARG;
    return DGN_OK;
}

}  // namespace

struct dgn_graph {
    GraphView v;
    int64_t P, T, Ein, Eout;
    int32_t G;
    int num_cus;
    bool topological;       // operator ids verified to be a topological order at build time
    bool multi_producer;    // some tensor is written by more than one operator
    int64_t max_graph_ops;  // largest graph of a packed batch (P for a single graph)
    uint64_t serial;        // unique per handle in this process
    // Hints only, taken from the last prune of this graph; a wrong one costs launches that return at once,
    // or a second batch, and corrects itself.  Kept apart for full prunes [0] and incremental ones [1],
    // whose traversals look nothing alike.
    //   wide_hint: wide levels were needed, so they are enqueued behind the first single-workgroup launch
    //     without waiting for its outcome;
    //   hint_runs, hint_run_len: how that prune alternated between stretches of wide levels and the
    //     single-workgroup kernel (lengths of the first stretches; 0 stretches: unknown); the launches are
    //     laid out the same way instead of in fixed groups.
    mutable std::atomic<int> wide_hint[2] = {};
    mutable std::atomic<int> hint_runs[2] = {};
    mutable std::atomic<int> hint_run_len[2][dgn::kMaxRuns] = {};
    //   exact_streak: prunes in a row whose traversal followed the hinted layout to the launch; after a few the
    //     spare launches at its end are dropped (a miss then costs one more batch, and brings them back)
    mutable std::atomic<int> exact_streak[2] = {};
    //   backward_passes: forward passes the last backward prune of this graph needed; the next one enqueues that many
    //     before it looks at their outcome
    mutable std::atomic<int> backward_passes = {};
};

namespace {

int finish_build(dgn_graph *h, const GraphLayout &L, const int64_t *op_off_host, const int64_t *t_off_host,
                 int32_t *status, const dgn_options *options, hipStream_t s, dgn_graph **out)
{
    DGN_HIP(launch_build_records(h->v, L.orec, L.prod1, status + kStatusMulti, s));
    if (h->G > 1) {
        DGN_HIP(hipMemcpyAsync(L.op_off, op_off_host, sizeof(int64_t) * (h->G + 1), hipMemcpyHostToDevice, s));
        DGN_HIP(hipMemcpyAsync(L.t_off, t_off_host, sizeof(int64_t) * (h->G + 1), hipMemcpyHostToDevice, s));
        h->v.op_off = L.op_off;
        h->v.t_off = L.t_off;
    }
    // The topological precondition is checked when the caller asks for validation, and for packed
    // batches, whose per-graph sweep is only chosen when it holds.  (One random access per edge: not
    // worth paying on every build of a big single graph, whose traversal does not depend on it.)  A packed batch
    // gets it in the walk over the edges that checks the graphs' ranges.
    const bool check_topo = (options && options->validate) || h->G >= kSweepMinGraphs;
    if (h->G > 1) DGN_HIP(launch_check_graph_ranges(h->v, status, check_topo, s));
    else if (check_topo) DGN_HIP(launch_check_topological(h->v, status, s));
    void *pin = nullptr;
    int rc = pinned_buffer(&pin);
    if (rc) return rc;
    DGN_HIP(hipMemcpyAsync(pin, status, (kStatusMulti + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    DGN_HIP(hipStreamSynchronize(s));
    int32_t bits = *static_cast<int32_t *>(pin);
    h->topological = check_topo && (bits & kErrTopo) == 0;
    h->multi_producer = static_cast<int32_t *>(pin)[kStatusMulti] != 0;
    if (!(options && options->validate)) bits &= ~kErrTopo;
    rc = error_bits_to_code(bits);
    if (rc) return rc;
    h->max_graph_ops = h->P;
    static std::atomic<uint64_t> next_serial{1};
    h->serial = next_serial.fetch_add(1, std::memory_order_relaxed);
    if (h->G > 1) {
        h->max_graph_ops = 0;
        for (int32_t i = 0; i < h->G; ++i)
            if (op_off_host[i + 1] - op_off_host[i] > h->max_graph_ops) h->max_graph_ops = op_off_host[i + 1] - op_off_host[i];
    }
    int dev = 0, cus = 0;
    DGN_HIP(hipGetDevice(&dev));
    DGN_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    h->num_cus = cus > 0 ? cus : 256;
    *out = h;
    return DGN_OK;
}

}  // namespace

extern "C" {

int dgn_version(void) { return DGN_VERSION; }
int dgn_last_hip_error(void) { return t_last_hip; }

const char *dgn_strerror(int code)
{
    switch (code) {
        case DGN_OK: return "ok";
        case DGN_ERR_INVALID_ARG: return "invalid argument";
        case DGN_ERR_NULL_PTR: return "required pointer is NULL";
        case DGN_ERR_TOO_LARGE: return "count too large for 32-bit ids";
        case DGN_ERR_ID_OUT_OF_RANGE: return "operator, tensor or target id out of range";
        case DGN_ERR_TOO_MANY_SETS: return "number of target sets must be 1..64";
        case DGN_ERR_WORKSPACE_TOO_SMALL: return "graph storage or scratch smaller than the queried size";
        case DGN_ERR_NOT_TOPOLOGICAL: return "operator ids are not a topological order";
        case DGN_ERR_HIP: return "HIP runtime error";
        case DGN_ERR_BAD_CSR: return "malformed CSR row pointers";
        default: return "unknown error";
    }
}

int dgn_graph_build_workspace(const dgn_coo_desc *d, size_t *graph_bytes, size_t *scratch_bytes)
{
    if (!d || !graph_bytes || !scratch_bytes) return DGN_ERR_NULL_PTR;
    int rc = check_sizes(d->num_ops, d->num_tensors, d->nnz_in, d->nnz_out, d->num_graphs, d->graph_op_offsets,
                         d->graph_tensor_offsets);
    if (rc) return rc;
    *graph_bytes = graph_layout(nullptr, d->num_ops, d->num_tensors, d->nnz_in, d->nnz_out, d->num_graphs, true).bytes;
    *scratch_bytes = build_scratch(nullptr, d->num_ops, d->num_tensors, d->nnz_in, d->nnz_out).bytes;
    return DGN_OK;
}

int dgn_graph_build(const dgn_coo_desc *d, void *graph_mem, size_t graph_bytes, void *scratch, size_t scratch_bytes,
                    const dgn_options *options, dgn_stream stream, dgn_graph **out)
{
    if (!d || !out) return DGN_ERR_NULL_PTR;
    *out = nullptr;
    size_t need_g = 0, need_s = 0;
    int rc = dgn_graph_build_workspace(d, &need_g, &need_s);
    if (rc) return rc;
    rc = check_options(options);
    if (rc) return rc;
    if (!graph_mem || !scratch) return DGN_ERR_NULL_PTR;
    if ((d->nnz_in > 0 && (!d->in_op || !d->in_tensor)) || (d->nnz_out > 0 && (!d->out_op || !d->out_tensor)))
        return DGN_ERR_NULL_PTR;
    if (graph_bytes < need_g || scratch_bytes < need_s) return DGN_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)graph_mem | (uintptr_t)scratch) & 7) return DGN_ERR_INVALID_ARG;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t P = d->num_ops, T = d->num_tensors, Ein = d->nnz_in, Eout = d->nnz_out;
    const GraphLayout L = graph_layout(graph_mem, P, T, Ein, Eout, d->num_graphs, true);
    const BuildScratch S = build_scratch(scratch, P, T, Ein, Eout);

    // One pass per edge list (all three in COO order) checks the ids, notes whether the keys ever decrease
    // (status[1..3]) and, on the assumption that they do not, already writes the finished rows: a graph
    // recorded operator by operator needs nothing more.  Reading the flags costs one synchronisation.
    FillRegion clr[1] = {{S.status, 256}};
    DGN_HIP(launch_clear(clr, 1, s));
    DGN_HIP(launch_scan_edges(d->in_op, d->in_tensor, Ein, (int32_t)P, (int32_t)T, L.in_idx, L.in_rowptr, S.status, S.status + 1, S.status + 5, s));
    DGN_HIP(launch_scan_edges(d->out_op, d->out_tensor, Eout, (int32_t)P, (int32_t)T, L.out_idx, L.out_rowptr, S.status, S.status + 2, S.status + 6, s));
    DGN_HIP(launch_scan_edges(d->out_tensor, d->out_op, Eout, (int32_t)T, (int32_t)P, L.prod_idx, L.prod_rowptr, S.status, S.status + 3, S.status + 7, s));
    void *pin = nullptr;
    rc = pinned_buffer(&pin);
    if (rc != DGN_OK) return rc;
    DGN_HIP(hipMemcpyAsync(pin, S.status, 8 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    DGN_HIP(hipStreamSynchronize(s));
    const int32_t *flags = static_cast<const int32_t *>(pin);
    if (flags[0]) return error_bits_to_code(flags[0]);       // bad ids: nothing is built from them
    const bool in_sorted = !flags[1], out_sorted = !flags[2];
    const bool prod_sorted = out_sorted && !flags[3];         // the third sort reads the outputs in operator order
    // Otherwise stable sorts: edges by operator (rows keep COO order), then outputs by tensor, which leaves each
    // tensor's producers ascending in operator id; row pointers from the sorted keys (first position of every
    // key): no histogram, no atomics.
    // (flags[5..7]: the pass met a long run of empty rows and left the row pointers to launch_row_bounds)
    if (!in_sorted) {
        DGN_HIP(launch_sort_pairs(d->in_op, d->in_tensor, S.sorted_keys, L.in_idx, Ein, key_bits_for(P), S.sort_tmp, s));
        DGN_HIP(launch_row_bounds(S.sorted_keys, Ein, (int32_t)P, L.in_rowptr, s));
    } else if (flags[5]) {
        DGN_HIP(launch_row_bounds(d->in_op, Ein, (int32_t)P, L.in_rowptr, s));
    }
    const int32_t *ops_of_out = d->out_op;                    // operator of every entry of out_idx
    if (!out_sorted) {
        DGN_HIP(launch_sort_pairs(d->out_op, d->out_tensor, S.sorted_ops, L.out_idx, Eout, key_bits_for(P), S.sort_tmp, s));
        DGN_HIP(launch_row_bounds(S.sorted_ops, Eout, (int32_t)P, L.out_rowptr, s));
        ops_of_out = S.sorted_ops;
    } else if (flags[6]) {
        DGN_HIP(launch_row_bounds(d->out_op, Eout, (int32_t)P, L.out_rowptr, s));
    }
    if (!prod_sorted) {
        DGN_HIP(launch_sort_pairs(L.out_idx, ops_of_out, S.sorted_keys, L.prod_idx, Eout, key_bits_for(T), S.sort_tmp, s));
        DGN_HIP(launch_row_bounds(S.sorted_keys, Eout, (int32_t)T, L.prod_rowptr, s));
    } else if (flags[7]) {
        DGN_HIP(launch_row_bounds(d->out_tensor, Eout, (int32_t)T, L.prod_rowptr, s));
    }

    dgn_graph *h = new (std::nothrow) dgn_graph();
    if (!h) return DGN_ERR_INVALID_ARG;
    h->P = P; h->T = T; h->Ein = Ein; h->Eout = Eout; h->G = d->num_graphs;
    h->v = GraphView{(int32_t)P, (int32_t)T, (int32_t)Ein, (int32_t)Eout, d->num_graphs, L.in_rowptr, L.in_idx,
                     L.out_rowptr, L.out_idx, L.prod_rowptr, L.prod_idx, nullptr, nullptr, L.orec, L.prod1};
    rc = finish_build(h, L, d->graph_op_offsets, d->graph_tensor_offsets, S.status, options, s, out);
    if (rc) delete h;
    return rc;
}

int dgn_graph_from_csr_workspace(const dgn_csr_desc *d, size_t *graph_bytes, size_t *scratch_bytes)
{
    if (!d || !graph_bytes || !scratch_bytes) return DGN_ERR_NULL_PTR;
    int rc = check_sizes(d->num_ops, d->num_tensors, d->nnz_in, d->nnz_out, d->num_graphs, d->graph_op_offsets,
                         d->graph_tensor_offsets);
    if (rc) return rc;
    *graph_bytes = graph_layout(nullptr, d->num_ops, d->num_tensors, d->nnz_in, d->nnz_out, d->num_graphs, false).bytes;
    *scratch_bytes = build_scratch(nullptr, d->num_ops, d->num_tensors, d->nnz_in, d->nnz_out).bytes;
    return DGN_OK;
}

int dgn_graph_from_csr(const dgn_csr_desc *d, void *graph_mem, size_t graph_bytes, void *scratch, size_t scratch_bytes,
                       const dgn_options *options, dgn_stream stream, dgn_graph **out)
{
    if (!d || !out) return DGN_ERR_NULL_PTR;
    *out = nullptr;
    size_t need_g = 0, need_s = 0;
    int rc = dgn_graph_from_csr_workspace(d, &need_g, &need_s);
    if (rc) return rc;
    rc = check_options(options);
    if (rc) return rc;
    if (!graph_mem || !scratch || !d->in_rowptr || !d->out_rowptr) return DGN_ERR_NULL_PTR;
    if ((d->nnz_in > 0 && !d->in_idx) || (d->nnz_out > 0 && !d->out_idx)) return DGN_ERR_NULL_PTR;
    if (graph_bytes < need_g || scratch_bytes < need_s) return DGN_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)graph_mem | (uintptr_t)scratch) & 7) return DGN_ERR_INVALID_ARG;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t P = d->num_ops, T = d->num_tensors, Ein = d->nnz_in, Eout = d->nnz_out;
    const GraphLayout L = graph_layout(graph_mem, P, T, Ein, Eout, d->num_graphs, false);
    const BuildScratch S = build_scratch(scratch, P, T, Ein, Eout);

    FillRegion clr[2] = {{L.prod_rowptr, align256((T + 1) * 4)}, {S.status, 256}};
    DGN_HIP(launch_clear(clr, 2, s));
    // the borrowed arrays are checked before any kernel trusts them
    DGN_HIP(launch_check_csr(d->in_rowptr, d->in_idx, (int32_t)P, (int32_t)Ein, (int32_t)T, S.status, s));
    DGN_HIP(launch_check_csr(d->out_rowptr, d->out_idx, (int32_t)P, (int32_t)Eout, (int32_t)T, S.status, s));
    void *pin = nullptr;
    rc = pinned_buffer(&pin);
    if (rc) return rc;
    DGN_HIP(hipMemcpyAsync(pin, S.status, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    DGN_HIP(hipStreamSynchronize(s));
    rc = error_bits_to_code(*static_cast<int32_t *>(pin));
    if (rc) return rc;

    DGN_HIP(launch_expand_rows(d->out_rowptr, (int32_t)P, S.sorted_ops, s));
    DGN_HIP(launch_degree_hist(d->out_idx, nullptr, Eout, (int32_t)T, 1, L.prod_rowptr, S.status, S.status + 3, s));
    DGN_HIP(launch_exclusive_scan(L.prod_rowptr, L.prod_rowptr, T, S.scan_tmp, s));
    DGN_HIP(launch_sort_pairs(d->out_idx, S.sorted_ops, nullptr, L.prod_idx, Eout, key_bits_for(T), S.sort_tmp, s));

    dgn_graph *h = new (std::nothrow) dgn_graph();
    if (!h) return DGN_ERR_INVALID_ARG;
    h->P = P; h->T = T; h->Ein = Ein; h->Eout = Eout; h->G = d->num_graphs;
    h->v = GraphView{(int32_t)P, (int32_t)T, (int32_t)Ein, (int32_t)Eout, d->num_graphs, d->in_rowptr, d->in_idx,
                     d->out_rowptr, d->out_idx, L.prod_rowptr, L.prod_idx, nullptr, nullptr, L.orec, L.prod1};
    rc = finish_build(h, L, d->graph_op_offsets, d->graph_tensor_offsets, S.status, options, s, out);
    if (rc) delete h;
    return rc;
}

int dgn_graph_get_csr(const dgn_graph *g, const int32_t **in_rowptr, const int32_t **in_idx, const int32_t **out_rowptr,
                      const int32_t **out_idx, const int32_t **prod_rowptr, const int32_t **prod_idx)
{
    if (!g) return DGN_ERR_NULL_PTR;
    if (in_rowptr) *in_rowptr = g->v.in_rowptr;
    if (in_idx) *in_idx = g->v.in_idx;
    if (out_rowptr) *out_rowptr = g->v.out_rowptr;
    if (out_idx) *out_idx = g->v.out_idx;
    if (prod_rowptr) *prod_rowptr = g->v.prod_rowptr;
    if (prod_idx) *prod_idx = g->v.prod_idx;
    return DGN_OK;
}

int dgn_graph_get_sizes(const dgn_graph *g, int64_t *num_ops, int64_t *num_tensors, int64_t *nnz_in, int64_t *nnz_out,
                        int32_t *num_graphs)
{
    if (!g) return DGN_ERR_NULL_PTR;
    if (num_ops) *num_ops = g->P;
    if (num_tensors) *num_tensors = g->T;
    if (nnz_in) *nnz_in = g->Ein;
    if (nnz_out) *nnz_out = g->Eout;
    if (num_graphs) *num_graphs = g->G;
    return DGN_OK;
}

void dgn_graph_destroy(dgn_graph *g) { delete g; }

int dgn_prune_workspace(const dgn_graph *g, int32_t num_sets, size_t *scratch_bytes)
{
    if (!g || !scratch_bytes) return DGN_ERR_NULL_PTR;
    if (num_sets < 1 || num_sets > DGN_MAX_SETS) return DGN_ERR_TOO_MANY_SETS;
    *scratch_bytes = prune_scratch(nullptr, g->P, g->T, g->G, 0).bytes;
    return DGN_OK;
}

// dgn_prune.  also_M [T] / also_K [P] (or NULL): two more arrays that the call zeroes with M and K -- all of them,
// or, with recycled buffers, the words that the previous call's log and kept list name (the caller vouches that
// they hold non-zero words nowhere else).
static int prune_impl(const dgn_graph *g, int32_t num_sets, int64_t num_targets, const int32_t *tgt_rowptr,
                      const int32_t *tgt_idx, uint64_t *tensor_mask, uint64_t *op_mask, uint8_t *op_flag, int32_t *kept_ops,
                      uint64_t *kept_masks, int64_t *kept_count, int64_t *per_query_count, void *scratch,
                      size_t scratch_bytes, const dgn_options *options, dgn_stats *stats, dgn_stream stream,
                      uint64_t *also_M, uint64_t *also_K)
{
    if (!g) return DGN_ERR_NULL_PTR;
    if (num_sets < 1 || num_sets > DGN_MAX_SETS) return DGN_ERR_TOO_MANY_SETS;
    if (num_targets < 0) return DGN_ERR_INVALID_ARG;
    if (num_targets > kMaxCount) return DGN_ERR_TOO_LARGE;
    int rc = check_options(options);
    if (rc) return rc;
    if (!tgt_rowptr || (num_targets > 0 && !tgt_idx) || !kept_count || !scratch) return DGN_ERR_NULL_PTR;
    if ((g->T > 0 && !tensor_mask) || (g->P > 0 && (!op_mask || !kept_ops))) return DGN_ERR_NULL_PTR;
    const PruneScratch S = prune_scratch(scratch, g->P, g->T, g->G, options ? options->max_queue_entries : 0);
    if (scratch_bytes < S.bytes) return DGN_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)scratch | (uintptr_t)tensor_mask | (uintptr_t)op_mask | (uintptr_t)kept_masks |
         (uintptr_t)kept_count | (uintptr_t)per_query_count) & 7)
        return DGN_ERR_INVALID_ARG;

    hipStream_t s = static_cast<hipStream_t>(stream);
    u64 *M = reinterpret_cast<u64 *>(tensor_mask);
    u64 *K = reinterpret_cast<u64 *>(op_mask);
    const size_t pq_bytes = per_query_count ? sizeof(int64_t) * 64 * (size_t)(g->G > 1 ? g->G : 1) : 0;
    int64_t launches = 0, level_launches = 0;
    // 0 start, 1 cleared, 2 seeded, 3 traversed, 4 counted, 5 scanned, 6 scattered.  An event between two
    // kernels costs a few microseconds of idle stream, so profile = 2 records only the two around the traversal.
    hipEvent_t *ev = nullptr;
    hipEvent_t *ev_trav = nullptr;
    if (options && options->profile && stats) {
        rc = profile_events(&ev_trav);
        if (rc) return rc;
        if (options->profile == 1) {
            ev = ev_trav;
            DGN_HIP(hipEventRecord(ev[0], s));
        }
    }

    // nothing marked yet: clear outputs, deferral markers and traversal state (an incremental call keeps
    // M and K: they hold a fixed point that the new target bits only add to).  With `recycle` the scratch
    // buffer may say that M, K and the kept list are still those of the previous prune of this graph: then
    // only what that prune set is zeroed, and this prune keeps a log of what it colours for the next one.
    const bool incremental = options && options->incremental;
    const bool sweep = !(options && options->traversal != 0) && g->G >= kSweepMinGraphs && g->topological &&
                       g->max_graph_ops <= kSweepMaxGraphOps;
    const bool recycle = options && options->recycle && !incremental && !sweep && g->P > 0;
    // The traversal sets a byte for every operator whose K leaves zero, which lets the count pass read P bytes
    // and the K of the kept operators instead of all of K.  The bytes are the caller's op_flag when that can be
    // cleared in whole 8-byte words, else a scratch array.  (Not for the per-graph sweep, which writes K
    // without atomics and finds nothing out about "first"; not for incremental calls, whose K comes from outside.)
    const bool use_flags = !sweep && !incremental && !(options && options->recompute_keep);
    uint8_t *flags = (op_flag && ((uintptr_t)op_flag & 7) == 0 && g->P % 8 == 0) ? op_flag : S.flagbuf;
    const size_t flag_bytes = flags == op_flag ? (size_t)g->P : S.db_bytes;
    const ColourLog log{recycle ? S.log.entries : nullptr, S.log.cnt, S.log.seg_cap};
    const RecycleHeader want{kRecycleMagic, g->serial, M, K, kept_ops, kept_count, flags, also_M, also_K, {0, 0, 0}};
    if (recycle) {
        // (the flag bytes are cleared whether or not this call's count pass reads them: the header this call leaves
        // names them, and the call that finds it zeroes them at this call's kept operators only)
        FillRegion big[6] = {{M, (size_t)g->T * 8}, {K, (size_t)g->P * 8}, {S.DB, S.db_bytes},
                             {flags, flag_bytes}, {also_M, (size_t)g->T * 8}, {also_K, (size_t)g->P * 8}};
        DGN_HIP(launch_clear_or_reset(big, 6, S.hdr, want, reinterpret_cast<u64 *>(S.state + 1), S.log, kept_ops, kept_count, M, K,
                                      S.DB, flags, s));
        // (the word behind the state header says which way the kernel above went: it comes back with the header)
        FillRegion small[6] = {{S.state, sizeof(TravState)}, {S.ctr, sizeof(TravCounters)}, {S.hdr, sizeof(RecycleHeader)},
                               {S.log.cnt, sizeof(SegCounter) * kMaxSeg}, {per_query_count, pq_bytes},
                               {S.pq_part, per_query_count ? S.pq_part_bytes : 0}};
        DGN_HIP(launch_clear(small, 6, s));
        ++launches;
    } else {
        // (the per-graph sweep stores K of every operator and uses no markers: it needs M cleared, nothing else)
        FillRegion clr[8] = {{M, incremental ? 0 : (size_t)g->T * 8}, {K, incremental || sweep ? 0 : (size_t)g->P * 8},
                             {S.DB, sweep ? 0 : S.db_bytes}, {S.state, 256 + sizeof(TravCounters)}, {S.hdr, 256},
                             {per_query_count, pq_bytes}, {S.pq_part, per_query_count ? S.pq_part_bytes : 0},
                             {flags, use_flags ? flag_bytes : 0}};
        DGN_HIP(launch_clear(clr, 8, s));
        if (also_M || also_K) {
            FillRegion more[2] = {{also_M, (size_t)g->T * 8}, {also_K, (size_t)g->P * 8}};
            DGN_HIP(launch_clear(more, 2, s));
            ++launches;
        }
    }
    if (ev) DGN_HIP(hipEventRecord(ev[1], s));
    // deferral schedule: threshold on the producer id, starting at decay*P and decaying geometrically
    const int defer_percent = options && options->defer_percent ? options->defer_percent : kDefaultDeferPercent;
    const int start_shift = options && options->defer_start_shift ? options->defer_start_shift : kDefaultStartShift;
    const int floor_shift = options && options->defer_floor_shift ? options->defer_floor_shift : kDefaultFloorShift;
    Schedule sch{1.0f, 0, 0, kSmallLevel};
    if (defer_percent < 100) {
        sch.decay = (float)defer_percent / 100.0f;
        sch.theta0 = (int32_t)(g->P >> start_shift);
        sch.theta_floor = (int32_t)(g->P >> floor_shift);
        if (sch.theta_floor < 64) sch.theta_floor = 64;
        if (sch.theta0 < sch.theta_floor) sch.theta0 = 0;
    }
    DGN_HIP(launch_seed(g->v, num_sets, num_targets, tgt_rowptr, tgt_idx, M, S.state, S.ctr, sweep ? nullptr : S.q0, S.qg,
                        sch.theta0, log, s));
    if (ev_trav) DGN_HIP(hipEventRecord(ev_trav[2], s));
    launches += 2;

    CompactArgs ca{};
    ca.g = g->v;
    ca.M = M;
    ca.K = K;
    ca.op_flag = op_flag;
    ca.kept_ops = kept_ops;
    ca.kept_masks = reinterpret_cast<u64 *>(kept_masks);
    ca.kept_count = kept_count;
    ca.per_query_count = per_query_count;
    ca.opbits = S.opbits;
    ca.block_counts = S.block_counts;
    ca.pq_part = S.pq_part;
    ca.pq_replicas = S.pq_replicas;
    ca.from_tensor_mask = options && options->recompute_keep;
    ca.flag_in = use_flags ? flags : nullptr;
    ca.hdr = recycle ? S.hdr : nullptr;
    ca.want = want;
    ca.error = &S.state->error;

    void *pin = nullptr;
    rc = pinned_buffer(&pin);
    if (rc) return rc;
    const TravState *hst = static_cast<const TravState *>(pin);

    // Packed batch of many small graphs in topological order: one wave sweeps each graph once (see
    // k_sweep_graphs); no frontier, no level loop, per-set counts come out of the sweep itself.
    if (sweep) {
        DGN_HIP(launch_sweep_graphs(g->v, M, K, ca.from_tensor_mask ? nullptr : per_query_count, g->multi_producer, s));
        ++launches;
        if (ev_trav) DGN_HIP(hipEventRecord(ev_trav[3], s));
        if (!ca.from_tensor_mask) ca.per_query_count = nullptr;   // already written by the sweep
        DGN_HIP(launch_keep_compact(ca, s, ev ? ev + 4 : nullptr));
        launches += 3 + (g->G > 1);
        DGN_HIP(hipMemcpyAsync(pin, S.state, sizeof(TravState), hipMemcpyDeviceToHost, s));
        DGN_HIP(hipStreamSynchronize(s));
        if (stats) {
            int32_t *user_trace = stats->level_trace;
            const int64_t user_cap = stats->level_trace_cap;
            memset(stats, 0, sizeof(*stats));
            stats->level_trace = user_trace;
            stats->level_trace_cap = user_cap;
            stats->launches = launches;
            stats->tensor_visits = g->P;
            if (ev) {
                for (int i = 0; i < 6; ++i) DGN_HIP(hipEventElapsedTime(&stats->phase_ms[i], ev[i], ev[i + 1]));
                DGN_HIP(hipEventElapsedTime(&stats->phase_ms[DGN_PHASE_TOTAL], ev[0], ev[6]));
            } else if (ev_trav) {
                DGN_HIP(hipEventElapsedTime(&stats->phase_ms[DGN_PHASE_TRAVERSE], ev_trav[2], ev_trav[3]));
            }
        }
        return error_bits_to_code(hst->error & ~kErrOverflow);
    }

    // Level loop.  The number of levels depends on the data, so the host enqueues kernels ahead and
    // reads the 64-byte state back at a few points:
    //   1. one single-workgroup launch walks all leading small levels (deep, thin graphs finish here);
    //   2. otherwise batches of wide levels with a single-workgroup launch after every few of them; the
    //      removal-rule/compaction passes are enqueued right behind the first batch and redone only if
    //      the traversal turns out unfinished.
    int grid = g->num_cus * kLevelBlocksPerCU;
    const int64_t max_useful = (g->T + 255) / 256;
    if (grid > max_useful) grid = (int)(max_useful > 0 ? max_useful : 1);
    const bool generic_only = options && options->traversal == 1;
    const int hk = (options && options->incremental) ? 1 : 0;      // which set of layout hints
    const int narrow_cap = generic_only ? 0 : kNarrowCap;
    int launch_no = 0;
    int32_t *user_trace = stats ? stats->level_trace : nullptr;
    const int64_t user_trace_cap = stats ? stats->level_trace_cap : 0;
    int4 *trace = (user_trace && user_trace_cap > 0) ? S.trace : nullptr;
    // the stand-alone removal-rule pass rewrites K, which the traversal still needs while unfinished
    const bool speculate = !ca.from_tensor_mask;
    bool done = false, compacted = false;
    // The record of a single-workgroup launch is a complete state (it leaves no tallies to fold in), so every
    // batch ends with one, and that record is what is read back.
    bool last_was_narrow = false;
    auto narrow = [&]() -> int {
        DGN_HIP(launch_narrow(g->v, S.state, S.ctr, launch_no, S.q0, S.q1, S.qg, S.DB, flags, M, K, narrow_cap, sch, log, trace, s));
        ++launch_no; ++launches;
        last_was_narrow = true;
        return DGN_OK;
    };
    auto read_state = [&]() -> int {
        if (!last_was_narrow) {
            const int e = narrow();
            if (e) return e;
        }
        DGN_HIP(hipMemcpyAsync(pin, S.state, 2 * sizeof(TravState), hipMemcpyDeviceToHost, s));
        DGN_HIP(hipStreamSynchronize(s));
        const LevelSlot &sl = hst->slot[(launch_no - 1) & 1];
        done = sl.n == 0 && !(sl.deferred_seen && sl.theta_hi > 0);
        return DGN_OK;
    };
    // A graph that needed wide levels last time starts with them at once: the wide kernel's second hop takes
    // the first two levels in one launch, where the single-workgroup kernel would stop after the first.
    if (!generic_only && !g->wide_hint[hk].load(std::memory_order_relaxed)) {
        rc = narrow();
        if (rc) return rc;
        rc = read_state();
        if (rc) return rc;
    }
    auto group = [&](int levels) -> int {            // `levels` wide launches, then the single-workgroup kernel
        for (int i = 0; i < levels; ++i) {
            // (a traversal that starts with a wide launch: that launch takes the seeds' level however small it is)
            const int cap = launch_no == 0 ? 0 : narrow_cap;
            DGN_HIP(launch_level(g->v, S.state, S.ctr, launch_no, S.q0, S.q1, S.qg, S.DB, flags, M, K, grid, cap, sch, log, trace, s));
            ++launch_no; ++launches; ++level_launches;
        }
        last_was_narrow = false;
        return narrow();
    };
    bool first = true;
    int batch = 0;
    int used_runs = 0, used_len[kMaxRuns] = {};       // the layout enqueued from the hints, if any
    while (!done) {
        const int hint_runs = generic_only ? 0 : g->hint_runs[hk].load(std::memory_order_relaxed);
        if (first && hint_runs > 0) {
            // the layout the previous prune of this graph turned out to need, plus a short tail
            int room = kMaxBatch;
            for (int r = 0; r < hint_runs && r < kMaxRuns && room > 0; ++r) {
                int len = g->hint_run_len[hk][r].load(std::memory_order_relaxed);
                len = len < 1 ? 1 : len > room ? room : len;
                rc = group(len);
                if (rc) return rc;
                room -= len + 1;
                used_len[used_runs++] = len;
            }
            if (g->exact_streak[hk].load(std::memory_order_relaxed) < kExactStreak) {
                rc = group(kTailLevels);
                if (rc) return rc;
            }
        } else {
            // unknown graph, or the layout fell short: groups of wide levels with the single-workgroup kernel
            // after each; a batch right after a hinted one is small (the hint was nearly right)
            const int groups = first ? kWideGroupsFirst : (hint_runs > 0 && batch == 1) ? 1 : kWideGroups;
            for (int i = 0; i < groups; ++i) {
                rc = group(kWidePerGroup);
                if (rc) return rc;
            }
        }
        ++batch;
        if (first && speculate) {
            if (ev_trav) DGN_HIP(hipEventRecord(ev_trav[3], s));
            DGN_HIP(launch_keep_compact(ca, s, ev ? ev + 4 : nullptr));
            launches += 3 + (g->G > 1);
            compacted = true;
        }
        rc = read_state();
        if (rc) return rc;
        if (!done) compacted = false;      // the speculative pass ran on unfinished masks
        first = false;
    }
    g->wide_hint[hk].store(hst->max_frontier > (u64)kNarrowCap ? 1 : 0, std::memory_order_relaxed);
    {
        const int nr = hst->n_runs < kMaxRuns ? hst->n_runs : kMaxRuns;
        bool exact = batch == 1 && used_runs > 0 && hst->n_runs == used_runs;
        for (int r = 0; r < nr; ++r) {
            if (exact && hst->wide_runs[r] != used_len[r]) exact = false;
            g->hint_run_len[hk][r].store(hst->wide_runs[r], std::memory_order_relaxed);
        }
        g->hint_runs[hk].store(nr, std::memory_order_relaxed);
        g->exact_streak[hk].store(exact ? g->exact_streak[hk].load(std::memory_order_relaxed) + 1 : 0,
                                  std::memory_order_relaxed);
    }
    if (recycle && (hst->error & (kErrOverflow | kErrLogFull))) {
        // the log is incomplete; a compaction enqueued ahead may have called it complete
        FillRegion hz[1] = {{S.hdr, sizeof(RecycleHeader)}};
        DGN_HIP(launch_clear(hz, 1, s));
        ++launches;
    }
    if (hst->error & kErrOverflow) {
        // A frontier queue overflowed and dropped entries: restore the fixed point with whole-graph
        // sweeps (each operator re-derives K from its outputs) until one of them changes nothing.
        compacted = false;
        int32_t *changed = &S.state->changed;
        for (;;) {
            FillRegion cz[1] = {{changed, 8}};
            DGN_HIP(launch_clear(cz, 1, s));
            DGN_HIP(launch_fix_sweep(g->v, M, K, flags, changed, grid, s));
            ++launches;
            DGN_HIP(hipMemcpyAsync(pin, S.state, sizeof(TravState), hipMemcpyDeviceToHost, s));
            DGN_HIP(hipStreamSynchronize(s));
            if (!hst->changed) break;
        }
    }
    if (!compacted) {
        if (pq_bytes) {
            FillRegion pq[2] = {{per_query_count, pq_bytes}, {S.pq_part, S.pq_part_bytes}};
            DGN_HIP(launch_clear(pq, 2, s));
            ++launches;
        }
        if (ev_trav) DGN_HIP(hipEventRecord(ev_trav[3], s));
        DGN_HIP(launch_keep_compact(ca, s, ev ? ev + 4 : nullptr));
        launches += 3 + (g->G > 1);
        DGN_HIP(hipStreamSynchronize(s));    // outputs are complete (and the phase events recorded) on return
    }
    if (stats) {
        memset(stats, 0, sizeof(*stats));
        stats->level_trace = user_trace;
        stats->level_trace_cap = user_trace_cap;
        stats->levels = hst->slot[(launch_no - 1) & 1].level;
        if (trace) {
            int64_t nrec = stats->levels < user_trace_cap ? stats->levels : user_trace_cap;
            if (nrec > kTraceLevels) nrec = kTraceLevels;
            if (nrec > 0) {
                DGN_HIP(hipMemcpyAsync(user_trace, S.trace, (size_t)nrec * sizeof(int4), hipMemcpyDeviceToHost, s));
                DGN_HIP(hipStreamSynchronize(s));
            }
        }
        stats->tensor_visits = (int64_t)hst->tensor_visits;
        stats->max_frontier = (int64_t)hst->max_frontier;
        stats->launches = launches;
        stats->level_launches = level_launches;
        stats->atomic_updates = (int64_t)hst->atomic_updates + num_targets;
        if (recycle) stats->recycled = *reinterpret_cast<const u64 *>(static_cast<const char *>(pin) + sizeof(TravState)) ? 1 : 0;
        if (ev) {
            for (int i = 0; i < 6; ++i) DGN_HIP(hipEventElapsedTime(&stats->phase_ms[i], ev[i], ev[i + 1]));
            DGN_HIP(hipEventElapsedTime(&stats->phase_ms[DGN_PHASE_TOTAL], ev[0], ev[6]));
        } else if (ev_trav) {
            DGN_HIP(hipEventElapsedTime(&stats->phase_ms[DGN_PHASE_TRAVERSE], ev_trav[2], ev_trav[3]));
        }
    }
    return error_bits_to_code(hst->error & ~(kErrOverflow | kErrLogFull));
}

int dgn_prune(const dgn_graph *g, int32_t num_sets, int64_t num_targets, const int32_t *tgt_rowptr,
              const int32_t *tgt_idx, uint64_t *tensor_mask, uint64_t *op_mask, uint8_t *op_flag, int32_t *kept_ops,
              uint64_t *kept_masks, int64_t *kept_count, int64_t *per_query_count, void *scratch, size_t scratch_bytes,
              const dgn_options *options, dgn_stats *stats, dgn_stream stream)
{
    return prune_impl(g, num_sets, num_targets, tgt_rowptr, tgt_idx, tensor_mask, op_mask, op_flag, kept_ops, kept_masks,
                      kept_count, per_query_count, scratch, scratch_bytes, options, stats, stream, nullptr, nullptr);
}

// Removal rule + compaction: K computed from tensor_mask_in (from_tensor_mask), or taken as it stands in op_mask.
// flag_in (or NULL): a byte per operator, 1 exactly where op_mask is not zero (then K is read there only).
static int keep_compact_impl(const dgn_graph *g, const uint64_t *tensor_mask_in, bool from_tensor_mask, uint64_t *op_mask,
                             uint8_t *op_flag, int32_t *kept_ops, uint64_t *kept_masks, int64_t *kept_count,
                             int64_t *per_query_count, void *scratch, size_t scratch_bytes, dgn_stream stream,
                             const uint8_t *flag_in = nullptr)
{
    if (!g) return DGN_ERR_NULL_PTR;
    if (!kept_count || !scratch) return DGN_ERR_NULL_PTR;
    if ((g->T > 0 && from_tensor_mask && !tensor_mask_in) || (g->P > 0 && (!op_mask || !kept_ops))) return DGN_ERR_NULL_PTR;
    const PruneScratch S = prune_scratch(scratch, g->P, g->T, g->G, 0);
    if (scratch_bytes < S.bytes) return DGN_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)scratch | (uintptr_t)tensor_mask_in | (uintptr_t)op_mask | (uintptr_t)kept_masks |
         (uintptr_t)kept_count | (uintptr_t)per_query_count) & 7)
        return DGN_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t pq_bytes = per_query_count ? sizeof(int64_t) * 64 * (size_t)(g->G > 1 ? g->G : 1) : 0;
    FillRegion pq[2] = {{per_query_count, pq_bytes}, {S.pq_part, per_query_count ? S.pq_part_bytes : 0}};
    DGN_HIP(launch_clear(pq, 2, s));
    CompactArgs ca{};
    ca.g = g->v;
    ca.M = reinterpret_cast<const u64 *>(tensor_mask_in);
    ca.K = reinterpret_cast<u64 *>(op_mask);
    ca.op_flag = op_flag;
    ca.kept_ops = kept_ops;
    ca.kept_masks = reinterpret_cast<u64 *>(kept_masks);
    ca.kept_count = kept_count;
    ca.per_query_count = per_query_count;
    ca.opbits = S.opbits;
    ca.block_counts = S.block_counts;
    ca.pq_part = S.pq_part;
    ca.pq_replicas = S.pq_replicas;
    ca.from_tensor_mask = from_tensor_mask;
    ca.flag_in = from_tensor_mask ? nullptr : flag_in;
    DGN_HIP(launch_keep_compact(ca, s));
    return DGN_OK;
}

int dgn_keep_compact(const dgn_graph *g, const uint64_t *tensor_mask_in, uint64_t *op_mask, uint8_t *op_flag,
                     int32_t *kept_ops, uint64_t *kept_masks, int64_t *kept_count, int64_t *per_query_count,
                     void *scratch, size_t scratch_bytes, dgn_stream stream)
{
    return keep_compact_impl(g, tensor_mask_in, true, op_mask, op_flag, kept_ops, kept_masks, kept_count, per_query_count,
                             scratch, scratch_bytes, stream);
}

// ---- removal rule + compaction for callers that cannot allocate ---------------------------------
// The passes' scratch (kept-operator bitmap, tile counts, replicated per-set counters) lives in an array
// of the code object itself, one copy per device; the host works with its device address, fetched once
// per device, never with the array's name.
constexpr int64_t kStaticMaxOps = (int64_t)1 << 26;
constexpr size_t kStaticBitmapBytes = (size_t)(kStaticMaxOps / 8);
constexpr size_t kStaticCountsBytes = ((size_t)(kStaticMaxOps / kCompactTile + 1) * sizeof(int32_t) + 255) & ~(size_t)255;
constexpr size_t kStaticPqBytes = sizeof(int64_t) * 64 * 64 * kPqStride;
constexpr size_t kStaticScratchBytes = kStaticBitmapBytes + kStaticCountsBytes + kStaticPqBytes;
static __device__ __align__(256) unsigned char static_scratch[kStaticScratchBytes];
constexpr int kStaticMaxDevices = 64;
static std::atomic<void *> g_static_scratch_ptr[kStaticMaxDevices];

// Device address of the current device's copy of the array.
static int static_scratch_address(char **out)
{
    int dev = -1;
    DGN_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticMaxDevices) return DGN_ERR_INVALID_ARG;
    void *p = g_static_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        DGN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch)));
        if (!p) return DGN_ERR_INVALID_ARG;
        g_static_scratch_ptr[dev].store(p, std::memory_order_release);   // (two threads racing here fetch the same address)
    }
    *out = static_cast<char *>(p);
    return DGN_OK;
}

int dgn_keep_compact_static_limits(int64_t *max_ops, size_t *static_bytes)
{
    if (max_ops) *max_ops = kStaticMaxOps;
    if (static_bytes) *static_bytes = kStaticScratchBytes;
    return DGN_OK;
}

int dgn_keep_compact_static(const dgn_graph *g, const uint64_t *tensor_mask_in, uint64_t *op_mask, uint8_t *op_flag,
                            int32_t *kept_ops, uint64_t *kept_masks, int64_t *kept_count, int64_t *per_query_count,
                            dgn_stream stream)
{
    if (!g || !kept_count) return DGN_ERR_NULL_PTR;
    if (g->P > kStaticMaxOps) return DGN_ERR_TOO_LARGE;
    if ((g->T > 0 && !tensor_mask_in) || (g->P > 0 && (!op_mask || !kept_ops))) return DGN_ERR_NULL_PTR;
    if (((uintptr_t)tensor_mask_in | (uintptr_t)op_mask | (uintptr_t)kept_masks | (uintptr_t)kept_count |
         (uintptr_t)per_query_count) & 7)
        return DGN_ERR_INVALID_ARG;
    char *base = nullptr;
    const int rc = static_scratch_address(&base);
    if (rc != DGN_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    CompactArgs ca{};
    ca.g = g->v;
    ca.M = reinterpret_cast<const u64 *>(tensor_mask_in);
    ca.K = reinterpret_cast<u64 *>(op_mask);
    ca.op_flag = op_flag;
    ca.kept_ops = kept_ops;
    ca.kept_masks = reinterpret_cast<u64 *>(kept_masks);
    ca.kept_count = kept_count;
    ca.per_query_count = per_query_count;
    ca.opbits = reinterpret_cast<u64 *>(base);
    ca.block_counts = reinterpret_cast<int32_t *>(base + kStaticBitmapBytes);
    // replicated per-set counters exactly as dgn_keep_compact lays them out: only with few graphs
    ca.pq_replicas = 1;
    while (ca.pq_replicas * 2 * (int64_t)g->G <= 64) ca.pq_replicas *= 2;
    const size_t pq_part_bytes = ca.pq_replicas > 1 ? sizeof(int64_t) * 64 * (size_t)g->G * ca.pq_replicas * kPqStride : 0;
    ca.pq_part = ca.pq_replicas > 1 ? reinterpret_cast<int64_t *>(base + kStaticBitmapBytes + kStaticCountsBytes) : nullptr;
    ca.from_tensor_mask = true;
    // the array keeps what the last call left: the counters must start at zero (a fill kernel, not a memset,
    // so that the call may be captured into a graph)
    const size_t pq_bytes = per_query_count ? sizeof(int64_t) * 64 * (size_t)(g->G > 1 ? g->G : 1) : 0;
    FillRegion pq[2] = {{per_query_count, pq_bytes}, {ca.pq_part, per_query_count ? pq_part_bytes : 0}};
    DGN_HIP(launch_clear(pq, 2, s));
    DGN_HIP(launch_keep_compact(ca, s));
    return DGN_OK;
}

int dgn_prune_words(const dgn_graph *g, int64_t num_sets, int64_t num_targets, const int32_t *tgt_rowptr,
                    const int32_t *tgt_idx, uint64_t *tensor_mask, uint64_t *op_mask, uint8_t *op_flag, int32_t *kept_ops,
                    uint64_t *kept_masks, int64_t *kept_count, int64_t *per_query_count, void *scratch,
                    size_t scratch_bytes, const dgn_options *options, dgn_stats *stats, dgn_stream stream)
{
    if (!g) return DGN_ERR_NULL_PTR;
    if (num_sets < 1 || num_sets > kMaxCount) return DGN_ERR_TOO_MANY_SETS;
    if (g->G > 1) return DGN_ERR_INVALID_ARG;        // a packed batch already numbers its sets graph by graph
    if (!tgt_rowptr) return DGN_ERR_NULL_PTR;
    const int64_t words = (num_sets + DGN_MAX_SETS - 1) / DGN_MAX_SETS;
    const size_t P = (size_t)g->P, T = (size_t)g->T;
    dgn_options per_word{};
    if (options) per_word = *options;
    if (words > 1) per_word.recycle = 0;             // one scratch buffer serves every word: its log covers the last only
    if (options) options = &per_word;
    dgn_stats total{};
    if (stats) total = *stats;
    total.levels = total.tensor_visits = total.launches = total.level_launches = 0;
    total.max_frontier = 0;
    for (int64_t w = 0; w < words; ++w) {
        const int32_t q = (int32_t)((num_sets - w * DGN_MAX_SETS) < DGN_MAX_SETS ? (num_sets - w * DGN_MAX_SETS) : DGN_MAX_SETS);
        // the sets of this word own entries [tgt_rowptr[64w], tgt_rowptr[64w + q]) of tgt_idx: the row
        // pointers hold absolute positions, so the slice is passed as it is and the seed step skips
        // every entry that lies outside it
        dgn_stats one{};
        if (stats) one = *stats;
        const int rc = dgn_prune(g, q, num_targets, tgt_rowptr + w * DGN_MAX_SETS, tgt_idx,
                                 tensor_mask ? tensor_mask + w * T : nullptr, op_mask ? op_mask + w * P : nullptr,
                                 op_flag ? op_flag + w * P : nullptr, kept_ops ? kept_ops + w * P : nullptr,
                                 kept_masks ? kept_masks + w * P : nullptr, kept_count ? kept_count + w : nullptr,
                                 per_query_count ? per_query_count + w * 64 : nullptr, scratch, scratch_bytes, options,
                                 stats ? &one : nullptr, stream);
        if (rc != DGN_OK) return rc;
        if (stats) {
            total.levels += one.levels;
            total.tensor_visits += one.tensor_visits;
            total.launches += one.launches;
            total.level_launches += one.level_launches;
            if (one.max_frontier > total.max_frontier) total.max_frontier = one.max_frontier;
            for (int i = 0; i < 8; ++i) total.phase_ms[i] = (w ? total.phase_ms[i] : 0.0f) + one.phase_ms[i];
        }
    }
    if (stats) *stats = total;
    return DGN_OK;
}

// ---- Backward Prune: scratch = [prune scratch][B: 8T][K of stage one: 8P][its kept list: 4P][small] ----
struct BackwardScratch {
    size_t prune_bytes;
    u64 *B, *KB;
    int32_t *kept, *tgt_rowptr, *flags;
    int64_t *kept_count;
    size_t bytes;
};

static BackwardScratch backward_scratch(void *mem, int64_t P, int64_t T, int32_t G)
{
    BackwardScratch b{};
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    b.prune_bytes = up(prune_scratch(nullptr, P, T, G, 0).bytes);
    char *p = static_cast<char *>(mem) + b.prune_bytes;
    b.B = reinterpret_cast<u64 *>(p); p += up((size_t)(T > 0 ? T : 1) * 8);
    b.KB = reinterpret_cast<u64 *>(p); p += up((size_t)(P > 0 ? P : 1) * 8);
    b.kept = reinterpret_cast<int32_t *>(p); p += up((size_t)(P > 0 ? P : 1) * 4);
    b.tgt_rowptr = reinterpret_cast<int32_t *>(p); p += 512;
    b.kept_count = reinterpret_cast<int64_t *>(p); p += up(sizeof(int64_t) * (size_t)(G > 1 ? G + 2 : 1));
    b.flags = reinterpret_cast<int32_t *>(p); p += 256;
    b.bytes = (size_t)(p - static_cast<char *>(mem));
    return b;
}

int dgn_backward_prune_workspace(const dgn_graph *g, size_t *scratch_bytes)
{
    if (!g || !scratch_bytes) return DGN_ERR_NULL_PTR;
    *scratch_bytes = backward_scratch(nullptr, g->P, g->T, g->G).bytes;
    return DGN_OK;
}

int dgn_backward_prune(const dgn_graph *g, int32_t num_pairs, const int32_t *obj, const int32_t *wrt,
                       uint64_t *tensor_mask, uint64_t *op_mask, uint8_t *op_flag, int32_t *kept_ops,
                       uint64_t *kept_masks, int64_t *kept_count, int64_t *per_query_count, void *scratch,
                       size_t scratch_bytes, const dgn_options *options, dgn_stats *stats, dgn_stream stream)
{
    if (!g) return DGN_ERR_NULL_PTR;
    if (num_pairs < 1 || num_pairs > DGN_MAX_SETS) return DGN_ERR_TOO_MANY_SETS;
    if (g->G > 1) return DGN_ERR_INVALID_ARG;        // pairs are not tied to the graphs of a packed batch
    if (!obj || !wrt || !kept_count || !scratch) return DGN_ERR_NULL_PTR;
    if ((g->T > 0 && !tensor_mask) || (g->P > 0 && (!op_mask || !kept_ops))) return DGN_ERR_NULL_PTR;
    const BackwardScratch S = backward_scratch(scratch, g->P, g->T, g->G);
    if (scratch_bytes < S.bytes) return DGN_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)scratch | (uintptr_t)tensor_mask | (uintptr_t)op_mask | (uintptr_t)kept_masks |
         (uintptr_t)kept_count | (uintptr_t)per_query_count) & 7)
        return DGN_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    u64 *F = reinterpret_cast<u64 *>(tensor_mask);

    // stage one: what every x_wrt depends on (bit i for pair i), and the operators kept for that
    DGN_HIP(launch_backward_seed(g->T, num_pairs, obj, wrt, S.tgt_rowptr, nullptr, nullptr, nullptr, true, s));
    dgn_options o1{};
    if (options) o1 = *options;
    o1.profile = 0;
    o1.incremental = 0;                              // stage one starts from nothing, in scratch memory
    // The marked masks F (the caller's tensor_mask) and the final K (its op_mask) are non-zero only inside stage
    // one's coloured set and kept list, so stage one zeroes them along with its own M and K: everything, or, when
    // the caller recycles the buffers, what the previous call's log and kept list name.
    // Stage one keeps its flag bytes (1 for every operator of its kept list) in the caller's op_flag when that can take
    // them, else in its scratch; the final removal rule turns them into the flags of the result, which spares the
    // last count pass the read of all of K.
    int rc = prune_impl(g, num_pairs, num_pairs, S.tgt_rowptr, wrt, reinterpret_cast<uint64_t *>(S.B),
                        reinterpret_cast<uint64_t *>(S.KB), op_flag, S.kept, nullptr, S.kept_count, nullptr, scratch,
                        S.prune_bytes, &o1, stats, stream, tensor_mask, op_mask);
    if (rc != DGN_OK) return rc;
    uint8_t *stage_flags = nullptr;
    if (!o1.recompute_keep)
        stage_flags = (op_flag && ((uintptr_t)op_flag & 7) == 0 && g->P % 8 == 0)
                          ? op_flag : prune_scratch(scratch, g->P, g->T, g->G, o1.max_queue_entries).flagbuf;

    // stage two: forwards from every x_obj, inside the coloured set of stage one
    FillRegion clr[1] = {{S.flags, 256}};
    DGN_HIP(launch_clear(clr, 1, s));
    DGN_HIP(launch_backward_seed(g->T, num_pairs, obj, wrt, nullptr, S.B, F, S.flags, false, s));
    void *pin = nullptr;
    rc = pinned_buffer(&pin);
    if (rc != DGN_OK) return rc;
    int32_t *host_flags = static_cast<int32_t *>(pin);
    const int grid = g->num_cus * 8;
    // Passes in batches, flags[2 + i] = "pass i of the batch added something", read back after each batch (a read-back
    // idles the GPU for about as long as half a pass takes).  The first batch is as long as the previous call's whole
    // run of passes, the following ones three passes each.
    int64_t passes = 0;
    int batch = g->backward_passes.load(std::memory_order_relaxed) + 1;      // (how far a pass gets varies a little)
    batch = batch < 3 ? 3 : batch > kBackwardMaxBatch ? kBackwardMaxBatch : batch;
    for (;;) {
        FillRegion again[1] = {{S.flags + 2, sizeof(int32_t) * (size_t)kBackwardMaxBatch}};
        if (passes) DGN_HIP(launch_clear(again, 1, s));
        for (int i = 0; i < batch; ++i)
            DGN_HIP(launch_forward_within(g->v, S.kept, S.kept_count, S.B, F, S.flags + 2 + i, grid, s));
        DGN_HIP(hipMemcpyAsync(host_flags, S.flags, 256, hipMemcpyDeviceToHost, s));
        DGN_HIP(hipStreamSynchronize(s));
        if (host_flags[0] & kErrIdRange) return DGN_ERR_ID_OUT_OF_RANGE;
        int quiet = 0;                               // the first pass of the batch that changed nothing
        while (quiet < batch && host_flags[2 + quiet] != 0) ++quiet;
        if (quiet < batch) {
            g->backward_passes.store((int)(passes + quiet + 1), std::memory_order_relaxed);
            passes += batch;
            break;
        }
        passes += batch;
        batch = 3;
    }
    if (stats) stats->reserved = (int32_t)passes;

    // Removal rule and ordered compaction on the marked set.  A marked tensor lies in stage one's coloured set,
    // so only operators of stage one's kept list can have a marked output: K is cleared and written for those.
    DGN_HIP(launch_keep_from_list(g->v, S.kept, S.kept_count, F, reinterpret_cast<u64 *>(op_mask), stage_flags, grid, s));
    return keep_compact_impl(g, tensor_mask, false, op_mask, op_flag, kept_ops, kept_masks, kept_count, per_query_count,
                             scratch, S.prune_bytes, stream, stage_flags);
}

int dgn_ignore_mask(const dgn_graph *g, const uint64_t *tensor_mask, const int32_t *kept_ops, const uint64_t *kept_masks,
                    const int64_t *kept_count, uint64_t *ignore_mask, int64_t *ignore_count, dgn_stream stream)
{
    if (!g || !kept_count) return DGN_ERR_NULL_PTR;
    if (g->T > 0 && (!tensor_mask || !ignore_mask)) return DGN_ERR_NULL_PTR;
    if (g->P > 0 && (!kept_ops || !kept_masks)) return DGN_ERR_NULL_PTR;
    if (((uintptr_t)tensor_mask | (uintptr_t)kept_masks | (uintptr_t)kept_count | (uintptr_t)ignore_mask |
         (uintptr_t)ignore_count) & 7)
        return DGN_ERR_INVALID_ARG;
    DGN_HIP(launch_ignore_mask(g->v, kept_ops, reinterpret_cast<const u64 *>(kept_masks), kept_count,
                               reinterpret_cast<const u64 *>(tensor_mask), reinterpret_cast<u64 *>(ignore_mask),
                               ignore_count, g->num_cus * 8, static_cast<hipStream_t>(stream)));
    return DGN_OK;
}

constexpr int kSetListBlocks = 2048;     // no graph handle here to ask for the number of compute units

int dgn_per_set_lists_workspace(int64_t num_kept, size_t *scratch_bytes)
{
    if (!scratch_bytes) return DGN_ERR_NULL_PTR;
    if (num_kept < 0) return DGN_ERR_INVALID_ARG;
    if (num_kept > kMaxCount / 64) return DGN_ERR_TOO_LARGE;
    *scratch_bytes = set_lists_scratch_bytes(num_kept);
    return DGN_OK;
}

int dgn_per_set_lists(const int32_t *kept_ops, const uint64_t *kept_masks, int64_t num_kept, int64_t *set_rowptr,
                      int32_t *set_ops, int64_t set_ops_capacity, void *scratch, size_t scratch_bytes, dgn_stream stream)
{
    if (num_kept < 0 || set_ops_capacity < 0) return DGN_ERR_INVALID_ARG;
    if (num_kept > kMaxCount / 64) return DGN_ERR_TOO_LARGE;      // slots are counted in int32
    if (!set_rowptr || !scratch) return DGN_ERR_NULL_PTR;
    if (num_kept > 0 && (!kept_ops || !kept_masks)) return DGN_ERR_NULL_PTR;
    if (set_ops_capacity > 0 && !set_ops) return DGN_ERR_NULL_PTR;
    if (scratch_bytes < set_lists_scratch_bytes(num_kept)) return DGN_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)kept_masks | (uintptr_t)set_rowptr | (uintptr_t)scratch) & 7) return DGN_ERR_INVALID_ARG;
    DGN_HIP(launch_set_lists(kept_ops, reinterpret_cast<const u64 *>(kept_masks), num_kept, set_rowptr, set_ops,
                             set_ops_capacity, scratch, kSetListBlocks, static_cast<hipStream_t>(stream)));
    return DGN_OK;
}

int dgn_target_digest_workspace(size_t *scratch_bytes)
{
    if (!scratch_bytes) return DGN_ERR_NULL_PTR;
    *scratch_bytes = digest_scratch_bytes();
    return DGN_OK;
}

int dgn_target_digest(const dgn_graph *g, int32_t num_sets, int64_t num_targets, const int32_t *tgt_rowptr,
                      const int32_t *tgt_idx, uint64_t *digest_out, void *scratch, size_t scratch_bytes, dgn_stream stream)
{
    if (!g || !tgt_rowptr || !digest_out || !scratch) return DGN_ERR_NULL_PTR;
    if (num_sets < 1 || num_sets > DGN_MAX_SETS) return DGN_ERR_TOO_MANY_SETS;
    if (num_targets < 0) return DGN_ERR_INVALID_ARG;
    if (num_targets > kMaxCount) return DGN_ERR_TOO_LARGE;
    if (num_targets > 0 && !tgt_idx) return DGN_ERR_NULL_PTR;
    if (scratch_bytes < digest_scratch_bytes()) return DGN_ERR_WORKSPACE_TOO_SMALL;
    if ((uintptr_t)scratch & 7) return DGN_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    u64 *dev = nullptr;
    DGN_HIP(launch_target_digest(num_sets, (int64_t)num_sets * g->G, tgt_rowptr, num_targets, tgt_idx, scratch, &dev, s));
    void *pin = nullptr;
    const int rc = pinned_buffer(&pin);
    if (rc != DGN_OK) return rc;
    DGN_HIP(hipMemcpyAsync(pin, dev, 2 * sizeof(u64), hipMemcpyDeviceToHost, s));
    DGN_HIP(hipStreamSynchronize(s));
    digest_out[0] = static_cast<const u64 *>(pin)[0];
    digest_out[1] = static_cast<const u64 *>(pin)[1];
    return DGN_OK;
}

int dgn_inplace_workspace(const dgn_graph *g, size_t *scratch_bytes)
{
    if (!g || !scratch_bytes) return DGN_ERR_NULL_PTR;
    *scratch_bytes = inplace_scratch_bytes(g->T);
    return DGN_OK;
}

static int inplace_impl(const dgn_graph *g, const uint64_t *op_mask, uint64_t select, const int32_t *kept_ops,
                        const int64_t *kept_count, int32_t *rename, int64_t *renamed_count, void *scratch,
                        size_t scratch_bytes, int32_t *rounds_out, dgn_stream stream)
{
    if (!g || !scratch) return DGN_ERR_NULL_PTR;
    if ((g->P > 0 && !op_mask) || (g->T > 0 && !rename)) return DGN_ERR_NULL_PTR;
    if (scratch_bytes < inplace_scratch_bytes(g->T)) return DGN_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)scratch | (uintptr_t)op_mask | (uintptr_t)renamed_count) & 7) return DGN_ERR_INVALID_ARG;
    if ((uintptr_t)rename & 3) return DGN_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const InplaceBuffers B = inplace_buffers(scratch, g->T);
    const int grid = g->num_cus * 8;
    DGN_HIP(launch_inplace_setup(g->v, reinterpret_cast<const u64 *>(op_mask), select, kept_ops, kept_count, rename,
                                 renamed_count, B, grid, s));
    void *pin = nullptr;
    int rc = pinned_buffer(&pin);
    if (rc != DGN_OK) return rc;
    int round = 0;
    for (;;) {                                       // four rounds per read-back of the "still alive" word
        for (int i = 0; i < 4 && round < kInplaceMaxRounds; ++i, ++round)
            DGN_HIP(launch_inplace_round(round, rename, renamed_count, B, grid, s));
        DGN_HIP(hipMemcpyAsync(pin, B.counters + round, sizeof(int32_t), hipMemcpyDeviceToHost, s));
        DGN_HIP(hipStreamSynchronize(s));
        if (*static_cast<int32_t *>(pin) == 0 || round >= kInplaceMaxRounds) break;
    }
    if (rounds_out) *rounds_out = round;
    return DGN_OK;
}

int dgn_inplace(const dgn_graph *g, const uint64_t *op_mask, uint64_t select, int32_t *rename, int64_t *renamed_count,
                void *scratch, size_t scratch_bytes, int32_t *rounds_out, dgn_stream stream)
{
    return inplace_impl(g, op_mask, select, nullptr, nullptr, rename, renamed_count, scratch, scratch_bytes, rounds_out,
                        stream);
}

int dgn_inplace_kept(const dgn_graph *g, const uint64_t *op_mask, uint64_t select, const int32_t *kept_ops,
                     const int64_t *kept_count, int32_t *rename, int64_t *renamed_count, void *scratch,
                     size_t scratch_bytes, int32_t *rounds_out, dgn_stream stream)
{
    if (g && g->P > 0 && (!kept_ops || !kept_count)) return DGN_ERR_NULL_PTR;
    if ((uintptr_t)kept_count & 7) return DGN_ERR_INVALID_ARG;
    return inplace_impl(g, op_mask, select, kept_ops, kept_count, rename, renamed_count, scratch, scratch_bytes,
                        rounds_out, stream);
}

}  // extern "C"
