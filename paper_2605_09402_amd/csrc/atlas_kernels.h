// Internal launch interface between the host state machine (atlas_api.hip)
// and the gfx950 kernels.  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace atlas {

// Device-side counters of one layer (int32 each, one 256-byte block).
enum Counter {
    CTR_READY_TAIL = 0,  // ready-list length (vertices completed so far)
    CTR_READY_HEAD = 1,  // ready-list prefix already flushed
    CTR_NUM_FLUSHES = 2,
    CTR_NEXT_RUN = 32,   // ticket counter of the grouped aggregation's dynamically assigned runs (its own cache line)
    CTR_COUNT = 64
};

// 64-bit counters (separate block): edges pushed so far.
// Bit of a pending count: the vertex's finished row already lies in its accumulator row as the update's
// 16-bit operand; only its own message is outstanding (see GroupedArgs::handover_self).
constexpr int32_t kPendingHanded = 0x40000000;

enum Counter64 { CTR64_EDGES = 0, CTR64_HANDED = 1 /* rows handed over to the update */, CTR64_COUNT = 8 };

// Bounded accumulator store (paper Sec. 3.5): a fixed number of slots in HBM,
// evicted partial states in pinned host memory.
enum HotCounter {
    HS_NEED = 0,        // vertices listed in need_list for the chunk being prepared
    HS_FREE_TOP = 1,    // height of the free-slot stack
    HS_CANDIDATES = 2,  // eviction candidates counted by the key kernel
    HS_RELOADS = 3,
    HS_EVICTIONS = 4,
    HS_OVERFLOW = 5,    // a list ran past its capacity (never expected: the host checks the counts)
    HS_PEAK = 6,        // most slots in use at once
    HS_COUNT = 16
};
struct HotStore {
    int32_t *slot_of = nullptr;     // [N] slot of the vertex's partial state; -1: none (not started, or
                                    // completed and released); -2: evicted, state in `cold`
    int32_t *slot_owner = nullptr;  // [slots] vertex held, -1: free
    int32_t *free_list = nullptr;   // [slots] stack of free slots
    int32_t *stamp = nullptr;       // [N] number (+1) of the last chunk that addressed the vertex
    int32_t *need_list = nullptr;   // [slots]
    int32_t *ctr = nullptr;         // [HS_COUNT]
    uint64_t *keys = nullptr, *keys_sorted = nullptr;   // [slots]
    float *hot = nullptr;           // [slots][d]
    float *cold = nullptr;          // [N][d], pinned host memory
    int64_t slots = 0;
    int d = 0;
};
hipError_t hot_init(const HotStore &h, int64_t n, hipStream_t s);
hipError_t hot_mark(const HotStore &h, const int32_t *grp_dst, int32_t dst_mask, int64_t n_groups, int64_t src_begin,
                    int64_t n_self, int32_t chunk_stamp, hipStream_t s);
hipError_t hot_build_keys(const HotStore &h, const int32_t *pending, int32_t chunk_stamp, int policy, hipStream_t s);
size_t hot_sort_temp_bytes(int64_t slots);
hipError_t hot_evict(const HotStore &h, int64_t n_evict, void *sort_temp, size_t sort_temp_bytes, hipStream_t s);
hipError_t hot_assign(const HotStore &h, int64_t need, hipStream_t s);
hipError_t hot_release(const HotStore &h, const int32_t *ready, const int32_t *counters, int64_t n, hipStream_t s);

// Attention state of a GAT layer (all [N][heads], fp32 unless noted).
// The running maximum is stored as an order-preserving int32 image of the
// float so that an integer atomicMax implements a float maximum.
struct GatState {
    const float *el = nullptr;   // a_src . z_u
    const float *er = nullptr;   // a_dst . z_v
    int32_t *m_cur = nullptr;    // reference maximum the accumulated state is relative to
    int32_t *m_next = nullptr;   // running maximum including the chunk being broadcast
    float *l = nullptr;          // running softmax denominator (relative to m_cur)
    int heads = 1;
    int dh = 0;                  // columns per head
    float slope = 0.2f;
};

struct AggregateArgs {
    const int64_t *off;    // row offsets addressed by global source id
    const int32_t *col;    // col[e - col_base] is the destination of edge e
    int64_t col_base;
    const void *emb;       // chunk rows; row u lives at (u - src_begin) * d
    int64_t src_begin, src_end;
    int d;                 // row width (elements)
    int in_dt;             // storage of the rows: 0 fp32, 1 bf16, 2 IEEE half (the atlas_dtype values)
    int model;             // atlas_model
    float *acc;            // [N][d] fp32
    int32_t *pending;      // [N]
    const int32_t *indeg;  // [N]
    int32_t *ready;        // [N]
    int32_t *counters;
    unsigned long long *counters64;
    GatState gat;          // model == GAT only
};

// S2+S3+S4: edge-balanced scatter-aggregate with fused pending decrement and
// wave-level ready compaction.
hipError_t launch_aggregate(const AggregateArgs &a, hipStream_t s);

// One planned chunk: its edges regrouped by destination.
struct PlanChunk {
    int64_t edge_base = 0;      // first edge of the chunk in CSR numbering
    int64_t n_edges = 0;
    int64_t n_groups = 0;       // distinct destinations the chunk sends to
    int32_t *grp_dst = nullptr;   // [n_groups] destination of each group, ascending; bit 31 set when no
                                  // earlier chunk sends to that destination (its first group of the layer)
    int32_t *tile_grp = nullptr;  // [ceil(n_edges/64)] group of the first edge of every 64-edge tile
    bool blocked = false;         // source-blocked order: grp_dst bit 30 marks destinations with several groups
    int32_t *zero_rows = nullptr; // device plans: destinations a planned-only layer clears before this chunk (their
    int64_t n_zero_rows = 0;      // first group is added to with atomics by several waves); may hold duplicates
    int32_t *zero_span = nullptr; // [n_zero_rows][2] first and last 64-edge tile of that first group, or {-1, -1}
                                  // for a destination with several groups: a launch whose runs keep the group
                                  // within one wave need not clear the row
    bool has_zero_rows = false;   // the list exists (plans of graphs with fewer than 2^30 vertices): planned-only
                                  // layers need it
    int64_t packed_off = 0;       // plans with 24-bit edge words: byte offset of the chunk's words in the plan's array
};

// 24-bit edge words of plans that live in pinned host memory (source offset within the chunk, bit 23 = group end)
size_t packed24_bytes(int64_t n_edges);
hipError_t launch_pack24(const int32_t *src_sorted, int64_t n_edges, int64_t src_begin, void *packed, hipStream_t s);
hipError_t launch_unpack24(const void *packed, int64_t n_edges, int64_t src_begin, int32_t *src_sorted, hipStream_t s);

struct GroupedArgs {
    const int32_t *src_sorted;  // chunk slice: source id of every edge in destination order,
                                // bit 31 set on the last edge of a destination's group
    int64_t n_edges;
    const int32_t *grp_dst;
    const int32_t *tile_grp;
    const void *emb;            // chunk rows; row u lives at (u - src_begin) * d
    int64_t src_begin;
    int d;
    int in_dt;
    int model;
    float *acc;
    int32_t *pending;
    const int32_t *indeg;
    int32_t *ready;
    int32_t *counters;
    unsigned long long *counters64;
    GatState gat;               // model == GAT only
    const int32_t *slot_of = nullptr;   // bounded store: row of `acc` that holds vertex v (nullptr: row v)
    int64_t n_groups = 0;
    int32_t multi_bit = 0;      // source-blocked chunk: 0x40000000, the grp_dst bit of destinations that have
                                // several groups in this chunk (all of them add with atomics); else 0
    float *scores = nullptr;    // GAT only: [n_edges][heads] attention logits of the chunk's edges, written
                                // by the max sweep and read by the aggregation
    int handover = 0;           // 1: a group this wave alone owns that completes its destination writes the finished
    int handover_dt = 1;        // row as the update's 16-bit operand (type handover_dt: 1 bf16, 2 IEEE half; normalised
    int handover_norm = 0;      // by 1/deg (0) or deg^-1/2 (1)) into the first half of the accumulator row, and the
                                // vertex's ready-list entry carries bit 31
    int handover_self = 0;      // 1 (layers whose vertices receive their own embedding as a message, with their own
    int64_t self_from = 0;      // chunk): a group that leaves only that message outstanding (destination >= self_from,
                                // the first source after this chunk) hands the row over as well and marks the
                                // vertex's pending count with kPendingHanded for k_self_message
    int forced_run = 0;         // the layer's run length (1..kMaxTilesPerRun), 0: chosen per launch
    int tiles_per_run = 1;      // consecutive 64-edge tiles one wave takes at a time (set by the launcher)
    int64_t tile_begin = 0;     // the launch covers tiles [tile_begin, tile_end) of the chunk (tile_end < 0: all).
    int64_t tile_end = -1;      // A chunk that arrives over the host link in pieces is pushed piece by piece;
                                // a group cut by a piece boundary is added with atomics like one cut by a run.
                                // (launch_zero_rows covers the whole chunk: once, before the first piece)
    // set by the launcher:
    int nruns = 0;              // runs in [tile_begin, tile_end): the first big_runs of tiles_per_run tiles,
    int big_runs = 0;           // the others (the launch's last tiles, taken when most waves are about to
    int small_run = 1;          // finish) of small_run tiles
    int dynamic = 0;            // 1: a wave's runs after its first are handed out by counters[CTR_NEXT_RUN]
    uint32_t run_base = 0;      // value of that counter when the launch begins
};

constexpr int kMaxTilesPerRun = 16;

// S2+S3+S4 over a planned chunk: per-destination register sums, one row update
// and one pending decrement per (chunk, destination) group.
// `run_tickets`: the layer's count of tickets drawn from counters[CTR_NEXT_RUN] so far (starts at 0 with the
// zeroed counter); every launch that hands out runs dynamically draws exactly one ticket per run and advances it.
hipError_t launch_aggregate_grouped(const GroupedArgs &a, uint32_t *run_tickets, hipStream_t s);
// Choose the launch's runs (tiles_per_run, nruns, big_runs, small_run, dynamic) ahead of the launch, for
// launch_zero_rows; a launch whose nruns is still 0 chooses them itself.
hipError_t plan_runs(GroupedArgs &a);

// Work arrays of the plan construction, kept from chunk to chunk (allocating and freeing tens of
// gigabytes per chunk costs more than some of the passes) and grown when a chunk needs more.
struct GrowBuf {
    void *p = nullptr;
    size_t cap = 0;
    hipError_t need(size_t bytes);
    void release();
};
struct PlanWork {
    GrowBuf tmp_src, dst_sorted, heads, temp, bkey, bkey_sorted, bpos, bpos_sorted, gstart, src_new, rows, cnt;
    GrowBuf part_flags, part_pos, part_dst, part_src;   // split of a first chunk into its dense part and the rest
    PlanWork() = default;
    PlanWork(const PlanWork &) = delete;
    PlanWork &operator=(const PlanWork &) = delete;
    ~PlanWork();
};

// Plan construction for one chunk (synchronous, on the default stream).  off_dev is addressed by global
// source id and col_dev by global edge number (only [src_begin, src_end] and
// [edge_begin, edge_end) are touched); `seen` is the plan-wide N-byte first-touch map
// (zeroed before the first chunk, chunks built in streaming order; nullptr: no group is marked as its
// destination's first, as for a chunk regrouped on its own, whose neighbours may have gone another way);
// src_sorted receives the chunk's
// edge_end - edge_begin entries; grp_dst and tile_grp (and, with want_zero_rows, the list of rows a
// planned-only layer clears) are allocated with hipMalloc.
// With `pairs` the chunk's edges are not read from the CSR but given as (destination, source) arrays of
// pairs->count entries in CSR order (a subset of the chunk's edges); pairs->src is overwritten.
struct EdgePairs {
    const uint32_t *dst;
    int32_t *src;
    int64_t count;
};
hipError_t build_plan_chunk(const int64_t *off_dev, const int32_t *col_dev, int64_t n, int64_t src_begin,
                            int64_t src_end, int64_t edge_begin, int64_t edge_end, int32_t *src_sorted,
                            uint8_t *seen, int64_t block_sources, int64_t hot_min_edges, bool want_zero_rows,
                            PlanWork &w, PlanChunk *out, const EdgePairs *pairs = nullptr);

// Dense part of a plan's first chunk (k_dense.hip): the multiplicities of the edges between the chunk's
// first sources and the first destinations as a staircase of matrices of 4-bit counts, one band per 256 destinations,
// and the same edges as an ordinary planned chunk (`list`) for layers the contraction does not serve.
constexpr int kDenseBuckets = 24;        // log-spaced rank buckets of the density histogram
constexpr int kDenseKstepBytes = 8192;   // cells of one band and k-step: 256 destinations x 64 sources x 4 bits
constexpr int kDenseKstepUnit = 12;      // a band's k-steps (of 64 sources) are a multiple of this
constexpr int kDenseItemKsteps = 192;    // most k-steps one workgroup contracts (a multiple of the unit, below 2^16)
struct DensePart {
    int64_t rows = 0;                 // destinations [0, rows), a multiple of 256 (may exceed N)
    int32_t n_bands = 0;              // rows / 256
    int32_t max_ksteps = 0;           // sources / 64 of the longest band (a multiple of kDenseKstepUnit)
    int32_t *band_ksteps = nullptr;   // device [n_bands]
    int64_t *band_off = nullptr;      // device [n_bands]: byte offset of the band's cells
    uint8_t *cells = nullptr;         // device
    size_t cell_bytes = 0;
    int32_t *msgs = nullptr;          // device [rows]: messages of the dense part to each destination
    int32_t *items = nullptr;         // device [n_items][3]: band, first k-step, k-steps (| 1 << 16: the band's
                                      // only item) of every work item
    int64_t n_items = 0;
    PlanChunk list;                   // the part's edges, grouped by destination
    int32_t *list_src = nullptr;      // plans of pinned-host graphs: the list's edge words (device memory, as all of
                                      // the dense part); device plans keep them in the plan's array at list.edge_base
    void release();
};
// Builds the first chunk of a plan in two parts.  max_bytes bounds the cells; cells_per_edge is the most
// cells a (source bucket, destination bucket) block may spend per edge it holds.  When no block is that
// dense the chunk is built as usual and dense->n_items stays 0.
hipError_t build_first_chunk_with_dense_part(const int64_t *off_dev, const int32_t *col_dev, int64_t n,
                                             int64_t src_begin, int64_t src_end, int64_t edge_begin,
                                             int64_t edge_end, int32_t *src_sorted, uint8_t *seen,
                                             int64_t block_sources, int64_t hot_min_edges, bool want_zero_rows,
                                             size_t max_bytes, int64_t cells_per_edge, PlanWork &w, PlanChunk *rest,
                                             DensePart *dense);
hipError_t launch_dense_histogram(const int32_t *src_of_edge, const int32_t *col, int64_t ne, int64_t src_begin,
                                  unsigned long long *hist, hipStream_t s);
hipError_t launch_dense_divert(const int32_t *src_of_edge, const int32_t *col, int64_t ne, int64_t src_begin,
                               const DensePart &p, uint8_t *flags, hipStream_t s);
hipError_t launch_dense_split(const int32_t *src_of_edge, const int32_t *col, const uint8_t *flags,
                              const uint32_t *flagged_before, int64_t ne, int64_t n_rest, uint32_t *dst_out,
                              int32_t *src_out, hipStream_t s);
struct DenseArgs {
    const uint8_t *cells;
    const int64_t *band_off;
    const int32_t *items;
    const void *xt;
    float *acc;
    int64_t n;
};
// Whether the contraction serves rows of this width and storage type (otherwise the layer pushes `list`).
bool dense_contract_takes(int d, int in_dt);
// Bytes of the repacked chunk rows the contraction reads (`xt` below).
size_t dense_packed_rows_bytes(const DensePart &p, int d);
// The dense part in three launches (the part is pushed before anything else of the layer):
//   prepare:  accumulator rows [0, rows) cleared, the chunk's rows (emb: chunk_rows of them, 16-bit, d wide)
//             repacked into xt;
//   contract: acc[v] += sum of the dense part's messages to v;
//   pending:  pending counts lowered, completed vertices appended to the ready list, edges counted.
hipError_t launch_dense_prepare(const DensePart &p, const void *emb, int64_t chunk_rows, int d, int in_dt, void *xt,
                                float *acc, int64_t n, hipStream_t s);
hipError_t launch_dense_contract(const DensePart &p, int d, int in_dt, const void *xt, float *acc, int64_t n,
                                 hipStream_t s);
hipError_t launch_dense_pending(const DensePart &p, int64_t n, int32_t *pending, int32_t *ready, int32_t *counters,
                                unsigned long long *counters64, hipStream_t s);

// indeg[v] += messages the chunk sends to v, for every destination of a planned chunk whose arrays are in
// device memory (src_sorted: the chunk's slice).  indeg must have been zeroed before the first chunk.
hipError_t launch_plan_chunk_in_degree(const PlanChunk &c, const int32_t *src_sorted, int32_t *indeg, hipStream_t s);

// Non-zero bytes of a device array (synchronous): how many destinations a plan's first-touch map has seen.
hipError_t count_nonzero_bytes(const uint8_t *p, int64_t n, int64_t *out);

// GAT, per chunk: raise m_next[v][h] to the largest logit any edge of the chunk
// sends to v (CSR order), then bring every destination whose maximum moved to
// the new reference (rescale l and acc, m_cur = m_next).
hipError_t launch_gat_chunk_max(const AggregateArgs &a, hipStream_t s);
hipError_t launch_gat_group_max(const GroupedArgs &a, hipStream_t s);   // the same over a planned chunk; also
                                                                        // stores every edge's logits in a.scores
// Planned GAT chunk, between the max sweep and the aggregation: destinations whose group is cut by a tile
// boundary are brought to the new maximum here (acc and l times exp(m_cur - m_next), m_cur = m_next), once
// per group; groups inside a tile are rescaled by the aggregation itself as part of their row update.
hipError_t launch_gat_rescale_cut_groups(const GroupedArgs &a, hipStream_t s);
hipError_t launch_gat_rescale(const GatState &g, float *acc, int d_out, int64_t n, hipStream_t s);
// GAT set-up and prepass.
hipError_t launch_fill_i32(int32_t *p, int32_t value, int64_t count, hipStream_t s);
int32_t gat_encoded_neg_inf();
hipError_t launch_gat_fold_attention(const void *W, const void *a_src, const void *a_dst, int w_dt, int d_in,
                                     int heads, int dh, float *wa, hipStream_t s);   // wa: [d_in][2*heads]
hipError_t launch_gat_prepass(const void *emb, int in_dt, int64_t src_begin, int64_t src_end, int d_in,
                              const float *wa, int heads, float *el, float *er, hipStream_t s);
// GAT flush: y = acc / l (+ bias, activation) for the ready rows.
struct GatFinalizeArgs {
    const float *acc;
    const float *l;
    const int32_t *ready;
    int32_t *counters;
    const float *bias;
    void *out;
    int d_out, heads, dh, activation, out_dt;
    int64_t n;
};
hipError_t launch_gat_finalize(const GatFinalizeArgs &a, hipStream_t s);

// Planned-only layers skip the accumulator zero fill: rows are first written by
// their first group.  A first group that several waves add to with atomics (it
// is cut by a run boundary, or its destination has one group per source block)
// has its row zeroed here before the chunk runs, from the list of candidates
// precomputed with the plan.  With `spans` and the runs of the launch that
// follows (`runs`, after plan_runs; nullptr: unknown, e.g. a chunk pushed in pieces) a row is left alone when
// its group lies inside one run: the run's wave then holds the whole sum and stores it.
hipError_t launch_zero_rows(const int32_t *rows, const int32_t *spans, int64_t n_rows, float *acc,
                            const int32_t *slot_of, int d, const GroupedArgs *runs, hipStream_t s);

// SAGE self message of sources [b, e): pending[u] -= 1 with ready compaction.
hipError_t launch_self_message(int64_t b, int64_t e, int32_t *pending, int32_t *ready,
                               int32_t *counters, hipStream_t s);

// S0 pieces.
// In-degree of every vertex.  With `scratch` of at least in_degree_scratch_bytes(n, num_edges) bytes of
// DEVICE memory (0: the graph is small, no scratch needed) and `col` in device memory, large graphs are
// counted bucket by bucket in LDS; without it (or for an edge array in host memory: pass nullptr) one
// atomic per edge.  The scratch must stay valid until the stream has passed the call.
size_t in_degree_scratch_bytes(int64_t n, int64_t num_edges);
hipError_t launch_in_degree(const int32_t *col, int64_t num_edges, int32_t *indeg, int64_t n, void *scratch,
                            size_t scratch_bytes, hipStream_t s);
hipError_t launch_init_pending(const int32_t *indeg, int32_t selfmsg, int64_t n, int32_t *pending,
                               int32_t *ready, int32_t *counters, hipStream_t s);
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s);

// Weight repack into MFMA B-fragment order (see k_update.hip).
size_t packed_weight_bytes(int K, int d_out, int compute_dt);
hipError_t launch_pack_weights(const void *W, int w_dt, int K, int d_out, int compute_dt,
                               void *packed, hipStream_t s);
hipError_t launch_to_f32(const void *src, int src_dt, int64_t count, float *dst, hipStream_t s);

struct UpdateArgs {
    int model;                // 0 SAGE (own row || mean), 1 GCN (deg^-1/2 sum), 2 plain rows of `acc`,
                              // 3 GIN (sum + self_scale * own row), 4 plain rows of `self_rows` (storage
                              // dtype, d_in up to 1024; with identity_rows)
    float self_scale;         // GIN: 1 + eps
    int d_in, d_out, K;       // K = 2*d_in (SAGE) or d_in
    int in_dt, out_dt, compute_dt;
    int activation;
    const float *acc;         // [N][d_in]
    const void *self_rows;    // SAGE: [N][d_in] in in_dtype
    const int32_t *indeg;
    const int32_t *ready;
    int32_t *counters;
    const void *packed_w;
    const float *bias;        // fp32 [d_out] or nullptr
    void *out;                // [N][d_out]
    void *out2;               // split > 0: columns split.. of the product go to out2 (column - split) and
    int split;                // columns below split to out, both with rows of `split` columns (a product
                              // with two weight matrices side by side); 0: one output of d_out columns
    int out2_dt;              // element type of out2 (out_dt is that of out)
    int64_t n;
    const int32_t *slot_of;   // bounded store: row of `acc` that holds vertex v (nullptr: row v)
    int handed_rows;          // 1: ready-list entries may carry bit 31 (rows handed over by the aggregation, see
                              // GroupedArgs::handover); only flushes for which update_takes_handed_rows() holds
    int64_t identity_rows;    // > 0: no ready list; rows 0..identity_rows-1 of `acc` (a dense
                              // row block, model 2 = plain X W) map to the same rows of `out`
};
// S5: gather ready rows, normalise, MFMA GEMM, bias, activation, scatter rows.
hipError_t launch_update(const UpdateArgs &a, hipStream_t s);
// Whether that flush (model: UpdateArgs::model) understands ready-list entries with bit 31 set: rows whose
// finished 16-bit operand the aggregation left in the first half of the accumulator row.
bool update_takes_handed_rows(int model, int d_in, int K, int d_out, int compute_dt);
// Transform-first layers: the ready rows' outputs from already-transformed sums,
// y_v = act(scale(deg_v) * acc[v] + self_scale * self_term[v] + b).
struct SumFinalizeArgs {
    const float *acc;         // [N or slots][d_out]
    const int32_t *slot_of;   // bounded store indirection or nullptr
    const float *self_term;   // [N][d_out] or nullptr
    float self_scale;
    int norm;                 // 0: 1/deg (mean), 1: deg^-1/2, 2: none
    const int32_t *indeg;
    const int32_t *ready;
    int32_t *counters;
    const float *bias;
    void *out;
    int d_out, activation, out_dt;
    int64_t n;
};
hipError_t launch_sum_finalize(const SumFinalizeArgs &a, hipStream_t s);

// SGC hop: out[v] = acc[v] * deg(v)^-1/2 for the ready rows (no contraction).
hipError_t launch_scale_rows(const UpdateArgs &a, hipStream_t s);
hipError_t launch_advance_head(int32_t *counters, hipStream_t s);

// Measured-peak probes (k_probe.hip).
hipError_t probe_copy(void *dst, const void *src, size_t bytes, hipStream_t s);
hipError_t probe_mix21(void *dst, const void *a, const void *b, size_t bytes, hipStream_t s);
size_t probe_gather_sink_bytes();
hipError_t probe_mfma(int waves_per_simd, int iters, void *sink, double *flops, hipStream_t s);
hipError_t probe_row_gather(const void *table, const int32_t *ids, int64_t n_ids, void *sink, hipStream_t s);

// Degree ordering.
hipError_t reorder_indegree_desc(const int32_t *indeg, int64_t n, int32_t *new_of_old,
                                 int32_t *old_of_new);
// The same order computed without any allocation, out of a fixed scratch array in device memory; enqueues
// on `s` and does not wait.  *too_large is set (and nothing is launched) when n exceeds
// kNoAllocMaxVertices or the sort's workspace would not fit the scratch.
constexpr int64_t kNoAllocMaxVertices = int64_t(1) << 20;
hipError_t reorder_indegree_desc_noalloc(const int32_t *indeg, int64_t n, int32_t *new_of_old, int32_t *old_of_new,
                                         hipStream_t s, bool *too_large);
hipError_t reorder_score_desc(const int64_t *off, const int32_t *col, const int32_t *indeg, int64_t n,
                              int32_t *new_of_old, int32_t *old_of_new);

// Sampling by disabling edges: keep, per destination, the `fanout` in-edges with the
// smallest keys (ties by CSR position); out_off [n+1] / out_col [<= e] receive the CSR
// of the kept edges.  Synchronous.
hipError_t sample_in_edges(const int64_t *off, const int32_t *col, int64_t n, int64_t e, const uint32_t *key,
                           int32_t fanout, int64_t *out_off, int32_t *out_col);

}  // namespace atlas
