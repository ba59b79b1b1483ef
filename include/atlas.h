/*
 * atlas.h -- C ABI of the broadcast-based GNN layer step for MI355X (gfx950).
 *
 * One layer of layer-wise full-graph inference is run as a stream of source
 * chunks (paper Sec. 3.1 "Broadcast Execution Model", Sec. 3.3 chunk iterator,
 * Sec. 3.4 orchestrator, Sec. 3.6 graduation):
 *
 *   atlas_layer_init       per-vertex pending-message counts, zeroed
 *                          accumulators, empty ready list        (Sec. 3.4)
 *   atlas_broadcast_chunk  push the embeddings of sources [b, e) along their
 *                          out-edges into per-destination accumulators; every
 *                          message decrements the destination's pending count;
 *                          destinations reaching zero are appended to the ready
 *                          list                                   (Sec. 3.1, 3.4)
 *   atlas_flush_ready      dense update of the ready ("graduated") rows and
 *                          write of their next-layer embeddings   (Sec. 3.6)
 *   atlas_layer_finish     exactly-once check, statistics, release (Sec. 3.1:
 *                          every embedding is consumed exactly once per layer)
 *
 * All work runs in HIP kernels on the current device; a process uses the
 * library with one device (its cache of device buffers, freed by
 * atlas_release_cache, and the chunk loader's copy stream belong to the device
 * that was current when they were first needed).  Every pointer is a plain
 * address whose residency (device / pinned host / pageable host) is stated
 * per argument; layer state is allocated by the library with hipMalloc.  No function
 * throws or aborts; every function returns ATLAS_OK (0) or a negative
 * atlas_status code and has no partial effect when it rejects its arguments.
 * A layer object must be used from one host thread at a time, and all calls on
 * one layer must be given the same HIP stream (or streams the caller orders).
 * The calls are not meant for HIP graph capture: atlas_layer_init allocates,
 * and the kernel arguments of a launch carry state of the layer at that call.
 * The functions documented as "Synchronous" (plans, orderings, sampling) take
 * no stream: they work on the default stream and return when their result is
 * complete, but they do not wait for work the caller has queued on other
 * non-blocking streams, so arrays written there must be complete before the
 * call (synchronise that stream first).
 */
#ifndef ATLAS_H
#define ATLAS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct atlas_layer atlas_layer_t; /* opaque, library-owned */
typedef struct atlas_plan atlas_plan_t;   /* opaque, library-owned: see atlas_plan_create */

enum atlas_status {
    ATLAS_OK = 0,
    ATLAS_E_NULL = -1,       /* a required pointer is NULL                                  */
    ATLAS_E_BAD_DIMS = -2,   /* unsupported width / heads / enum value                      */
    ATLAS_E_RANGE = -3,      /* chunk bounds outside [0, N] or longer than max_chunk_sources */
    ATLAS_E_ORDER = -4,      /* chunks must be contiguous and ascending, starting at 0      */
    ATLAS_E_INCOMPLETE = -5, /* finish before every vertex was completed and flushed        */
    ATLAS_E_OVERFLOW = -6,   /* N >= 2^31 (vertex ids and counts are int32)                 */
    ATLAS_E_HIP = -7,        /* a HIP call failed; see atlas_last_hip_error()               */
    ATLAS_E_NOMEM = -8,      /* device or host allocation failed                            */
    ATLAS_E_STATE = -9,      /* call not valid in the layer's current state                 */
    ATLAS_E_TOO_LARGE = -10  /* input exceeds the fixed scratch of a no-allocation entry point */
};

enum atlas_residency { ATLAS_RESIDENT_DEVICE = 0, ATLAS_RESIDENT_PINNED_HOST = 1 };
/* The layer types the paper evaluates (GraphConv, SAGEConv, GINConv: Sec. 4.1) and the two it names as
 * adoptable into the same execution model (GAT, SGC: Sec. 3.9). */
enum atlas_model {
    ATLAS_MODEL_SAGE_MEAN = 0,
    ATLAS_MODEL_GCN_SYM = 1,
    ATLAS_MODEL_GAT = 2,
    ATLAS_MODEL_GIN = 3,     /* sum aggregation, (1 + gin_eps) x own embedding added, one linear map */
    ATLAS_MODEL_SGC_HOP = 4  /* one propagation step of SGC: the symmetric-normalised neighbour sum
                                without weights; K hops = K-1 such layers and one GCN_SYM layer */
};
enum atlas_dtype {
    ATLAS_DTYPE_F32 = 0,
    ATLAS_DTYPE_BF16 = 1,
    ATLAS_DTYPE_F16 = 2  /* IEEE half (the paper's largest feature set is stored so, Sec. 4.1); sums are kept in
                            fp32, the contraction runs on half operands.  Not for GAT; GIN only together with
                            ATLAS_FLAG_TRANSFORM_FIRST (a hub's plain sum leaves the range of half) */
};
enum atlas_activation { ATLAS_ACT_NONE = 0, ATLAS_ACT_RELU = 1, ATLAS_ACT_ELU = 2 };
enum atlas_flags {
    ATLAS_FLAG_TIMING = 1,       /* record per-stage GPU time with HIP events                  */
    ATLAS_FLAG_EMB_RESIDENT = 2, /* embeddings in device memory, SAGE_MEAN / GIN: the caller promises that every
                                    `emb` given to atlas_broadcast_chunk is the row range
                                    [src_begin, src_end) of ONE contiguous N x d_in matrix that
                                    stays valid until atlas_layer_finish; the library then reads
                                    a vertex's own row from that matrix instead of keeping a
                                    copy (E_STATE if two chunks disagree about the matrix base) */
    ATLAS_FLAG_PLANNED_ONLY = 4, /* SAGE_MEAN / GCN_SYM on a graph with a plan: the caller promises
                                    that every chunk coincides with a planned chunk
                                    (atlas_broadcast_chunk returns E_RANGE otherwise).  The layer
                                    then skips the zero fill of the accumulators: a row is first
                                    written by its destination's first group, and the accumulator
                                    of a vertex without in-edges is never read.  Ignored without
                                    a plan, for GAT and for graphs of 2^30 vertices or more (their
                                    plans lack the list of rows to clear).  With it, ATLAS_DBG_ACC rows of vertices
                                    that have received nothing yet are undefined. */
    ATLAS_FLAG_NO_HANDOVER = 32, /* switch the fused part of the flush off (see atlas_flush_ready); for comparisons */
    ATLAS_FLAG_NO_DENSE = 64,    /* push the dense part of a plan (see atlas_plan_create_dense) as the planned
                                    chunk it also is instead of a contraction; for comparisons */
    ATLAS_FLAG_CSR_STREAM = 16,  /* never regroup a chunk on the fly: a chunk without a planned chunk is pushed
                                    straight from the CSR with fp32 atomics, whatever its length (see
                                    atlas_broadcast_chunk) */
    ATLAS_FLAG_TRANSFORM_FIRST = 8 /* SAGE_MEAN / GCN_SYM / GIN: the weight matrix is
                                    applied to each chunk's rows before they are pushed (the linear map
                                    commutes with the neighbour sum), so messages and accumulators are
                                    d_out wide instead of d_in.  Pays when d_out is well below d_in (wide
                                    input features); d_in may then be up to 1024 (fp32 embeddings: 512)
                                    and d_out must be a multiple of 64.  The pushed products are messages
                                    and travel in the embeddings' storage type (SAGE_MEAN, GCN_SYM; GIN
                                    pushes fp32), sums stay fp32: results equal the default order up to
                                    one rounding of each product to that type.  Ignored for other
                                    models. */
};

/* The graph: CSR by SOURCE vertex (paper Sec. 3.2: out-edges, read sequentially
 * by offsets).  Vertex ids are the (re-ordered) ids the chunks are streamed in.
 * Multi-edges and self-edges are ordinary edges.  Caller-owned; must stay valid
 * and unchanged until atlas_layer_finish returns. */
typedef struct {
    int64_t num_vertices;       /* N, 0 <= N < 2^31                                        */
    int64_t num_edges;          /* E = row_offsets[N]                                      */
    const int64_t *row_offsets; /* N+1 ascending edge offsets; DEVICE: device memory,
                                   PINNED_HOST: pinned host memory                         */
    const int32_t *col_indices; /* E destination ids; same residency as row_offsets        */
    const int32_t *in_degree;   /* N in-degrees (multiplicity counted) in DEVICE memory,
                                   or NULL: the library counts them at init                */
    int32_t residency;          /* atlas_residency of row_offsets / col_indices            */
    const atlas_plan_t *plan;   /* optional result of atlas_plan_create on THIS graph, or
                                   NULL: chunks are then pushed straight from the CSR      */
} atlas_graph_t;

/* Layer shape.  d_in must be a multiple of 64 (one wavefront holds a row),
 * at most 512 (fp32 SAGE_MEAN: at most 256); d_out a multiple of 16, at most
 * 256.  GAT: 1 <= heads <= 8, d_out a multiple of 64 and of heads, and
 * (d_out / heads) a multiple of (d_out / 64); no bounded accumulator store.
 * SGC_HOP: d_out == d_in (up to 512), activation NONE. */
typedef struct {
    int32_t model;             /* atlas_model                                              */
    int32_t d_in, d_out;       /* input / output embedding width                           */
    int32_t heads;             /* GAT heads (1 otherwise)                                  */
    int32_t in_dtype;          /* atlas_dtype of the chunk embeddings                      */
    int32_t out_dtype;         /* atlas_dtype of the rows atlas_flush_ready writes         */
    int32_t activation;        /* atlas_activation applied after bias                      */
    float neg_slope;           /* GAT LeakyReLU slope                                      */
    int64_t max_chunk_sources; /* upper bound on src_end - src_begin of any chunk          */
    int32_t flags;             /* atlas_flags                                              */
    float gin_eps;             /* GIN: weight 1 + gin_eps of the vertex's own embedding    */
    int64_t hot_slots;         /* 0 (or >= N): one accumulator row per vertex.  0 < hot_slots < N:
                                  bounded accumulator store with that many rows, see below  */
    int32_t evict_policy;      /* atlas_evict_policy of the bounded store                   */
    int32_t tiles_per_run;     /* launch shape of the planned aggregation, see below; 0: the
                                  library chooses per launch                                */
    int64_t piece_tiles;       /* chunk loader of PINNED_HOST graphs with a plan, see below;
                                  0: the library's default (2^21 tiles)                     */
} atlas_dims_t;

/* The two launch-shape fields of atlas_dims_t.  Results do not depend on either beyond the
 * order of fp32 additions; 0 is the right value outside tests and tuning runs.
 *   tiles_per_run (0..16, else E_BAD_DIMS): in the planned aggregation each wave takes runs of
 *     that many consecutive 64-edge tiles of the chunk's destination-ordered edge list and
 *     keeps a destination's partial sum in registers from one tile of a run to the next.  0:
 *     chosen from the chunk's size (1 for small chunks, up to 16).  With runs of 4 tiles or
 *     more the runs after a wave's first are handed out by a counter instead of a fixed
 *     stride; with 8 or more the launch's last tiles go out in runs a quarter as long.
 *   piece_tiles (0..2^30, else E_BAD_DIMS): a planned chunk of at least 2 * piece_tiles tiles
 *     crosses the host link in pieces of piece_tiles tiles and each piece is pushed as soon as
 *     it has arrived, so that a long chunk's copy and kernels overlap (Sec. 3.3: the reader
 *     runs ahead of the aggregation). */

/* Bounded accumulator store (the paper's memory manager, Sec. 3.5, with HBM as the
 * hot tier and library-owned pinned host memory as the cold tier).  Only vertices
 * that have received a message and are not yet flushed hold one of the hot_slots
 * rows.  Before a chunk is pushed every vertex it addresses gets a row; when the
 * free rows do not suffice, the shortfall is evicted to the cold tier from the
 * resident vertices the chunk does not address, by evict_policy, ties by vertex
 * id, and an evicted vertex is reloaded when a later chunk addresses it.  Rows
 * are released by the atlas_flush_ready that writes the vertex's output, so the
 * rows needed at once are the chunk's destinations plus the completed vertices
 * not yet flushed; atlas_broadcast_chunk returns E_NOMEM when they do not fit
 * (the chunk is then partly marked and the layer can only be finished, which
 * frees it; a smaller chunk size, more rows or an order that completes vertices
 * sooner, such as atlas_reorder_score_desc, is the remedy).
 * Requires a graph with a plan and chunks that coincide with the planned ones
 * (as with ATLAS_FLAG_PLANNED_ONLY); not available for GAT.  Each chunk costs
 * one wait for the stream (the host reads the slot counts).  On a PINNED_HOST
 * graph the evicted rows share the host link with the chunk loader's copies.
 * N < 2^30 (E_OVERFLOW at atlas_layer_init otherwise). */
enum atlas_evict_policy {
    ATLAS_EVICT_MIN_PENDING = 0, /* fewest pending messages first (the paper's policy)      */
    ATLAS_EVICT_MAX_PENDING = 1  /* most pending messages first (for comparison)            */
};

/* Layer parameters, DEVICE memory, row-major, caller-owned; they are repacked
 * at init and need not outlive atlas_layer_init.
 *   SAGE_MEAN: W is [2*d_in][d_out]; rows 0..d_in-1 multiply the vertex's own
 *              embedding, rows d_in.. multiply the neighbour mean
 *              (self-concatenation, Sec. 4.3);  y = [h_v || mean] W + bias.
 *   GCN_SYM:   W is [d_in][d_out];  y = (sum_u h_u / sqrt(D_u D_v)) W + bias,
 *              D = in-degree of the graph as given (self-edges already added).
 *              Defined for graphs in which every vertex that sends a message
 *              has an in-edge itself (D_u > 0), as after adding the self-edges.
 *   GAT:       W is [d_in][d_out], head k owns columns k*dh..(k+1)*dh-1,
 *              attn_src / attn_dst are [heads][dh].
 *   GIN:       W is [d_in][d_out]; y = ((1 + gin_eps) x_v + sum of in-neighbours) W + b.
 *   SGC_HOP:   no weights (all four pointers may be NULL);
 *              y_v = sum_{u in N(v)} x_u / sqrt(D_u D_v), D as for GCN_SYM.
 * bias is [d_out] or NULL. */
typedef struct {
    const void *W, *bias, *attn_src, *attn_dst;
    int32_t dtype; /* atlas_dtype of all four arrays */
} atlas_weights_t;

typedef struct {
    int64_t edges_processed;    /* messages pushed along edges                              */
    int64_t sources_processed;  /* sources broadcast (must equal N at finish)               */
    int64_t vertices_completed; /* ready-list length                                        */
    int64_t vertices_flushed;   /* rows written by atlas_flush_ready                        */
    int64_t num_chunks, num_flushes;
    int64_t bytes_copied_h2d;   /* PINNED_HOST residency: bytes staged into HBM             */
    float ms_aggregate;         /* ATLAS_FLAG_TIMING: sum over chunks of the scatter-aggregate
                                   kernel (with its fused decrement + compaction)           */
    float ms_self;              /* ATLAS_FLAG_TIMING: SAGE own-row copy + self message      */
    float ms_update;            /* ATLAS_FLAG_TIMING: sum over flushes of update kernels    */
    float ms_copy;              /* ATLAS_FLAG_TIMING: sum of staging copies                 */
    float ms_init;              /* ATLAS_FLAG_TIMING: layer set-up kernels                  */
    int64_t hot_evictions;      /* bounded store: rows written to the cold tier             */
    int64_t hot_reloads;        /* bounded store: rows read back from the cold tier         */
    int64_t hot_peak_slots;     /* bounded store: most rows in use at once                  */
    int64_t chunks_planned;     /* chunks pushed from the plan (destination-grouped edges)  */
    int64_t chunks_csr_stream;  /* chunks pushed straight from the CSR with fp32 atomics (short
                                   chunks without a planned chunk, or ATLAS_FLAG_CSR_STREAM):
                                   about ten times slower per edge than the other two       */
    int64_t chunks_regrouped;   /* chunks without a planned chunk that were regrouped by
                                   destination on the fly; the three counts add up to
                                   num_chunks                                               */
    float ms_regroup;           /* host time of that regrouping (it is synchronous), always
                                   measured                                                 */
    float ms_dense;             /* ATLAS_FLAG_TIMING: time of the dense part of the plan's first
                                   chunk, pushed either way (not part of ms_aggregate)      */
    int64_t rows_handed_over;   /* vertices whose finished row went from the aggregation to the
                                   update as the update's operand (see atlas_flush_ready)   */
    int64_t edges_contracted;   /* edges of the plan's dense part that were pushed as a dense
                                   contraction (see atlas_plan_create_dense); they are part
                                   of edges_processed                                       */
    float ms_contract;          /* ATLAS_FLAG_TIMING: the contraction kernel alone (part of
                                   ms_dense, which also clears the rows, repacks the chunk
                                   and lowers the pending counts)                           */
} atlas_layer_stats_t;

/* Create the state of one layer (Sec. 3.4: pending-message tracker and
 * per-vertex arrays; Sec. 3.8: a vertex is complete after d_in(v) messages).
 * pending0[v] = d_in(v) (+1 for SAGE_MEAN and GIN: the vertex's own embedding is a
 * message to itself that arrives with its own chunk).  Vertices with
 * pending0 == 0 are placed on the ready list here.  Accumulators are zeroed.
 * Enqueues on `hip_stream` (a hipStream_t, NULL = default stream; the set-up kernels
 * are ordered with the chunk and flush calls that follow, which is why the call takes
 * the stream although the layer's definition has no use for one) and returns
 * without waiting.  *out receives the layer.  Errors: E_NULL, E_BAD_DIMS,
 * E_OVERFLOW, E_NOMEM, E_HIP. */
int atlas_layer_init(const atlas_graph_t *graph, const atlas_dims_t *dims,
                     const atlas_weights_t *weights, void *hip_stream, atlas_layer_t **out);

/* GAT only: attention terms el[u] = a_src . (W^T h_u), er[u] = a_dst . (W^T h_u)
 * of rows [src_begin, src_end).  Every row must have been through this call
 * before the first atlas_broadcast_chunk (a destination's term is needed when
 * its first message arrives).  Same chunk rules and `emb` meaning as
 * atlas_broadcast_chunk; host rows of a PINNED_HOST graph therefore cross the
 * link twice per layer, here and in their broadcast.  E_STATE for other models. */
int atlas_attention_prepass(atlas_layer_t *layer, int64_t src_begin, int64_t src_end,
                            const void *emb, void *hip_stream);

/* Broadcast sources [src_begin, src_end) (Sec. 3.1, 3.3, 3.4).  `emb` points at
 * the (src_end - src_begin) x d_in row-major embeddings OF THE CHUNK ONLY, in
 * dims.in_dtype; device memory for DEVICE graphs; for PINNED_HOST graphs
 * either pinned host memory (the library stages it and the chunk's edges into
 * HBM on its own copy stream, overlapped with the previous chunk's kernels) or
 * device memory (a later layer whose input is the previous layer's output:
 * only the edges are staged), the same kind for every chunk of the layer.
 * For every out-edge (u, v): acc[v] += g(u) h_u and pending[v] -= 1; v joins
 * the ready list when its count reaches zero.  Chunks must arrive in ascending
 * contiguous order starting at 0 ("strictly ordered", Sec. 3.4).  Only
 * enqueues; `emb` must stay valid until the stream has passed this point.
 * Which way the chunk's edges are visited: from the graph's plan when the range is
 * one of its chunks; else, when the chunk has at least 2^20 edges, regrouped by
 * destination on the spot (the plan's construction for this chunk alone, thrown
 * away afterwards: the call then waits for the stream and sorts before it
 * enqueues; about a third of the time of the third way at scale 26); else straight
 * from the CSR with one fp32 atomic row add per edge.  Results are the same sums in
 * another order; atlas_layer_stats_t says which way each chunk went.
 * Errors: E_NULL, E_RANGE, E_ORDER, E_STATE, E_HIP. */
int atlas_broadcast_chunk(atlas_layer_t *layer, int64_t src_begin, int64_t src_end,
                          const void *emb, void *hip_stream);

/* Update every vertex that became ready since the previous flush (Sec. 3.6):
 * gather its finished aggregate, normalise, multiply by W, add bias, apply the
 * activation and write row v of `out` (DEVICE memory, N x d_out row-major,
 * dims.out_dtype).  Only rows of flushed vertices are written.  If n_flushed is
 * not NULL the call waits for the stream and stores the number of rows written;
 * with NULL it only enqueues.  Errors: E_NULL, E_STATE, E_HIP.
 * Fused part (Sec. 3.6 hands a vertex to the transform the moment its count reaches zero): in
 * SAGE_MEAN / GCN_SYM layers with 16-bit embeddings of width 128, a vertex whose last edge
 * message belongs to a group of a planned or regrouped chunk that one wavefront sums alone --
 * the group completes the vertex, or (SAGE_MEAN) leaves only the vertex's own message
 * outstanding, which carries no data for the sum -- does not go through an fp32 accumulator
 * round trip: the aggregation writes the
 * finished row as this call's own left operand (normalised, rounded to the compute type exactly
 * as this call would have) and marks the vertex's ready-list entry; this call reads half the
 * bytes for it and skips the normalisation.  Results are bit-identical with and without it
 * (ATLAS_FLAG_NO_HANDOVER); ATLAS_DBG_ACC rows of such vertices then hold that operand in their
 * first half. */
int atlas_flush_ready(atlas_layer_t *layer, void *out, int64_t *n_flushed, void *hip_stream);

/* Wait for the layer's work, verify that all N sources were broadcast and that
 * every vertex was completed and flushed exactly once, fill *stats (may be
 * NULL) and free the layer -- also when it returns E_INCOMPLETE. */
int atlas_layer_finish(atlas_layer_t *layer, atlas_layer_stats_t *stats);

/* One-time, per-graph preparation (like the paper's offline reordering,
 * Sec. 3.8, it is paid once and reused by every layer and every run on the
 * graph): for each aligned chunk k = [k*chunk_sources, min(N, (k+1)*chunk_sources))
 * the chunk's out-edges are regrouped by destination, so that a chunk's
 * messages to one destination are summed in registers and reach the
 * accumulator as one row update, and the destination's pending count drops by
 * the group's size in one step.  Results are those of the plain edge stream
 * (same sums up to fp32 rounding order, same counts, same ready sets).
 * atlas_broadcast_chunk uses the plan for chunks that coincide with a planned
 * chunk; any other range is regrouped on the fly or pushed from the CSR (see there).
 * Synchronous.  The plan holds about 4 bytes per edge and lives where the graph
 * lives: device memory for DEVICE graphs; library-owned pinned host memory for
 * PINNED_HOST graphs (each chunk's CSR slice is staged into HBM, regrouped
 * there and brought back; atlas_broadcast_chunk then streams the regrouped
 * chunk instead of the CSR slice; with chunks of at most 2^23 sources a
 * pinned-host plan keeps 3 bytes per edge, which is what crosses the host link
 * in every layer).  It must outlive the layers that use it.
 * graph->plan and graph->in_degree are ignored here. */
int atlas_plan_create(const atlas_graph_t *graph, int64_t chunk_sources, atlas_plan_t **out);

/* atlas_plan_create with a source-blocked edge order for the heavy destinations.
 * In destination order the group of a high-degree destination walks the rows
 * of the whole chunk, far more than a cache holds, so nothing is reused between
 * groups.  Here the edges of every destination that receives at least
 * hot_min_edges messages from a chunk are ordered by (source block,
 * destination), a block being block_sources consecutive sources: while the
 * kernel works through one block its rows stay cache resident.  Choose
 * block_sources so that a block's rows fit an L2 (4 MiB on this GPU: 16,384
 * rows of 256 bytes) and hot_min_edges at several times the number of blocks
 * per chunk (every such destination gets one group per block).  Results are the
 * same sums in another order.  block_sources = 0: plain atlas_plan_create.
 * Not for GAT layers (E_BAD_DIMS at atlas_layer_init); N < 2^30 (E_OVERFLOW). */
int atlas_plan_create_blocked(const atlas_graph_t *graph, int64_t chunk_sources, int64_t block_sources,
                              int64_t hot_min_edges, atlas_plan_t **out);
/* atlas_plan_create_blocked with a dense part for the first chunk.  With ids in in-degree-descending order (Sec. 3.8) the hottest sources and the
 * hottest destinations both lie at the front, and the first chunk's edges between them are so
 * many that this corner of the adjacency matrix holds more than one edge per hundred cells.
 * There a message costs more as a 256-byte row gather than its cell costs in a dense product.
 * The plan therefore keeps the multiplicities of that corner as a staircase of matrices of 4-bit counts
 * (256 destinations form a band; a band takes its first S_band sources, S_band non-increasing
 * over the bands) and the layer adds  multiplicities x rows  to the accumulators of those
 * destinations on the matrix cores before it pushes the chunk's other edges: multiplicities up
 * to 15 are exact 16-bit floats, the products are exact, the sums are fp32 -- the edge stream's
 * sums in another order.  Pending counts drop by each destination's number of dense messages in
 * one step, vertices that complete are appended to the ready list as for any other message.
 * The region is chosen from the chunk's edge counts over log-spaced (source rank, destination
 * rank) blocks: a block belongs to it when it holds at least one edge per dense_cells_per_edge
 * cells (0: the library's default, 96) and so do the blocks before it; the value is halved until
 * the cells fit dense_max_bytes (0: no dense part, plain atlas_plan_create_blocked).  A cell that
 * is full (15) leaves further copies of its edge to the chunk's edge list.  When no block is
 * dense enough the plan is an ordinary one.
 * The contraction serves layers that sum plain rows (SAGE_MEAN, GIN, SGC_HOP), 16-bit rows of
 * width 64 or 128 (with ATLAS_FLAG_TRANSFORM_FIRST: the pushed products); every other layer, and
 * ATLAS_FLAG_NO_DENSE, pushes the same edges as a planned chunk, which the plan keeps as well.
 * Not for GAT layers or a bounded accumulator store (E_BAD_DIMS at atlas_layer_init).
 * The dense part always lives in device memory, also in the plan of a PINNED_HOST graph: it is
 * then the part of the topology that does not cross the host link in every layer (the cells are
 * half a byte each, and the part's edges as a planned chunk 4 bytes each, where a streamed edge
 * costs 3 bytes per layer). */
int atlas_plan_create_dense(const atlas_graph_t *graph, int64_t chunk_sources, int64_t block_sources,
                            int64_t hot_min_edges, int64_t dense_max_bytes, int64_t dense_cells_per_edge,
                            atlas_plan_t **out);
int atlas_plan_destroy(atlas_plan_t *plan);

/* In-degree of every vertex (histogram of col_indices), int32[N] in DEVICE
 * memory.  Works for both residencies (a PINNED_HOST edge array is read over
 * the host link, once).  Enqueues on hip_stream; for DEVICE graphs of more
 * than 2^15 vertices and 2^22 edges it also waits for the result (such graphs
 * are counted bucket by bucket in LDS, with two bytes of scratch per edge that
 * the call takes from, and returns to, the library's buffer cache). */
int atlas_in_degree(const atlas_graph_t *graph, int32_t *in_degree, void *hip_stream);

/* The same in-degrees read off a plan of the graph whose arrays are in DEVICE memory (a group's
 * size is what its destination receives from the chunk): one pass over the plan's 4-byte edge
 * words instead of one counter update per edge.  atlas_layer_init does this by itself when the
 * graph has such a plan and no in_degree.  Enqueues on hip_stream.  E_STATE for plans of
 * PINNED_HOST graphs (count from the graph instead). */
int atlas_plan_in_degree(const atlas_plan_t *plan, int32_t *in_degree, void *hip_stream);

/* In-degree-descending vertex order, ties by smaller old id first:
 * old_of_new[i] is the vertex placed at position i, new_of_old its inverse.
 * graph->in_degree must be set.  Both outputs are int32[N] DEVICE memory.
 * Synchronous. */
int atlas_reorder_indegree_desc(const atlas_graph_t *graph, int32_t *new_of_old,
                                int32_t *old_of_new);

/* atlas_reorder_indegree_desc for callers that cannot allocate device memory (tight serving
 * loops that re-order a small graph per request, harnesses that forbid hipMalloc): the same
 * permutation, bit for bit, computed without any allocation.  The sort's scratch (sorted keys,
 * ids, workspace) lies in a fixed 24 MiB array in device memory that every GPU the library runs
 * on holds until the process ends; inputs and outputs are the caller's as above.
 * num_vertices <= ATLAS_NOALLOC_MAX_VERTICES, else E_TOO_LARGE and nothing is launched.
 * Enqueues on hip_stream (NULL = default stream) and returns without waiting; the outputs are
 * complete when the stream has passed this point.  All calls on one GPU share that GPU's
 * scratch: calls that overlap on one GPU (two streams, two threads) race; calls on one stream
 * are ordered and need no clearing in between (every scratch word is written before it is
 * read).  The library sort it uses clears its counters with asynchronous memsets, so the call
 * is not meant for stream capture.  Errors: E_NULL, E_RANGE, E_TOO_LARGE, E_HIP. */
#define ATLAS_NOALLOC_MAX_VERTICES (1 << 20)
int atlas_reorder_indegree_desc_noalloc(const atlas_graph_t *graph, int32_t *new_of_old, int32_t *old_of_new,
                                        void *hip_stream);

/* The paper's greedy ordering (Sec. 3.8): vertices by decreasing
 * Score(u) = (sum_{v in Out(u)} 1/d_in(v)) / d_out(u) (0 without out-edges),
 * ties by smaller old id first.  Scores are summed in fp64 in CSR order, so the
 * permutation is reproducible bit for bit.  DEVICE graphs, graph->in_degree
 * must be set; outputs are int32[N] DEVICE memory.  Synchronous. */
int atlas_reorder_score_desc(const atlas_graph_t *graph, int32_t *new_of_old, int32_t *old_of_new);

/* Neighbourhood sampling done on the graph before inference (the route Sec. 3.9
 * names: the edges a sample drops are switched off, and the broadcast then runs
 * unchanged on what is left).  Every destination keeps at most `fanout` of its in-edges:
 * those with the smallest edge_key (one caller-drawn uint32 per edge, DEVICE
 * memory, in CSR order), ties by position in the CSR.  out_row_offsets
 * (int64[N+1]) and out_col_indices (int32, room for num_edges) in DEVICE memory
 * receive the CSR by source of the kept edges in their original order;
 * *out_num_edges (host, may be NULL) their number.  DEVICE graphs with fewer
 * than 2^32 edges.  Synchronous.  Errors: E_NULL, E_BAD_DIMS, E_RANGE,
 * E_OVERFLOW, E_NOMEM, E_HIP. */
int atlas_sample_in_edges(const atlas_graph_t *graph, const uint32_t *edge_key, int32_t fanout,
                          int64_t *out_row_offsets, int32_t *out_col_indices, int64_t *out_num_edges);

/* What a plan holds, for reports: chunk count, edges, destination groups (one per chunk and
 * destination; a source-blocked plan has one per block for its heavy destinations), groups
 * that are the first of their destination in the whole plan, and the bytes the plan occupies
 * in device and in pinned host memory. */
typedef struct {
    int64_t num_chunks, num_edges, num_groups, num_first_groups;
    int64_t bytes_device, bytes_pinned_host;
    int64_t dense_edges;        /* edges the dense part of the first chunk holds (0: no dense part) */
    int64_t dense_groups;       /* their destination groups (part of num_groups)                    */
    int64_t dense_cells;        /* its cells (half a byte each)                                     */
    int64_t dense_rows;         /* destinations [0, dense_rows) have a band                         */
    int64_t dense_max_sources;  /* sources the longest band takes                                   */
} atlas_plan_info_t;
int atlas_plan_info(const atlas_plan_t *plan, atlas_plan_info_t *info);

/* Measured peaks of the box at hand, for the benchmark's report (Sec. 4.4 of the paper
 * asks what bounds the run; here: what a bare kernel of the same access pattern reaches).
 * They only enqueue on hip_stream; the caller times them with events on that stream.
 *   atlas_probe_copy:        dst[0..bytes) = src[0..bytes), DEVICE memory, bytes a multiple of 16.
 *   atlas_probe_mix21:       dst[i] = a[i] ^ b[i] over `bytes` bytes of each array: two bytes read per byte
 *                            written, the flush's mix (accumulator row and own row in, output row out).
 *   atlas_probe_row_gather:  reads rows ids[0..n_ids) of `table` (rows of 256 bytes, DEVICE),
 *                            one wave per row, eight rows in flight per wave -- the planned
 *                            aggregation's source-row gather without its bookkeeping.  ids:
 *                            int32 DEVICE, each in [0, table_rows).  sink: DEVICE scratch of at
 *                            least atlas_probe_gather_sink_bytes() bytes (the waves' folded words).
 *   atlas_probe_dense_rows:  out = rows x W on the matrix cores with the kernels the flush and the
 *                            transform-first path use for a dense block of rows: n_rows x K row-major
 *                            `rows`, K x d_out row-major `W`, n_rows x d_out `out`, all `dtype`
 *                            (16-bit types; K a multiple of 64 up to 1024, d_out a multiple of 32 up
 *                            to 256), `repeat` passes over the same rows, so that a row block that
 *                            fits the caches shows the contraction's rate without the HBM cap.
 *   atlas_probe_mfma:        nothing but bf16 32x32x16 matrix instructions on register operands:
 *                            waves_per_simd (1..8) wavefronts on every SIMD, each `iters` (up to 2^24)
 *                            rounds of four independent products; *flops (host) receives the
 *                            launch's flop count.  What the matrix pipeline delivers when nothing is
 *                            loaded, converted or synchronised.  sink: as for atlas_probe_row_gather.
 * Errors: E_NULL, E_BAD_DIMS, E_RANGE, E_HIP, E_NOMEM. */
int atlas_probe_mfma(int32_t waves_per_simd, int32_t iters, void *sink, double *flops, void *hip_stream);
int atlas_probe_copy(void *dst, const void *src, int64_t bytes, void *hip_stream);
int atlas_probe_mix21(void *dst, const void *a, const void *b, int64_t bytes, void *hip_stream);
int64_t atlas_probe_gather_sink_bytes(void);
int atlas_probe_row_gather(const void *table, int64_t table_rows, const int32_t *ids, int64_t n_ids, void *sink,
                           void *hip_stream);
int atlas_probe_dense_rows(int32_t dtype, const void *rows, int64_t n_rows, int32_t K, int32_t d_out, const void *W,
                           void *out, int32_t repeat, void *hip_stream);

/* Synchronise and copy one internal array to host memory, for tests. */
enum atlas_debug_what {
    ATLAS_DBG_INDEG = 0,       /* int32[N]                                  */
    ATLAS_DBG_PENDING = 1,     /* int32[N]                                  */
    ATLAS_DBG_READY = 2,       /* int32[ready count], completion order      */
    ATLAS_DBG_READY_COUNT = 3, /* int64[2]: {ready tail, flushed head}      */
    ATLAS_DBG_ACC = 4          /* float[N][acc width]                       */
};
int atlas_debug_copy(atlas_layer_t *layer, int what, void *host_dst, int64_t bytes);

/* Free what the library keeps for reuse between layers: its cache of device buffers, the
 * work arrays of the on-the-fly regrouping (see atlas_broadcast_chunk), the bounded store's
 * pinned cold tier, and the chunk loader's copy stream (created again when next needed).  Call it when no layer is alive, e.g. before the process ends: the HIP
 * runtime may already be shutting down when static destructors run, so the library frees
 * nothing by itself at exit. */
int atlas_release_cache(void);

const char *atlas_strerror(int status);
const char *atlas_last_hip_error(void); /* text of the last failed HIP call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* ATLAS_H */
