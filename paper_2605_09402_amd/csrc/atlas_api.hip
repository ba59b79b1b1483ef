// Host side of the C ABI declared in include/atlas.h: argument checks, the
// per-layer state machine (strictly ordered chunks, paper Sec. 3.4), buffer
// ownership, the pinned-host chunk loader on a second stream (the reader that
// runs ahead of the orchestrator, Sec. 3.3) and the exactly-once check at the
// end of a layer (Sec. 3.1).
#include "../../include/atlas.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "atlas_kernels.h"

using namespace atlas;

namespace {

thread_local std::string g_hip_error;

int hip_fail(hipError_t e, const char *what) {
    g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return e == hipErrorOutOfMemory ? ATLAS_E_NOMEM : ATLAS_E_HIP;
}

#define HIP_TRY(expr)                                     \
    do {                                                  \
        hipError_t e_ = (expr);                           \
        if (e_ != hipSuccess) return hip_fail(e_, #expr); \
    } while (0)

// ---- device buffer cache: layers of one model reuse each other's buffers ----
struct CachedBuf { void *p; size_t bytes; };
std::mutex g_cache_mu;
std::vector<CachedBuf> g_cache;

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

hipError_t cache_alloc(void **out, size_t bytes) {
    bytes = round_up(bytes > 0 ? bytes : 1, 256);
    {
        std::lock_guard<std::mutex> lk(g_cache_mu);
        int best = -1;
        for (int i = 0; i < static_cast<int>(g_cache.size()); ++i)
            if (g_cache[i].bytes >= bytes && g_cache[i].bytes <= bytes + bytes / 4 &&
                (best < 0 || g_cache[i].bytes < g_cache[best].bytes))
                best = i;
        if (best >= 0) {
            *out = g_cache[best].p;
            g_cache.erase(g_cache.begin() + best);
            return hipSuccess;
        }
    }
    return hipMalloc(out, bytes);
}

struct Buf {
    void *p = nullptr;
    size_t bytes = 0;
    hipError_t alloc(size_t n) {
        bytes = round_up(n > 0 ? n : 1, 256);
        return cache_alloc(&p, bytes);
    }
    void release() {
        if (!p) return;
        std::lock_guard<std::mutex> lk(g_cache_mu);
        g_cache.push_back({p, bytes});
        p = nullptr;
    }
};

size_t dtype_size(int dt) { return dt == ATLAS_DTYPE_F32 ? 4 : 2; }

// Cold tier of the bounded accumulator store: one pinned host buffer per
// process, grown on demand and kept until atlas_release_cache (pinning tens of
// gigabytes takes seconds; layers with a bounded store run one after another
// and reuse it).
// Work arrays of the on-the-fly regrouping (tens of gigabytes for a long chunk), parked between layers so that
// a run without a plan does not allocate and free them per layer; one set: a second layer that regroups at the
// same time gets its own.  Freed by atlas_release_cache.
PlanWork *g_regroup_work = nullptr;
PlanWork *take_regroup_work() {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    PlanWork *w = g_regroup_work;
    g_regroup_work = nullptr;
    return w;
}
void park_regroup_work(PlanWork *w) {
    if (!w) return;
    {
        std::lock_guard<std::mutex> lk(g_cache_mu);
        if (!g_regroup_work) {
            g_regroup_work = w;
            return;
        }
    }
    delete w;
}

void *g_cold = nullptr;
size_t g_cold_bytes = 0;
hipError_t cold_buffer(size_t bytes, void **out) {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    if (g_cold_bytes < bytes) {
        if (g_cold) (void)hipHostFree(g_cold);
        g_cold = nullptr;
        g_cold_bytes = 0;
        hipError_t e = hipHostMalloc(&g_cold, bytes, hipHostMallocDefault);
        if (e != hipSuccess) return e;
        g_cold_bytes = bytes;
    }
    *out = g_cold;
    return hipSuccess;
}

// tiles per piece of a long pinned-host chunk unless dims.piece_tiles says otherwise: 2^21 tiles = 2^27 edges
constexpr int64_t kDefaultPieceTiles = int64_t(1) << 21;
// A block of the first chunk goes to the dense part when it holds at least one edge per this many cells: a
// cell costs a byte of the contraction's stream, an edge a 256-byte row gather.
constexpr int64_t kDefaultDenseCellsPerEdge = 96;

// The chunk loader's copy stream is created once per process and shared by
// all layers: HIP spreads streams over a few hardware queues, and a stream
// created anew for every layer can land on the queue that carries the caller's
// kernels, which silently serialises the copies with them.
hipStream_t g_copy_stream = nullptr;
hipError_t loader_stream(hipStream_t *out) {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    if (!g_copy_stream) {
        hipError_t e = hipStreamCreateWithFlags(&g_copy_stream, hipStreamNonBlocking);
        if (e != hipSuccess) return e;
    }
    *out = g_copy_stream;
    return hipSuccess;
}

struct TimedSpan { hipEvent_t a, b; };

}  // namespace

struct atlas_plan {
    int64_t n = 0, e = 0, chunk = 0;
    bool host = false;              // arrays live in pinned host memory (plan of a PINNED_HOST graph)
    int32_t *src_sorted = nullptr;  // [E] destination-ordered source ids of all chunks
    uint8_t *src_packed = nullptr;  // host plans with chunks of at most 2^23 sources: the same words in 3 bytes
    size_t packed_bytes = 0;        // (PlanChunk::packed_off locates a chunk's words); src_sorted is then unused
    int64_t *dev_off = nullptr;     // host plans: device copy of the graph's row offsets, so that layers need not
                                    // bring them over the link again
    bool blocked = false;           // some chunk is in source-blocked order (grp_dst bit 30 in use)
    std::vector<PlanChunk> chunks;  // grp_dst / tile_grp: device, or pinned host when `host`
    size_t max_stage_bytes = 0;     // host plans: largest staging slot any chunk needs
    int64_t n_first = 0;            // destinations that receive a message from some chunk (first-touch groups)
    DensePart dense;                // device plans made by atlas_plan_create_dense: the dense part of chunk 0
                                    // (dense.n_items > 0), pushed before chunks[0], which holds the chunk's other edges
};

namespace {
size_t stage_bytes_of(const PlanChunk &c, bool packed) {
    const size_t words = packed ? packed24_bytes(c.n_edges) : static_cast<size_t>(c.n_edges) * 4;
    return round_up(words, 256) + round_up(static_cast<size_t>(c.n_groups) * 4, 256) +
           round_up(static_cast<size_t>((c.n_edges + 63) / 64) * 4, 256);
}
}  // namespace

struct atlas_layer {
    atlas_graph_t g{};
    atlas_dims_t dims{};
    int64_t n = 0, e = 0;
    int K = 0;
    int compute_dt = 0;
    int selfmsg = 0;
    int acc_width = 0;

    Buf indeg_scratch;   // scratch of the in-degree count when the library counts (large DEVICE graphs)
    Buf indeg_own, pending, ready, counters, counters64, acc, self_rows, packed_w, bias, dev_off;
    Buf gat_el, gat_er, gat_mcur, gat_mnext, gat_l, gat_wa, gat_z;   // GAT state
    Buf gat_scores;                                                  // GAT, planned chunks: per-edge logits
    Buf dense_rows;                                                  // chunk 0's rows repacked for the dense part
    int64_t edges_contracted = 0;                                    // edges pushed as a dense contraction
    int64_t prepass_next = 0, num_prepass = 0;
    const int32_t *indeg = nullptr;
    const int64_t *off_dev = nullptr;  // device-visible row offsets

    // bounded accumulator store (dims.hot_slots > 0)
    bool bounded = false;
    HotStore hs{};
    Buf hs_slot_of, hs_owner, hs_free, hs_stamp, hs_need, hs_ctr, hs_keys, hs_keys_sorted, hs_sort_temp;
    int64_t hot_evictions = 0, hot_reloads = 0;

    // transform-first layers
    bool tf = false;
    Buf unpacked;   // pinned-host plans with 24-bit edge words: the current chunk's words as the kernels read them
    Buf tf_z;       // [chunk][d_out] in the storage type: the chunk's rows times W (SAGE: W_neigh)
    Buf tf_self;    // [N][d_out] fp32: SAGE x_v W_self, GIN x_v W
    Buf packed_w2;  // SAGE: W_self in fragment order

    bool handover = false;             // rows completed inside the grouped aggregation leave as the update's operand
    bool planned_only = false;         // every chunk runs from the plan: no accumulator zero fill
    bool emb_resident = false;         // own rows are read from the caller's matrix
    const char *x_base = nullptr;      // base of that matrix (set by the first chunk)
    int emb_on_device = -1;            // PINNED_HOST graphs: the chunks' embeddings are device memory (1), host (0),
                                       // not yet known (-1); e.g. a later layer whose input is the previous output

    int64_t next_src = 0;
    uint32_t run_tickets = 0;          // tickets drawn so far from the grouped aggregation's run counter
    int64_t num_chunks = 0, num_flushes = 0;
    int64_t chunks_planned = 0, chunks_csr = 0, chunks_regrouped = 0;   // which aggregation path each chunk took
    // Chunks without a planned chunk are regrouped by destination on the fly (the plan's construction, for
    // this chunk only, thrown away afterwards) when they are long enough to pay for the sort.
    PlanWork *regroup_work = nullptr;
    PlanChunk cur_regroup{};          // arrays of the chunk regrouped last; freed before the next one is built
    Buf regroup_src;                  // its edge words
    double ms_regroup = 0.0;          // host time spent regrouping (the sort is synchronous)
    int64_t bytes_h2d = 0;

    // pinned-host loader
    hipStream_t copy_stream = nullptr;
    // Staging ring of the chunk loader.  With four slots the copies of the chunks after a long one
    // (the first chunk of a degree-ordered graph: 75 ms of kernels at scale 26) keep going while its
    // kernels run; with two the copy stream sat idle for most of that time.  A slot's edge buffer is
    // allocated for the first chunk that needs it and grows on demand, so only the slots that ever
    // see a large chunk are large.
    static constexpr int kStageSlots = 4;
    hipEvent_t slot_loaded[kStageSlots] = {};
    hipEvent_t slot_free[kStageSlots] = {};
    bool slot_used[kStageSlots] = {};
    Buf stage_col[kStageSlots], stage_emb[kStageSlots];
    std::vector<hipEvent_t> piece_ev[kStageSlots];   // a long chunk's edge words arrive in pieces: one event each

    std::vector<TimedSpan> t_agg, t_self, t_upd, t_copy, t_init, t_dense, t_contract;
    hipStream_t last_stream = nullptr;

    int32_t *ctr() { return static_cast<int32_t *>(counters.p); }

    void free_regrouped() {
        if (cur_regroup.grp_dst) (void)hipFree(cur_regroup.grp_dst);
        if (cur_regroup.tile_grp) (void)hipFree(cur_regroup.tile_grp);
        cur_regroup = PlanChunk{};
    }

    void destroy() {
        for (Buf *b : {&indeg_scratch, &indeg_own, &pending, &ready, &counters, &counters64, &acc, &self_rows, &packed_w, &bias,
                       &dev_off, &gat_el, &gat_er,
                       &gat_mcur, &gat_mnext, &gat_l, &gat_wa, &gat_z, &gat_scores, &dense_rows, &hs_slot_of, &hs_owner, &hs_free,
                       &hs_stamp, &hs_need, &hs_ctr, &hs_keys, &hs_keys_sorted, &hs_sort_temp, &tf_z, &tf_self, &unpacked,
                       &packed_w2})
            b->release();
        free_regrouped();
        park_regroup_work(regroup_work);
        regroup_work = nullptr;
        regroup_src.release();
        for (auto &v : piece_ev)
            for (hipEvent_t e : v) (void)hipEventDestroy(e);
        for (Buf &b : stage_col) b.release();
        for (Buf &b : stage_emb) b.release();
        for (auto *v : {&t_agg, &t_self, &t_upd, &t_copy, &t_init, &t_dense, &t_contract})
            for (auto &sp : *v) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
        for (int i = 0; i < kStageSlots; ++i) {
            if (slot_loaded[i]) (void)hipEventDestroy(slot_loaded[i]);
            if (slot_free[i]) (void)hipEventDestroy(slot_free[i]);
        }
    }
};

namespace {

// Transform first (ATLAS_FLAG_TRANSFORM_FIRST): the linear map commutes with the
// sum, so each chunk's rows are multiplied by W before they are pushed and the
// accumulators are d_out wide.
bool transform_first(const atlas_dims_t &d) {
    return (d.flags & ATLAS_FLAG_TRANSFORM_FIRST) &&
           (d.model == ATLAS_MODEL_SAGE_MEAN || d.model == ATLAS_MODEL_GCN_SYM || d.model == ATLAS_MODEL_GIN);
}

// layers whose update uses the vertex's own embedding: it travels as a self message
bool has_self_term(int model) { return model == ATLAS_MODEL_SAGE_MEAN || model == ATLAS_MODEL_GIN; }
// the aggregation kernels know three kinds of sum: plain, source-scaled by deg^-1/2, attention-weighted
int aggregate_kind(int model) {
    if (model == ATLAS_MODEL_GCN_SYM || model == ATLAS_MODEL_SGC_HOP) return 1;
    return model == ATLAS_MODEL_GAT ? 2 : 0;
}

int check_dims(const atlas_dims_t &d, const atlas_weights_t &w) {
    if (d.model < ATLAS_MODEL_SAGE_MEAN || d.model > ATLAS_MODEL_SGC_HOP) return ATLAS_E_BAD_DIMS;
    if (d.model == ATLAS_MODEL_SGC_HOP) {
        // propagation only: no weights, the output row is the scaled accumulator row
        if (d.d_out != d.d_in || d.activation != ATLAS_ACT_NONE) return ATLAS_E_BAD_DIMS;
    } else if (!w.W) {
        return ATLAS_E_NULL;
    }
    if (d.model == ATLAS_MODEL_GAT) {
        // a wave holds a transformed row and each lane's elements must fall into one head
        if (d.heads < 1 || d.heads > 8 || d.d_out % 64 != 0 || d.d_out % d.heads != 0) return ATLAS_E_BAD_DIMS;
        if ((d.d_out / d.heads) % (d.d_out / 64) != 0) return ATLAS_E_BAD_DIMS;
        if (!w.attn_src || !w.attn_dst) return ATLAS_E_NULL;
    }
    const bool tf = transform_first(d);
    if (d.d_in <= 0 || d.d_in % 64 != 0 || d.d_in > (tf ? 1024 : 512)) return ATLAS_E_BAD_DIMS;
    if (tf && d.d_out % 64 != 0) return ATLAS_E_BAD_DIMS;   // a wave holds one d_out-wide product row
    if (d.d_out <= 0 || d.d_out % 16 != 0 || (d.d_out > 256 && d.model != ATLAS_MODEL_SGC_HOP))
        return ATLAS_E_BAD_DIMS;
    for (int dt : {d.in_dtype, d.out_dtype, w.dtype})
        if (dt != ATLAS_DTYPE_F32 && dt != ATLAS_DTYPE_BF16 && dt != ATLAS_DTYPE_F16) return ATLAS_E_BAD_DIMS;
    if (d.activation < ATLAS_ACT_NONE || d.activation > ATLAS_ACT_ELU) return ATLAS_E_BAD_DIMS;
    if (d.max_chunk_sources <= 0) return ATLAS_E_BAD_DIMS;
    if (d.hot_slots < 0 || d.evict_policy < ATLAS_EVICT_MIN_PENDING || d.evict_policy > ATLAS_EVICT_MAX_PENDING)
        return ATLAS_E_BAD_DIMS;
    if (d.hot_slots > 0 && d.model == ATLAS_MODEL_GAT) return ATLAS_E_BAD_DIMS;
    if (d.tiles_per_run < 0 || d.tiles_per_run > atlas::kMaxTilesPerRun) return ATLAS_E_BAD_DIMS;
    if (d.piece_tiles < 0 || d.piece_tiles > (int64_t(1) << 30)) return ATLAS_E_BAD_DIMS;
    const int K = d.model == ATLAS_MODEL_SAGE_MEAN && !tf ? 2 * d.d_in : d.d_in;
    // GIN forms (1 + eps) x_v + sum in the compute type before the contraction: a hub's sum leaves the
    // range of IEEE half, so half-precision GIN runs transform-first only (products summed in fp32)
    if (d.model == ATLAS_MODEL_GIN && d.in_dtype == ATLAS_DTYPE_F16 && !tf) return ATLAS_E_BAD_DIMS;
    const bool bf16c = d.in_dtype != ATLAS_DTYPE_F32;
    const size_t lds = 256 + static_cast<size_t>(64) * (K + (bf16c ? 8 : 1)) * (bf16c ? 2 : 4);
    if (lds > 160 * 1024) return ATLAS_E_BAD_DIMS;
    return ATLAS_OK;
}

int start_span(atlas_layer *L, std::vector<TimedSpan> &v, hipStream_t s) {
    if (!(L->dims.flags & ATLAS_FLAG_TIMING)) return ATLAS_OK;
    TimedSpan sp{};
    HIP_TRY(hipEventCreate(&sp.a));
    HIP_TRY(hipEventCreate(&sp.b));
    v.push_back(sp);
    HIP_TRY(hipEventRecord(sp.a, s));
    return ATLAS_OK;
}
int end_span(atlas_layer *L, std::vector<TimedSpan> &v, hipStream_t s) {
    if (!(L->dims.flags & ATLAS_FLAG_TIMING)) return ATLAS_OK;
    HIP_TRY(hipEventRecord(v.back().b, s));
    return ATLAS_OK;
}
float sum_spans(std::vector<TimedSpan> &v) {
    float total = 0.f;
    for (auto &sp : v) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sp.a, sp.b) == hipSuccess) total += ms;
    }
    return total;
}

int init_impl(atlas_layer *L, const atlas_weights_t *w, hipStream_t s) {
    const atlas_dims_t &d = L->dims;
    const int64_t n = L->n;
    const size_t n1 = static_cast<size_t>(n > 0 ? n : 1);
    HIP_TRY(L->counters.alloc(CTR_COUNT * sizeof(int32_t)));
    HIP_TRY(L->counters64.alloc(CTR64_COUNT * sizeof(unsigned long long)));
    HIP_TRY(L->pending.alloc(n1 * sizeof(int32_t)));
    HIP_TRY(L->ready.alloc(n1 * sizeof(int32_t)));
    // A bounded store needs the per-chunk destination lists of a plan; it implies the planned-only promise.
    L->bounded = d.hot_slots > 0 && d.hot_slots < n;
    // a plan with a dense part serves sum-aggregating layers whose accumulators are addressed by vertex id
    if (L->g.plan && L->g.plan->dense.n_items > 0 && (L->bounded || d.model == ATLAS_MODEL_GAT)) return ATLAS_E_BAD_DIMS;
    if (L->bounded) {
        const atlas_plan *pl = L->g.plan;
        if (!pl || pl->host != (L->g.residency == ATLAS_RESIDENT_PINNED_HOST) || pl->n != n || pl->e != L->e)
            return ATLAS_E_STATE;
        // slots are never zero-filled: the store relies on the plan's list of rows to clear
        if (d.hot_slots >= (int64_t(1) << 31) || n >= (int64_t(1) << 30)) return ATLAS_E_OVERFLOW;
    }
    const size_t acc_rows = L->bounded ? static_cast<size_t>(d.hot_slots) : n1;
    HIP_TRY(L->acc.alloc(acc_rows * L->acc_width * sizeof(float)));
    // (PINNED_HOST graphs: honoured when the embeddings turn out to be device memory, see the first chunk)
    L->emb_resident = has_self_term(d.model) && (d.flags & ATLAS_FLAG_EMB_RESIDENT) && !L->tf;
    if (L->tf) {
        const size_t rows = static_cast<size_t>(std::min<int64_t>(d.max_chunk_sources, std::max<int64_t>(n, 1)));
        if (d.model != ATLAS_MODEL_GIN) HIP_TRY(L->tf_z.alloc(rows * d.d_out * dtype_size(d.in_dtype)));
        if (has_self_term(d.model)) HIP_TRY(L->tf_self.alloc(n1 * d.d_out * sizeof(float)));
        // SAGE: W_neigh and W_self side by side in one fragment-ordered buffer (column blocks of the
        // first, then of the second), so that one pass over the chunk's rows yields both products
        if (d.model == ATLAS_MODEL_SAGE_MEAN)
            HIP_TRY(L->packed_w2.alloc(2 * packed_weight_bytes(L->K, d.d_out, L->compute_dt)));
    }
    if (has_self_term(d.model) && !L->emb_resident && !L->tf)
        HIP_TRY(L->self_rows.alloc(n1 * d.d_in * dtype_size(d.in_dtype)));
    HIP_TRY(L->packed_w.alloc(packed_weight_bytes(L->K, d.d_out, L->compute_dt)));
    HIP_TRY(launch_fill_zero(L->counters.p, L->counters.bytes, s));
    HIP_TRY(launch_fill_zero(L->counters64.p, L->counters64.bytes, s));
    // With ATLAS_FLAG_PLANNED_ONLY every row is first written (not added to) by
    // its destination's first group, so the zero fill is skipped.  GAT rescales
    // its accumulators and keeps the fill.
    L->planned_only = ((d.flags & ATLAS_FLAG_PLANNED_ONLY) || L->bounded) && L->g.plan && d.model != ATLAS_MODEL_GAT &&
                      L->g.plan->host == (L->g.residency == ATLAS_RESIDENT_PINNED_HOST) &&
                      L->g.plan->n == n && L->g.plan->e == L->e &&
                      n < (int64_t(1) << 30);   // the plan lists the rows to clear only below 2^30 vertices
    if (!L->planned_only)
        HIP_TRY(launch_fill_zero(L->acc.p, static_cast<size_t>(n) * L->acc_width * sizeof(float), s));
    // Fused part of the flush: 16-bit SAGE / GCN layers of width 128 whose flush runs the kernel that knows
    // handed-over rows, accumulators addressed by vertex id.
    L->handover = !(d.flags & ATLAS_FLAG_NO_HANDOVER) && !L->tf && !L->bounded &&
                  (d.model == ATLAS_MODEL_SAGE_MEAN || d.model == ATLAS_MODEL_GCN_SYM) &&
                  update_takes_handed_rows(d.model, d.d_in, L->K, d.d_out, L->compute_dt);
    if (L->bounded) {
        const size_t S = static_cast<size_t>(d.hot_slots);
        HIP_TRY(L->hs_slot_of.alloc(n1 * sizeof(int32_t)));
        HIP_TRY(L->hs_stamp.alloc(n1 * sizeof(int32_t)));
        HIP_TRY(L->hs_owner.alloc(S * sizeof(int32_t)));
        HIP_TRY(L->hs_free.alloc(S * sizeof(int32_t)));
        HIP_TRY(L->hs_need.alloc(S * sizeof(int32_t)));
        HIP_TRY(L->hs_ctr.alloc(HS_COUNT * sizeof(int32_t)));
        HIP_TRY(L->hs_keys.alloc(S * sizeof(uint64_t)));
        HIP_TRY(L->hs_keys_sorted.alloc(S * sizeof(uint64_t)));
        HIP_TRY(L->hs_sort_temp.alloc(hot_sort_temp_bytes(d.hot_slots)));
        void *cold = nullptr;
        if (hipError_t e = cold_buffer(n1 * L->acc_width * sizeof(float), &cold); e != hipSuccess) {
            (void)hip_fail(e, "hipHostMalloc(cold store)");
            return ATLAS_E_NOMEM;
        }
        L->hs.slot_of = static_cast<int32_t *>(L->hs_slot_of.p);
        L->hs.stamp = static_cast<int32_t *>(L->hs_stamp.p);
        L->hs.slot_owner = static_cast<int32_t *>(L->hs_owner.p);
        L->hs.free_list = static_cast<int32_t *>(L->hs_free.p);
        L->hs.need_list = static_cast<int32_t *>(L->hs_need.p);
        L->hs.ctr = static_cast<int32_t *>(L->hs_ctr.p);
        L->hs.keys = static_cast<uint64_t *>(L->hs_keys.p);
        L->hs.keys_sorted = static_cast<uint64_t *>(L->hs_keys_sorted.p);
        L->hs.hot = static_cast<float *>(L->acc.p);
        L->hs.cold = static_cast<float *>(cold);
        L->hs.slots = d.hot_slots;
        L->hs.d = L->acc_width;
        HIP_TRY(hot_init(L->hs, n, s));
    }

    if (L->g.residency == ATLAS_RESIDENT_PINNED_HOST) {
        // row offsets are small next to the edge array: keep a device copy for the kernels
        HIP_TRY(loader_stream(&L->copy_stream));
        for (int i = 0; i < atlas_layer::kStageSlots; ++i) {
            HIP_TRY(hipEventCreateWithFlags(&L->slot_loaded[i], hipEventDisableTiming));
            HIP_TRY(hipEventCreateWithFlags(&L->slot_free[i], hipEventDisableTiming));
        }
        // Every host-to-device copy of the layer goes through the copy stream, this one included.  A
        // copy issued on the compute stream here is still in flight when the first chunk's copies
        // start; the two streams then hold a copy engine each, the copy stream is given one that
        // moves host memory at about half the link rate (31 instead of 57 GB/s measured) and keeps
        // it for the whole layer.
        if (L->g.plan && L->g.plan->host && L->g.plan->dev_off && L->g.plan->n == n) {
            L->off_dev = L->g.plan->dev_off;   // the plan of this graph already holds them on the device
        } else {
            HIP_TRY(L->dev_off.alloc((n1 + 1) * sizeof(int64_t)));
            HIP_TRY(hipMemcpyAsync(L->dev_off.p, L->g.row_offsets, (static_cast<size_t>(n) + 1) * sizeof(int64_t),
                                   hipMemcpyHostToDevice, L->copy_stream));
            HIP_TRY(hipEventRecord(L->slot_loaded[0], L->copy_stream));
            HIP_TRY(hipStreamWaitEvent(s, L->slot_loaded[0], 0));
            L->off_dev = static_cast<const int64_t *>(L->dev_off.p);
            L->bytes_h2d += (n + 1) * static_cast<int64_t>(sizeof(int64_t));
        }
        // staging slots are allocated by the first chunk that uses them (atlas_broadcast_chunk)
    } else {
        L->off_dev = L->g.row_offsets;
    }

    if (L->g.in_degree) {
        L->indeg = L->g.in_degree;
    } else {
        HIP_TRY(L->indeg_own.alloc(n1 * sizeof(int32_t)));
        const atlas_plan *pl = L->g.plan;
        if (pl && !pl->host && pl->n == n && pl->e == L->e && n > 0) {
            // the plan already has every destination's messages side by side: group sizes, no pass over the CSR
            int rc = atlas_plan_in_degree(pl, static_cast<int32_t *>(L->indeg_own.p), s);
            if (rc != ATLAS_OK) return rc;
            L->indeg = static_cast<const int32_t *>(L->indeg_own.p);
        } else {
            // an edge array in host memory is read over the link once, with one atomic per edge; in device
            // memory large graphs are counted bucket by bucket (scratch: two bytes per edge, kept until finish)
            const size_t sb = L->g.residency == ATLAS_RESIDENT_DEVICE ? in_degree_scratch_bytes(n, L->e) : 0;
            if (sb) HIP_TRY(L->indeg_scratch.alloc(sb));
            HIP_TRY(launch_in_degree(L->g.col_indices, L->e, static_cast<int32_t *>(L->indeg_own.p), n,
                                     L->indeg_scratch.p, sb, s));
            L->indeg = static_cast<const int32_t *>(L->indeg_own.p);
        }
    }
    if (d.model == ATLAS_MODEL_GAT) {
        // the attention sweeps assume one group per destination and chunk
        if (L->g.plan && L->g.plan->blocked) return ATLAS_E_BAD_DIMS;
        const size_t nh = n1 * d.heads;
        HIP_TRY(L->gat_el.alloc(nh * sizeof(float)));
        HIP_TRY(L->gat_er.alloc(nh * sizeof(float)));
        HIP_TRY(L->gat_mcur.alloc(nh * sizeof(int32_t)));
        HIP_TRY(L->gat_mnext.alloc(nh * sizeof(int32_t)));
        HIP_TRY(L->gat_l.alloc(nh * sizeof(float)));
        HIP_TRY(L->gat_wa.alloc(static_cast<size_t>(d.d_in) * 2 * d.heads * sizeof(float)));
        HIP_TRY(L->gat_z.alloc(static_cast<size_t>(std::min<int64_t>(d.max_chunk_sources, std::max<int64_t>(n, 1))) *
                               d.d_out * sizeof(float)));
        if (L->g.plan) {   // room for the logits of the largest planned chunk
            int64_t most = 1;
            for (const PlanChunk &c : L->g.plan->chunks) most = std::max(most, c.n_edges);
            HIP_TRY(L->gat_scores.alloc(static_cast<size_t>(most) * d.heads * sizeof(float)));
        }
        HIP_TRY(launch_fill_i32(static_cast<int32_t *>(L->gat_mcur.p), gat_encoded_neg_inf(), n * d.heads, s));
        HIP_TRY(launch_fill_i32(static_cast<int32_t *>(L->gat_mnext.p), gat_encoded_neg_inf(), n * d.heads, s));
        HIP_TRY(launch_fill_zero(L->gat_l.p, static_cast<size_t>(n) * d.heads * sizeof(float), s));
        HIP_TRY(launch_gat_fold_attention(w->W, w->attn_src, w->attn_dst, w->dtype, d.d_in,
                                          d.heads, d.d_out / d.heads, static_cast<float *>(L->gat_wa.p), s));
    }
    HIP_TRY(launch_init_pending(L->indeg, L->selfmsg, n, static_cast<int32_t *>(L->pending.p),
                                static_cast<int32_t *>(L->ready.p), L->ctr(), s));
    if (L->tf && d.model == ATLAS_MODEL_SAGE_MEAN) {
        // rows 0..d_in-1 of W multiply the own embedding, rows d_in.. the neighbour mean
        const char *w_neigh = static_cast<const char *>(w->W) +
                              static_cast<size_t>(d.d_in) * d.d_out * dtype_size(w->dtype);
        char *second = static_cast<char *>(L->packed_w2.p) + packed_weight_bytes(L->K, d.d_out, L->compute_dt);
        HIP_TRY(launch_pack_weights(w_neigh, w->dtype, L->K, d.d_out, L->compute_dt,
                                    L->packed_w2.p, s));
        HIP_TRY(launch_pack_weights(w->W, w->dtype, L->K, d.d_out, L->compute_dt, second, s));
    } else if (d.model != ATLAS_MODEL_SGC_HOP)
        HIP_TRY(launch_pack_weights(w->W, w->dtype, L->K, d.d_out, L->compute_dt,
                                    L->packed_w.p, s));
    if (w->bias && d.model != ATLAS_MODEL_SGC_HOP) {
        HIP_TRY(L->bias.alloc(d.d_out * sizeof(float)));
        HIP_TRY(launch_to_f32(w->bias, w->dtype, d.d_out, static_cast<float *>(L->bias.p), s));
    }
    return ATLAS_OK;
}


// PINNED_HOST graphs: the caller's embeddings are pinned host memory (staged per chunk) or device memory
// (a later layer reading the previous layer's output: read in place).  One kind per layer.
int note_emb_location(atlas_layer *L, const void *emb) {
    hipPointerAttribute_t attr{};
    int on_device = 0;
    if (hipPointerGetAttributes(&attr, emb) == hipSuccess) on_device = attr.type == hipMemoryTypeDevice ? 1 : 0;
    else (void)hipGetLastError();   // pageable memory is unknown to the runtime: host
    if (L->emb_on_device >= 0 && L->emb_on_device != on_device) return ATLAS_E_STATE;
    L->emb_on_device = on_device;
    return ATLAS_OK;
}

// Rows of a staging slot of the chunk loader, allocated at first use (every chunk fits the layer's largest).
int stage_emb_slot(atlas_layer *L, int slot) {
    if (L->stage_emb[slot].p) return ATLAS_OK;
    const size_t rows = static_cast<size_t>(std::min<int64_t>(L->dims.max_chunk_sources, std::max<int64_t>(L->n, 1)));
    HIP_TRY(L->stage_emb[slot].alloc(rows * L->dims.d_in * dtype_size(L->dims.in_dtype)));
    return ATLAS_OK;
}

// What atlas_broadcast_chunk knows about a chunk staged from pinned host memory.
struct StagedChunk {
    int slot = -1;            // staging slot of the ring (-1: DEVICE graph, nothing staged)
    int npieces = 1;          // a long planned chunk crosses the host link, and is pushed, in pieces
    int64_t piece_tiles = 0;  // 64-edge tiles per piece
    bool packed = false;      // its edge words travel in 3 bytes and are unpacked piece by piece
};

// S1, the chunk loader (Sec. 3.3): stage the chunk into HBM on the copy stream; the compute
// stream only waits for this chunk's event, so the copy of chunk k+1 (enqueued by the next call)
// overlaps the kernels of chunk k.  Fills the staged addresses into `a` (CSR slice) and `ga`
// (planned chunk).
int stage_pinned_chunk(atlas_layer *L, const atlas_plan *plan, const PlanChunk *pc, int64_t src_begin,
                       int64_t src_end, const void *emb, size_t emb_bytes, bool emb_dev, char *self_dst,
                       hipStream_t s, AggregateArgs &a, GroupedArgs &ga, StagedChunk &st) {
    const atlas_dims_t &d = L->dims;
    const int slot = st.slot = static_cast<int>(L->num_chunks % atlas_layer::kStageSlots);
    const int64_t e0 = L->g.row_offsets[src_begin], e1 = L->g.row_offsets[src_end];
    const bool packed = pc && plan->src_packed;
    const size_t col_bytes = pc ? stage_bytes_of(*pc, packed) : static_cast<size_t>(e1 - e0) * sizeof(int32_t);
    if (!L->stage_col[slot].p || col_bytes > L->stage_col[slot].bytes) {
        // first use of the slot, or a chunk larger than those it has held: wait for the slot, then grow it
        if (L->slot_used[slot]) HIP_TRY(hipEventSynchronize(L->slot_free[slot]));
        Buf bigger;
        HIP_TRY(bigger.alloc(col_bytes));
        L->stage_col[slot].release();
        L->stage_col[slot] = bigger;
    }
    if (L->slot_used[slot]) HIP_TRY(hipStreamWaitEvent(L->copy_stream, L->slot_free[slot], 0));
    int rc = start_span(L, L->t_copy, L->copy_stream);
    if (rc != ATLAS_OK) return rc;
    const void *emb_dst = emb;   // device-resident embeddings are read where they are
    if (!emb_dev) {
        if (!self_dst && (rc = stage_emb_slot(L, slot)) != ATLAS_OK) return rc;
        void *stage = self_dst ? static_cast<void *>(self_dst) : L->stage_emb[slot].p;
        HIP_TRY(hipMemcpyAsync(stage, emb, emb_bytes, hipMemcpyHostToDevice, L->copy_stream));
        emb_dst = stage;
    }
    size_t staged_bytes = 0;
    if (pc) {
        // planned chunk: its regrouped edges travel instead of the CSR slice (3 or 4 bytes per edge)
        char *base = static_cast<char *>(L->stage_col[slot].p);
        const size_t sb = packed ? packed24_bytes(pc->n_edges) : static_cast<size_t>(pc->n_edges) * 4,
                     gb = static_cast<size_t>(pc->n_groups) * 4, tb = static_cast<size_t>((pc->n_edges + 63) / 64) * 4;
        char *g_dev = base + round_up(sb, 256), *t_dev = g_dev + round_up(gb, 256);
        if (sb) {
            const char *words = packed ? reinterpret_cast<const char *>(plan->src_packed + pc->packed_off)
                                       : reinterpret_cast<const char *>(plan->src_sorted + pc->edge_base);
            // the group arrays first: every piece needs them
            HIP_TRY(hipMemcpyAsync(g_dev, pc->grp_dst, gb, hipMemcpyHostToDevice, L->copy_stream));
            HIP_TRY(hipMemcpyAsync(t_dev, pc->tile_grp, tb, hipMemcpyHostToDevice, L->copy_stream));
            const int64_t ntiles = (pc->n_edges + 63) / 64;
            // (a GAT chunk is pushed in one piece: its maximum sweep reads all of the chunk's edges first)
            if (ntiles >= 2 * st.piece_tiles && d.model != ATLAS_MODEL_GAT)
                st.npieces = static_cast<int>((ntiles + st.piece_tiles - 1) / st.piece_tiles);
            auto &evs = L->piece_ev[slot];
            while (static_cast<int>(evs.size()) < st.npieces) {
                hipEvent_t ev = nullptr;
                HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
                evs.push_back(ev);
            }
            const size_t tile_bytes = packed ? 192 : 256;   // 64 words of 3 or 4 bytes
            for (int p = 0; p < st.npieces; ++p) {
                const size_t lo = static_cast<size_t>(p) * st.piece_tiles * tile_bytes;
                const size_t hi = p + 1 < st.npieces ? lo + st.piece_tiles * tile_bytes : sb;
                HIP_TRY(hipMemcpyAsync(base + lo, words + lo, hi - lo, hipMemcpyHostToDevice, L->copy_stream));
                HIP_TRY(hipEventRecord(evs[p], L->copy_stream));
            }
        }
        ga.src_sorted = reinterpret_cast<const int32_t *>(base);
        ga.grp_dst = reinterpret_cast<const int32_t *>(g_dev);
        ga.tile_grp = reinterpret_cast<const int32_t *>(t_dev);
        staged_bytes = sb + gb + tb;
    } else if (col_bytes) {
        HIP_TRY(hipMemcpyAsync(L->stage_col[slot].p, L->g.col_indices + e0, col_bytes, hipMemcpyHostToDevice,
                               L->copy_stream));
        staged_bytes = col_bytes;
    }
    rc = end_span(L, L->t_copy, L->copy_stream);
    if (rc != ATLAS_OK) return rc;
    HIP_TRY(hipEventRecord(L->slot_loaded[slot], L->copy_stream));
    // the compute stream goes on when the rows, the group arrays and the first piece are there
    HIP_TRY(hipStreamWaitEvent(s, st.npieces > 1 ? L->piece_ev[slot][0] : L->slot_loaded[slot], 0));
    if (packed && pc->n_edges > 0) {
        // 24-bit words as they came over the link -> the 32-bit words the kernels read (piece by piece, below)
        const size_t need = static_cast<size_t>((pc->n_edges + 3) / 4) * 16;
        if (!L->unpacked.p || L->unpacked.bytes < need) {
            HIP_TRY(hipStreamSynchronize(s));   // the previous chunk's kernels may still read the old buffer
            L->unpacked.release();
            HIP_TRY(L->unpacked.alloc(need));
        }
        st.packed = true;
        ga.src_sorted = static_cast<const int32_t *>(L->unpacked.p);
        if (st.npieces == 1)
            HIP_TRY(launch_unpack24(static_cast<const char *>(L->stage_col[slot].p), pc->n_edges, src_begin,
                                    static_cast<int32_t *>(L->unpacked.p), s));
    }
    L->bytes_h2d += static_cast<int64_t>((emb_dev ? 0 : emb_bytes) + staged_bytes);
    a.col = static_cast<const int32_t *>(L->stage_col[slot].p);
    a.col_base = e0;
    a.emb = emb_dst;
    return ATLAS_OK;
}

// Transform-first layers: multiply the chunk's rows by W on the matrix cores; the products are
// what is pushed (`a` is pointed at them).
int transform_chunk_first(atlas_layer *L, int64_t src_begin, int64_t src_end, hipStream_t s, AggregateArgs &a) {
    const atlas_dims_t &d = L->dims;
    int rc = start_span(L, L->t_self, s);
    if (rc != ATLAS_OK) return rc;
    UpdateArgs u{};
    u.model = 4;
    u.d_in = d.d_in;
    u.d_out = d.d_out;
    u.K = L->K;
    u.in_dt = d.in_dtype;
    u.compute_dt = L->compute_dt;
    u.self_rows = a.emb;
    u.counters = L->ctr();
    u.n = src_end - src_begin;
    u.identity_rows = src_end - src_begin;
    float *self_rows_out = L->tf_self.p ? static_cast<float *>(L->tf_self.p) + static_cast<size_t>(src_begin) * d.d_out
                                        : nullptr;
    // The products that are pushed are messages: they travel in the storage type of the embeddings
    // (half the bytes per edge for 16-bit storage).  A vertex's own product is read once and stays
    // fp32; GIN pushes that same buffer.
    const int push_dt = d.model == ATLAS_MODEL_GIN ? 0 : d.in_dtype;
    if (d.model == ATLAS_MODEL_SAGE_MEAN) {
        const size_t half = packed_weight_bytes(L->K, d.d_out, L->compute_dt);
        if (d.d_out % 32 == 0 && 2 * d.d_out <= 256) {
            // one pass over the rows: [x W_neigh | x W_self], the halves go to the two buffers
            u.packed_w = L->packed_w2.p;
            u.d_out = 2 * d.d_out;
            u.split = d.d_out;
            u.out = L->tf_z.p;
            u.out_dt = push_dt;
            u.out2 = self_rows_out;
            u.out2_dt = 0;
            HIP_TRY(launch_update(u, s));
        } else {
            u.packed_w = L->packed_w2.p;
            u.out = L->tf_z.p;
            u.out_dt = push_dt;
            HIP_TRY(launch_update(u, s));
            u.packed_w = static_cast<char *>(L->packed_w2.p) + half;
            u.out = self_rows_out;
            u.out_dt = 0;
            HIP_TRY(launch_update(u, s));
        }
    } else {
        u.packed_w = L->packed_w.p;
        u.out = d.model == ATLAS_MODEL_GIN ? static_cast<void *>(self_rows_out) : L->tf_z.p;
        u.out_dt = push_dt;
        HIP_TRY(launch_update(u, s));
    }
    if ((rc = end_span(L, L->t_self, s)) != ATLAS_OK) return rc;
    a.emb = d.model == ATLAS_MODEL_GIN ? static_cast<const void *>(self_rows_out) : L->tf_z.p;
    a.d = d.d_out;
    a.in_dt = push_dt;
    return ATLAS_OK;
}

// Bounded accumulator store (Sec. 3.5): every vertex this chunk addresses gets a slot before the
// chunk is pushed; the counts come back to the host, which sizes the eviction and checks that
// the chunk fits.
int make_room_for_chunk(atlas_layer *L, const PlanChunk *pc, int64_t src_begin, int64_t src_end, hipStream_t s,
                        const AggregateArgs &a, GroupedArgs &ga) {
    const atlas_dims_t &d = L->dims;
    const int32_t stamp = static_cast<int32_t>(L->num_chunks + 1);
    HIP_TRY(hot_mark(L->hs, ga.grp_dst, 0x7fffffff & ~ga.multi_bit, pc->n_groups, src_begin, L->selfmsg ? src_end - src_begin : 0, stamp, s));
    int32_t hc[HS_COUNT];
    HIP_TRY(hipMemcpyAsync(hc, L->hs.ctr, sizeof(hc), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (hc[HS_OVERFLOW]) return ATLAS_E_NOMEM;
    const int64_t need = hc[HS_NEED], free_slots = hc[HS_FREE_TOP];
    if (need > free_slots) {
        const int64_t n_evict = need - free_slots;
        HIP_TRY(hot_build_keys(L->hs, a.pending, stamp, d.evict_policy, s));
        HIP_TRY(hipMemcpyAsync(hc, L->hs.ctr, sizeof(hc), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        if (hc[HS_CANDIDATES] < n_evict) return ATLAS_E_NOMEM;   // the chunk's destinations do not fit the slots
        HIP_TRY(hot_evict(L->hs, n_evict, L->hs_sort_temp.p, L->hs_sort_temp.bytes, s));
        L->hot_evictions += n_evict;
    }
    HIP_TRY(hot_assign(L->hs, need, s));
    ga.slot_of = L->hs.slot_of;
    return ATLAS_OK;
}

// A chunk of at least this many edges that has no planned chunk is regrouped on the fly.
constexpr int64_t kRegroupMinEdges = int64_t(1) << 20;

// Regroup the edges [e0, e1) of sources [src_begin, src_end) by destination, as a plan would have
// (Sec. 3.3: the chunk is what is streamed; only the order in which its edges are visited changes).
// `col` is addressed by global edge number.  Synchronous: the construction sorts on the default stream,
// and the arrays of the chunk regrouped before this one are released first, so the layer's stream is
// drained before and the result is complete after.
int regroup_chunk(atlas_layer *L, int64_t src_begin, int64_t src_end, int64_t e0, int64_t e1, const int32_t *col,
                  hipStream_t s) {
    const auto t0 = std::chrono::steady_clock::now();
    HIP_TRY(hipStreamSynchronize(s));
    if (L->copy_stream) HIP_TRY(hipStreamSynchronize(L->copy_stream));
    L->free_regrouped();
    if (!L->regroup_work) {
        L->regroup_work = take_regroup_work();
        if (!L->regroup_work) L->regroup_work = new (std::nothrow) PlanWork();
        if (!L->regroup_work) return ATLAS_E_NOMEM;
    }
    const size_t words = static_cast<size_t>(e1 - e0) * sizeof(int32_t);
    if (!L->regroup_src.p || L->regroup_src.bytes < words) {
        L->regroup_src.release();
        HIP_TRY(L->regroup_src.alloc(words));
    }
    HIP_TRY(build_plan_chunk(L->off_dev, col, L->n, src_begin, src_end, e0, e1, static_cast<int32_t *>(L->regroup_src.p),
                             nullptr, 0, 0, false, *L->regroup_work, &L->cur_regroup));
    L->ms_regroup += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    return ATLAS_OK;
}

GatState gat_state(atlas_layer *L) {
    GatState g;
    g.el = static_cast<const float *>(L->gat_el.p);
    g.er = static_cast<const float *>(L->gat_er.p);
    g.m_cur = static_cast<int32_t *>(L->gat_mcur.p);
    g.m_next = static_cast<int32_t *>(L->gat_mnext.p);
    g.l = static_cast<float *>(L->gat_l.p);
    g.heads = L->dims.heads;
    g.dh = L->dims.d_out / L->dims.heads;
    g.slope = L->dims.neg_slope;
    return g;
}

}  // namespace

extern "C" {

int atlas_layer_init(const atlas_graph_t *graph, const atlas_dims_t *dims, const atlas_weights_t *weights,
                     void *hip_stream, atlas_layer_t **out) {
    if (!graph || !dims || !weights || !out) return ATLAS_E_NULL;
    if (graph->num_vertices < 0 || graph->num_edges < 0) return ATLAS_E_RANGE;
    if (graph->num_vertices >= (int64_t(1) << 31)) return ATLAS_E_OVERFLOW;
    if (!graph->row_offsets || (graph->num_edges > 0 && !graph->col_indices)) return ATLAS_E_NULL;
    if (graph->residency != ATLAS_RESIDENT_DEVICE && graph->residency != ATLAS_RESIDENT_PINNED_HOST)
        return ATLAS_E_BAD_DIMS;
    int rc = check_dims(*dims, *weights);
    if (rc != ATLAS_OK) return rc;

    atlas_layer *L = new (std::nothrow) atlas_layer();
    if (!L) return ATLAS_E_NOMEM;
    L->g = *graph;
    L->dims = *dims;
    L->n = graph->num_vertices;
    L->e = graph->num_edges;
    L->selfmsg = has_self_term(dims->model) ? 1 : 0;
    L->tf = transform_first(*dims);
    L->K = dims->model == ATLAS_MODEL_SAGE_MEAN && !L->tf ? 2 * dims->d_in : dims->d_in;
    L->compute_dt = dims->in_dtype;
    L->acc_width = dims->model == ATLAS_MODEL_GAT || L->tf ? dims->d_out : dims->d_in;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    L->last_stream = s;
    rc = start_span(L, L->t_init, s);
    if (rc == ATLAS_OK) rc = init_impl(L, weights, s);
    if (rc == ATLAS_OK) rc = end_span(L, L->t_init, s);
    if (rc != ATLAS_OK) {
        (void)hipStreamSynchronize(s);
        L->destroy();
        delete L;
        return rc;
    }
    *out = L;
    return ATLAS_OK;
}

int atlas_attention_prepass(atlas_layer_t *L, int64_t src_begin, int64_t src_end, const void *emb,
                            void *hip_stream) {
    if (!L || !emb) return ATLAS_E_NULL;
    if (L->dims.model != ATLAS_MODEL_GAT || L->next_src != 0) return ATLAS_E_STATE;
    if (src_begin < 0 || src_end > L->n || src_begin >= src_end ||
        src_end - src_begin > L->dims.max_chunk_sources)
        return ATLAS_E_RANGE;
    if (src_begin != L->prepass_next) return ATLAS_E_ORDER;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    L->last_stream = s;
    const void *rows = emb;
    int slot = -1;
    if (L->g.residency == ATLAS_RESIDENT_PINNED_HOST) {
        int rc = note_emb_location(L, emb);
        if (rc != ATLAS_OK) return rc;
        if (!L->emb_on_device) {
            // host rows cross the link here and once more when their chunk is broadcast: the attention
            // terms of all vertices must exist before the first message (Sec. 3.9)
            slot = static_cast<int>(L->num_prepass % atlas_layer::kStageSlots);
            if ((rc = stage_emb_slot(L, slot)) != ATLAS_OK) return rc;
            if (L->slot_used[slot]) HIP_TRY(hipStreamWaitEvent(L->copy_stream, L->slot_free[slot], 0));
            const size_t bytes = static_cast<size_t>(src_end - src_begin) * L->dims.d_in * dtype_size(L->dims.in_dtype);
            if ((rc = start_span(L, L->t_copy, L->copy_stream)) != ATLAS_OK) return rc;
            HIP_TRY(hipMemcpyAsync(L->stage_emb[slot].p, emb, bytes, hipMemcpyHostToDevice, L->copy_stream));
            if ((rc = end_span(L, L->t_copy, L->copy_stream)) != ATLAS_OK) return rc;
            HIP_TRY(hipEventRecord(L->slot_loaded[slot], L->copy_stream));
            HIP_TRY(hipStreamWaitEvent(s, L->slot_loaded[slot], 0));
            L->bytes_h2d += static_cast<int64_t>(bytes);
            rows = L->stage_emb[slot].p;
        }
    }
    HIP_TRY(launch_gat_prepass(rows, L->dims.in_dtype, src_begin, src_end, L->dims.d_in, static_cast<const float *>(L->gat_wa.p),
                               L->dims.heads, static_cast<float *>(L->gat_el.p), static_cast<float *>(L->gat_er.p), s));
    if (slot >= 0) {
        HIP_TRY(hipEventRecord(L->slot_free[slot], s));
        L->slot_used[slot] = true;
    }
    L->num_prepass += 1;
    L->prepass_next = src_end;
    return ATLAS_OK;
}

int atlas_broadcast_chunk(atlas_layer_t *L, int64_t src_begin, int64_t src_end, const void *emb,
                          void *hip_stream) {
    if (!L || !emb) return ATLAS_E_NULL;
    if (src_begin < 0 || src_end > L->n || src_begin >= src_end ||
        src_end - src_begin > L->dims.max_chunk_sources)
        return ATLAS_E_RANGE;
    if (src_begin != L->next_src) return ATLAS_E_ORDER;
    // GAT: a destination's attention term must exist before its first message
    if (L->dims.model == ATLAS_MODEL_GAT && L->prepass_next != L->n) return ATLAS_E_STATE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    L->last_stream = s;
    const atlas_dims_t &d = L->dims;
    const size_t row_bytes = static_cast<size_t>(d.d_in) * dtype_size(d.in_dtype);
    const size_t emb_bytes = static_cast<size_t>(src_end - src_begin) * row_bytes;

    AggregateArgs a{};
    a.off = L->off_dev;
    a.src_begin = src_begin;
    a.src_end = src_end;
    a.d = d.d_in;
    a.in_dt = d.in_dtype;
    a.model = aggregate_kind(d.model);
    a.acc = static_cast<float *>(L->acc.p);
    a.pending = static_cast<int32_t *>(L->pending.p);
    a.indeg = L->indeg;
    a.ready = static_cast<int32_t *>(L->ready.p);
    a.counters = L->ctr();
    a.counters64 = static_cast<unsigned long long *>(L->counters64.p);

    if (L->g.residency == ATLAS_RESIDENT_PINNED_HOST) {
        // where the caller keeps this layer's embeddings: pinned host memory (staged per chunk) or device
        // memory (a later layer reading the previous layer's output; read in place)
        int rc = note_emb_location(L, emb);
        if (rc != ATLAS_OK) return rc;
        if (L->emb_resident && !L->emb_on_device) {
            // host embeddings cannot be read in place: keep a copy of the own rows after all
            L->emb_resident = false;
            const size_t n1 = static_cast<size_t>(std::max<int64_t>(L->n, 1));
            HIP_TRY(L->self_rows.alloc(n1 * d.d_in * dtype_size(d.in_dtype)));
        }
    }
    const bool emb_dev = L->g.residency == ATLAS_RESIDENT_DEVICE || L->emb_on_device == 1;
    if (L->emb_resident) {
        const char *base = static_cast<const char *>(emb) - static_cast<size_t>(src_begin) * row_bytes;
        if (L->x_base && base != L->x_base) return ATLAS_E_STATE;
        L->x_base = base;
    }
    char *self_dst = has_self_term(d.model) && !L->emb_resident && !L->tf
                         ? static_cast<char *>(L->self_rows.p) + static_cast<size_t>(src_begin) * row_bytes
                         : nullptr;
    // a chunk that coincides with a planned chunk runs from its destination-ordered edges
    const atlas_plan *plan = L->g.plan;
    if (plan && plan->host != (L->g.residency == ATLAS_RESIDENT_PINNED_HOST)) plan = nullptr;
    const PlanChunk *pc = nullptr;
    if (plan && plan->chunk > 0 && src_begin % plan->chunk == 0 &&
        src_end == std::min(L->n, src_begin + plan->chunk))
        pc = &plan->chunks[static_cast<size_t>(src_begin / plan->chunk)];
    if (L->planned_only && !pc) return ATLAS_E_RANGE;  // the layer promised planned chunks only
    GroupedArgs ga{};

    // A long planned chunk crosses the host link in pieces, and each piece is pushed as soon as it has
    // arrived, so the chunk's copy and its kernels overlap (the first chunk of a degree-ordered graph
    // holds most of the edges).
    StagedChunk st;
    st.piece_tiles = d.piece_tiles > 0 ? d.piece_tiles : kDefaultPieceTiles;
    if (L->g.residency == ATLAS_RESIDENT_PINNED_HOST) {
        int rc = stage_pinned_chunk(L, plan, pc, src_begin, src_end, emb, emb_bytes, emb_dev, self_dst, s, a, ga, st);
        if (rc != ATLAS_OK) return rc;
    } else {
        a.col = L->g.col_indices;
        a.col_base = 0;
        a.emb = emb;
    }

    int rc = ATLAS_OK;
    bool regrouped = false;
    if (!pc && !(d.flags & ATLAS_FLAG_CSR_STREAM) && L->n > 0 &&
        static_cast<double>(src_end - src_begin) * (static_cast<double>(L->e) / static_cast<double>(L->n)) >=
            static_cast<double>(kRegroupMinEdges)) {
        // long enough on the graph's average: look at the chunk's real edge count
        int64_t eb[2] = {0, 0};
        if (L->g.residency == ATLAS_RESIDENT_PINNED_HOST) {
            eb[0] = L->g.row_offsets[src_begin];
            eb[1] = L->g.row_offsets[src_end];
        } else {
            HIP_TRY(hipMemcpy(&eb[0], L->g.row_offsets + src_begin, sizeof(int64_t), hipMemcpyDeviceToHost));
            HIP_TRY(hipMemcpy(&eb[1], L->g.row_offsets + src_end, sizeof(int64_t), hipMemcpyDeviceToHost));
        }
        if (eb[1] - eb[0] >= kRegroupMinEdges && eb[1] - eb[0] < (int64_t(1) << 32)) {
            if ((rc = regroup_chunk(L, src_begin, src_end, eb[0], eb[1], a.col - a.col_base, s)) != ATLAS_OK) return rc;
            pc = &L->cur_regroup;
            regrouped = true;
        }
    }
    if (L->selfmsg) {
        if ((rc = start_span(L, L->t_self, s)) != ATLAS_OK) return rc;
        if (self_dst && emb_dev)
            HIP_TRY(hipMemcpyAsync(self_dst, emb, emb_bytes, hipMemcpyDeviceToDevice, s));
        HIP_TRY(launch_self_message(src_begin, src_end, a.pending, a.ready, a.counters, s));
        if ((rc = end_span(L, L->t_self, s)) != ATLAS_OK) return rc;
    }
    if (L->tf && (rc = transform_chunk_first(L, src_begin, src_end, s, a)) != ATLAS_OK) return rc;
    if (d.model == ATLAS_MODEL_GAT) {
        // transform the chunk (z = x W on the matrix cores), raise the running
        // maxima with the chunk's logits, move the touched destinations to them
        if ((rc = start_span(L, L->t_self, s)) != ATLAS_OK) return rc;
        UpdateArgs u{};
        u.d_in = d.d_in;
        u.d_out = d.d_out;
        u.K = L->K;
        if (d.in_dtype == ATLAS_DTYPE_F32) {
            u.model = 2;                       // plain fp32 rows
            u.acc = static_cast<const float *>(a.emb);
        } else {
            u.model = 4;                       // plain rows in the 16-bit storage type, 16-bit matrix instructions
            u.self_rows = a.emb;
            u.in_dt = d.in_dtype;
            u.compute_dt = L->compute_dt;
        }
        u.counters = L->ctr();
        u.packed_w = L->packed_w.p;
        u.out = L->gat_z.p;
        u.n = src_end - src_begin;
        u.identity_rows = src_end - src_begin;
        HIP_TRY(launch_update(u, s));
        a.gat = gat_state(L);
        a.emb = L->gat_z.p;
        a.d = d.d_out;
        a.in_dt = 0;
    }
    if (pc) {
        if (regrouped) {
            ga.src_sorted = static_cast<const int32_t *>(L->regroup_src.p);
            ga.grp_dst = pc->grp_dst;
            ga.tile_grp = pc->tile_grp;
        } else if (!plan->host) {
            ga.src_sorted = plan->src_sorted + pc->edge_base;
            ga.grp_dst = pc->grp_dst;
            ga.tile_grp = pc->tile_grp;
        }
        ga.n_edges = pc->n_edges;
        ga.n_groups = pc->n_groups;
        ga.multi_bit = pc->blocked ? 0x40000000 : 0;
        ga.emb = a.emb;
        ga.gat = a.gat;
        ga.src_begin = src_begin;
        ga.d = a.d;
        ga.in_dt = a.in_dt;
        ga.model = a.model;
        ga.acc = a.acc;
        ga.pending = a.pending;
        ga.indeg = a.indeg;
        ga.ready = a.ready;
        ga.counters = a.counters;
        ga.counters64 = a.counters64;
        ga.forced_run = d.tiles_per_run;
        ga.handover = L->handover ? 1 : 0;
        ga.handover_dt = d.in_dtype;
        ga.handover_norm = d.model == ATLAS_MODEL_GCN_SYM ? 1 : 0;
        ga.handover_self = L->handover && L->selfmsg ? 1 : 0;
        ga.self_from = src_end;
    }
    if (d.model == ATLAS_MODEL_GAT) {
        if (pc) {
            // logits of the chunk's edges, kept between the max sweep and the aggregation
            const size_t need = static_cast<size_t>(std::max<int64_t>(pc->n_edges, 1)) * d.heads * sizeof(float);
            if (L->gat_scores.bytes < need) {
                HIP_TRY(hipStreamSynchronize(s));   // the previous chunk may still read the old buffer
                L->gat_scores.release();
                HIP_TRY(L->gat_scores.alloc(need));
            }
            ga.scores = static_cast<float *>(L->gat_scores.p);
            HIP_TRY(launch_gat_group_max(ga, s));
            HIP_TRY(launch_gat_rescale_cut_groups(ga, s));   // other groups: rescaled by the aggregation
        } else {
            HIP_TRY(launch_gat_chunk_max(a, s));
            HIP_TRY(launch_gat_rescale(a.gat, a.acc, d.d_out, L->n, s));
        }
        if ((rc = end_span(L, L->t_self, s)) != ATLAS_OK) return rc;
    }
    if (L->bounded && (rc = make_room_for_chunk(L, pc, src_begin, src_end, s, a, ga)) != ATLAS_OK) return rc;
    if (pc && !regrouped && src_begin == 0 && plan->dense.n_items > 0) {
        if ((rc = start_span(L, L->t_dense, s)) != ATLAS_OK) return rc;
        // the first chunk's dense part goes first: as a contraction on the matrix cores where the kernel
        // serves the rows' width and type, else as the planned chunk the plan keeps of the same edges
        const DensePart &dp = plan->dense;
        if (!(d.flags & ATLAS_FLAG_NO_DENSE) && a.model == 0 && dense_contract_takes(a.d, a.in_dt)) {
            const size_t need = dense_packed_rows_bytes(dp, a.d);
            if (L->dense_rows.bytes < need) {
                L->dense_rows.release();
                HIP_TRY(L->dense_rows.alloc(need));
            }
            HIP_TRY(launch_dense_prepare(dp, a.emb, src_end - src_begin, a.d, a.in_dt, L->dense_rows.p, a.acc, L->n, s));
            if ((rc = start_span(L, L->t_contract, s)) != ATLAS_OK) return rc;
            HIP_TRY(launch_dense_contract(dp, a.d, a.in_dt, L->dense_rows.p, a.acc, L->n, s));
            if ((rc = end_span(L, L->t_contract, s)) != ATLAS_OK) return rc;
            HIP_TRY(launch_dense_pending(dp, L->n, a.pending, a.ready, a.counters, a.counters64, s));
            L->edges_contracted += dp.list.n_edges;
        } else {
            GroupedArgs gd = ga;
            gd.src_sorted = dp.list_src ? dp.list_src : plan->src_sorted + dp.list.edge_base;
            gd.grp_dst = dp.list.grp_dst;
            gd.tile_grp = dp.list.tile_grp;
            gd.n_edges = dp.list.n_edges;
            gd.n_groups = dp.list.n_groups;
            gd.multi_bit = 0;
            if (gd.n_edges > 0) HIP_TRY(plan_runs(gd));
            if (L->planned_only)
                HIP_TRY(launch_zero_rows(dp.list.zero_rows, dp.list.zero_span, dp.list.n_zero_rows, gd.acc, gd.slot_of,
                                         gd.d, &gd, s));
            HIP_TRY(launch_aggregate_grouped(gd, &L->run_tickets, s));
        }
        if ((rc = end_span(L, L->t_dense, s)) != ATLAS_OK) return rc;
    }
    if ((rc = start_span(L, L->t_agg, s)) != ATLAS_OK) return rc;
    if (pc) {
        for (int p = 0; p < st.npieces; ++p) {
            if (st.npieces > 1) {
                if (p > 0) HIP_TRY(hipStreamWaitEvent(s, L->piece_ev[st.slot][p], 0));
                ga.tile_begin = p * st.piece_tiles;
                ga.tile_end = p + 1 < st.npieces ? (p + 1) * st.piece_tiles : -1;
            }
            if (st.packed && st.npieces > 1) {
                const int64_t e_lo = ga.tile_begin * 64;
                const int64_t e_hi = ga.tile_end < 0 ? pc->n_edges : std::min<int64_t>(pc->n_edges, ga.tile_end * 64);
                HIP_TRY(launch_unpack24(static_cast<const char *>(L->stage_col[st.slot].p) + e_lo * 3, e_hi - e_lo, src_begin,
                                        static_cast<int32_t *>(L->unpacked.p) + e_lo, s));
            }
            // a chunk pushed in one launch: its runs are chosen here, so that the rows of groups that stay
            // within one run need not be cleared
            if (st.npieces == 1 && ga.n_edges > 0) HIP_TRY(plan_runs(ga));
            // the list (device memory, also in plans of pinned-host graphs) covers the whole chunk: cleared
            // once, before the first piece adds anything
            if (L->planned_only && p == 0)
                HIP_TRY(launch_zero_rows(pc->zero_rows, pc->zero_span, pc->n_zero_rows, ga.acc, ga.slot_of, ga.d,
                                         st.npieces == 1 ? &ga : nullptr, s));
            HIP_TRY(launch_aggregate_grouped(ga, &L->run_tickets, s));
        }
    } else {
        HIP_TRY(launch_aggregate(a, s));
    }
    rc = end_span(L, L->t_agg, s);
    if (rc != ATLAS_OK) return rc;
    if (st.slot >= 0) {
        HIP_TRY(hipEventRecord(L->slot_free[st.slot], s));
        L->slot_used[st.slot] = true;
    }
    L->next_src = src_end;
    L->num_chunks += 1;
    (regrouped ? L->chunks_regrouped : pc ? L->chunks_planned : L->chunks_csr) += 1;
    return ATLAS_OK;
}

int atlas_flush_ready(atlas_layer_t *L, void *out, int64_t *n_flushed, void *hip_stream) {
    if (!L || !out) return ATLAS_E_NULL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    L->last_stream = s;
    const atlas_dims_t &d = L->dims;
    int32_t before[2] = {0, 0};
    if (n_flushed) {
        HIP_TRY(hipMemcpyAsync(before, L->ctr(), sizeof(before), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
    }
    UpdateArgs u{};
    u.model = d.model == ATLAS_MODEL_GIN ? 3 : d.model;
    u.self_scale = 1.0f + d.gin_eps;
    u.d_in = d.d_in;
    u.d_out = d.d_out;
    u.K = L->K;
    u.in_dt = d.in_dtype;
    u.out_dt = d.out_dtype;
    u.compute_dt = L->compute_dt;
    u.activation = d.activation;
    u.acc = static_cast<const float *>(L->acc.p);
    u.self_rows = L->emb_resident ? static_cast<const void *>(L->x_base) : L->self_rows.p;
    u.indeg = L->indeg;
    u.ready = static_cast<const int32_t *>(L->ready.p);
    u.counters = L->ctr();
    u.packed_w = L->packed_w.p;
    u.bias = static_cast<const float *>(L->bias.p);
    u.out = out;
    u.n = L->n;
    u.slot_of = L->bounded ? L->hs.slot_of : nullptr;
    u.handed_rows = L->handover ? 1 : 0;
    int rc = start_span(L, L->t_upd, s);
    if (rc != ATLAS_OK) return rc;
    if (d.model == ATLAS_MODEL_GAT) {
        GatFinalizeArgs f{};
        f.acc = u.acc;
        f.l = static_cast<const float *>(L->gat_l.p);
        f.ready = u.ready;
        f.counters = u.counters;
        f.bias = u.bias;
        f.out = out;
        f.d_out = d.d_out;
        f.heads = d.heads;
        f.dh = d.d_out / d.heads;
        f.activation = d.activation;
        f.out_dt = u.out_dt;
        f.n = L->n;
        HIP_TRY(launch_gat_finalize(f, s));
    } else if (L->tf) {
        SumFinalizeArgs f{};
        f.acc = u.acc;
        f.slot_of = u.slot_of;
        f.self_term = static_cast<const float *>(L->tf_self.p);
        f.self_scale = d.model == ATLAS_MODEL_GIN ? 1.0f + d.gin_eps : 1.0f;
        f.norm = d.model == ATLAS_MODEL_SAGE_MEAN ? 0 : (d.model == ATLAS_MODEL_GCN_SYM ? 1 : 2);
        f.indeg = u.indeg;
        f.ready = u.ready;
        f.counters = u.counters;
        f.bias = u.bias;
        f.out = out;
        f.d_out = d.d_out;
        f.activation = d.activation;
        f.out_dt = u.out_dt;
        f.n = L->n;
        HIP_TRY(launch_sum_finalize(f, s));
    } else if (d.model == ATLAS_MODEL_SGC_HOP) {
        HIP_TRY(launch_scale_rows(u, s));
    } else
    // SAGE / GIN rows become ready only after their own chunk: before the first
    // broadcast there is nothing to update (and no matrix to read own rows from)
    if (!(L->emb_resident && !L->x_base)) HIP_TRY(launch_update(u, s));
    if (L->bounded) HIP_TRY(hot_release(L->hs, u.ready, u.counters, L->n, s));   // flushed vertices give their slots back
    HIP_TRY(launch_advance_head(L->ctr(), s));
    rc = end_span(L, L->t_upd, s);
    if (rc != ATLAS_OK) return rc;
    L->num_flushes += 1;
    if (n_flushed) *n_flushed = static_cast<int64_t>(before[CTR_READY_TAIL]) - before[CTR_READY_HEAD];
    return ATLAS_OK;
}

int atlas_layer_finish(atlas_layer_t *L, atlas_layer_stats_t *stats) {
    if (!L) return ATLAS_E_NULL;
    int rc = ATLAS_OK;
    int32_t c[CTR_COUNT] = {0};
    unsigned long long c64[CTR64_COUNT] = {0};
    hipError_t e = hipStreamSynchronize(L->last_stream);
    if (e == hipSuccess && L->copy_stream) e = hipStreamSynchronize(L->copy_stream);
    if (e == hipSuccess) e = hipMemcpy(c, L->counters.p, sizeof(c), hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(c64, L->counters64.p, sizeof(c64), hipMemcpyDeviceToHost);
    if (e != hipSuccess) rc = hip_fail(e, "atlas_layer_finish");
    if (stats) {
        *stats = atlas_layer_stats_t{};
        stats->edges_processed = static_cast<int64_t>(c64[CTR64_EDGES]);
        stats->sources_processed = L->next_src;
        stats->vertices_completed = c[CTR_READY_TAIL];
        stats->vertices_flushed = c[CTR_READY_HEAD];
        stats->num_chunks = L->num_chunks;
        stats->num_flushes = L->num_flushes;
        stats->bytes_copied_h2d = L->bytes_h2d;
        stats->chunks_planned = L->chunks_planned;
        stats->chunks_csr_stream = L->chunks_csr;
        stats->chunks_regrouped = L->chunks_regrouped;
        stats->rows_handed_over = static_cast<int64_t>(c64[CTR64_HANDED]);
        stats->ms_regroup = static_cast<float>(L->ms_regroup);
        if (L->bounded) {
            int32_t hc[HS_COUNT] = {0};
            if (hipMemcpy(hc, L->hs.ctr, sizeof(hc), hipMemcpyDeviceToHost) == hipSuccess) {
                stats->hot_evictions = hc[HS_EVICTIONS];
                stats->hot_reloads = hc[HS_RELOADS];
                stats->hot_peak_slots = hc[HS_PEAK];
            }
        }
        if (rc == ATLAS_OK) {
            stats->edges_contracted = L->edges_contracted;
            stats->ms_aggregate = sum_spans(L->t_agg);
            stats->ms_dense = sum_spans(L->t_dense);
            stats->ms_contract = sum_spans(L->t_contract);
            stats->ms_self = sum_spans(L->t_self);
            stats->ms_init = sum_spans(L->t_init);
            stats->ms_update = sum_spans(L->t_upd);
            stats->ms_copy = sum_spans(L->t_copy);
        }
    }
    if (rc == ATLAS_OK &&
        (L->next_src != L->n || c[CTR_READY_TAIL] != L->n || c[CTR_READY_HEAD] != L->n ||
         static_cast<int64_t>(c64[CTR64_EDGES]) != L->e))
        rc = ATLAS_E_INCOMPLETE;
    L->destroy();
    delete L;
    return rc;
}

int atlas_plan_create(const atlas_graph_t *graph, int64_t chunk_sources, atlas_plan_t **out) {
    return atlas_plan_create_blocked(graph, chunk_sources, 0, 0, out);
}

int atlas_plan_create_blocked(const atlas_graph_t *graph, int64_t chunk_sources, int64_t block_sources,
                              int64_t hot_min_edges, atlas_plan_t **out) {
    return atlas_plan_create_dense(graph, chunk_sources, block_sources, hot_min_edges, 0, 0, out);
}

int atlas_plan_create_dense(const atlas_graph_t *graph, int64_t chunk_sources, int64_t block_sources,
                            int64_t hot_min_edges, int64_t dense_max_bytes, int64_t dense_cells_per_edge,
                            atlas_plan_t **out) {
    if (!graph || !out) return ATLAS_E_NULL;
    if (block_sources < 0 || hot_min_edges < 0 || dense_max_bytes < 0 || dense_cells_per_edge < 0)
        return ATLAS_E_BAD_DIMS;
    if (dense_max_bytes > 0 && dense_cells_per_edge == 0) dense_cells_per_edge = kDefaultDenseCellsPerEdge;
    // bit 30 of a stored destination id marks destinations with several groups per chunk
    if (block_sources > 0 && graph->num_vertices >= (int64_t(1) << 30)) return ATLAS_E_OVERFLOW;
    if (!graph->row_offsets || (graph->num_edges > 0 && !graph->col_indices)) return ATLAS_E_NULL;
    if (chunk_sources <= 0) return ATLAS_E_BAD_DIMS;
    if (graph->residency != ATLAS_RESIDENT_DEVICE && graph->residency != ATLAS_RESIDENT_PINNED_HOST)
        return ATLAS_E_BAD_DIMS;
    if (graph->num_vertices < 0 || graph->num_edges < 0) return ATLAS_E_RANGE;
    if (graph->num_vertices >= (int64_t(1) << 31)) return ATLAS_E_OVERFLOW;
    atlas_plan *P = new (std::nothrow) atlas_plan();
    if (!P) return ATLAS_E_NOMEM;
    P->n = graph->num_vertices;
    P->e = graph->num_edges;
    P->chunk = chunk_sources;
    P->host = graph->residency == ATLAS_RESIDENT_PINNED_HOST;
    const int64_t nchunks = (P->n + chunk_sources - 1) / chunk_sources;
    const size_t e_bytes = static_cast<size_t>(std::max<int64_t>(P->e, 1)) * sizeof(int32_t);
    int rc = ATLAS_OK;
    // a plan that is copied to the device in every layer keeps its edge words in 3 bytes
    const bool packed = P->host && chunk_sources <= (int64_t(1) << 23);
    hipError_t e = hipSuccess;
    if (packed) {
        // every chunk's words start on a 256-byte boundary
        P->packed_bytes = static_cast<size_t>(std::max<int64_t>(P->e, 1)) * 3 + static_cast<size_t>(nchunks + 1) * 268;
        e = hipHostMalloc(reinterpret_cast<void **>(&P->src_packed), P->packed_bytes, hipHostMallocDefault);
    } else {
        e = P->host ? hipHostMalloc(reinterpret_cast<void **>(&P->src_sorted), e_bytes, hipHostMallocDefault)
                    : hipMalloc(reinterpret_cast<void **>(&P->src_sorted), e_bytes);
    }
    if (e != hipSuccess) rc = hip_fail(e, "alloc(plan)");
    size_t packed_off = 0;

    auto offset_at = [&](int64_t u, int64_t *v) -> hipError_t {
        if (P->host) { *v = graph->row_offsets[u]; return hipSuccess; }
        return hipMemcpy(v, graph->row_offsets + u, sizeof(int64_t), hipMemcpyDeviceToHost);
    };
    uint8_t *seen = nullptr;  // first-touch map of the whole plan
    if (rc == ATLAS_OK) {
        const size_t nb = static_cast<size_t>(std::max<int64_t>(P->n, 1));
        if ((e = hipMalloc(reinterpret_cast<void **>(&seen), nb)) != hipSuccess ||
            (e = hipMemset(seen, 0, nb)) != hipSuccess)
            rc = hip_fail(e, "alloc(plan first-touch map)");
    }
    int64_t ebeg = 0;
    PlanWork work;   // freed when this function returns
    GrowBuf off_stage, col_stage, src_stage;   // host plans: the chunk's CSR slice and regrouped words in HBM
    if (rc == ATLAS_OK && nchunks > 0 && (e = offset_at(0, &ebeg)) != hipSuccess) rc = hip_fail(e, "row_offsets");
    for (int64_t k = 0; rc == ATLAS_OK && k < nchunks; ++k) {
        const int64_t b = k * chunk_sources, en = std::min(P->n, b + chunk_sources);
        int64_t eend = 0;
        if ((e = offset_at(en, &eend)) != hipSuccess) { rc = hip_fail(e, "row_offsets"); break; }
        const int64_t ne = eend - ebeg;
        PlanChunk pc;
        if (!P->host) {
            if (k == 0 && dense_max_bytes > 0)
                e = build_first_chunk_with_dense_part(graph->row_offsets, graph->col_indices, P->n, b, en, ebeg, eend,
                                                      P->src_sorted + ebeg, seen, block_sources, hot_min_edges, true,
                                                      static_cast<size_t>(dense_max_bytes), dense_cells_per_edge, work,
                                                      &pc, &P->dense);
            else
                e = build_plan_chunk(graph->row_offsets, graph->col_indices, P->n, b, en, ebeg, eend,
                                     P->src_sorted + ebeg, seen, block_sources, hot_min_edges, true, work, &pc);
            if (e != hipSuccess) { rc = hip_fail(e, "build_plan_chunk"); break; }
        } else {
            // stage the chunk's CSR slice into HBM, regroup there, bring the result back
            const size_t nsrc = static_cast<size_t>(en - b);
            const size_t ne1 = static_cast<size_t>(std::max<int64_t>(ne, 1));
            if ((e = off_stage.need((nsrc + 1) * sizeof(int64_t))) == hipSuccess &&
                (e = col_stage.need((ne1 + 3) * 4)) == hipSuccess &&   // also holds the packed words
                (e = src_stage.need(ne1 * 4)) == hipSuccess) {
                int64_t *off_tmp = static_cast<int64_t *>(off_stage.p);
                int32_t *col_tmp = static_cast<int32_t *>(col_stage.p), *src_tmp = static_cast<int32_t *>(src_stage.p);
                e = hipMemcpy(off_tmp, graph->row_offsets + b, (nsrc + 1) * sizeof(int64_t), hipMemcpyHostToDevice);
                if (e == hipSuccess && ne > 0)
                    e = hipMemcpy(col_tmp, graph->col_indices + ebeg, static_cast<size_t>(ne) * 4, hipMemcpyHostToDevice);
                if (e == hipSuccess && k == 0 && dense_max_bytes > 0) {
                    // The dense part stays in HBM (cells, and its edges as a planned chunk): it is the part of the
                    // topology that never crosses the host link again; the chunk's other edges go to host memory.
                    e = build_first_chunk_with_dense_part(off_tmp - b, col_tmp - ebeg, P->n, b, en, ebeg, eend, src_tmp, seen,
                                                          block_sources, hot_min_edges, true,
                                                          static_cast<size_t>(dense_max_bytes), dense_cells_per_edge, work,
                                                          &pc, &P->dense);
                    if (e == hipSuccess && P->dense.n_items > 0) {
                        const size_t lb = static_cast<size_t>(P->dense.list.n_edges) * 4;
                        if ((e = hipMalloc(reinterpret_cast<void **>(&P->dense.list_src), lb)) == hipSuccess)
                            e = hipMemcpy(P->dense.list_src, src_tmp + pc.n_edges, lb, hipMemcpyDeviceToDevice);
                    }
                } else if (e == hipSuccess) {
                    e = build_plan_chunk(off_tmp - b, col_tmp - ebeg, P->n, b, en, ebeg, eend, src_tmp, seen, block_sources,
                                         hot_min_edges, true, work, &pc);
                }
                const int64_t pe = pc.n_edges;   // the chunk's edges that go to host memory
                if (e == hipSuccess && pe > 0 && packed) {
                    // the CSR slice is no longer needed: its buffer takes the packed words
                    const size_t pb = packed24_bytes(pe);
                    pc.packed_off = static_cast<int64_t>(packed_off);
                    if (packed_off + pb > P->packed_bytes) e = hipErrorInvalidValue;
                    if (e == hipSuccess) e = launch_pack24(src_tmp, pe, b, col_tmp, nullptr);
                    if (e == hipSuccess) e = hipMemcpy(P->src_packed + packed_off, col_tmp, pb, hipMemcpyDeviceToHost);
                    packed_off += round_up(pb, 256);
                } else if (e == hipSuccess && pe > 0) {
                    e = hipMemcpy(P->src_sorted + ebeg, src_tmp, static_cast<size_t>(pe) * 4, hipMemcpyDeviceToHost);
                }
                if (e == hipSuccess && pe > 0) {
                    int32_t *g_h = nullptr, *t_h = nullptr;
                    const size_t gb = static_cast<size_t>(pc.n_groups) * 4, tb = static_cast<size_t>((pe + 63) / 64) * 4;
                    if ((e = hipHostMalloc(reinterpret_cast<void **>(&g_h), gb, hipHostMallocDefault)) == hipSuccess &&
                        (e = hipHostMalloc(reinterpret_cast<void **>(&t_h), tb, hipHostMallocDefault)) == hipSuccess &&
                        (e = hipMemcpy(g_h, pc.grp_dst, gb, hipMemcpyDeviceToHost)) == hipSuccess)
                        e = hipMemcpy(t_h, pc.tile_grp, tb, hipMemcpyDeviceToHost);
                    (void)hipFree(pc.grp_dst);
                    (void)hipFree(pc.tile_grp);
                    pc.grp_dst = g_h;
                    pc.tile_grp = t_h;
                }
            }
            if (e != hipSuccess) {
                P->chunks.push_back(pc);  // so that destroy releases what was allocated
                rc = hip_fail(e, "build_plan_chunk(host)");
                break;
            }
        }
        P->blocked = P->blocked || pc.blocked;
        P->chunks.push_back(pc);
        P->max_stage_bytes = std::max(P->max_stage_bytes, stage_bytes_of(pc, packed));
        ebeg = eend;
    }
    for (GrowBuf *gb : {&off_stage, &col_stage, &src_stage}) gb->release();
    if (rc == ATLAS_OK && seen && (e = count_nonzero_bytes(seen, P->n, &P->n_first)) != hipSuccess)
        rc = hip_fail(e, "plan first-touch count");
    if (seen) (void)hipFree(seen);
    if (rc == ATLAS_OK && P->host) {
        const size_t ob = (static_cast<size_t>(P->n) + 1) * sizeof(int64_t);
        if ((e = hipMalloc(reinterpret_cast<void **>(&P->dev_off), ob)) != hipSuccess ||
            (e = hipMemcpy(P->dev_off, graph->row_offsets, ob, hipMemcpyHostToDevice)) != hipSuccess)
            rc = hip_fail(e, "plan row offsets");
    }
    if (rc != ATLAS_OK) {
        atlas_plan_destroy(P);
        return rc;
    }
    *out = P;
    return ATLAS_OK;
}

int atlas_plan_destroy(atlas_plan_t *P) {
    if (!P) return ATLAS_E_NULL;
    (void)hipDeviceSynchronize();
    for (auto &c : P->chunks) {
        if (c.grp_dst) (void)(P->host ? hipHostFree(c.grp_dst) : hipFree(c.grp_dst));
        if (c.tile_grp) (void)(P->host ? hipHostFree(c.tile_grp) : hipFree(c.tile_grp));
        if (c.zero_rows) (void)hipFree(c.zero_rows);
        if (c.zero_span) (void)hipFree(c.zero_span);
    }
    if (P->src_sorted) (void)(P->host ? hipHostFree(P->src_sorted) : hipFree(P->src_sorted));
    if (P->src_packed) (void)hipHostFree(P->src_packed);
    if (P->dev_off) (void)hipFree(P->dev_off);
    P->dense.release();
    delete P;
    return ATLAS_OK;
}

int atlas_plan_info(const atlas_plan_t *P, atlas_plan_info_t *info) {
    if (!P || !info) return ATLAS_E_NULL;
    *info = atlas_plan_info_t{};
    info->num_chunks = static_cast<int64_t>(P->chunks.size());
    info->num_edges = P->e;
    info->num_first_groups = P->n_first;
    size_t dev = 0, host = 0;
    for (const PlanChunk &c : P->chunks) {
        info->num_groups += c.n_groups;
        const size_t arrays = static_cast<size_t>(c.n_groups) * 4 + static_cast<size_t>((c.n_edges + 63) / 64) * 4;
        (P->host ? host : dev) += arrays;
        dev += static_cast<size_t>(c.n_zero_rows) * 12;
    }
    if (P->dense.n_items > 0) {
        const PlanChunk &c = P->dense.list;
        info->num_groups += c.n_groups;
        dev += static_cast<size_t>(c.n_groups) * 4 + static_cast<size_t>((c.n_edges + 63) / 64) * 4 +
               static_cast<size_t>(c.n_zero_rows) * 12;
        dev += P->dense.cell_bytes + static_cast<size_t>(P->dense.rows) * 4 + static_cast<size_t>(P->dense.n_bands) * 12 +
               static_cast<size_t>(P->dense.n_items) * 12 + (P->dense.list_src ? static_cast<size_t>(c.n_edges) * 4 : 0);
        info->dense_edges = c.n_edges;
        info->dense_groups = c.n_groups;
        info->dense_cells = static_cast<int64_t>(P->dense.cell_bytes) * 2;   // half a byte each
        info->dense_rows = std::min(P->dense.rows, P->n);
        info->dense_max_sources = static_cast<int64_t>(P->dense.max_ksteps) * 64;
    }
    if (P->src_packed) host += P->packed_bytes;
    else (P->host ? host : dev) += static_cast<size_t>(P->e) * 4;
    if (P->dev_off) dev += (static_cast<size_t>(P->n) + 1) * sizeof(int64_t);
    info->bytes_device = static_cast<int64_t>(dev);
    info->bytes_pinned_host = static_cast<int64_t>(host);
    return ATLAS_OK;
}

int atlas_plan_in_degree(const atlas_plan_t *P, int32_t *in_degree, void *hip_stream) {
    if (!P || !in_degree) return ATLAS_E_NULL;
    if (P->host) return ATLAS_E_STATE;   // the plan's arrays are in host memory: count from the graph instead
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    HIP_TRY(launch_fill_zero(in_degree, static_cast<size_t>(P->n) * sizeof(int32_t), s));
    for (const PlanChunk &c : P->chunks)
        HIP_TRY(launch_plan_chunk_in_degree(c, P->src_sorted + c.edge_base, in_degree, s));
    if (P->dense.n_items > 0)
        HIP_TRY(launch_plan_chunk_in_degree(P->dense.list, P->dense.list_src ? P->dense.list_src
                                                                            : P->src_sorted + P->dense.list.edge_base,
                                            in_degree, s));
    return ATLAS_OK;
}

int atlas_probe_copy(void *dst, const void *src, int64_t bytes, void *hip_stream) {
    if (!dst || !src) return ATLAS_E_NULL;
    if (bytes < 0 || bytes % 16 != 0) return ATLAS_E_RANGE;
    HIP_TRY(probe_copy(dst, src, static_cast<size_t>(bytes), static_cast<hipStream_t>(hip_stream)));
    return ATLAS_OK;
}

int atlas_probe_mix21(void *dst, const void *a, const void *b, int64_t bytes, void *hip_stream) {
    if (!dst || !a || !b) return ATLAS_E_NULL;
    if (bytes < 0 || bytes % 16 != 0) return ATLAS_E_RANGE;
    HIP_TRY(probe_mix21(dst, a, b, static_cast<size_t>(bytes), static_cast<hipStream_t>(hip_stream)));
    return ATLAS_OK;
}

int atlas_probe_mfma(int32_t waves_per_simd, int32_t iters, void *sink, double *flops, void *hip_stream) {
    if (!sink || !flops) return ATLAS_E_NULL;
    if (waves_per_simd < 1 || waves_per_simd > 8 || iters < 1 || iters > (1 << 24)) return ATLAS_E_RANGE;
    HIP_TRY(probe_mfma(waves_per_simd, iters, sink, flops, static_cast<hipStream_t>(hip_stream)));
    return ATLAS_OK;
}

int64_t atlas_probe_gather_sink_bytes(void) { return static_cast<int64_t>(probe_gather_sink_bytes()); }

int atlas_probe_row_gather(const void *table, int64_t table_rows, const int32_t *ids, int64_t n_ids, void *sink,
                           void *hip_stream) {
    if (!table || !ids || !sink) return ATLAS_E_NULL;
    if (table_rows <= 0 || table_rows >= (int64_t(1) << 31) || n_ids < 0) return ATLAS_E_RANGE;
    HIP_TRY(probe_row_gather(table, ids, n_ids, sink, static_cast<hipStream_t>(hip_stream)));
    return ATLAS_OK;
}

int atlas_probe_dense_rows(int32_t dtype, const void *rows, int64_t n_rows, int32_t K, int32_t d_out, const void *W,
                           void *out, int32_t repeat, void *hip_stream) {
    if (!rows || !W || !out) return ATLAS_E_NULL;
    if (dtype != ATLAS_DTYPE_BF16 && dtype != ATLAS_DTYPE_F16) return ATLAS_E_BAD_DIMS;
    if (K <= 0 || K % 64 != 0 || K > 1024 || d_out <= 0 || d_out % 32 != 0 || d_out > 256) return ATLAS_E_BAD_DIMS;
    if (n_rows <= 0 || n_rows >= (int64_t(1) << 31) || repeat < 1) return ATLAS_E_RANGE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Buf packed, counters;
    HIP_TRY(packed.alloc(packed_weight_bytes(K, d_out, dtype)));
    hipError_t e = counters.alloc(CTR_COUNT * sizeof(int32_t));
    if (e == hipSuccess) e = launch_fill_zero(counters.p, counters.bytes, s);
    if (e == hipSuccess) e = launch_pack_weights(W, dtype, K, d_out, dtype, packed.p, s);
    UpdateArgs u{};
    u.model = 4;           // plain rows in the storage type
    u.d_in = K;
    u.d_out = d_out;
    u.K = K;
    u.in_dt = u.out_dt = u.compute_dt = dtype;
    u.self_rows = rows;
    u.counters = static_cast<int32_t *>(counters.p);
    u.packed_w = packed.p;
    u.out = out;
    u.n = n_rows;
    u.identity_rows = n_rows;
    for (int r = 0; e == hipSuccess && r < repeat; ++r) e = launch_update(u, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);   // the packed weights go back to the cache below
    packed.release();
    counters.release();
    if (e != hipSuccess) return hip_fail(e, "atlas_probe_dense_rows");
    return ATLAS_OK;
}

int atlas_in_degree(const atlas_graph_t *graph, int32_t *in_degree, void *hip_stream) {
    if (!graph || !in_degree) return ATLAS_E_NULL;
    if (graph->num_edges > 0 && !graph->col_indices) return ATLAS_E_NULL;
    if (graph->num_vertices < 0 || graph->num_edges < 0) return ATLAS_E_RANGE;
    if (graph->num_vertices >= (int64_t(1) << 31)) return ATLAS_E_OVERFLOW;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const size_t sb = graph->residency == ATLAS_RESIDENT_DEVICE
                          ? in_degree_scratch_bytes(graph->num_vertices, graph->num_edges) : 0;
    Buf scratch;
    if (sb) HIP_TRY(scratch.alloc(sb));
    hipError_t e = launch_in_degree(graph->col_indices, graph->num_edges, in_degree, graph->num_vertices, scratch.p, sb, s);
    if (sb) {
        // the scratch goes back to the library's cache: the count must be over first
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        scratch.release();
    }
    if (e != hipSuccess) return hip_fail(e, "atlas_in_degree");
    return ATLAS_OK;
}

int atlas_reorder_indegree_desc(const atlas_graph_t *graph, int32_t *new_of_old, int32_t *old_of_new) {
    if (!graph || !new_of_old || !old_of_new || !graph->in_degree) return ATLAS_E_NULL;
    if (graph->num_vertices < 0) return ATLAS_E_RANGE;
    if (graph->num_vertices >= (int64_t(1) << 31)) return ATLAS_E_OVERFLOW;
    HIP_TRY(reorder_indegree_desc(graph->in_degree, graph->num_vertices, new_of_old, old_of_new));
    return ATLAS_OK;
}

int atlas_reorder_indegree_desc_noalloc(const atlas_graph_t *graph, int32_t *new_of_old, int32_t *old_of_new,
                                        void *hip_stream) {
    if (!graph || !new_of_old || !old_of_new || !graph->in_degree) return ATLAS_E_NULL;
    if (graph->num_vertices < 0) return ATLAS_E_RANGE;
    static_assert(atlas::kNoAllocMaxVertices == ATLAS_NOALLOC_MAX_VERTICES, "header and kernel limit differ");
    if (graph->num_vertices > ATLAS_NOALLOC_MAX_VERTICES) return ATLAS_E_TOO_LARGE;
    bool too_large = false;
    HIP_TRY(reorder_indegree_desc_noalloc(graph->in_degree, graph->num_vertices, new_of_old, old_of_new,
                                          static_cast<hipStream_t>(hip_stream), &too_large));
    return too_large ? ATLAS_E_TOO_LARGE : ATLAS_OK;
}

int atlas_reorder_score_desc(const atlas_graph_t *graph, int32_t *new_of_old, int32_t *old_of_new) {
    if (!graph || !new_of_old || !old_of_new || !graph->in_degree || !graph->row_offsets) return ATLAS_E_NULL;
    if (graph->num_edges > 0 && !graph->col_indices) return ATLAS_E_NULL;
    if (graph->residency != ATLAS_RESIDENT_DEVICE) return ATLAS_E_BAD_DIMS;
    if (graph->num_vertices < 0) return ATLAS_E_RANGE;
    if (graph->num_vertices >= (int64_t(1) << 31)) return ATLAS_E_OVERFLOW;
    HIP_TRY(reorder_score_desc(graph->row_offsets, graph->col_indices, graph->in_degree, graph->num_vertices,
                               new_of_old, old_of_new));
    return ATLAS_OK;
}

int atlas_sample_in_edges(const atlas_graph_t *graph, const uint32_t *edge_key, int32_t fanout,
                          int64_t *out_row_offsets, int32_t *out_col_indices, int64_t *out_num_edges) {
    if (!graph || !out_row_offsets || !graph->row_offsets) return ATLAS_E_NULL;
    if (graph->num_edges > 0 && (!graph->col_indices || !edge_key || !out_col_indices)) return ATLAS_E_NULL;
    if (graph->residency != ATLAS_RESIDENT_DEVICE) return ATLAS_E_BAD_DIMS;
    if (graph->num_vertices < 0 || graph->num_edges < 0 || fanout < 0) return ATLAS_E_RANGE;
    if (graph->num_vertices >= (int64_t(1) << 31) || graph->num_edges >= (int64_t(1) << 32)) return ATLAS_E_OVERFLOW;
    HIP_TRY(sample_in_edges(graph->row_offsets, graph->col_indices, graph->num_vertices, graph->num_edges, edge_key,
                            fanout, out_row_offsets, out_col_indices));
    if (out_num_edges)
        HIP_TRY(hipMemcpy(out_num_edges, out_row_offsets + graph->num_vertices, sizeof(int64_t), hipMemcpyDeviceToHost));
    return ATLAS_OK;
}

int atlas_debug_copy(atlas_layer_t *L, int what, void *host_dst, int64_t bytes) {
    if (!L || !host_dst) return ATLAS_E_NULL;
    if (bytes < 0) return ATLAS_E_RANGE;
    HIP_TRY(hipStreamSynchronize(L->last_stream));
    const void *src = nullptr;
    int64_t avail = 0;
    int32_t c[2] = {0, 0};
    HIP_TRY(hipMemcpy(c, L->counters.p, sizeof(c), hipMemcpyDeviceToHost));
    int64_t pair[2] = {c[CTR_READY_TAIL], c[CTR_READY_HEAD]};
    switch (what) {
        case ATLAS_DBG_INDEG: src = L->indeg; avail = L->n * 4; break;
        case ATLAS_DBG_PENDING: src = L->pending.p; avail = L->n * 4; break;
        case ATLAS_DBG_READY: src = L->ready.p; avail = static_cast<int64_t>(c[CTR_READY_TAIL]) * 4; break;
        case ATLAS_DBG_ACC:
            if (L->bounded) return ATLAS_E_STATE;   // rows live in slots or in the cold tier
            src = L->acc.p;
            avail = L->n * L->acc_width * 4;
            break;
        case ATLAS_DBG_READY_COUNT:
            if (bytes < static_cast<int64_t>(sizeof(pair))) return ATLAS_E_RANGE;
            static_cast<int64_t *>(host_dst)[0] = pair[0];
            static_cast<int64_t *>(host_dst)[1] = pair[1];
            return ATLAS_OK;
        default: return ATLAS_E_BAD_DIMS;
    }
    if (bytes > avail) return ATLAS_E_RANGE;
    if (bytes > 0) HIP_TRY(hipMemcpy(host_dst, src, static_cast<size_t>(bytes), hipMemcpyDeviceToHost));
    if (what == ATLAS_DBG_READY) {   // bit 31 of an entry says how the row reaches the update, not which vertex
        int32_t *ids = static_cast<int32_t *>(host_dst);
        for (int64_t i = 0; i < bytes / 4; ++i) ids[i] &= 0x7fffffff;
    }
    if (what == ATLAS_DBG_PENDING) {   // likewise bit 30 of a count (see kPendingHanded)
        int32_t *cnt = static_cast<int32_t *>(host_dst);
        for (int64_t i = 0; i < bytes / 4; ++i) cnt[i] &= ~kPendingHanded;
    }
    return ATLAS_OK;
}

int atlas_release_cache(void) {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    hipError_t first = hipSuccess;
    for (auto &b : g_cache) {
        hipError_t e = hipFree(b.p);
        if (e != hipSuccess && first == hipSuccess) first = e;
    }
    g_cache.clear();
    delete g_regroup_work;
    g_regroup_work = nullptr;
    if (g_cold) {
        hipError_t e = hipHostFree(g_cold);
        if (e != hipSuccess && first == hipSuccess) first = e;
        g_cold = nullptr;
        g_cold_bytes = 0;
    }
    if (g_copy_stream) {
        // no layer is alive (the caller's promise), so nothing is queued on it any more
        hipError_t e = hipStreamSynchronize(g_copy_stream);
        if (e == hipSuccess) e = hipStreamDestroy(g_copy_stream);
        if (e != hipSuccess && first == hipSuccess) first = e;
        g_copy_stream = nullptr;
    }
    if (first != hipSuccess) return hip_fail(first, "hipFree");
    return ATLAS_OK;
}

const char *atlas_strerror(int status) {
    switch (status) {
        case ATLAS_OK: return "ok";
        case ATLAS_E_NULL: return "required pointer is NULL";
        case ATLAS_E_BAD_DIMS: return "unsupported dimensions or enum value";
        case ATLAS_E_RANGE: return "chunk bounds or size out of range";
        case ATLAS_E_ORDER: return "chunks must be contiguous and ascending from 0";
        case ATLAS_E_INCOMPLETE: return "layer finished before every vertex was completed and flushed";
        case ATLAS_E_OVERFLOW: return "vertex count does not fit int32";
        case ATLAS_E_HIP: return "HIP call failed";
        case ATLAS_E_NOMEM: return "out of memory";
        case ATLAS_E_STATE: return "call not valid in this state";
        case ATLAS_E_TOO_LARGE: return "input exceeds the fixed scratch of the no-allocation entry point";
        default: return "unknown status";
    }
}

const char *atlas_last_hip_error(void) { return g_hip_error.c_str(); }

}  // extern "C"
