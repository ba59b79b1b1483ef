// Broadcast step of one source chunk: push every source row along its
// out-edges into the per-destination fp32 accumulators, decrement the
// destination's pending-message count once per message, and append the
// destinations whose count reaches zero to the ready list.
// (Paper Sec. 3.1 broadcast model; Sec. 3.4 message construction and the
// pending-message tracker; Sec. 3.6 completion when the count reaches zero.)
//
// Work is split by EDGES, not by sources: a wavefront owns 64 consecutive
// edges of the chunk's CSR slice, so a source with a million out-edges and a
// run of sources with one edge each cost the same.  The wave finds the source
// of its first edge with a 64-ary search over the row offsets, resolves the
// source of every edge in registers, then walks its edges: the 64 lanes hold
// one source row (d/64 elements per lane, lane-contiguous so that every
// atomic instruction covers whole cache lines of the destination row).
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>
#include <type_traits>

namespace atlas {
namespace {

constexpr int kWave = 64;
constexpr int kTileEdges = 64;
constexpr int kMaxHeads = 8;   // attention heads (checked at layer init)
constexpr int kBlock = 256;

__device__ __forceinline__ float load_as_f32(const float *p) { return *p; }
__device__ __forceinline__ float load_as_f32(const uint16_t *p) {   // bf16
    return __uint_as_float(static_cast<uint32_t>(*p) << 16);
}
__device__ __forceinline__ float load_as_f32(const _Float16 *p) { return static_cast<float>(*p); }
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

// Largest u in [lo, hi) with off[u] <= e.  Requires off[lo] <= e < off[hi].
// All 64 lanes take part; the result is wave-uniform.
__device__ __forceinline__ int64_t wave_find_source(const int64_t *__restrict__ off, int64_t lo,
                                                    int64_t hi, int64_t e, int lane) {
    while (hi - lo > 1) {
        const int64_t step = (hi - lo + 63) >> 6;
        const int64_t p = lo + static_cast<int64_t>(lane) * step;
        bool ok = false;
        if (p < hi) ok = off[p] <= e;
        const int c = __popcll(__ballot(ok));  // offsets ascend: a prefix of lanes says yes
        lo += static_cast<int64_t>(c - 1) * step;
        const int64_t nh = lo + step;
        hi = nh < hi ? nh : hi;
    }
    return lo;
}

// Ready-list appends are staged per wave in LDS: every wave appends the
// vertices it completes to its own buffer and moves them to the global list
// 256 at a time.  The list's tail counter is one address for the whole GPU and
// same-address atomics retire at roughly one per 10 ns, so it must see one
// atomic per few hundred completed vertices, not one per tile.  `count` is
// wave-uniform and stays below kStageFlush between calls.
constexpr int kStageFlush = 256;
constexpr int kStageCap = kStageFlush + kWave;

template <int FLUSH = kStageFlush>
__device__ __forceinline__ void stage_ready(bool is_ready, int32_t v, int32_t *stage, int &count,
                                            int32_t *ready, int32_t *counters, int lane) {
    const uint64_t m = __ballot(is_ready);
    if (m == 0) return;
    if (is_ready) stage[count + __popcll(m & ((1ull << lane) - 1ull))] = v;
    count += __popcll(m);
    __builtin_amdgcn_wave_barrier();
    if (count >= FLUSH) {
        int base = 0;
        if (lane == 0) base = atomicAdd(&counters[CTR_READY_TAIL], FLUSH);
        base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
        for (int k = 0; k < FLUSH / kWave; ++k) ready[base + k * kWave + lane] = stage[k * kWave + lane];
        const int rem = count - FLUSH;
        int32_t t = 0;
        if (lane < rem) t = stage[FLUSH + lane];
        __builtin_amdgcn_wave_barrier();
        if (lane < rem) stage[lane] = t;
        __builtin_amdgcn_wave_barrier();
        count = rem;
    }
}

__device__ __forceinline__ void drain_ready(const int32_t *stage, int count, int32_t *ready,
                                            int32_t *counters, int lane) {
    if (count <= 0) return;
    int base = 0;
    if (lane == 0) base = atomicAdd(&counters[CTR_READY_TAIL], count);
    base = __builtin_amdgcn_readfirstlane(base);
    for (int k = lane; k < count; k += kWave) ready[base + k] = stage[k];
}

// Sources and destinations of the 64 edges [e0, e0 + cnt) of a CSR tile:
// returns the source u0 of the first edge; lane j gets the destination of edge
// j in `v` and its source as an offset from u0 in `my_src`.  Lane k fetches
// the end offset of source ubase+k; an edge's source is the number of row ends
// at or before it, found by a binary search over the 64 lane-held ends.  A
// tile spanning more than 64 sources (long runs of sources without out-edges)
// re-anchors with another search.
__device__ __forceinline__ int64_t resolve_tile(const AggregateArgs &a, int64_t e0, int cnt, int lane,
                                                int32_t &v, int &my_src) {
    const int64_t u0 = wave_find_source(a.off, a.src_begin, a.src_end, e0, lane);
    v = 0;
    if (lane < cnt) v = a.col[e0 + lane - a.col_base];
    my_src = 0;
    bool found = lane >= cnt;
    int64_t ubase = u0;
    while (true) {
        const int64_t u = ubase + lane;
        int relend = kTileEdges;
        if (u < a.src_end) {
            const int64_t r = a.off[u + 1] - e0;
            relend = r < kTileEdges ? static_cast<int>(r) : kTileEdges;
        }
        int lo = 0, hi = kWave;
#pragma unroll
        for (int it = 0; it < 7; ++it) {
            const int mid = (lo + hi) >> 1;
            const int r = __shfl(relend, mid & (kWave - 1));
            const bool open = lo < hi;
            const bool le = r <= lane;
            if (open && le) lo = mid + 1;
            if (open && !le) hi = mid;
        }
        if (!found && lo < kWave) {
            my_src = static_cast<int>(ubase - u0) + lo;
            found = true;
        }
        const uint64_t todo = __ballot(!found);
        if (todo == 0) break;
        const int first = __ffsll(static_cast<unsigned long long>(todo)) - 1;
        ubase = wave_find_source(a.off, ubase, a.src_end, e0 + first, lane);
    }
    return u0;
}

__device__ __forceinline__ int32_t encode_max(float f) {
    const int32_t b = __float_as_int(f);
    return b >= 0 ? b : b ^ 0x7fffffff;
}
__device__ __forceinline__ float decode_max(int32_t e) { return __int_as_float(e >= 0 ? e : e ^ 0x7fffffff); }
__device__ __forceinline__ float leaky(float s, float slope) { return s > 0.f ? s : slope * s; }

template <typename T, int VPL, int MODEL>
__global__ __launch_bounds__(kBlock) void k_aggregate(AggregateArgs a) {
    constexpr int D = VPL * kWave;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / kWave);
    const int64_t ebeg = a.off[a.src_begin];
    const int64_t eend = a.off[a.src_end];
    const int64_t ntiles = (eend - ebeg + kTileEdges - 1) / kTileEdges;
    const T *__restrict__ emb = static_cast<const T *>(a.emb);
    __shared__ int32_t stage_all[(kBlock / kWave) * kStageCap];
    int32_t *stage = stage_all + (threadIdx.x >> 6) * kStageCap;
    int staged = 0;

    if (wave == 0 && lane == 0)
        atomicAdd(&a.counters64[CTR64_EDGES], static_cast<unsigned long long>(eend - ebeg));

    for (int64_t t = wave; t < ntiles; t += nwaves) {
        const int64_t e0 = ebeg + t * kTileEdges;
        const int64_t left = eend - e0;
        const int cnt = left < kTileEdges ? static_cast<int>(left) : kTileEdges;
        int32_t v;
        int my_src;
        const int64_t u0 = resolve_tile(a, e0, cnt, lane, v, my_src);

        float x[VPL];
        float elu[VPL];  // GAT: source attention term of the head each element belongs to
#pragma unroll
        for (int i = 0; i < VPL; ++i) x[i] = elu[i] = 0.f;
        int uprev = -1;
        for (int j = 0; j < cnt; ++j) {
            const int so = __builtin_amdgcn_readlane(my_src, j);
            const int32_t vj = __builtin_amdgcn_readlane(v, j);
            if (so != uprev) {
                uprev = so;
                const int64_t u = u0 + so;
                const T *row = emb + (u - a.src_begin) * D + lane;
                float g = 1.f;
                if (MODEL == 1) {  // GCN: source side of the symmetric normalisation
                    const int32_t du = a.indeg[u];
                    g = 1.0f / sqrtf(static_cast<float>(du > 0 ? du : 1));
                }
#pragma unroll
                for (int i = 0; i < VPL; ++i) x[i] = load_as_f32(row + i * kWave) * g;
                if (MODEL == 2) {
#pragma unroll
                    for (int i = 0; i < VPL; ++i) elu[i] = a.gat.el[u * a.gat.heads + (lane + i * kWave) / a.gat.dh];
                }
            }
            float *dst = a.acc + static_cast<int64_t>(vj) * D + lane;
            if (MODEL == 2) {
                // weight exp(s - m_cur) <= 1: m_cur already covers every logit of this chunk
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    const int c = lane + i * kWave;
                    const int64_t vh = static_cast<int64_t>(vj) * a.gat.heads + c / a.gat.dh;
                    const float sc = leaky(elu[i] + a.gat.er[vh], a.gat.slope);
                    const float wgt = expf(sc - decode_max(a.gat.m_cur[vh]));
                    unsafeAtomicAdd(dst + i * kWave, x[i] * wgt);
                    if (c % a.gat.dh == 0) unsafeAtomicAdd(a.gat.l + vh, wgt);
                }
            } else {
#pragma unroll
                for (int i = 0; i < VPL; ++i) unsafeAtomicAdd(dst + i * kWave, x[i]);
            }
        }

        // One pending-count decrement per message; the message that takes the
        // count to zero completes the destination.
        bool is_ready = false;
        if (lane < cnt) is_ready = atomicSub(&a.pending[v], 1) == 1;
        stage_ready(is_ready, v, stage, staged, a.ready, a.counters, lane);
    }
    drain_ready(stage, staged, a.ready, a.counters, lane);
}

// GAT, first sweep of a chunk: every edge raises m_next[v][h] to its logit.
__global__ __launch_bounds__(kBlock) void k_gat_chunk_max(AggregateArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / kWave);
    const int64_t ebeg = a.off[a.src_begin];
    const int64_t eend = a.off[a.src_end];
    const int64_t ntiles = (eend - ebeg + kTileEdges - 1) / kTileEdges;
    const int H = a.gat.heads;
    for (int64_t t = wave; t < ntiles; t += nwaves) {
        const int64_t e0 = ebeg + t * kTileEdges;
        const int64_t left = eend - e0;
        const int cnt = left < kTileEdges ? static_cast<int>(left) : kTileEdges;
        int32_t v;
        int my_src;
        const int64_t u0 = resolve_tile(a, e0, cnt, lane, v, my_src);
        if (lane < cnt) {
            const int64_t u = u0 + my_src;
            for (int h = 0; h < H; ++h) {
                const float sc = leaky(a.gat.el[u * H + h] + a.gat.er[static_cast<int64_t>(v) * H + h], a.gat.slope);
                atomicMax(&a.gat.m_next[static_cast<int64_t>(v) * H + h], encode_max(sc));
            }
        }
    }
}

// The self message of SAGE: every source of the chunk sends its own row to
// itself, one pending-count decrement.  No other kernel runs on the layer's
// stream at the same time and each thread owns one vertex, so the decrement
// is a plain read-modify-write.
__global__ __launch_bounds__(kBlock) void k_self_message(int64_t b, int64_t e, int32_t *pending,
                                                         int32_t *ready, int32_t *counters) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / kWave);
    const int64_t span = e - b;
    // about half the vertices of a power-law graph complete by this message alone: few waves with a large
    // staging buffer each keep the number of appends to the one ready-tail counter (about 10 ns each,
    // serialised) down; four independent counts per lane are in flight to cover the latency instead
    constexpr int kSelfFlush = 2048;
    constexpr int kPer = 4;
    __shared__ int32_t stage_all[(kBlock / kWave) * (kSelfFlush + kWave)];
    int32_t *stage = stage_all + (threadIdx.x >> 6) * (kSelfFlush + kWave);
    int staged = 0;
    for (int64_t i0 = wave * (kWave * kPer); i0 < span; i0 += nwaves * (kWave * kPer)) {
        int32_t left[kPer], mark[kPer];
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int64_t i = i0 + k * kWave + lane;
            const int32_t p = i < span ? pending[b + i] : 0;
            // bit 30: the aggregation has already left the vertex's finished row as the update's 16-bit operand
            mark[k] = p & kPendingHanded;
            left[k] = i < span ? (p & ~kPendingHanded) - 1 : -1;
        }
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int64_t i = i0 + k * kWave + lane;
            if (i < span) pending[b + i] = left[k];
            const int32_t entry = static_cast<int32_t>(b + i) | (mark[k] ? static_cast<int32_t>(0x80000000u) : 0);
            stage_ready<kSelfFlush>(i < span && left[k] == 0, entry, stage, staged, ready, counters, lane);
        }
    }
    drain_ready(stage, staged, ready, counters, lane);
}

// ---- planned chunk: edges regrouped by destination --------------------------
//
// A tile is 64 consecutive edges of the chunk's destination-ordered edge list
// and a wave owns runs of consecutive tiles.  Every edge is one coalesced read
// of its source row; the rows of one destination are summed in registers and
// reach the accumulator as a single row update.  A destination whose edges all
// lie inside one run is touched by this wave only (plain read-add-write); a
// group cut by a run boundary is added with atomics by every run that holds a
// piece of it.  The pending count drops tile by tile, by the size of the
// group's piece in the tile.

template <typename T, int VPL>
__device__ __forceinline__ void load_row(const T *__restrict__ p, float (&x)[VPL]) {
    if constexpr (std::is_same<T, _Float16>::value) {   // IEEE half rows: one vector load, then conversions
        if constexpr (VPL == 2) {
            const f16x2_t w = *reinterpret_cast<const f16x2_t *>(p);
            x[0] = static_cast<float>(w[0]); x[1] = static_cast<float>(w[1]);
        } else if constexpr (VPL == 4) {
            const f16x4_t w = *reinterpret_cast<const f16x4_t *>(p);
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = static_cast<float>(w[i]);
        } else if constexpr (VPL == 8) {
            const f16x8_t w = *reinterpret_cast<const f16x8_t *>(p);
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = static_cast<float>(w[i]);
        } else {
#pragma unroll
            for (int i = 0; i < VPL; ++i) x[i] = load_as_f32(p + i);
        }
    } else if constexpr (sizeof(T) == 2) {
        if constexpr (VPL == 2) {
            const uint32_t w = *reinterpret_cast<const uint32_t *>(p);
            x[0] = __uint_as_float(w << 16);
            x[1] = __uint_as_float(w & 0xffff0000u);
        } else if constexpr (VPL == 4) {
            const uint2 w = *reinterpret_cast<const uint2 *>(p);
            x[0] = __uint_as_float(w.x << 16); x[1] = __uint_as_float(w.x & 0xffff0000u);
            x[2] = __uint_as_float(w.y << 16); x[3] = __uint_as_float(w.y & 0xffff0000u);
        } else if constexpr (VPL == 8) {
            const uint4 w = *reinterpret_cast<const uint4 *>(p);
            x[0] = __uint_as_float(w.x << 16); x[1] = __uint_as_float(w.x & 0xffff0000u);
            x[2] = __uint_as_float(w.y << 16); x[3] = __uint_as_float(w.y & 0xffff0000u);
            x[4] = __uint_as_float(w.z << 16); x[5] = __uint_as_float(w.z & 0xffff0000u);
            x[6] = __uint_as_float(w.w << 16); x[7] = __uint_as_float(w.w & 0xffff0000u);
        } else {
#pragma unroll
            for (int i = 0; i < VPL; ++i) x[i] = load_as_f32(p + i);
        }
    } else {
        if constexpr (VPL == 2) {
            const float2 w = *reinterpret_cast<const float2 *>(p);
            x[0] = w.x; x[1] = w.y;
        } else if constexpr (VPL == 4) {
            const float4 w = *reinterpret_cast<const float4 *>(p);
            x[0] = w.x; x[1] = w.y; x[2] = w.z; x[3] = w.w;
        } else if constexpr (VPL == 8) {
            const float4 w0 = *reinterpret_cast<const float4 *>(p);
            const float4 w1 = *reinterpret_cast<const float4 *>(p + 4);
            x[0] = w0.x; x[1] = w0.y; x[2] = w0.z; x[3] = w0.w;
            x[4] = w1.x; x[5] = w1.y; x[6] = w1.z; x[7] = w1.w;
        } else {
#pragma unroll
            for (int i = 0; i < VPL; ++i) x[i] = p[i];
        }
    }
}

// Accumulator rows are touched once per chunk: their loads and stores carry
// the streaming hint so that they displace as little as possible in L2.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int VPL>
__device__ __forceinline__ void row_add_owned(float *p, const float (&x)[VPL]) {
    if constexpr (VPL == 2) {
        f32x2_t v = __builtin_nontemporal_load(reinterpret_cast<f32x2_t *>(p));
        v[0] += x[0]; v[1] += x[1];
        __builtin_nontemporal_store(v, reinterpret_cast<f32x2_t *>(p));
    } else if constexpr (VPL == 4 || VPL == 8) {
#pragma unroll
        for (int q = 0; q < VPL / 4; ++q) {
            f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<f32x4_t *>(p + 4 * q));
            v[0] += x[4 * q]; v[1] += x[4 * q + 1]; v[2] += x[4 * q + 2]; v[3] += x[4 * q + 3];
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t *>(p + 4 * q));
        }
    } else {
#pragma unroll
        for (int i = 0; i < VPL; ++i) p[i] += x[i];
    }
}

template <int VPL>
__device__ __forceinline__ void row_store(float *p, const float (&x)[VPL]) {
    if constexpr (VPL == 2) {
        f32x2_t v; v[0] = x[0]; v[1] = x[1];
        __builtin_nontemporal_store(v, reinterpret_cast<f32x2_t *>(p));
    } else if constexpr (VPL == 4 || VPL == 8) {
#pragma unroll
        for (int q = 0; q < VPL / 4; ++q) {
            f32x4_t v; v[0] = x[4 * q]; v[1] = x[4 * q + 1]; v[2] = x[4 * q + 2]; v[3] = x[4 * q + 3];
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t *>(p + 4 * q));
        }
    } else {
#pragma unroll
        for (int i = 0; i < VPL; ++i) p[i] = x[i];
    }
}

// p = p * f + x for the only writer of the row
template <int VPL>
__device__ __forceinline__ void row_scale_add_owned(float *p, float f, const float (&x)[VPL]) {
    float y[VPL];
    if constexpr (VPL == 2) {
        const float2 o = *reinterpret_cast<const float2 *>(p);
        y[0] = o.x * f + x[0];
        y[1] = o.y * f + x[1];
    } else if constexpr (VPL == 4 || VPL == 8) {
#pragma unroll
        for (int q = 0; q < VPL / 4; ++q) {
            const float4 o = *reinterpret_cast<const float4 *>(p + 4 * q);
            y[4 * q] = o.x * f + x[4 * q];
            y[4 * q + 1] = o.y * f + x[4 * q + 1];
            y[4 * q + 2] = o.z * f + x[4 * q + 2];
            y[4 * q + 3] = o.w * f + x[4 * q + 3];
        }
    } else {
#pragma unroll
        for (int i = 0; i < VPL; ++i) y[i] = p[i] * f + x[i];
    }
    row_store<VPL>(p, y);
}

template <int VPL>
__device__ __forceinline__ void row_add_shared(float *p, const float (&x)[VPL]) {
#pragma unroll
    for (int i = 0; i < VPL; ++i) unsafeAtomicAdd(p + i, x[i]);
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
// two fp32 -> one word of two 16-bit values (round to nearest even); dt: 1 bf16, 2 IEEE half
__device__ __forceinline__ uint32_t pack_pair(int dt, float lo, float hi) {
    const f32x2_t v = {lo, hi};
    if (dt == 2) {
        const f16x2_t h = __builtin_convertvector(v, f16x2_t);
        return *reinterpret_cast<const uint32_t *>(&h);
    }
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<const uint32_t *>(&b);
}

// Hand-over of a finished row to the update (the fused part of the flush, Sec. 3.6: a vertex graduates the
// moment its count reaches zero).  When a group that this wave alone owns takes its destination's count to
// zero, the finished sum is in the wave's registers: it leaves as the update's own left operand --
// normalised and rounded to the 16-bit compute type exactly as the update would have done -- in the first
// half of the accumulator row, instead of as fp32 sums that the update reads back, scales and rounds.  The
// ready-list entry of such a vertex carries kHandedOver.  `row` is the start of the accumulator row, `x` the
// group's sum of this lane's elements lane * VPL ..; the row so far is added unless the group is the
// destination's first.  (Every lane's old values are in registers before any lane stores: the stores
// depend on the loads of the same instruction.)
constexpr int32_t kHandedOver = static_cast<int32_t>(0x80000000u);
template <int VPL>
__device__ __forceinline__ void row_hand_over(float *row, int lane, const float (&x)[VPL], bool first, float scale,
                                              int dt) {
    static_assert(VPL % 2 == 0, "pairs of elements");
    float t[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) t[i] = x[i];
    if (!first) {
#pragma unroll
        for (int q = 0; q < VPL / 2; ++q) {
            const f32x2_t v = __builtin_nontemporal_load(reinterpret_cast<f32x2_t *>(row + lane * VPL + 2 * q));
            t[2 * q] += v[0];
            t[2 * q + 1] += v[1];
        }
    }
    uint32_t *o = reinterpret_cast<uint32_t *>(row) + lane * (VPL / 2);
#pragma unroll
    for (int q = 0; q < VPL / 2; ++q) o[q] = pack_pair(dt, t[2 * q] * scale, t[2 * q + 1] * scale);
}

// Second half of a tile's pending-count update: `old` is what the lane's read
// (or atomic) returned.  The sole writer stores the new count here.
__device__ __forceinline__ void finish_pending(bool closes, bool shared, int32_t old, int32_t c, int32_t dst,
                                               bool handed, bool handed_early, const GroupedArgs &a, int32_t *stage,
                                               int &staged, int lane) {
    bool is_ready = false;
    if (closes) {
        is_ready = old == c;
        // handed_early: only the vertex's own message is outstanding and the row is already the update's operand;
        // the count carries the mark to k_self_message, which completes the vertex
        if (!shared) a.pending[dst] = (old - c) | (handed_early ? kPendingHanded : 0);
    }
    // a handed-over row was written because the count read ahead equalled c: the same value as `old`
    stage_ready(is_ready, handed ? dst | kHandedOver : dst, stage, staged, a.ready, a.counters, lane);
}

template <typename T, int VPL, int MODEL, bool FUSE>
// The kernel is latency-bound on the row gathers.  Instantiations whose eight
// rows in flight take at most 16 registers are held to all 8 waves of a SIMD
// (scalar registers beyond that budget spill to lanes, nothing to memory), the
// narrow GAT ones to 6.
__global__ __launch_bounds__(kBlock)
__attribute__((amdgpu_waves_per_eu(MODEL == 2 ? (VPL <= 2 ? 6 : 1) : (VPL * sizeof(T) <= 8 ? 8 : 1), 8)))
void k_aggregate_grouped(GroupedArgs a) {
    constexpr int D = VPL * kWave;
    constexpr int U = 8;  // source rows in flight per wave
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6);
    const int nwaves = gridDim.x * (kBlock / kWave);
    const int ntiles = static_cast<int>((a.n_edges + kTileEdges - 1) / kTileEdges);  // < 2^31: checked by the launcher
    const T *__restrict__ emb = static_cast<const T *>(a.emb);
    __shared__ int32_t stage_all[(kBlock / kWave) * kStageCap];
    int32_t *stage = stage_all + (threadIdx.x >> 6) * kStageCap;
    int staged = 0;
    // GAT: the tile's attention weights, [edge][head], written by the edge's lane and read per row
    __shared__ float wgt_all[MODEL == 2 ? (kBlock / kWave) * kTileEdges * kMaxHeads : 1];
    float *wl = wgt_all + (MODEL == 2 ? (threadIdx.x >> 6) * kTileEdges * kMaxHeads : 0);

    // the launch's share of the chunk's tiles
    const int t_lo = static_cast<int>(a.tile_begin);
    const int t_hi = a.tile_end < 0 || a.tile_end > ntiles ? ntiles : static_cast<int>(a.tile_end);
    if (wave == 0 && lane == 0) {
        const int64_t e_lo = static_cast<int64_t>(t_lo) * kTileEdges;
        const int64_t e_hi = t_hi == ntiles ? a.n_edges : static_cast<int64_t>(t_hi) * kTileEdges;
        atomicAdd(&a.counters64[CTR64_EDGES], static_cast<unsigned long long>(e_hi > e_lo ? e_hi - e_lo : 0));
    }

    // A wave takes runs of `run` consecutive tiles.  A group that is open at
    // the end of a tile stays in the wave's registers when the next tile is
    // the wave's own, so a long group costs one shared add per run, not per tile.
    //
    // The loop is software-pipelined: a tile's edge words, first group index
    // and group destinations are fetched while the tile before it gathers
    // rows, and the result of a tile's pending-count reads is consumed during
    // the next tile, so that the only memory waits on the wave's critical
    // path are those of the row gathers.
    //
    // Waves do not advance at the same speed: a CU issues for its oldest waves
    // first, and with equal shares the workgroup that reached a CU first is
    // done a third earlier than the one that came last, which then works on
    // with few waves left to hide its gathers.  Long launches therefore hand
    // out the runs after a wave's first through a ticket counter (one atomic
    // per run, fetched a run ahead); short ones, where one atomic per tile or
    // two would be more than one address sustains, keep the fixed stride.
    // The launch's last tiles go out in shorter runs, so that the waves end
    // within a short run's time of each other.
    const int run = a.tiles_per_run;
    const int nruns = a.nruns;
    const int big = a.big_runs;
    const int t_small = t_lo + big * run;   // first tile of the short runs
    const int small = a.small_run;
    float sum[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) sum[i] = 0.f;
    float lsum = 0.f;
    // `cut`: other waves may add to the current group's destination row
    // (the group began before this run); it persists from tile to tile.
    bool cut = false;
    bool open_prev = false;

    // the tile in hand (fetched ahead)
    int rn = wave;
    int t = rn >= nruns ? -1 : rn < big ? t_lo + rn * run : t_small + (rn - big) * small;
    int t_end = t + (rn < big ? run : small);
    t_end = t_end < t_hi ? t_end : t_hi;
    bool run_start = true;
    int32_t ticket = 0;   // lane 0: counter value drawn for the wave's next run
    if (a.dynamic && t >= 0 && lane == 0) ticket = atomicAdd(&a.counters[CTR_NEXT_RUN], 1);
    int32_t s = 0, g0 = 0, prev_word = -1, gd = 0;
    // FUSE: count and in-degree of the destination of every group that ends in the tile, read a tile ahead
    int32_t pend_pre = 0, deg_pre = 1;
    auto read_ahead = [&](bool ends, int32_t gdw, int32_t &pend, int32_t &deg) {
        if constexpr (FUSE) {
            if (ends) {
                const int32_t v = gdw & 0x7fffffff & ~a.multi_bit;
                pend = a.pending[v];
                deg = a.indeg[v];
            }
        }
    };
    if (t >= 0) {
        const int64_t e0 = static_cast<int64_t>(t) * kTileEdges;
        const int64_t left = a.n_edges - e0;
        const int cnt = left < kTileEdges ? static_cast<int>(left) : kTileEdges;
        if (lane < cnt) s = a.src_sorted[e0 + lane];
        g0 = a.tile_grp[t];
        if (e0 > 0) prev_word = a.src_sorted[e0 - 1];
        const bool is_end = lane < cnt && s < 0;
        const uint64_t below = __ballot(is_end) & ((1ull << lane) - 1ull);
        if (is_end || lane == cnt - 1) gd = a.grp_dst[g0 + __popcll(below)];
        read_ahead(is_end, gd, pend_pre, deg_pre);
    }
    // pending-count update of the tile before, not yet consumed
    bool pd_closes = false, pd_shared = false, pd_handed = false, pd_early = false;
    int n_handed = 0;   // wave-uniform
    int32_t pd_old = 0, pd_c = 0, pd_dst = 0;

    while (t >= 0) {
        // which tile comes next, and its edge words
        int rn_n = rn, t_n = t + 1, t_end_n = t_end;
        bool run_start_n = false;
        if (t_n == t_end) {
            if (a.dynamic) {
                // tickets count up from run_base; ticket k stands for run nwaves + k
                const uint32_t k = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(ticket)) - a.run_base;
                rn_n = k < static_cast<uint32_t>(nruns) ? nwaves + static_cast<int>(k) : nruns;
            } else {
                rn_n = rn + nwaves;
            }
            t_n = rn_n >= nruns ? -1 : rn_n < big ? t_lo + rn_n * run : t_small + (rn_n - big) * small;
            t_end_n = t_n + (rn_n < big ? run : small);
            t_end_n = t_end_n < t_hi ? t_end_n : t_hi;
            run_start_n = true;
            // a wave draws until a ticket lies beyond the last run: one ticket per run over the whole launch
            if (a.dynamic && t_n >= 0 && lane == 0) ticket = atomicAdd(&a.counters[CTR_NEXT_RUN], 1);
        }
        int32_t s_n = 0, g0_n = 0, prev_word_n = -1, gd_n = 0;
        int32_t pend_n = 0, deg_n = 1;
        int cnt_n = 0;
        if (t_n >= 0) {
            const int64_t e0n = static_cast<int64_t>(t_n) * kTileEdges;
            const int64_t leftn = a.n_edges - e0n;
            cnt_n = leftn < kTileEdges ? static_cast<int>(leftn) : kTileEdges;
            if (lane < cnt_n) s_n = a.src_sorted[e0n + lane];
            g0_n = a.tile_grp[t_n];
            prev_word_n = a.src_sorted[e0n - 1];   // e0n > 0: the wave's first tile was fetched above
        }
        bool ahead_done = false;

        const int64_t e0 = static_cast<int64_t>(t) * kTileEdges;
        const int64_t left = a.n_edges - e0;
        const int cnt = left < kTileEdges ? static_cast<int>(left) : kTileEdges;
        const bool is_end = lane < cnt && s < 0;
        const uint64_t endmask = __ballot(is_end);
        const int src = s & 0x7fffffff;
        // the tile's first group continues one that started in an earlier tile?
        bool cut0 = open_prev;
        if (run_start) {
            cut = prev_word >= 0;
            cut0 = cut;
        }
        const uint64_t below = endmask & ((1ull << lane) - 1ull);
        const bool closes = is_end || lane == cnt - 1;  // last edge of a group, or of the tile
        int32_t dstv = 0;
        bool first_touch = false;  // no earlier chunk sent to this destination: its row holds nothing yet
        bool multi = false;        // source-blocked chunk: other groups of this launch address the same destination
        if (closes) {
            first_touch = gd < 0;
            multi = (gd & a.multi_bit) != 0;
            dstv = gd & 0x7fffffff & ~a.multi_bit;
        }
        const uint64_t firstmask = __ballot(first_touch);
        const uint64_t multimask = __ballot(multi);
        // FUSE: groups that lie wholly inside the tile are this wave's alone (sums, count); one of them that takes
        // its destination's count to zero hands the finished row over instead of adding it
        const int prev_end0 = below ? 63 - __clzll(static_cast<long long>(below)) : -1;
        bool hands = false, hands_early = false;
        float hscale = 1.f;
        if constexpr (FUSE) {
            const bool owned = is_end && !(below == 0 && cut0) && !multi;
            hands = owned && pend_pre == lane - prev_end0;
            // the same when the one message still outstanding is the vertex's own, which comes with its own
            // (later) chunk and carries no data for the sum: the row is final now
            hands_early = owned && a.handover_self && dstv >= a.self_from && pend_pre == lane - prev_end0 + 1;
            hands = hands || hands_early;
            const float fd = static_cast<float>(deg_pre > 0 ? deg_pre : 1);
            hscale = a.handover_norm == 0 ? 1.0f / fd : 1.0f / sqrtf(fd);
        }
        const uint64_t handmask = FUSE ? __ballot(hands) : 0ull;
        if constexpr (FUSE) n_handed += __popcll(handmask);
        // accumulator row of the destination: the vertex id, or its slot in a bounded store
        int32_t rowv = dstv;
        if (MODEL != 2 && a.slot_of && closes) rowv = a.slot_of[dstv];
        float gs = 1.f;
        if (MODEL == 1 && lane < cnt) {  // GCN: source side of the symmetric normalisation
            const int32_t du = a.indeg[src];
            gs = 1.0f / sqrtf(static_cast<float>(du > 0 ? du : 1));
        }

        // GAT: every lane's elements belong to one head (dh is a multiple of VPL)
        const int hl = MODEL == 2 ? (lane * VPL) / a.gat.dh : 0;
        const bool head_first = MODEL == 2 && (lane * VPL) % a.gat.dh == 0;
        if (MODEL == 2) {
            // lane e: weights of edge e for every head, exp(logit - new maximum of its destination) <= 1;
            // the destination is held by the lane that closes the edge's group
            const int H = a.gat.heads;
            const uint64_t rest = endmask >> lane;
            int closer = rest ? lane + __ffsll(static_cast<unsigned long long>(rest)) - 1 : cnt - 1;
            const int64_t ve = __shfl(dstv, closer);
            if (lane < cnt)
                for (int h = 0; h < H; ++h)
                    wl[lane * H + h] = expf(a.scores[(e0 + lane) * H + h] - decode_max(a.gat.m_next[ve * H + h]));
            __builtin_amdgcn_wave_barrier();   // the weights are read across lanes below
        }

        for (int j0 = 0; j0 < cnt; j0 += U) {
            if (j0 == U) {
                // the words fetched before the first batch have arrived with it
                ahead_done = true;
                if (t_n >= 0) {
                    const bool is_end_n = lane < cnt_n && s_n < 0;
                    const uint64_t below_n = __ballot(is_end_n) & ((1ull << lane) - 1ull);
                    if (is_end_n || lane == cnt_n - 1) gd_n = a.grp_dst[g0_n + __popcll(below_n)];
                    read_ahead(is_end_n, gd_n, pend_n, deg_n);
                }
                finish_pending(pd_closes, pd_shared, pd_old, pd_c, pd_dst, pd_handed, pd_early, a, stage, staged, lane);
                pd_closes = false;
            }
            float r[U][VPL];
            float wgt[U];
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const int j = j0 + i < cnt ? j0 + i : cnt - 1;
                const int sj = __builtin_amdgcn_readlane(src, j);
                load_row<T, VPL>(emb + (static_cast<int64_t>(sj) - a.src_begin) * D + lane * VPL, r[i]);
                if (MODEL == 1) {
                    const float g = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(gs), j));
#pragma unroll
                    for (int q = 0; q < VPL; ++q) r[i][q] *= g;
                }
                if (MODEL == 2) wgt[i] = wl[j * a.gat.heads + hl];
            }
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const int j = j0 + i;
                if (j < cnt) {
                    if (MODEL == 2) {
#pragma unroll
                        for (int q = 0; q < VPL; ++q) sum[q] += wgt[i] * r[i][q];
                        lsum += wgt[i];
                    } else {
#pragma unroll
                        for (int q = 0; q < VPL; ++q) sum[q] += r[i][q];
                    }
                    if ((endmask >> j) & 1ull) {
                        const int32_t v = __builtin_amdgcn_readlane(dstv, j);
                        float *dst = a.acc + static_cast<int64_t>(__builtin_amdgcn_readlane(rowv, j)) * D + lane * VPL;
                        if (MODEL == 2) {
                            const int64_t vh = static_cast<int64_t>(v) * a.gat.heads + hl;
                            if (cut) {   // already at the new maximum (k_gat_rescale_cut_groups)
                                row_add_shared<VPL>(dst, sum);
                                if (head_first) unsafeAtomicAdd(a.gat.l + vh, lsum);
                            } else {     // sole writer: move the row to the new maximum while adding
                                const int32_t mc = a.gat.m_cur[vh], mn = a.gat.m_next[vh];
                                const float f = mc == mn ? 1.f : expf(decode_max(mc) - decode_max(mn));
                                row_scale_add_owned<VPL>(dst, f, sum);
                                if (head_first) {
                                    a.gat.l[vh] = a.gat.l[vh] * f + lsum;
                                    a.gat.m_cur[vh] = mn;
                                }
                            }
                        } else if (FUSE && ((handmask >> j) & 1ull)) {
                            if constexpr (FUSE)
                                row_hand_over<VPL>(dst - lane * VPL, lane, sum, ((firstmask >> j) & 1ull) != 0,
                                                   __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(hscale), j)),
                                                   a.handover_dt);
                        } else if (cut || ((multimask >> j) & 1ull)) {
                            row_add_shared<VPL>(dst, sum);
                        } else if ((firstmask >> j) & 1ull) {
                            row_store<VPL>(dst, sum);
                        } else {
                            row_add_owned<VPL>(dst, sum);
                        }
                        cut = false;
                        lsum = 0.f;
#pragma unroll
                        for (int q = 0; q < VPL; ++q) sum[q] = 0.f;
                    }
                }
            }
        }
        open_prev = !((endmask >> (cnt - 1)) & 1ull);
        if (open_prev && t + 1 == t_end) {  // open group that continues in another wave's tile
            const int32_t v = __builtin_amdgcn_readlane(dstv, cnt - 1);
            row_add_shared<VPL>(a.acc + static_cast<int64_t>(__builtin_amdgcn_readlane(rowv, cnt - 1)) * D + lane * VPL, sum);
            if (MODEL == 2 && head_first)
                unsafeAtomicAdd(a.gat.l + static_cast<int64_t>(v) * a.gat.heads + hl, lsum);
#pragma unroll
            for (int q = 0; q < VPL; ++q) sum[q] = 0.f;
            lsum = 0.f;
        }
        if (!ahead_done) {   // a tile of one batch (the chunk's last)
            if (t_n >= 0) {
                const bool is_end_n = lane < cnt_n && s_n < 0;
                const uint64_t below_n = __ballot(is_end_n) & ((1ull << lane) - 1ull);
                if (is_end_n || lane == cnt_n - 1) gd_n = a.grp_dst[g0_n + __popcll(below_n)];
                read_ahead(is_end_n, gd_n, pend_n, deg_n);
            }
            finish_pending(pd_closes, pd_shared, pd_old, pd_c, pd_dst, pd_handed, pd_early, a, stage, staged, lane);
        }

        // pending count: minus the number of this tile's messages to the group.
        // A group that lies wholly inside the tile is the only writer of its
        // destination's count during this kernel, so a plain read-modify-write
        // is enough; pieces of a cut group use the atomic.  The value read is
        // used (and the plain write made) while the next tile gathers.
        pd_closes = closes;
        pd_dst = dstv;
        pd_handed = hands && !hands_early;
        pd_early = hands_early;
        if (closes) {
            const int prev_end = prev_end0;
            pd_c = lane - prev_end;
            pd_shared = (below == 0 && cut0) || !is_end || multi;
            if (pd_shared) pd_old = atomicSub(&a.pending[dstv], pd_c);
            else pd_old = a.pending[dstv];
        }

        rn = rn_n; t = t_n; t_end = t_end_n; run_start = run_start_n;
        s = s_n; g0 = g0_n; prev_word = prev_word_n; gd = gd_n;
        pend_pre = pend_n; deg_pre = deg_n;
    }
    finish_pending(pd_closes, pd_shared, pd_old, pd_c, pd_dst, pd_handed, pd_early, a, stage, staged, lane);
    drain_ready(stage, staged, a.ready, a.counters, lane);
    if (FUSE && lane == 0 && n_handed > 0)
        atomicAdd(&a.counters64[CTR64_HANDED], static_cast<unsigned long long>(n_handed));
}

// GAT, first sweep of a planned chunk: one lane per edge of a 64-edge tile of
// the destination-ordered list, a segmented max-scan over the lanes of each
// destination's group, and one update of m_next per (group, head) -- plain for
// a group that lies inside the tile, atomic for a group cut by a tile boundary.
__global__ __launch_bounds__(kBlock) void k_gat_group_max(GroupedArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / kWave);
    const int64_t ntiles = (a.n_edges + kTileEdges - 1) / kTileEdges;
    const int H = a.gat.heads;
    for (int64_t t = wave; t < ntiles; t += nwaves) {
        const int64_t e0 = t * kTileEdges;
        const int64_t left = a.n_edges - e0;
        const int cnt = left < kTileEdges ? static_cast<int>(left) : kTileEdges;
        const int g0 = a.tile_grp[t];
        int32_t s = 0;
        if (lane < cnt) s = a.src_sorted[e0 + lane];
        const bool is_end = lane < cnt && s < 0;
        const uint64_t endmask = __ballot(is_end);
        const int64_t src = s & 0x7fffffff;
        bool cut = false;
        if (e0 > 0) cut = a.src_sorted[e0 - 1] >= 0;
        const uint64_t below = endmask & ((1ull << lane) - 1ull);
        const bool closes = is_end || lane == cnt - 1;
        int32_t dstv = 0;
        if (closes) dstv = a.grp_dst[g0 + __popcll(below)] & 0x7fffffff;
        // my edge's destination is held by the lane that closes my group
        const uint64_t rest = endmask >> lane;
        int closer = rest ? lane + __ffsll(static_cast<unsigned long long>(rest)) - 1 : cnt - 1;
        if (closer < 0) closer = 0;
        const int64_t v = __shfl(dstv, closer);
        const int start = below ? 64 - __clzll(static_cast<long long>(below)) : 0;  // first lane of my group
        const bool shared = (below == 0 && cut) || !is_end;
        for (int h = 0; h < H; ++h) {
            float sc = -INFINITY;
            if (lane < cnt) {
                sc = leaky(a.gat.el[src * H + h] + a.gat.er[v * H + h], a.gat.slope);
                a.scores[(e0 + lane) * H + h] = sc;   // the aggregation reuses the logit
            }
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const float up = __shfl_up(sc, o);
                if (lane - o >= start) sc = fmaxf(sc, up);
            }
            if (closes) {
                int32_t *m = a.gat.m_next + v * H + h;
                const int32_t enc = encode_max(sc);
                if (shared) atomicMax(m, enc);
                else if (enc > *m) *m = enc;
            }
        }
    }
}

// Planned GAT chunk: one lane per tile boundary.  A group cut by tile boundaries
// is added to by several waves with atomics, so its destination is moved to the
// new maximum beforehand, by the lane of the FIRST boundary that cuts it (the
// group starts in the previous tile): acc and l times
// exp(m_cur - m_next) per head, then m_cur = m_next.  A first touch
// (m_cur = -inf, state still zero) only moves the reference.
__global__ __launch_bounds__(kBlock) void k_gat_rescale_cut_groups(GroupedArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t ntiles = (a.n_edges + kTileEdges - 1) / kTileEdges;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const int H = a.gat.heads;
    for (int64_t t0 = 1 + static_cast<int64_t>(blockIdx.x) * kBlock + (threadIdx.x & ~(kWave - 1)); t0 < ntiles;
         t0 += stride) {
        const int64_t t = t0 + lane;
        int64_t v = -1;
        if (t < ntiles && a.src_sorted[t * kTileEdges - 1] >= 0) {   // the previous tile ends inside a group
            const int32_t g = a.tile_grp[t];                          // group of the tile's first edge = the cut one
            // first boundary of the group: it starts inside the previous tile, or exactly on that tile's first edge
            if (a.tile_grp[t - 1] != g || t == 1 || a.src_sorted[(t - 1) * kTileEdges - 1] < 0)
                v = a.grp_dst[g] & 0x7fffffff;
        }
        bool rows = false;
        if (v >= 0)
            for (int h = 0; h < H; ++h) {
                const int32_t mc = a.gat.m_cur[v * H + h];
                if (mc != a.gat.m_next[v * H + h] && decode_max(mc) != -INFINITY) rows = true;
            }
        uint64_t todo = __ballot(rows);
        while (todo) {  // the whole wave rescales one destination row at a time
            const int j = __ffsll(static_cast<unsigned long long>(todo)) - 1;
            todo &= todo - 1;
            const int64_t vv = __shfl(v, j);
            for (int c = lane; c < a.d; c += kWave) {
                const int h = c / a.gat.dh;
                a.acc[vv * a.d + c] *= expf(decode_max(a.gat.m_cur[vv * H + h]) - decode_max(a.gat.m_next[vv * H + h]));
            }
            if (lane < H)
                a.gat.l[vv * H + lane] *= expf(decode_max(a.gat.m_cur[vv * H + lane]) - decode_max(a.gat.m_next[vv * H + lane]));
        }
        // every lane has finished reading m_cur of the rows above before any lane moves it
        __builtin_amdgcn_wave_barrier();
        if (v >= 0)
            for (int h = 0; h < H; ++h) a.gat.m_cur[v * H + h] = a.gat.m_next[v * H + h];
    }
}

// A wave takes 64 listed rows at a time, one per lane for the test, then clears those that need it
// together.  run > 0: the runs of the launch that follows are known (the first `big` of `run` tiles,
// then runs of `small`); a group whose first and last tile fall into one run needs no clearing.
__global__ __launch_bounds__(kBlock) void k_zero_rows(const int32_t *__restrict__ rows,
                                                     const int32_t *__restrict__ spans, int64_t n_rows, float *acc,
                                                     const int32_t *__restrict__ slot_of, int d, int run, int big,
                                                     int small) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / kWave);
    const int t_small = big * run;
    for (int64_t base = wave * kWave; base < n_rows; base += nwaves * kWave) {
        const int64_t i = base + lane;
        bool need = i < n_rows;
        int32_t v = 0;
        if (need && run > 0) {
            const int t0 = spans[2 * i], t1 = spans[2 * i + 1];
            if (t0 >= 0) {
                const int r0 = t0 < t_small ? t0 / run : big + (t0 - t_small) / small;
                const int r1 = t1 < t_small ? t1 / run : big + (t1 - t_small) / small;
                need = r0 != r1;
            }
        }
        if (need) {
            v = rows[i];
            if (slot_of) v = slot_of[v];
        }
        uint64_t todo = __ballot(need);
        while (todo) {
            const int j = __ffsll(static_cast<unsigned long long>(todo)) - 1;
            todo &= todo - 1;
            float *row = acc + static_cast<int64_t>(__builtin_amdgcn_readlane(v, j)) * d;
            for (int c = lane; c < d; c += kWave) row[c] = 0.f;
        }
    }
}

constexpr int kMinDynamicRun = 4;
constexpr int kMinSplitRun = 8;

// The runs of a launch over tiles [tile_begin, tile_end) on a grid of `grid` workgroups.
hipError_t plan_runs_on(GroupedArgs &a, int grid) {
    // runs of several tiles only where every wave still gets many runs
    const int64_t ntiles = (a.n_edges + kTileEdges - 1) / kTileEdges;
    const int64_t nwaves = static_cast<int64_t>(grid) * (kBlock / kWave);
    const int64_t mine = (a.tile_end < 0 || a.tile_end > ntiles ? ntiles : a.tile_end) - a.tile_begin;
    if (a.tile_begin < 0 || mine < 0) return hipErrorInvalidValue;
    a.nruns = 0;
    if (mine == 0) return hipSuccess;
    const int64_t fit = mine / (4 * nwaves);
    a.tiles_per_run = static_cast<int>(fit < 1 ? 1 : fit > kMaxTilesPerRun ? kMaxTilesPerRun : fit);
    if (a.forced_run > 0) a.tiles_per_run = a.forced_run > kMaxTilesPerRun ? kMaxTilesPerRun : a.forced_run;
    if (ntiles > 0x7fffffff) return hipErrorInvalidValue;   // tile indices are 32-bit in the kernel
    a.nruns = static_cast<int>((mine + a.tiles_per_run - 1) / a.tiles_per_run);
    a.big_runs = a.nruns;
    a.small_run = a.tiles_per_run;
    // runs by ticket where a run is long enough to hide the counter's latency and the launch's
    // tickets (one per run) stay well below what one address sustains
    a.dynamic = a.tiles_per_run >= kMinDynamicRun ? 1 : 0;
    if (a.dynamic && a.tiles_per_run >= kMinSplitRun) {
        // the last run of every wave, in quarters
        const int64_t whole = mine / a.tiles_per_run;
        a.big_runs = static_cast<int>(whole > nwaves ? whole - nwaves : 0);
        a.small_run = a.tiles_per_run / 4;
        const int64_t rest = mine - static_cast<int64_t>(a.big_runs) * a.tiles_per_run;
        a.nruns = a.big_runs + static_cast<int>((rest + a.small_run - 1) / a.small_run);
    }
    return hipSuccess;
}

template <typename T, int MODEL>
hipError_t launch_grouped_vpl(const GroupedArgs &a_in, int grid, uint32_t *run_tickets, hipStream_t s) {
    GroupedArgs a = a_in;
    if (!run_tickets) return hipErrorInvalidValue;
    if (a.nruns == 0) {
        const hipError_t e = plan_runs_on(a, grid);
        if (e != hipSuccess) return e;
        if (a.nruns == 0) return hipSuccess;   // no tiles
    }
    if (a.dynamic) {
        // Tickets drawn by the launch: the counter hands out consecutive values, ticket k stands for run
        // nwaves + k, so the first max(nruns - nwaves, 0) drawn are valid and every later one is not.  A wave
        // that has a first run (min(nwaves, nruns) of them) draws once at its start, once more after every
        // valid ticket and stops at its first invalid one: valid tickets + one per such wave = nruns.
        a.run_base = *run_tickets;
        *run_tickets += static_cast<uint32_t>(a.nruns);
    }
    if constexpr (MODEL != 2 && sizeof(T) == 2) {
        // finished rows are handed over in the 16-bit compute type: rows of 128 elements (the width whose flush
        // kernel knows the hand-over), accumulators addressed by vertex id
        // ... and only in launches whose groups are short on average: a group must lie inside a 64-edge tile to
        // be handed over, and the hand-over's read-ahead (count and degree of every group end) costs a launch of
        // long groups (the first chunk of a degree-ordered stream: 58 edges per group, nothing completes) more
        // than it saves.
        // Where vertices also receive their own embedding as a message (handover_self), most low-degree vertices
        // have all their edge messages in by the first chunk and wait for that message only: there the hand-over
        // pays in every launch.
        if (a.handover && !a.slot_of && a.d == 2 * kWave && a.n_groups > 0 &&
            (a.handover_self || a.n_edges / a.n_groups < 32)) {
            hipLaunchKernelGGL((k_aggregate_grouped<T, 2, MODEL, true>), dim3(grid), dim3(kBlock), 0, s, a);
            return hipGetLastError();
        }
    }
    switch (a.d / kWave) {
        case 1: hipLaunchKernelGGL((k_aggregate_grouped<T, 1, MODEL, false>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 2: hipLaunchKernelGGL((k_aggregate_grouped<T, 2, MODEL, false>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 3: hipLaunchKernelGGL((k_aggregate_grouped<T, 3, MODEL, false>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 4: hipLaunchKernelGGL((k_aggregate_grouped<T, 4, MODEL, false>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 5: hipLaunchKernelGGL((k_aggregate_grouped<T, 5, MODEL, false>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 6: hipLaunchKernelGGL((k_aggregate_grouped<T, 6, MODEL, false>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 7: hipLaunchKernelGGL((k_aggregate_grouped<T, 7, MODEL, false>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 8: hipLaunchKernelGGL((k_aggregate_grouped<T, 8, MODEL, false>), dim3(grid), dim3(kBlock), 0, s, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <typename T, int MODEL>
hipError_t launch_vpl(const AggregateArgs &a, int grid, hipStream_t s) {
    switch (a.d / kWave) {
        case 1: hipLaunchKernelGGL((k_aggregate<T, 1, MODEL>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 2: hipLaunchKernelGGL((k_aggregate<T, 2, MODEL>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 3: hipLaunchKernelGGL((k_aggregate<T, 3, MODEL>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 4: hipLaunchKernelGGL((k_aggregate<T, 4, MODEL>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 5: hipLaunchKernelGGL((k_aggregate<T, 5, MODEL>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 6: hipLaunchKernelGGL((k_aggregate<T, 6, MODEL>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 7: hipLaunchKernelGGL((k_aggregate<T, 7, MODEL>), dim3(grid), dim3(kBlock), 0, s, a); break;
        case 8: hipLaunchKernelGGL((k_aggregate<T, 8, MODEL>), dim3(grid), dim3(kBlock), 0, s, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

int persistent_grid(int blocks_per_cu) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 1024;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return 1024;
    return cus * blocks_per_cu;
}

}  // namespace

hipError_t launch_aggregate(const AggregateArgs &a, hipStream_t s) {
    if (a.d % kWave != 0) return hipErrorInvalidValue;
    const int grid = persistent_grid(8);
    // model 1 (GCN) scales the source row; every other model pushes it as is
    if (a.model == 2) return a.in_dt ? hipErrorInvalidValue : launch_vpl<float, 2>(a, grid, s);
    if (a.in_dt == 2) return a.model == 1 ? launch_vpl<_Float16, 1>(a, grid, s) : launch_vpl<_Float16, 0>(a, grid, s);
    if (a.in_dt == 1) return a.model == 1 ? launch_vpl<uint16_t, 1>(a, grid, s) : launch_vpl<uint16_t, 0>(a, grid, s);
    return a.model == 1 ? launch_vpl<float, 1>(a, grid, s) : launch_vpl<float, 0>(a, grid, s);
}

hipError_t launch_gat_group_max(const GroupedArgs &a, hipStream_t s) {
    if (a.n_edges <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_gat_group_max, dim3(persistent_grid(8)), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t plan_runs(GroupedArgs &a) { return plan_runs_on(a, persistent_grid(8)); }

hipError_t launch_zero_rows(const int32_t *rows, const int32_t *spans, int64_t n_rows, float *acc,
                            const int32_t *slot_of, int d, const GroupedArgs *runs, hipStream_t s) {
    if (n_rows <= 0) return hipSuccess;
    // the runs are counted from the chunk's first tile: only for a launch over the whole chunk
    const bool known = runs && spans && runs->nruns > 0 && runs->tile_begin == 0 && runs->small_run > 0;
    int64_t blocks = (n_rows + kBlock - 1) / kBlock;   // 64 listed rows per wave and round
    const int cap = persistent_grid(8);
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(k_zero_rows, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, rows, spans, n_rows, acc,
                       slot_of, d, known ? runs->tiles_per_run : 0, known ? runs->big_runs : 0,
                       known ? runs->small_run : 1);
    return hipGetLastError();
}

hipError_t launch_gat_rescale_cut_groups(const GroupedArgs &a, hipStream_t s) {
    const int64_t ntiles = (a.n_edges + kTileEdges - 1) / kTileEdges;
    if (ntiles <= 1) return hipSuccess;
    int64_t blocks = (ntiles + kBlock - 1) / kBlock;
    const int cap = persistent_grid(8);
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(k_gat_rescale_cut_groups, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gat_chunk_max(const AggregateArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(k_gat_chunk_max, dim3(persistent_grid(8)), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_aggregate_grouped(const GroupedArgs &a, uint32_t *run_tickets, hipStream_t s) {
    if (a.d % kWave != 0) return hipErrorInvalidValue;
    if (a.n_edges <= 0) return hipSuccess;
    const int grid = persistent_grid(8);
    if (a.model == 2) {
        if (a.in_dt || a.gat.dh % (a.d / kWave) != 0) return hipErrorInvalidValue;
        return launch_grouped_vpl<float, 2>(a, grid, run_tickets, s);
    }
    if (a.in_dt == 2)
        return a.model == 1 ? launch_grouped_vpl<_Float16, 1>(a, grid, run_tickets, s) : launch_grouped_vpl<_Float16, 0>(a, grid, run_tickets, s);
    if (a.in_dt == 1)
        return a.model == 1 ? launch_grouped_vpl<uint16_t, 1>(a, grid, run_tickets, s) : launch_grouped_vpl<uint16_t, 0>(a, grid, run_tickets, s);
    return a.model == 1 ? launch_grouped_vpl<float, 1>(a, grid, run_tickets, s) : launch_grouped_vpl<float, 0>(a, grid, run_tickets, s);
}

hipError_t launch_self_message(int64_t b, int64_t e, int32_t *pending, int32_t *ready,
                               int32_t *counters, hipStream_t s) {
    if (e <= b) return hipSuccess;
    int64_t blocks = (e - b + kBlock * 4 - 1) / (kBlock * 4);
    const int cap = persistent_grid(2);
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(k_self_message, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, b, e,
                       pending, ready, counters);
    return hipGetLastError();
}

}  // namespace atlas
