// Dense update of ready ("graduated") vertices: gather the finished aggregate
// of every vertex on the ready list, normalise it, multiply by the layer's
// weight matrix on the matrix cores, add bias, apply the activation and write
// the row of the next-layer embedding matrix.  (Paper Sec. 3.6: the linear
// transformation and non-linearity applied to completed vertices; Sec. 3.4 for
// the mean normalisation; Sec. 4.3 for the self-concatenation of SAGE.)
//
// A workgroup (4 waves) takes a tile of 64 ready rows.  The rows are gathered
// with whole-row coalesced loads, normalised (1/deg for the SAGE mean,
// deg^-1/2 for GCN), converted to the MFMA input type and staged in LDS as the
// A operand [64][K].  W is repacked once per layer into the per-lane
// B-fragment order of the 32x32 MFMA, so a wave fetches a fragment with one
// contiguous 1 KiB (bf16) / 256 B (fp32) load that stays L2 resident.
// The 64 x d_out output tile is cut into 32x32 blocks dealt round-robin to the
// four waves.  Workgroups loop over tiles (the ready count lives on the device,
// the host never reads it).
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>
#include <type_traits>

namespace atlas {
namespace {

constexpr int kBlock = 256;
constexpr int kTileRows = 64;

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);  // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
    return __uint_as_float(static_cast<uint32_t>(h) << 16);
}

__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
    const _Float16 h = static_cast<_Float16>(f);   // round to nearest even
    return *reinterpret_cast<const uint16_t *>(&h);
}
__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) {
    return static_cast<float>(*reinterpret_cast<const _Float16 *>(&b));
}

// Compute type CT of the contraction, the atlas_dtype of the layer's embeddings:
// 0 fp32, 1 bf16, 2 IEEE half.  16-bit operands are held as raw bits.
template <int CT> struct Elem { using type = uint16_t; };
template <> struct Elem<0> { using type = float; };

template <int CT> __device__ __forceinline__ typename Elem<CT>::type to_elem(float f);
template <> __device__ __forceinline__ float to_elem<0>(float f) { return f; }
template <> __device__ __forceinline__ uint16_t to_elem<1>(float f) { return f32_to_bf16_rne(f); }
template <> __device__ __forceinline__ uint16_t to_elem<2>(float f) { return f32_to_f16_bits(f); }

__host__ __device__ constexpr int lds_pad(bool sixteen_bit) { return sixteen_bit ? 8 : 1; }

// Output column that row m (0..31) of a 32x32 block computed as D^T stands for.
// A lane of the result holds rows m = 8q + 4h + t (q, t < 4; h = lane / 32).
// fp32 operands: the identity, a lane's four runs of four columns are 16-byte
// stores and the two halves of the wave complete 32 bytes of a row per store.
// 16-bit operands: rows are assigned so that a lane holds two runs of EIGHT
// consecutive columns (16 + 16 bytes of a 16-bit output row) and the halves
// again sit side by side: column 16 (q / 2) + 8 h + 4 (q % 2) + t.  The 8-byte
// stores of the identity order cost four store instructions per block, each
// touching 32 rows; the texture unit spends a cycle per row and instruction.
template <int CT>
__host__ __device__ constexpr int block_column(int m) {
    if (CT == 0) return m;
    const int q = m >> 3, h = (m >> 2) & 1, t = m & 3;
    return 16 * (q >> 1) + 8 * h + 4 * (q & 1) + t;
}

// Packed-W element index.  bf16: fragment (nb, kk) is 64 lanes x 8 values,
// value t of lane l is W[kk*16 + (l/32)*8 + t][nb*32 + block_column(l%32)].
// fp32: fragment (nb, kk) is 64 lanes x 1 value, W[kk*2 + l/32][nb*32 + l%32].
template <int CT>
__global__ __launch_bounds__(kBlock) void k_pack_weights(const void *W, int w_dt, int K, int d_out,
                                                         typename Elem<CT>::type *packed) {
    constexpr int kStepK = CT ? 16 : 2;
    constexpr int kPerLane = CT ? 8 : 1;
    const int NB = (d_out + 31) / 32;
    const int KS = K / kStepK;
    const int64_t total = static_cast<int64_t>(NB) * KS * 64 * kPerLane;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= total) return;
    const int t = static_cast<int>(i % kPerLane);
    const int l = static_cast<int>((i / kPerLane) % 64);
    const int64_t frag = i / (kPerLane * 64);
    const int kk = static_cast<int>(frag % KS);
    const int nb = static_cast<int>(frag / KS);
    const int k = kk * kStepK + (l / 32) * kPerLane + t;
    const int j = nb * 32 + block_column<CT>(l % 32);
    float w = 0.f;
    if (j < d_out) {
        const int64_t src = static_cast<int64_t>(k) * d_out + j;
        if (w_dt == 2) w = f16_bits_to_f32(static_cast<const uint16_t *>(W)[src]);
        else w = w_dt == 1 ? bf16_to_f32(static_cast<const uint16_t *>(W)[src]) : static_cast<const float *>(W)[src];
    }
    packed[i] = to_elem<CT>(w);
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16x2 (round to nearest even, one hardware instruction)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<const uint32_t *>(&b);
}

// two fp32 -> packed IEEE half pair (round to nearest even)
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    const f16x2_t b = __builtin_convertvector(v, f16x2_t);
    return *reinterpret_cast<const uint32_t *>(&b);
}
// ... in the compute type CT (1 or 2), or by a run-time dtype code
template <int CT>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    if constexpr (CT == 2) return pack_f16x2(lo, hi);
    else return pack_bf16x2(lo, hi);
}
__device__ __forceinline__ uint32_t pack2_dt(int dt, float lo, float hi) {
    return dt == 2 ? pack_f16x2(lo, hi) : pack_bf16x2(lo, hi);
}

// per-lane operand of one matrix instruction and the instruction itself, by compute type
template <int CT> struct Frag { using type = float; };
template <> struct Frag<1> { using type = bf16x8_t; };
template <> struct Frag<2> { using type = f16x8_t; };
template <int CT>
__device__ __forceinline__ f32x16_t mfma_block(typename Frag<CT>::type b, typename Frag<CT>::type a, f32x16_t c) {
    if constexpr (CT == 1) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c, 0, 0, 0);
    else if constexpr (CT == 2) return __builtin_amdgcn_mfma_f32_32x32x16_f16(b, a, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x2f32(b, a, c, 0, 0, 0);
}

__device__ __forceinline__ float apply_activation(float y, int act) {
    if (act == 1) return y > 0.f ? y : 0.f;
    if (act == 2) return y > 0.f ? y : expm1f(y);
    return y;
}

// Epilogue of one 32x32 block computed as D^T (W fragment as the first MFMA
// operand): lane l then holds, for tile row l%32, sixteen output columns of
// block nb, value 4q + t being column 32 nb + block_column(8q + 4 (l/32) + t).
// `half` = l / 32.
template <bool ADD_BIAS>
__device__ __forceinline__ void store_block_row(const UpdateArgs &a, const f32x16_t &c, int64_t out_row,
                                                int nb, int half, const float *bias16) {
    float y[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) y[r] = ADD_BIAS ? c[r] + bias16[r] : c[r];
    if (a.activation == 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) y[r] = fmaxf(y[r], 0.f);
    } else if (a.activation == 2) {
#pragma unroll
        for (int r = 0; r < 16; ++r) y[r] = y[r] > 0.f ? y[r] : expm1f(y[r]);
    }
    // two weight matrices side by side: the block lies wholly in one of the two outputs
    void *outp = a.out;
    int cols = a.d_out;
    int odt = a.out_dt;
    int base = nb * 32;
    if (a.split > 0) {
        cols = a.split;
        if (base >= a.split) {
            outp = a.out2;
            odt = a.out2_dt;
            base -= a.split;
        }
    }
    const int limit = a.split > 0 ? a.split : a.d_out;
    if (a.compute_dt != 0) {
        // two runs of eight columns: 16 s + 8 half + (0..7), values 8 s .. 8 s + 7
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const int col = base + 16 * s2 + 8 * half;
            if (col >= limit) continue;
            const float *v = y + 8 * s2;
            if (odt) {
                uint16_t *o = static_cast<uint16_t *>(outp) + out_row * cols + col;
                *reinterpret_cast<uint4 *>(o) = make_uint4(pack2_dt(odt, v[0], v[1]), pack2_dt(odt, v[2], v[3]),
                                                           pack2_dt(odt, v[4], v[5]), pack2_dt(odt, v[6], v[7]));
            } else {
                float *o = static_cast<float *>(outp) + out_row * cols + col;
                *reinterpret_cast<float4 *>(o) = make_float4(v[0], v[1], v[2], v[3]);
                *reinterpret_cast<float4 *>(o + 4) = make_float4(v[4], v[5], v[6], v[7]);
            }
        }
    } else {
        // four runs of four columns: 8 q + 4 half + (0..3)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = base + 8 * q + 4 * half;
            if (col >= limit) continue;
            if (odt) {
                uint16_t *o = static_cast<uint16_t *>(outp) + out_row * cols + col;
                *reinterpret_cast<uint2 *>(o) =
                    make_uint2(pack2_dt(odt, y[4 * q], y[4 * q + 1]), pack2_dt(odt, y[4 * q + 2], y[4 * q + 3]));
            } else {
                float *o = static_cast<float *>(outp) + out_row * cols + col;
                *reinterpret_cast<float4 *>(o) = make_float4(y[4 * q], y[4 * q + 1], y[4 * q + 2], y[4 * q + 3]);
            }
        }
    }
}

// the bias of the sixteen columns a lane holds, in the order of its values
__device__ __forceinline__ void load_bias16(const UpdateArgs &a, int nb, int half, float (&bias16)[16]) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int m = 8 * q + 4 * half + t;
            const int n = nb * 32 + (a.compute_dt != 0 ? block_column<1>(m) : m);
            bias16[4 * q + t] = (a.bias && n < a.d_out) ? a.bias[n] : 0.f;
        }
}

// Stage the wave's eight rows of the tile (generic kernel).  A row is covered
// by 256-column segments of 4 columns per lane; every load is issued
// unconditionally (rows past the end of the ready list, lanes past the row
// width and vertices without in-edges read a valid dummy location whose value
// is dropped) and kept raw in registers, so all loads of the wave are in flight
// together before the first is used (skipping the dummy loads with a wave-uniform
// branch was measured: 2.69 against 2.58 ms at d = 256).  d_in <= 512: at most 16 items.
template <int CT> struct OwnRaw4 { using type = float4; };
template <> struct OwnRaw4<1> { using type = uint2; };
template <> struct OwnRaw4<2> { using type = uint2; };
template <int CT> __device__ __forceinline__ float4 own_to_f32(typename OwnRaw4<CT>::type u);
template <> __device__ __forceinline__ float4 own_to_f32<2>(uint2 u) {   // four IEEE halves -> fp32
    return make_float4(f16_bits_to_f32(static_cast<uint16_t>(u.x)), f16_bits_to_f32(static_cast<uint16_t>(u.x >> 16)),
                       f16_bits_to_f32(static_cast<uint16_t>(u.y)), f16_bits_to_f32(static_cast<uint16_t>(u.y >> 16)));
}
template <> __device__ __forceinline__ float4 own_to_f32<1>(uint2 u) {   // four bf16 -> fp32
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                       __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u));
}
template <> __device__ __forceinline__ float4 own_to_f32<0>(float4 v) { return v; }

template <int CT, int SEGS>
__device__ __forceinline__ void gather_own_rows(const UpdateArgs &a, typename Elem<CT>::type *A, int stride,
                                                int w, int lane, int32_t idv);

template <int CT, int SEGS>
__device__ __forceinline__ void gather_rows(const UpdateArgs &a, typename Elem<CT>::type *A, int stride,
                                            int w, int lane, int32_t idv, int32_t rowv, float scalev,
                                            int has_aggv) {
    constexpr int kRows = kTileRows / 8;  // rows per wave
    constexpr int nitems = SEGS * kRows;  // 256-column segments per row x rows
    constexpr int kBatch = 8;             // loads in flight per pass
    const int d = a.d_in;
    const int c4 = lane * 4;
    const int acc_base = a.model == 0 ? d : 0;  // SAGE: own row first, then the neighbour mean
    auto row_of = [&](int item) { return item / SEGS; };
    auto col_of = [&](int item) { return (item % SEGS) * 256 + c4; };
    if (a.model == 3) {   // GIN: sum + self_scale * own row, rounded once
#pragma unroll
        for (int base = 0; base < nitems; base += kBatch) {
            float4 v[kBatch];
            typename OwnRaw4<CT>::type o[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const int rr = row_of(base + i), col = col_of(base + i);
                const int32_t id = __builtin_amdgcn_readlane(idv, rr);
                const bool fetch = id >= 0 && __builtin_amdgcn_readlane(has_aggv, rr) != 0;
                const int cc = col < d ? col : 0;
                const int32_t ar = __builtin_amdgcn_readlane(rowv, rr);
                v[i] = *reinterpret_cast<const float4 *>(a.acc + static_cast<int64_t>(fetch ? ar : 0) * d + cc);
                const int64_t oo = static_cast<int64_t>(id >= 0 ? id : 0) * d + cc;
                if constexpr (CT) o[i] = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(a.self_rows) + oo);
                else o[i] = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.self_rows) + oo);
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const int rr = row_of(base + i), col = col_of(base + i);
                if (col >= d) continue;
                const bool has_agg = __builtin_amdgcn_readlane(has_aggv, rr) != 0;
                const float4 own = own_to_f32<CT>(o[i]);
                const float x0 = (has_agg ? v[i].x : 0.f) + a.self_scale * own.x;
                const float x1 = (has_agg ? v[i].y : 0.f) + a.self_scale * own.y;
                const float x2 = (has_agg ? v[i].z : 0.f) + a.self_scale * own.z;
                const float x3 = (has_agg ? v[i].w : 0.f) + a.self_scale * own.w;
                typename Elem<CT>::type *dst = A + (w * kRows + rr) * stride + col;
                if constexpr (CT) {
                    *reinterpret_cast<uint2 *>(dst) = make_uint2(pack2<CT>(x0, x1), pack2<CT>(x2, x3));
                } else {
                    dst[0] = x0;
                    dst[1] = x1;
                    dst[2] = x2;
                    dst[3] = x3;
                }
            }
        }
        return;
    }
#pragma unroll
    for (int base = 0; base < nitems; base += kBatch) {
        float4 v[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int rr = row_of(base + i), col = col_of(base + i);
            const int32_t id = __builtin_amdgcn_readlane(idv, rr);
            const bool fetch = id >= 0 && __builtin_amdgcn_readlane(has_aggv, rr) != 0;
            const int32_t ar = __builtin_amdgcn_readlane(rowv, rr);
            const int64_t o = static_cast<int64_t>(fetch ? ar : 0) * d + (col < d ? col : 0);
            v[i] = *reinterpret_cast<const float4 *>(a.acc + o);
        }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int rr = row_of(base + i), col = col_of(base + i);
            if (col >= d) continue;
            const float g = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(scalev), rr));
            // a vertex without in-edges never had its accumulator written: its aggregate is zero
            const bool has_agg = __builtin_amdgcn_readlane(has_aggv, rr) != 0;
            typename Elem<CT>::type *dst = A + (w * kRows + rr) * stride + acc_base + col;
            if constexpr (CT) {
                const uint32_t lo = pack2<CT>(v[i].x * g, v[i].y * g), hi = pack2<CT>(v[i].z * g, v[i].w * g);
                *reinterpret_cast<uint2 *>(dst) = make_uint2(has_agg ? lo : 0u, has_agg ? hi : 0u);
            } else {
                dst[0] = has_agg ? v[i].x * g : 0.f;
                dst[1] = has_agg ? v[i].y * g : 0.f;
                dst[2] = has_agg ? v[i].z * g : 0.f;
                dst[3] = has_agg ? v[i].w * g : 0.f;
            }
        }
    }
    if (a.model != 0) return;
    gather_own_rows<CT, SEGS>(a, A, stride, w, lane, idv);
}

// Rows of `self_rows` (storage dtype) into columns [0, d_in) of the A tile: the
// SAGE own rows, or the whole operand of a plain row transform (model 4).
template <int CT, int SEGS>
__device__ __forceinline__ void gather_own_rows(const UpdateArgs &a, typename Elem<CT>::type *A, int stride,
                                                int w, int lane, int32_t idv) {
    constexpr int kRows = kTileRows / 8;
    constexpr int nitems = SEGS * kRows;
    constexpr int kBatch = 8;
    const int d = a.d_in;
    const int c4 = lane * 4;
    auto row_of = [&](int item) { return item / SEGS; };
    auto col_of = [&](int item) { return (item % SEGS) * 256 + c4; };
    // rows past the list's end are stored as loaded and never used
#pragma unroll
    for (int base = 0; base < nitems; base += kBatch) {
        typename OwnRaw4<CT>::type v[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int rr = row_of(base + i), col = col_of(base + i);
            const int32_t id = __builtin_amdgcn_readlane(idv, rr);
            const int64_t o = static_cast<int64_t>(id >= 0 ? id : 0) * d + (col < d ? col : 0);
            if constexpr (CT) v[i] = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(a.self_rows) + o);
            else v[i] = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.self_rows) + o);
        }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int rr = row_of(base + i), col = col_of(base + i);
            if (col >= d) continue;
            typename Elem<CT>::type *dst = A + (w * kRows + rr) * stride + col;
            if constexpr (CT) {
                *reinterpret_cast<uint2 *>(dst) = v[i];   // bf16 rows go in as loaded
            } else {
                dst[0] = v[i].x;
                dst[1] = v[i].y;
                dst[2] = v[i].z;
                dst[3] = v[i].w;
            }
        }
    }
}

// ---- generic variant: W streamed from L2, one A tile in LDS ------------------
//
// A workgroup of 8 waves takes a tile of 64 ready rows; two or more workgroups
// share a CU, so one's gather overlaps another's contraction.  BOTH_MB (more
// than four column blocks): wave w computes column block w for both 32-row
// halves, so a W fragment fetched from L2 feeds two matrix instructions;
// otherwise wave w computes column block w % 4 of half w / 4.  The W fragments
// of the next four k-steps are fetched while the current four are multiplied.
constexpr int kGenBlock = 512;

template <int CT, bool BOTH_MB>
__global__ __launch_bounds__(kGenBlock, 4) void k_update(UpdateArgs a) {
    using elem_t = typename Elem<CT>::type;
    using frag_t = typename Frag<CT>::type;
    extern __shared__ __align__(16) unsigned char smem[];
    int32_t *ids = reinterpret_cast<int32_t *>(smem);                 // [64]
    elem_t *A = reinterpret_cast<elem_t *>(smem + kTileRows * sizeof(int32_t));
    const int K = a.K;
    const int stride = K + lds_pad(CT);
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int NB = (a.d_out + 31) / 32;
    constexpr int kStepK = CT ? 16 : 2;   // k per matrix instruction
    constexpr int kFrag = CT ? 8 : 1;     // W / A elements per lane and instruction
    constexpr int kUnroll = 4;
    constexpr int kMB = BOTH_MB ? 2 : 1;
    constexpr int kRows = kTileRows / 8;
    const int KS = K / kStepK;
    const int G = KS / kUnroll;              // K is a multiple of 64: KS is a multiple of 4

    const bool dense = a.identity_rows > 0;
    const int head = dense ? 0 : a.counters[CTR_READY_HEAD];
    const int tail = dense ? static_cast<int>(a.identity_rows) : a.counters[CTR_READY_TAIL];
    const int ntiles = (tail - head + kTileRows - 1) / kTileRows;

    const int nb = BOTH_MB ? w : (w & 3);
    const int mb0 = BOTH_MB ? 0 : (w >> 2);
    const bool works = nb < NB;                               // waves past the last block compute and discard
    const int nbc = works ? nb : NB - 1;
    const elem_t *wp = static_cast<const elem_t *>(a.packed_w) + (static_cast<size_t>(nbc) * KS * 64 + lane) * kFrag;
    const int a_off = (mb0 * 32 + (lane & 31)) * stride + (lane >> 5) * kFrag;
    auto load_w = [&](int g, frag_t (&f)[kUnroll]) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            f[u] = *reinterpret_cast<const frag_t *>(wp + static_cast<size_t>(g * kUnroll + u) * 64 * kFrag);
    };

    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        __syncthreads();  // previous tile's LDS readers are done
        // ---- gather: wave w stages rows w*8 .. w*8+7; lane r < 8 holds row r's id ----
        int32_t idv = -1;
        int32_t rowv = 0;   // accumulator row of the vertex: its id, or its slot in a bounded store
        float scalev = 1.f;
        int has_aggv = 1;
        if (lane < kRows) {
            const int idx = head + tile * kTileRows + w * kRows + lane;
            if (idx < tail) {
                idv = dense ? idx : a.ready[idx];
                const int32_t deg = a.indeg ? a.indeg[idv] : 1;
                if (deg <= 0) has_aggv = 0;
                rowv = a.slot_of ? a.slot_of[idv] : idv;
                const float fd = static_cast<float>(deg > 0 ? deg : 1);
                // SAGE: mean = sum * (1/deg); GCN: deg^-1/2; a plain linear map (model 2): 1
                scalev = a.model == 0 ? 1.0f / fd : (a.model == 1 ? 1.0f / sqrtf(fd) : 1.0f);
            }
            ids[w * kRows + lane] = idv;
        }
        frag_t wcur[kUnroll];
        load_w(0, wcur);   // on its way while the rows are gathered
        if (a.model == 4) {   // plain rows in the storage dtype, up to 1024 wide
            if (a.d_in > 512) gather_own_rows<CT, 4>(a, A, stride, w, lane, idv);
            else if (a.d_in > 256) gather_own_rows<CT, 2>(a, A, stride, w, lane, idv);
            else gather_own_rows<CT, 1>(a, A, stride, w, lane, idv);
        } else if (a.d_in > 256) {
            gather_rows<CT, 2>(a, A, stride, w, lane, idv, rowv, scalev, has_aggv);
        } else {
            gather_rows<CT, 1>(a, A, stride, w, lane, idv, rowv, scalev, has_aggv);
        }
        __syncthreads();

        // ---- contraction, as D^T blocks; the bias is the initial accumulator ----
        f32x16_t c[kMB];
        {
            float b16[16];   // re-read per tile (cache hit) rather than held in registers
            load_bias16(a, nbc, lane >> 5, b16);
#pragma unroll
            for (int m = 0; m < kMB; ++m)
#pragma unroll
                for (int r = 0; r < 16; ++r) c[m][r] = b16[r];
        }
        for (int g = 0; g < G; ++g) {
            frag_t wnxt[kUnroll];
            load_w(g + 1 < G ? g + 1 : g, wnxt);   // the last group re-reads itself
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int kk = g * kUnroll + u;
#pragma unroll
                for (int m = 0; m < kMB; ++m) {
                    const frag_t av = *reinterpret_cast<const frag_t *>(A + a_off + m * 32 * stride + kk * kStepK);
                    c[m] = mfma_block<CT>(wcur[u], av, c[m]);
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) wcur[u] = wnxt[u];
        }

        // ---- epilogue: activation, store row of the next layer ----
        if (works) {
#pragma unroll
            for (int m = 0; m < kMB; ++m) {
                const int32_t id = ids[(mb0 + m) * 32 + (lane & 31)];
                if (id >= 0) store_block_row<false>(a, c[m], id, nb, lane >> 5, nullptr);
            }
        }
    }
}

// ---- dense transform: contiguous 16-bit rows times W, K-sliced ---------------
//
// The chunk transform of the transform-first order multiplies a dense block
// of rows (up to 1024 wide) by W.  The generic kernel stages whole rows (one
// workgroup per CU at that width) and every wave streams its W fragments from
// L2 once per 64 rows, which is what bounds it.  Here a workgroup of 8 waves
// owns 128 rows and walks K in slices of 64 columns: the next slice of the
// rows is in flight from HBM to registers (and the wave's next W fragments
// from L2) while the matrix cores work on the current one out of a
// double-buffered LDS tile of 2 x 18 KB, two workgroups per CU.  Wave w
// computes all 128 rows times column block w, so a W fragment is fetched once
// per 128 rows.
constexpr int kDenseRows = 128;
constexpr int kDenseSlice = 64;
constexpr int kDenseStride = kDenseSlice + 8;   // elements; 144 B rows keep 16-byte reads aligned and spread banks
constexpr int kDenseBlock = 512;
constexpr int kDenseMB = kDenseRows / 32;

template <int CT>
__global__ __launch_bounds__(kDenseBlock, 2) void k_dense_transform(UpdateArgs a) {
    static_assert(CT == 1 || CT == 2, "16-bit compute types only");
    using frag_t = typename Frag<CT>::type;
    __shared__ __align__(16) uint16_t A[2][kDenseRows * kDenseStride];
    const int K = a.K;
    const int KS = K / 16;                     // k-steps of one matrix instruction
    const int nslices = K / kDenseSlice;
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int NB = (a.d_out + 31) / 32;
    const bool works = w < NB;
    const int nb = works ? w : NB - 1;         // waves past the last column block compute and discard
    const int64_t n = a.identity_rows;
    const int64_t ntiles = (n + kDenseRows - 1) / kDenseRows;
    const uint16_t *X = static_cast<const uint16_t *>(a.self_rows);
    const uint16_t *Wp = static_cast<const uint16_t *>(a.packed_w) + (static_cast<size_t>(nb) * KS * 64 + lane) * 8;

    // staging: thread t moves 16 bytes of row t / 8 (and of row 64 + t / 8), columns (t % 8) * 8 .. + 7 of the slice
    const int st_row = threadIdx.x >> 3;
    const int st_col = (threadIdx.x & 7) * 8;
    const int a_off = (lane & 31) * kDenseStride + (lane >> 5) * 8;

    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t row0 = tile * kDenseRows;
        int64_t r0 = row0 + st_row, r1 = row0 + 64 + st_row;
        if (r0 >= n) r0 = n - 1;               // rows past the end read the last row; their results are dropped
        if (r1 >= n) r1 = n - 1;
        const uint16_t *x0 = X + r0 * K + st_col;
        const uint16_t *x1 = X + r1 * K + st_col;
        auto load_w = [&](int slice, frag_t (&f)[4]) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                f[u] = *reinterpret_cast<const frag_t *>(Wp + static_cast<size_t>(slice * 4 + u) * 64 * 8);
        };

        f32x16_t c[kDenseMB];
#pragma unroll
        for (int m = 0; m < kDenseMB; ++m)
#pragma unroll
            for (int r = 0; r < 16; ++r) c[m][r] = 0.f;

        frag_t wcur[4];
        load_w(0, wcur);
        uint4 g0 = *reinterpret_cast<const uint4 *>(x0);
        uint4 g1 = *reinterpret_cast<const uint4 *>(x1);
        *reinterpret_cast<uint4 *>(&A[0][st_row * kDenseStride + st_col]) = g0;
        *reinterpret_cast<uint4 *>(&A[0][(64 + st_row) * kDenseStride + st_col]) = g1;
        __syncthreads();
        for (int sl = 0; sl < nslices; ++sl) {
            const bool more = sl + 1 < nslices;
            frag_t wnxt[4];
            if (more) {
                g0 = *reinterpret_cast<const uint4 *>(x0 + (sl + 1) * kDenseSlice);
                g1 = *reinterpret_cast<const uint4 *>(x1 + (sl + 1) * kDenseSlice);
            }
            load_w(more ? sl + 1 : sl, wnxt);  // the last slice re-reads itself
            const uint16_t *Ab = A[sl & 1] + a_off;
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int m = 0; m < kDenseMB; ++m) {
                    const frag_t av = *reinterpret_cast<const frag_t *>(Ab + m * 32 * kDenseStride + u * 16);
                    c[m] = mfma_block<CT>(wcur[u], av, c[m]);
                }
            if (more) {
                uint16_t *An = A[(sl + 1) & 1];
                *reinterpret_cast<uint4 *>(&An[st_row * kDenseStride + st_col]) = g0;
                *reinterpret_cast<uint4 *>(&An[(64 + st_row) * kDenseStride + st_col]) = g1;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) wcur[u] = wnxt[u];
            __syncthreads();   // the slice just written is complete; the one just read may be overwritten
        }

        if (works) {
#pragma unroll
            for (int m = 0; m < kDenseMB; ++m) {
                const int64_t row = row0 + m * 32 + (lane & 31);
                if (row < n) store_block_row<false>(a, c[m], row, nb, lane >> 5, nullptr);
            }
        }
    }
}

// ---- pipelined variant: W resident in LDS, double-buffered A tile -----------
//
// Used when d_in <= 128 and W plus two A tiles fit in LDS.  One workgroup of
// 8 waves per CU loops over 64-row tiles.  While the matrix cores work on tile
// t (A and W both read from LDS), the global loads of tile t+1's rows are
// already in flight into registers and the ready ids of tile t+2 are being
// fetched, so the gather latency is hidden behind the contraction instead of
// being exposed once per tile.
//
// With two waves per SIMD the kernel is bound by instruction issue long before
// the matrix cores or HBM are busy, so the staging code is written for few
// vector instructions per row: half a wave covers a row (16 bytes of the
// accumulator and 8 or 16 bytes of the own row per lane, two rows per load
// instruction), per-row values sit in the lanes of a quad and are spread with
// DPP quad broadcasts, the bias is the initial value of the MFMA accumulator,
// and the k-loop is fully unrolled so every LDS read has an immediate offset.
constexpr int kPipeBlock = 512;
constexpr int kPipeRows = kTileRows / (kPipeBlock / 64);  // rows staged per wave = 8
constexpr int kPipeIters = kPipeRows / 2;                 // two rows per load instruction

template <int CT>
struct RowRegs {
    float4 acc[kPipeIters];
    typename OwnRaw4<CT>::type own[kPipeIters];
};

template <int CTRL>
__device__ __forceinline__ int32_t dpp_quad(int32_t v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
// value held by lane (quad base + i) of every lane's quad; i is a constant after unrolling
__device__ __forceinline__ int32_t quad_bcast(int32_t v, int i) {
    switch (i) {
        case 0: return dpp_quad<0x00>(v);
        case 1: return dpp_quad<0x55>(v);
        case 2: return dpp_quad<0xAA>(v);
        default: return dpp_quad<0xFF>(v);
    }
}

// Issue the loads of the wave's 8 rows: lanes 0..31 take row 2i, lanes 32..63
// row 2i+1 in round i.  `idv` / `degv` hold, in lane l, the values of row
// 2 (l % 4) + l / 32.  Rows past the end of the ready list read row 0 and are
// dropped when the tile is stored.  The accumulator of a vertex without
// in-edges is not loaded (nothing was ever added to its row): the half-wave
// of that row is masked off for the load, which costs no wait, while a dummy
// load of a cached row still took its 512 bytes of the CU's load path (half
// of all vertices at scale 26: 11.2 -> 10.6 ms per layer).
// A vertex whose row was handed over by the aggregation (bit 31 of its ready-list entry, `handv` != 0 in the
// lane that holds the row's id) has the finished operand -- normalised, rounded to the compute type -- in the
// first half of its accumulator row.  The load stays one unconditional 16-byte load per lane; only its
// address differs: lanes 2k and 2k + 1 of the half-wave both read bytes 16 k .. 16 k + 15 of the row (eight
// 16-bit values, four for each of them), so such a row costs 256 bytes of traffic instead of 512, and
// pipe_store_rows picks the lane's half.  Straight-line code: this kernel is bound by instruction issue.
template <int CT, int OWN, bool HAND>
__device__ __forceinline__ void pipe_issue_rows(const UpdateArgs &a, int32_t idv, int32_t degv, int32_t slotv,
                                                int32_t handv, int lane, RowRegs<CT> &r) {
    const int d = a.d_in;
    const int c4 = (lane & 31) * 4;
    const int col = c4 < d ? c4 : 0;
    const int col_handed = ((lane & 31) >> 1) * 4;   // in floats: byte 16 * (l / 2) of the row
#pragma unroll
    for (int i = 0; i < kPipeIters; ++i) {
        const int32_t id = quad_bcast(idv, i);
        const int32_t dg = quad_bcast(degv, i);
        const int32_t row = id >= 0 ? id : 0;
        const int32_t arow = a.slot_of ? quad_bcast(slotv, i) : row;
        r.acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        int acol = col;
        if constexpr (HAND) acol = quad_bcast(handv, i) != 0 ? col_handed : col;
        if (dg > 0) r.acc[i] = *reinterpret_cast<const float4 *>(a.acc + static_cast<int64_t>(arow) * d + acol);
        if constexpr (OWN != 0) {
            const int64_t o = static_cast<int64_t>(row) * d + col;
            if constexpr (CT) r.own[i] = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(a.self_rows) + o);
            else r.own[i] = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.self_rows) + o);
        }
    }
}

// Normalise and convert the rows loaded by pipe_issue_rows and store them into
// the A tile.  Rows past the end of the ready list are stored as they came:
// a row of A only feeds the same row of the product, which is never written.
template <int CT, int OWN, bool HAND>
__device__ __forceinline__ void pipe_store_rows(const UpdateArgs &a, typename Elem<CT>::type *A, int stride,
                                                int w, int lane, const RowRegs<CT> &r, int32_t degv, int32_t handv) {
    const int d = a.d_in;
    const int c4 = (lane & 31) * 4;
    const float fd = static_cast<float>(degv > 0 ? degv : 1);
    // SAGE: mean = sum * (1/deg); GCN: deg^-1/2; plain linear map: 1
    const float scalev = a.model == 0 ? 1.0f / fd : (a.model == 1 ? 1.0f / sqrtf(fd) : 1.0f);
    if (c4 >= d) return;
    typename Elem<CT>::type *row0 = A + (w * kPipeRows + (lane >> 5)) * stride + c4 + (OWN == 1 ? d : 0);
#pragma unroll
    for (int i = 0; i < kPipeIters; ++i) {
        const float g = __uint_as_float(static_cast<uint32_t>(quad_bcast(static_cast<int32_t>(__float_as_uint(scalev)), i)));
        // a vertex without in-edges never had its accumulator written: its aggregate is zero
        const bool has_agg = quad_bcast(degv, i) > 0;
        typename Elem<CT>::type *row = row0 + 2 * i * stride;
        float4 v = r.acc[i];
        v.x *= g;
        v.y *= g;
        v.z *= g;
        v.w *= g;
        if constexpr (OWN == 2) {   // GIN: sum + self_scale * own row, rounded once
            const float4 own = own_to_f32<CT>(r.own[i]);
            v.x = (has_agg ? v.x : 0.f) + a.self_scale * own.x;
            v.y = (has_agg ? v.y : 0.f) + a.self_scale * own.y;
            v.z = (has_agg ? v.z : 0.f) + a.self_scale * own.z;
            v.w = (has_agg ? v.w : 0.f) + a.self_scale * own.w;
        }
        const bool keep = OWN == 2 || has_agg;
        if constexpr (CT) {
            uint32_t lo = pack2<CT>(v.x, v.y), hi = pack2<CT>(v.z, v.w);
            if constexpr (HAND) {
                // handed over: the 16 bytes loaded are the operand's values of this lane and its neighbour
                const bool handed = quad_bcast(handv, i) != 0;
                const bool odd = (lane & 1) != 0;
                const uint32_t hlo = __float_as_uint(odd ? r.acc[i].z : r.acc[i].x);
                const uint32_t hhi = __float_as_uint(odd ? r.acc[i].w : r.acc[i].y);
                lo = handed ? hlo : lo;
                hi = handed ? hhi : hi;
            }
            *reinterpret_cast<uint2 *>(row) = make_uint2(keep ? lo : 0u, keep ? hi : 0u);
            // bf16 own rows go to LDS as they were loaded; the aggregate is rounded once
            if constexpr (OWN == 1) *reinterpret_cast<uint2 *>(row - d) = r.own[i];
        } else {
            row[0] = keep ? v.x : 0.f;
            row[1] = keep ? v.y : 0.f;
            row[2] = keep ? v.z : 0.f;
            row[3] = keep ? v.w : 0.f;
            if constexpr (OWN == 1) {
                row[0 - d] = r.own[i].x;
                row[1 - d] = r.own[i].y;
                row[2 - d] = r.own[i].z;
                row[3 - d] = r.own[i].w;
            }
        }
    }
}

// acc (+)= A[32 rows of mb] x W[32 columns of nb] over KS k-steps, as D^T.
// KS > 0: compile-time trip count, fully unrolled (immediate LDS offsets);
// KS == 0: run-time trip count `ks`, a multiple of 4, in groups of four whose
// LDS reads are issued one group ahead of the matrix instructions.
template <int CT, int KS>
__device__ __forceinline__ void contract_block(const typename Elem<CT>::type *arow,
                                               const typename Elem<CT>::type *wfrag, int ks, f32x16_t &c) {
    if constexpr (CT && KS > 0) {
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            using frag16_t = typename Frag<CT>::type;
            const frag16_t av = *reinterpret_cast<const frag16_t *>(arow + kk * 16);
            const frag16_t bv = *reinterpret_cast<const frag16_t *>(wfrag + kk * 64 * 8);
            c = mfma_block<CT>(bv, av, c);
        }
    } else {
        constexpr int kUnroll = 4;
        using frag_t = typename Frag<CT>::type;
        auto load = [&](int kk, frag_t &af, frag_t &bf) {
            if constexpr (CT) {
                af = *reinterpret_cast<const frag_t *>(arow + kk * 16);
                bf = *reinterpret_cast<const frag_t *>(wfrag + static_cast<size_t>(kk) * 64 * 8);
            } else {
                af = arow[kk * 2];
                bf = wfrag[static_cast<size_t>(kk) * 64];
            }
        };
        frag_t av[kUnroll], bv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) load(u, av[u], bv[u]);
        for (int kk = 0; kk < ks; kk += kUnroll) {
            frag_t an[kUnroll], bn[kUnroll];
            const int nxt = kk + kUnroll < ks ? kk + kUnroll : kk;  // the last group re-reads itself
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) load(nxt + u, an[u], bn[u]);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                c = mfma_block<CT>(bv[u], av[u], c);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                av[u] = an[u];
                bv[u] = bn[u];
            }
        }
    }
}

template <int CT, int PPW, int OWN, bool HAND>
__global__ __launch_bounds__(kPipeBlock) void k_update_pipelined(UpdateArgs a) {
    using elem_t = typename Elem<CT>::type;
    extern __shared__ __align__(16) unsigned char smem[];
    const int K = a.K;
    const int stride = K + lds_pad(CT);
    const int NB = (a.d_out + 31) / 32;
    constexpr int kStepK = CT ? 16 : 2;
    const int KS = K / kStepK;
    const size_t w_elems = static_cast<size_t>(NB) * 32 * K;
    const size_t a_elems = static_cast<size_t>(kTileRows) * stride;
    int32_t *ids = reinterpret_cast<int32_t *>(smem);  // [2][64]
    elem_t *Wl = reinterpret_cast<elem_t *>(smem + 2 * kTileRows * sizeof(int32_t));
    elem_t *A0 = Wl + ((w_elems + 7) & ~static_cast<size_t>(7));
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int my_row = 2 * (lane & 3) + (lane >> 5);   // the row of the wave's eight whose id this lane holds

    const bool dense = a.identity_rows > 0;
    const int head = dense ? 0 : a.counters[CTR_READY_HEAD];
    const int tail = dense ? static_cast<int>(a.identity_rows) : a.counters[CTR_READY_TAIL];
    const int ntiles = (tail - head + kTileRows - 1) / kTileRows;
    if (static_cast<int>(blockIdx.x) >= ntiles) return;

    {  // W -> LDS, 16 bytes per thread per step
        const uint4 *src = static_cast<const uint4 *>(a.packed_w);
        uint4 *dst = reinterpret_cast<uint4 *>(Wl);
        const size_t vecs = w_elems * sizeof(elem_t) / 16;
        for (size_t i = threadIdx.x; i < vecs; i += kPipeBlock) dst[i] = src[i];
    }

    // ready-list entries: vertex id, bit 31 set when the aggregation handed the finished row over; -1: no row
    auto load_ids = [&](int tile) -> int32_t {
        int32_t id = -1;
        if (tile < ntiles) {
            const int idx = head + tile * kTileRows + w * kPipeRows + my_row;
            if (idx < tail) id = dense ? idx : a.ready[idx];
        }
        return id;
    };
    auto handed_of = [](int32_t raw) -> int32_t { return HAND && raw != -1 && raw < 0 ? 1 : 0; };
    auto vertex_of = [](int32_t raw) -> int32_t { return HAND ? (raw == -1 ? -1 : raw & 0x7fffffff) : raw; };
    auto load_deg = [&](int32_t id) -> int32_t { return (a.indeg && id >= 0) ? a.indeg[id] : 1; };
    // bounded store: the slot that holds the vertex's accumulator row (-1 for vertices without in-edges,
    // whose row is never fetched)
    auto load_slot = [&](int32_t id) -> int32_t { return (a.slot_of && id >= 0) ? a.slot_of[id] : 0; };

    // per (mb, nb) block of this wave: LDS addresses and the bias as the initial accumulator
    f32x16_t bj[PPW];
    int a_off[PPW];
    const elem_t *wfrag[PPW];
#pragma unroll
    for (int i = 0; i < PPW; ++i) {
        const int p = w + 8 * i;
        const int nb = p % NB, mb = (p / NB) & 1;   // waves past the last block compute and discard
        float b16[16];
        load_bias16(a, nb, lane >> 5, b16);
#pragma unroll
        for (int r = 0; r < 16; ++r) bj[i][r] = b16[r];
        if constexpr (CT) {
            a_off[i] = (mb * 32 + (lane & 31)) * stride + (lane >> 5) * 8;
            wfrag[i] = Wl + (static_cast<size_t>(nb) * KS * 64 + lane) * 8;
        } else {
            a_off[i] = (mb * 32 + (lane & 31)) * stride + (lane >> 5);
            wfrag[i] = Wl + static_cast<size_t>(nb) * KS * 64 + lane;
        }
    }

    // Two tiles of rows are in flight in registers (r0: this workgroup's next
    // tile, r1: the one after it); the in-degrees of the tile after those and
    // the ready ids of the one after that are on their way.  Every step stores
    // one register set to LDS, refills it with the tile two steps ahead and
    // runs the contraction of the stored tile.
    int tile = blockIdx.x;
    const int G = gridDim.x;
    int32_t raw0 = load_ids(tile), raw1 = load_ids(tile + G), raw_a = load_ids(tile + 2 * G);
    int32_t id_b = load_ids(tile + 3 * G);   // still raw: cleaned when it moves up
    int32_t id0 = vertex_of(raw0), id1 = vertex_of(raw1), id_a = vertex_of(raw_a);
    int32_t hand0 = handed_of(raw0), hand1 = handed_of(raw1), hand_a = handed_of(raw_a);
    int32_t deg0 = load_deg(id0), deg1 = load_deg(id1), deg_a = load_deg(id_a);
    int32_t slot_a = load_slot(id_a);
    RowRegs<CT> r0, r1;
    pipe_issue_rows<CT, OWN, HAND>(a, id0, deg0, load_slot(id0), hand0, lane, r0);
    __builtin_amdgcn_sched_barrier(0);   // keep the two sets' loads in this order, as in the loop
    pipe_issue_rows<CT, OWN, HAND>(a, id1, deg1, load_slot(id1), hand1, lane, r1);

    auto step = [&](RowRegs<CT> &regs, int32_t &idv, int32_t &degv, int32_t &handv, int buf) {
        elem_t *A = A0 + buf * a_elems;
        int32_t *tids = ids + buf * kTileRows;
        pipe_store_rows<CT, OWN, HAND>(a, A, stride, w, lane, regs, degv, handv);
        if ((lane & 31) < 4) tids[w * kPipeRows + my_row] = idv;
        __syncthreads();
        idv = id_a;
        degv = deg_a;
        handv = hand_a;
        const int32_t slotv = slot_a;
        id_a = vertex_of(id_b);
        hand_a = handed_of(id_b);
        deg_a = load_deg(id_a);
        slot_a = load_slot(id_a);
        id_b = load_ids(tile + 4 * G);
        pipe_issue_rows<CT, OWN, HAND>(a, idv, degv, slotv, handv, lane, regs);

        f32x16_t c[PPW];
#pragma unroll
        for (int i = 0; i < PPW; ++i) {
            c[i] = bj[i];
            const elem_t *arow = A + a_off[i];
            if constexpr (CT) {
                switch (KS) {
                    case 4: contract_block<CT, 4>(arow, wfrag[i], KS, c[i]); break;
                    case 8: contract_block<CT, 8>(arow, wfrag[i], KS, c[i]); break;
                    case 16: contract_block<CT, 16>(arow, wfrag[i], KS, c[i]); break;
                    default: contract_block<CT, 0>(arow, wfrag[i], KS, c[i]); break;
                }
            } else {
                contract_block<0, 0>(arow, wfrag[i], KS, c[i]);
            }
        }
#pragma unroll
        for (int i = 0; i < PPW; ++i) {
            const int p = w + 8 * i;
            if (p >= 2 * NB) continue;
            const int nb = p % NB, mb = p / NB;
            const int32_t id = tids[mb * 32 + (lane & 31)];
            if (id >= 0) store_block_row<false>(a, c[i], id, nb, lane >> 5, nullptr);
        }
    };

    // Both steps run in every round (the second on an empty tile when the
    // workgroup's tile count is odd: ids of -1, nothing stored).  With an exit
    // between them the compiler has to assume that a round may start right
    // after the first step's loads were issued, and then waits for them all.
    for (; tile < ntiles; tile += G) {
        step(r0, id0, deg0, hand0, 0);
        tile += G;
        step(r1, id1, deg1, hand1, 1);
    }
}

size_t pipelined_lds_bytes(int K, int d_out, bool bf16c) {
    const int NB = (d_out + 31) / 32;
    const size_t es = bf16c ? 2 : 4;
    const size_t w_elems = (static_cast<size_t>(NB) * 32 * K + 7) & ~static_cast<size_t>(7);
    return 2 * kTileRows * sizeof(int32_t) + w_elems * es +
           2 * static_cast<size_t>(kTileRows) * (K + lds_pad(bf16c)) * es;
}

template <int CT, int PPW, int OWN, bool HAND>
hipError_t launch_pipelined_t(const UpdateArgs &a, int grid, hipStream_t s) {
    const size_t lds = pipelined_lds_bytes(a.K, a.d_out, CT);
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_update_pipelined<CT, PPW, OWN, HAND>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL((k_update_pipelined<CT, PPW, OWN, HAND>), dim3(grid), dim3(kPipeBlock), lds, s, a);
    return hipGetLastError();
}

template <int CT, int OWN>
hipError_t launch_pipelined_o(const UpdateArgs &a, int grid, hipStream_t s) {
    const int NB = (a.d_out + 31) / 32;
    if constexpr (CT != 0 && OWN != 2) {
        // the ready list may hold rows handed over by the aggregation (bit 31 of the entry)
        if (a.handed_rows)
            return 2 * NB <= 8 ? launch_pipelined_t<CT, 1, OWN, true>(a, grid, s)
                               : launch_pipelined_t<CT, 2, OWN, true>(a, grid, s);
    }
    return 2 * NB <= 8 ? launch_pipelined_t<CT, 1, OWN, false>(a, grid, s)
                       : launch_pipelined_t<CT, 2, OWN, false>(a, grid, s);
}

// own row: concatenated (SAGE), added (GIN) or unused
template <int CT>
hipError_t launch_pipelined_c(const UpdateArgs &a, int grid, hipStream_t s) {
    if (a.model == 0) return launch_pipelined_o<CT, 1>(a, grid, s);
    if (a.model == 3) return launch_pipelined_o<CT, 2>(a, grid, s);
    return launch_pipelined_o<CT, 0>(a, grid, s);
}

// Transform-first layers: one wave per ready row, four columns per lane and round.
__global__ __launch_bounds__(kBlock) void k_sum_finalize(SumFinalizeArgs a) {
    // One thread per (ready row, run of four columns), four such items in
    // flight per thread: the vertex ids of all four are read first, then their
    // degrees and rows, so a thread waits for memory three times per four
    // items instead of three times per item.
    constexpr int U = 4;
    const int head = a.counters[CTR_READY_HEAD];
    const int tail = a.counters[CTR_READY_TAIL];
    const int d = a.d_out;
    const int quads = d / 4;
    const int64_t total = static_cast<int64_t>(tail - head) * quads;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t it0 = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; it0 < total; it0 += U * stride) {
        int64_t v[U];
        int c[U];
        bool live[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            int64_t it = it0 + k * stride;
            live[k] = it < total;
            if (!live[k]) it = it0;          // a valid item; its result is dropped
            c[k] = static_cast<int>(it % quads) * 4;
            v[k] = a.ready[head + it / quads];
        }
        int32_t deg[U];
        int64_t arow[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            deg[k] = a.indeg[v[k]];
            arow[k] = a.slot_of ? static_cast<int64_t>(a.slot_of[v[k]]) : v[k];
        }
        float4 x[U], t[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            x[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            t[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (deg[k] > 0)   // the accumulator of a vertex without in-edges was never written
                x[k] = *reinterpret_cast<const float4 *>(a.acc + arow[k] * d + c[k]);
            if (a.self_term) t[k] = *reinterpret_cast<const float4 *>(a.self_term + v[k] * d + c[k]);
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const float fd = static_cast<float>(deg[k] > 0 ? deg[k] : 1);
            const float g = a.norm == 0 ? 1.0f / fd : (a.norm == 1 ? 1.0f / sqrtf(fd) : 1.0f);
            float y[4] = {x[k].x * g + a.self_scale * t[k].x, x[k].y * g + a.self_scale * t[k].y,
                          x[k].z * g + a.self_scale * t[k].z, x[k].w * g + a.self_scale * t[k].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (a.bias) y[e] += a.bias[c[k] + e];
                if (a.activation == 1) y[e] = fmaxf(y[e], 0.f);
                else if (a.activation == 2) y[e] = y[e] > 0.f ? y[e] : expm1f(y[e]);
            }
            if (!live[k]) continue;
            if (a.out_dt)
                *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(a.out) + v[k] * d + c[k]) =
                    make_uint2(pack2_dt(a.out_dt, y[0], y[1]), pack2_dt(a.out_dt, y[2], y[3]));
            else
                *reinterpret_cast<float4 *>(static_cast<float *>(a.out) + v[k] * d + c[k]) =
                    make_float4(y[0], y[1], y[2], y[3]);
        }
    }
}

// SGC hop: the ready rows of the accumulator times deg^-1/2, one wave per row.
__global__ __launch_bounds__(kBlock) void k_scale_rows(UpdateArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / 64) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / 64);
    const int head = a.counters[CTR_READY_HEAD];
    const int tail = a.counters[CTR_READY_TAIL];
    const int d = a.d_in;
    for (int64_t i = head + wave; i < tail; i += nwaves) {
        const int64_t v = a.ready[i];
        const int32_t deg = a.indeg[v];
        const float g = deg > 0 ? 1.0f / sqrtf(static_cast<float>(deg)) : 0.f;
        for (int c = lane * 4; c < d; c += 256) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (deg > 0)   // never written otherwise
                x = *reinterpret_cast<const float4 *>(a.acc + (a.slot_of ? static_cast<int64_t>(a.slot_of[v]) : v) * d + c);
            if (a.out_dt)
                *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(a.out) + v * d + c) =
                    make_uint2(pack2_dt(a.out_dt, x.x * g, x.y * g), pack2_dt(a.out_dt, x.z * g, x.w * g));
            else
                *reinterpret_cast<float4 *>(static_cast<float *>(a.out) + v * d + c) =
                    make_float4(x.x * g, x.y * g, x.z * g, x.w * g);
        }
    }
}

__global__ void k_advance_head(int32_t *counters) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        counters[CTR_READY_HEAD] = counters[CTR_READY_TAIL];
        counters[CTR_NUM_FLUSHES] += 1;
    }
}

size_t update_lds_bytes(int K, bool bf16c) {
    return kTileRows * sizeof(int32_t) +
           static_cast<size_t>(kTileRows) * (K + lds_pad(bf16c)) * (bf16c ? 2 : 4);
}

template <int CT, bool BOTH_MB>
hipError_t launch_update_t(const UpdateArgs &a, int grid, hipStream_t s) {
    const size_t lds = update_lds_bytes(a.K, CT);
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_update<CT, BOTH_MB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL((k_update<CT, BOTH_MB>), dim3(grid), dim3(kGenBlock), lds, s, a);
    return hipGetLastError();
}

template <int CT>
hipError_t launch_update_c(const UpdateArgs &a, int grid, hipStream_t s) {
    const int NB = (a.d_out + 31) / 32;
    if (NB > 8 || a.d_in > (a.model == 4 ? 1024 : 512)) return hipErrorInvalidValue;
    return NB > 4 ? launch_update_t<CT, true>(a, grid, s) : launch_update_t<CT, false>(a, grid, s);
}

}  // namespace

size_t packed_weight_bytes(int K, int d_out, int compute_dt) {
    const int NB = (d_out + 31) / 32;
    return static_cast<size_t>(NB) * 32 * K * (compute_dt ? 2 : 4);
}

hipError_t launch_pack_weights(const void *W, int w_dt, int K, int d_out, int compute_dt,
                               void *packed, hipStream_t s) {
    const int NB = (d_out + 31) / 32;
    const int64_t total = static_cast<int64_t>(NB) * 32 * K;
    const unsigned blocks = static_cast<unsigned>((total + kBlock - 1) / kBlock);
    if (compute_dt == 2)
        hipLaunchKernelGGL(k_pack_weights<2>, dim3(blocks), dim3(kBlock), 0, s, W, w_dt, K, d_out,
                           static_cast<uint16_t *>(packed));
    else if (compute_dt == 1)
        hipLaunchKernelGGL(k_pack_weights<1>, dim3(blocks), dim3(kBlock), 0, s, W, w_dt, K, d_out,
                           static_cast<uint16_t *>(packed));
    else
        hipLaunchKernelGGL(k_pack_weights<0>, dim3(blocks), dim3(kBlock), 0, s, W, w_dt, K, d_out,
                           static_cast<float *>(packed));
    return hipGetLastError();
}

// Whether launch_update runs the pipelined kernel for a flush of this shape (the kernel that knows rows handed
// over by the aggregation).
bool update_takes_handed_rows(int model, int d_in, int K, int d_out, int compute_dt) {
    return compute_dt != 0 && (model == 0 || model == 1) && d_in == 128 &&
           pipelined_lds_bytes(K, d_out, true) <= 160 * 1024;
}

hipError_t launch_update(const UpdateArgs &a, hipStream_t s) {
    if (update_lds_bytes(a.K, a.compute_dt != 0) > 160 * 1024) return hipErrorInvalidValue;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus <= 0) cus = 256;
    if (a.model == 4 && a.compute_dt != 0 && a.in_dt == a.compute_dt && a.identity_rows > 0 && a.K == a.d_in &&
        a.K % kDenseSlice == 0 && a.activation == 0 && !a.bias && a.d_out > 128) {
        // a dense block of 16-bit rows times a W of more than four column blocks: the K-sliced kernel
        if (a.d_out > 256 || a.d_in > 1024) return hipErrorInvalidValue;
        int64_t grid = static_cast<int64_t>(cus) * 2;
        const int64_t max_tiles = (a.identity_rows + kDenseRows - 1) / kDenseRows;
        if (grid > max_tiles) grid = max_tiles;
        const dim3 g(static_cast<unsigned>(grid)), b(kDenseBlock);
        if (a.compute_dt == 1) hipLaunchKernelGGL((k_dense_transform<1>), g, b, 0, s, a);
        else hipLaunchKernelGGL((k_dense_transform<2>), g, b, 0, s, a);
        return hipGetLastError();
    }
    if (a.model != 4 && a.d_in <= 128 && pipelined_lds_bytes(a.K, a.d_out, a.compute_dt != 0) <= 160 * 1024) {
        int64_t grid = cus;
        const int64_t max_tiles = (a.n + kTileRows - 1) / kTileRows;
        if (grid > max_tiles) grid = max_tiles;
        if (grid < 1) grid = 1;
        if (a.compute_dt == 2) return launch_pipelined_c<2>(a, static_cast<int>(grid), s);
        return a.compute_dt == 1 ? launch_pipelined_c<1>(a, static_cast<int>(grid), s)
                                 : launch_pipelined_c<0>(a, static_cast<int>(grid), s);
    }
    const size_t lds = update_lds_bytes(a.K, a.compute_dt != 0);
    int per_cu = static_cast<int>((160 * 1024) / lds);
    if (per_cu < 1) per_cu = 1;
    if (per_cu > 4) per_cu = 4;   // 8 waves per workgroup, 32 per CU
    int64_t grid = static_cast<int64_t>(cus) * per_cu;
    const int64_t max_tiles = (a.n + kTileRows - 1) / kTileRows;
    if (grid > max_tiles) grid = max_tiles;
    if (grid < 1) grid = 1;
    if (a.compute_dt == 2) return launch_update_c<2>(a, static_cast<int>(grid), s);
    return a.compute_dt == 1 ? launch_update_c<1>(a, static_cast<int>(grid), s)
                             : launch_update_c<0>(a, static_cast<int>(grid), s);
}

hipError_t launch_sum_finalize(const SumFinalizeArgs &a, hipStream_t s) {
    if (a.n <= 0) return hipSuccess;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus <= 0) cus = 256;
    const int64_t items = a.n * (a.d_out / 4);            // a.n bounds the rows the ready list holds
    int64_t blocks = (items + 4 * kBlock - 1) / (4 * kBlock);
    if (blocks < 1) blocks = 1;
    if (blocks > static_cast<int64_t>(cus) * 8) blocks = static_cast<int64_t>(cus) * 8;
    hipLaunchKernelGGL(k_sum_finalize, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_scale_rows(const UpdateArgs &a, hipStream_t s) {
    if (a.n <= 0) return hipSuccess;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus <= 0) cus = 256;
    int64_t blocks = (a.n + (kBlock / 64) - 1) / (kBlock / 64);
    if (blocks > static_cast<int64_t>(cus) * 8) blocks = static_cast<int64_t>(cus) * 8;
    hipLaunchKernelGGL(k_scale_rows, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_advance_head(int32_t *counters, hipStream_t s) {
    hipLaunchKernelGGL(k_advance_head, dim3(1), dim3(64), 0, s, counters);
    return hipGetLastError();
}

}  // namespace atlas
