// GAT pieces that are not edge sweeps: attention-vector folding, the attention
// prepass, the per-chunk rescale of the running softmax state, and the final
// normalisation of ready rows.  The paper names attention layers as adoptable
// but does not implement them (Sec. 3.9); the layer is the textbook GAT, run
// in the paper's broadcast form with a per-destination running maximum, sum
// and weighted accumulator.
//
// Softmax is invariant to the shift used, so the accumulated state of a
// destination is kept relative to a reference maximum m_cur that only moves
// between chunks: before a chunk's messages are added, m_next collects the
// largest logit of the chunk per (destination, head) (integer atomicMax on an
// order-preserving image of the float), destinations whose maximum moved are
// rescaled by exp(m_cur - m_next), and the chunk's messages are then added
// with weights exp(s - m_cur) <= 1.
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>

#include <type_traits>

namespace atlas {
namespace {

constexpr int kBlock = 256;

__device__ __forceinline__ float decode_max(int32_t e) {
    return __int_as_float(e >= 0 ? e : e ^ 0x7fffffff);
}

__global__ __launch_bounds__(kBlock) void k_fill_i32(int32_t *p, int32_t value, int64_t count) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < count; i += stride) p[i] = value;
}

// parameter i of an array stored as fp32 (0), bf16 (1) or IEEE half (2)
__device__ __forceinline__ float param_f32(const void *p, int dt, int64_t i) {
    if (dt == 2) return static_cast<float>(static_cast<const _Float16 *>(p)[i]);
    return dt == 1 ? __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t *>(p)[i]) << 16)
                   : static_cast<const float *>(p)[i];
}

// wa[c][h] = sum_j W[c][h*dh + j] a_src[h][j],  wa[c][heads + h] likewise with a_dst:
// a . (W^T x) = (W a) . x, so the attention terms need no transformed row.
__global__ __launch_bounds__(kBlock) void k_gat_fold_attention(const void *W, const void *a_src, const void *a_dst,
                                                               int w_dt, int d_in, int heads, int dh, float *wa) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= d_in * 2 * heads) return;
    const int c = i / (2 * heads);
    const int k = i % (2 * heads);
    const int h = k % heads;
    const void *av = k < heads ? a_src : a_dst;
    float s = 0.f;
    for (int j = 0; j < dh; ++j)
        s += param_f32(W, w_dt, static_cast<int64_t>(c) * heads * dh + h * dh + j) * param_f32(av, w_dt, h * dh + j);
    wa[i] = s;
}

// One wave per row: el[u][h] and er[u][h] for the rows of the chunk.  A lane
// keeps the folded attention columns of its (up to four) row elements in
// registers for all the rows it sees.  The 16 partial sums are reduced with a
// halving butterfly: at each of the first four steps a lane hands half of its
// values to its partner and keeps the other half, so 15 + 2 shuffles replace
// 16 x 6.
// element c of a row stored as fp32, bf16 (uint16_t) or IEEE half
template <typename T>
__device__ __forceinline__ float row_elem(const T *row, int c) {
    if constexpr (std::is_same<T, _Float16>::value) return static_cast<float>(row[c]);
    else if constexpr (sizeof(T) == 2) return __uint_as_float(static_cast<uint32_t>(row[c]) << 16);
    else return row[c];
}

template <typename T>
__global__ __launch_bounds__(kBlock) void k_gat_prepass(const T *__restrict__ emb, int64_t src_begin, int64_t src_end,
                                                        int d_in, const float *__restrict__ wa, int heads, float *el,
                                                        float *er) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / 64) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / 64);
    const int H2 = 2 * heads;
    constexpr int kRegCols = 4;  // columns lane, lane+64, lane+128, lane+192 live in registers
    float wreg[kRegCols][16];
#pragma unroll
    for (int i = 0; i < kRegCols; ++i)
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int c = lane + 64 * i;
            wreg[i][k] = (c < d_in && k < H2) ? wa[c * H2 + k] : 0.f;
        }
    // value k ends up on the lanes whose low four bits spell k with bit 0 first:
    // bit0 -> 8, bit1 -> 4, bit2 -> 2, bit3 -> 1
    const int my_k = ((lane & 1) << 3) | ((lane & 2) << 1) | ((lane & 4) >> 1) | ((lane & 8) >> 3);
    for (int64_t u = src_begin + wave; u < src_end; u += nwaves) {
        const T *row = emb + (u - src_begin) * d_in;
        float part[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) part[k] = 0.f;
#pragma unroll
        for (int i = 0; i < kRegCols; ++i) {
            const int c = lane + 64 * i;
            float x = 0.f;
            if (c < d_in) x = row_elem(row, c);
#pragma unroll
            for (int k = 0; k < 16; ++k) part[k] += x * wreg[i][k];
        }
        for (int c = lane + 64 * kRegCols; c < d_in; c += 64) {  // wider rows: the rest from memory
            const float x = row_elem(row, c);
#pragma unroll
            for (int k = 0; k < 16; ++k)
                if (k < H2) part[k] += x * wa[c * H2 + k];
        }
        // halving steps: 16 -> 8 -> 4 -> 2 -> 1 values per lane
        float p8[8], p4[4], p2[2], p1;
        {
            const bool hi = lane & 1;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float give = hi ? part[k] : part[k + 8];
                const float keep = hi ? part[k + 8] : part[k];
                p8[k] = keep + __shfl_xor(give, 1);
            }
        }
        {
            const bool hi = lane & 2;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float give = hi ? p8[k] : p8[k + 4];
                const float keep = hi ? p8[k + 4] : p8[k];
                p4[k] = keep + __shfl_xor(give, 2);
            }
        }
        {
            const bool hi = lane & 4;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const float give = hi ? p4[k] : p4[k + 2];
                const float keep = hi ? p4[k + 2] : p4[k];
                p2[k] = keep + __shfl_xor(give, 4);
            }
        }
        {
            const bool hi = lane & 8;
            const float give = hi ? p2[0] : p2[1];
            const float keep = hi ? p2[1] : p2[0];
            p1 = keep + __shfl_xor(give, 8);
        }
        p1 += __shfl_xor(p1, 16);
        p1 += __shfl_xor(p1, 32);
        if (lane < 16 && my_k < H2) {
            if (my_k < heads) el[u * heads + my_k] = p1;
            else er[u * heads + (my_k - heads)] = p1;
        }
    }
}

// Bring destinations whose running maximum moved in this chunk to the new
// reference: l and acc are multiplied by exp(m_cur - m_next) per head.  A first
// touch (m_cur = -inf, state still zero) only moves the reference.
__global__ __launch_bounds__(kBlock) void k_gat_rescale(GatState g, float *acc, int d_out, int64_t n) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / 64) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / 64);
    const int H = g.heads;
    const int64_t nbatches = (n + 63) / 64;
    for (int64_t bt = wave; bt < nbatches; bt += nwaves) {
        const int64_t v = bt * 64 + lane;
        bool moved = false, rows = false;
        if (v < n) {
            for (int h = 0; h < H; ++h) {
                const int32_t mc = g.m_cur[v * H + h], mn = g.m_next[v * H + h];
                if (mn != mc) {
                    moved = true;
                    if (decode_max(mc) != -INFINITY) rows = true;
                }
            }
        }
        uint64_t todo = __ballot(rows);
        while (todo) {  // the whole wave rescales one destination row at a time
            const int src_lane = __ffsll(static_cast<unsigned long long>(todo)) - 1;
            todo &= todo - 1;
            const int64_t vv = bt * 64 + src_lane;
            for (int c = lane; c < d_out; c += 64) {
                const int h = c / g.dh;
                const float f = expf(decode_max(g.m_cur[vv * H + h]) - decode_max(g.m_next[vv * H + h]));
                acc[vv * d_out + c] *= f;
            }
            if (lane < H) {
                const float f = expf(decode_max(g.m_cur[vv * H + lane]) - decode_max(g.m_next[vv * H + lane]));
                g.l[vv * H + lane] *= f;
            }
        }
        // every lane has finished reading m_cur of the rows above before any lane moves it
        __builtin_amdgcn_wave_barrier();
        if (moved)
            for (int h = 0; h < H; ++h) g.m_cur[v * H + h] = g.m_next[v * H + h];
    }
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// y_r = acc_r / l_r per head (0 where nothing arrived) + bias, activation.
__global__ __launch_bounds__(kBlock) void k_gat_finalize(GatFinalizeArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / 64) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / 64);
    const int head = a.counters[CTR_READY_HEAD];
    const int tail = a.counters[CTR_READY_TAIL];
    for (int64_t i = head + wave; i < tail; i += nwaves) {
        const int64_t v = a.ready[i];
        for (int c = lane; c < a.d_out; c += 64) {
            const float l = a.l[v * a.heads + c / a.dh];
            float y = l > 0.f ? a.acc[v * a.d_out + c] / l : 0.f;
            if (a.bias) y += a.bias[c];
            if (a.activation == 1) y = y > 0.f ? y : 0.f;
            else if (a.activation == 2) y = y > 0.f ? y : expm1f(y);
            if (a.out_dt == 2) static_cast<_Float16 *>(a.out)[v * a.d_out + c] = static_cast<_Float16>(y);
            else if (a.out_dt == 1) static_cast<uint16_t *>(a.out)[v * a.d_out + c] = f32_to_bf16_rne(y);
            else static_cast<float *>(a.out)[v * a.d_out + c] = y;
        }
    }
}

int grid_cap(int per_cu) {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus <= 0) cus = 256;
    return cus * per_cu;
}

int grid_for_waves(int64_t waves_wanted) {
    int64_t blocks = (waves_wanted + 3) / 4;
    const int cap = grid_cap(8);
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return static_cast<int>(blocks);
}

}  // namespace

int32_t gat_encoded_neg_inf() {
    const uint32_t bits = 0xff800000u;  // -inf
    return static_cast<int32_t>(bits ^ 0x7fffffffu);
}

hipError_t launch_fill_i32(int32_t *p, int32_t value, int64_t count, hipStream_t s) {
    if (count <= 0) return hipSuccess;
    int64_t blocks = (count + kBlock - 1) / kBlock;
    const int cap = grid_cap(16);
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(k_fill_i32, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, p, value, count);
    return hipGetLastError();
}

hipError_t launch_gat_fold_attention(const void *W, const void *a_src, const void *a_dst, int w_dt, int d_in,
                                     int heads, int dh, float *wa, hipStream_t s) {
    const int total = d_in * 2 * heads;
    hipLaunchKernelGGL(k_gat_fold_attention, dim3((total + kBlock - 1) / kBlock), dim3(kBlock), 0, s, W, a_src, a_dst,
                       w_dt, d_in, heads, dh, wa);
    return hipGetLastError();
}

hipError_t launch_gat_prepass(const void *emb, int in_dt, int64_t src_begin, int64_t src_end, int d_in,
                              const float *wa, int heads, float *el, float *er, hipStream_t s) {
    if (src_end <= src_begin) return hipSuccess;
    if (heads > 8) return hipErrorInvalidValue;
    const int grid = grid_for_waves(src_end - src_begin);
    if (in_dt == 2)
        hipLaunchKernelGGL(k_gat_prepass<_Float16>, dim3(grid), dim3(kBlock), 0, s,
                           static_cast<const _Float16 *>(emb), src_begin, src_end, d_in, wa, heads, el, er);
    else if (in_dt == 1)
        hipLaunchKernelGGL(k_gat_prepass<uint16_t>, dim3(grid), dim3(kBlock), 0, s,
                           static_cast<const uint16_t *>(emb), src_begin, src_end, d_in, wa, heads, el, er);
    else
        hipLaunchKernelGGL(k_gat_prepass<float>, dim3(grid), dim3(kBlock), 0, s, static_cast<const float *>(emb),
                           src_begin, src_end, d_in, wa, heads, el, er);
    return hipGetLastError();
}

hipError_t launch_gat_rescale(const GatState &g, float *acc, int d_out, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_gat_rescale, dim3(grid_for_waves((n + 63) / 64)), dim3(kBlock), 0, s, g, acc, d_out, n);
    return hipGetLastError();
}

hipError_t launch_gat_finalize(const GatFinalizeArgs &a, hipStream_t s) {
    if (a.n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_gat_finalize, dim3(grid_for_waves(a.n)), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace atlas
