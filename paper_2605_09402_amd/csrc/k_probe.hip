// Measured peaks of the machine, taken with kernels of this library's own
// shape, for the benchmark's report: a plain device copy (what "HBM bandwidth"
// means for a 1 read : 1 write stream) and the wave-per-row gather of random
// 256-byte rows that the planned aggregation is made of (one coalesced row read
// per message, paper Sec. 3.1 / 3.4), without any of its bookkeeping.  The
// roofline fractions the benchmark prints are against the published peak; these
// figures say how much of that peak a bare kernel of the same access pattern
// reaches on the box at hand.
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>

namespace atlas {
namespace {

constexpr int kBlock = 256;
constexpr int kWave = 64;

__global__ __launch_bounds__(kBlock) void k_probe_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                       size_t vecs) {
    const size_t stride = static_cast<size_t>(gridDim.x) * kBlock;
    for (size_t i = static_cast<size_t>(blockIdx.x) * kBlock + threadIdx.x; i < vecs; i += stride) dst[i] = src[i];
}

// Two reads for one write (dst = a ^ b): the read/write mix of the flush (accumulator row and own row in,
// output row out) without its gather or its contraction.
__global__ __launch_bounds__(kBlock) void k_probe_mix21(const uint4 *__restrict__ a, const uint4 *__restrict__ b,
                                                        uint4 *__restrict__ dst, size_t vecs) {
    const size_t stride = static_cast<size_t>(gridDim.x) * kBlock;
    for (size_t i = static_cast<size_t>(blockIdx.x) * kBlock + threadIdx.x; i < vecs; i += stride) {
        const uint4 x = a[i], y = b[i];
        dst[i] = make_uint4(x.x ^ y.x, x.y ^ y.y, x.z ^ y.z, x.w ^ y.w);
    }
}

// A wave reads 64 row ids with one coalesced load, then gathers the rows, U at a
// time: the 64 lanes hold one 256-byte row, 4 bytes each.  The words are folded
// into one register per lane so that no load can be dropped; each wave writes
// its 64 folded words once, at the end.
template <int U>
__global__ __launch_bounds__(kBlock) void k_probe_row_gather(const uint32_t *__restrict__ table,
                                                             const int32_t *__restrict__ ids, int64_t n_ids,
                                                             uint32_t *__restrict__ sink) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / kWave);
    uint32_t fold = 0;
    for (int64_t base = wave * kWave; base < n_ids; base += nwaves * kWave) {
        const int64_t left = n_ids - base;
        const int cnt = left < kWave ? static_cast<int>(left) : kWave;
        int32_t id = 0;
        if (lane < cnt) id = ids[base + lane];
        for (int j0 = 0; j0 < cnt; j0 += U) {
            uint32_t r[U];
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const int j = j0 + i < cnt ? j0 + i : cnt - 1;
                const int64_t row = __builtin_amdgcn_readlane(id, j);
                r[i] = table[row * kWave + lane];
            }
#pragma unroll
            for (int i = 0; i < U; ++i) fold ^= r[i];
        }
    }
    sink[wave * kWave + lane] = fold;
}

// Nothing but matrix instructions: every wave keeps `ACCS` independent 32x32 accumulators and issues
// bf16 32x32x16 products on them from registers, `iters` rounds; what the matrix pipeline delivers when
// nothing has to be loaded, converted or synchronised.
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
template <int ACCS>
__global__ __launch_bounds__(kBlock) void k_probe_mfma(int iters, float *__restrict__ sink) {
    const int lane = threadIdx.x & (kWave - 1);
    uint4 qa = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);   // ones
    uint4 qb = make_uint4(lane & 1 ? 0x3f800000u : 0u, 0u, 0u, 0u);
    const probe_bf16x8 a = __builtin_bit_cast(probe_bf16x8, qa), b = __builtin_bit_cast(probe_bf16x8, qb);
    probe_f32x16 c[ACCS];
#pragma unroll
    for (int k = 0; k < ACCS; ++k)
#pragma unroll
        for (int i = 0; i < 16; ++i) c[k][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < ACCS; ++k) c[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[k], 0, 0, 0);
    }
    float fold = 0.f;
#pragma unroll
    for (int k = 0; k < ACCS; ++k)
#pragma unroll
        for (int i = 0; i < 16; ++i) fold += c[k][i];
    sink[static_cast<size_t>(blockIdx.x) * kBlock + threadIdx.x] = fold;
}

int cu_count() {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    return cus > 0 ? cus : 256;
}

}  // namespace

hipError_t probe_copy(void *dst, const void *src, size_t bytes, hipStream_t s) {
    const size_t vecs = bytes / 16;
    if (vecs == 0) return hipSuccess;
    hipLaunchKernelGGL(k_probe_copy, dim3(cu_count() * 16), dim3(kBlock), 0, s, static_cast<const uint4 *>(src),
                       static_cast<uint4 *>(dst), vecs);
    return hipGetLastError();
}

hipError_t probe_mix21(void *dst, const void *a, const void *b, size_t bytes, hipStream_t s) {
    const size_t vecs = bytes / 16;
    if (vecs == 0) return hipSuccess;
    hipLaunchKernelGGL(k_probe_mix21, dim3(cu_count() * 16), dim3(kBlock), 0, s, static_cast<const uint4 *>(a),
                       static_cast<const uint4 *>(b), static_cast<uint4 *>(dst), vecs);
    return hipGetLastError();
}

hipError_t probe_mfma(int waves_per_simd, int iters, void *sink, double *flops, hipStream_t s) {
    // sink: at least probe_gather_sink_bytes() bytes (8 workgroups of 256 threads per CU)
    if (waves_per_simd < 1 || waves_per_simd > 8 || iters < 1) return hipErrorInvalidValue;
    const int blocks = cu_count() * waves_per_simd;   // a workgroup of 4 waves puts one wave on every SIMD of its CU
    constexpr int kAccs = 4;
    *flops = static_cast<double>(blocks) * (kBlock / kWave) * static_cast<double>(iters) * kAccs * 2.0 * 32 * 32 * 16;
    hipLaunchKernelGGL((k_probe_mfma<kAccs>), dim3(blocks), dim3(kBlock), 0, s, iters, static_cast<float *>(sink));
    return hipGetLastError();
}

size_t probe_gather_sink_bytes() { return static_cast<size_t>(cu_count()) * 8 * kBlock * sizeof(uint32_t); }

hipError_t probe_row_gather(const void *table, const int32_t *ids, int64_t n_ids, void *sink, hipStream_t s) {
    if (n_ids <= 0) return hipSuccess;
    // 8 workgroups of 4 waves per CU, 8 rows in flight per wave: the aggregation's own shape
    hipLaunchKernelGGL(k_probe_row_gather<8>, dim3(cu_count() * 8), dim3(kBlock), 0, s,
                       static_cast<const uint32_t *>(table), ids, n_ids, static_cast<uint32_t *>(sink));
    return hipGetLastError();
}

}  // namespace atlas
