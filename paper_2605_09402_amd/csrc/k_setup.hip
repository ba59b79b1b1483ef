// Layer set-up kernels: in-degree histogram, pending-count initialisation with
// seeding of the ready list, zero fill, parameter conversion.
// (Paper Sec. 3.4: per-vertex degree / pending arrays created at layer start;
// Sec. 3.8: a vertex is complete once it has received d_in(v) messages.)
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>

namespace atlas {
namespace {

constexpr int kBlock = 256;

int grid_for(int64_t items, int per_cu = 8) {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus <= 0) cus = 256;
    int64_t blocks = (items + kBlock - 1) / kBlock;
    const int64_t cap = static_cast<int64_t>(cus) * per_cu;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return static_cast<int>(blocks);
}

__global__ __launch_bounds__(kBlock) void k_in_degree(const int32_t *__restrict__ col, int64_t num_edges,
                                                      int32_t *indeg) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; e < num_edges; e += stride)
        atomicAdd(&indeg[col[e]], 1);
}

__global__ __launch_bounds__(kBlock) void k_init_pending(const int32_t *__restrict__ indeg, int32_t selfmsg,
                                                         int64_t n, int32_t *pending, int32_t *ready,
                                                         int32_t *counters) {
    const int lane = threadIdx.x & 63;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const int64_t rounded = (n + kBlock - 1) / kBlock * kBlock;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < rounded; i += stride) {
        bool is_ready = false;
        if (i < n) {
            const int32_t p = indeg[i] + selfmsg;
            pending[i] = p;
            is_ready = p == 0;  // nothing will ever arrive: complete at layer start
        }
        // seeding happens once per layer and is rare (GAT vertices without
        // in-edges): one tail update per wave is enough here
        const uint64_t m = __ballot(is_ready);
        if (m) {
            const int leader = __ffsll(static_cast<unsigned long long>(m)) - 1;
            int base = 0;
            if (lane == leader) base = atomicAdd(&counters[CTR_READY_TAIL], __popcll(m));
            base = __shfl(base, leader);
            if (is_ready) ready[base + __popcll(m & ((1ull << lane) - 1ull))] = static_cast<int32_t>(i);
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_fill_zero(uint4 *p, size_t vecs) {
    const size_t stride = static_cast<size_t>(gridDim.x) * kBlock;
    for (size_t i = static_cast<size_t>(blockIdx.x) * kBlock + threadIdx.x; i < vecs; i += stride)
        p[i] = make_uint4(0, 0, 0, 0);
}

__global__ __launch_bounds__(kBlock) void k_to_f32(const void *src, int src_dt, int64_t count, float *dst) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= count) return;
    if (src_dt == 2)        // IEEE half
        dst[i] = static_cast<float>(static_cast<const _Float16 *>(src)[i]);
    else if (src_dt == 1)   // bf16
        dst[i] = __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t *>(src)[i]) << 16);
    else
        dst[i] = static_cast<const float *>(src)[i];
}

}  // namespace

hipError_t launch_in_degree(const int32_t *col, int64_t num_edges, int32_t *indeg, int64_t n,
                            hipStream_t s) {
    hipError_t err = launch_fill_zero(indeg, static_cast<size_t>(n) * sizeof(int32_t), s);
    if (err != hipSuccess) return err;
    if (num_edges == 0) return hipSuccess;
    hipLaunchKernelGGL(k_in_degree, dim3(grid_for(num_edges, 16)), dim3(kBlock), 0, s, col, num_edges, indeg);
    return hipGetLastError();
}

hipError_t launch_init_pending(const int32_t *indeg, int32_t selfmsg, int64_t n, int32_t *pending,
                               int32_t *ready, int32_t *counters, hipStream_t s) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_init_pending, dim3(grid_for(n)), dim3(kBlock), 0, s, indeg, selfmsg, n, pending,
                       ready, counters);
    return hipGetLastError();
}

// Buffers handed to this function are 256-byte aligned device allocations
// whose size is rounded up to 16 bytes by the allocator in atlas_api.hip.
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s) {
    const size_t vecs = (bytes + 15) / 16;
    if (vecs == 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_zero, dim3(grid_for(static_cast<int64_t>(vecs), 16)), dim3(kBlock), 0, s,
                       static_cast<uint4 *>(p), vecs);
    return hipGetLastError();
}

hipError_t launch_to_f32(const void *src, int src_dt, int64_t count, float *dst, hipStream_t s) {
    if (count == 0) return hipSuccess;
    const unsigned blocks = static_cast<unsigned>((count + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(k_to_f32, dim3(blocks), dim3(kBlock), 0, s, src, src_dt, count, dst);
    return hipGetLastError();
}

}  // namespace atlas
