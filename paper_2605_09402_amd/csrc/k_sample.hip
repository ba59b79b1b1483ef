// Neighbourhood sampling done on the graph ahead of inference: the paper notes
// that sampled inference fits the broadcast model once the edges a sample
// drops have been switched off (Sec. 3.9).  Every destination keeps at most
// `fanout` of its in-edges -- those with the smallest caller-supplied random
// keys, ties by position in the CSR -- and the kept edges are written out as a
// new CSR by source in their original order.  Integer work only: one stable
// radix sort of (destination, key) with the edge position as payload, a
// max-scan that gives every sorted position the start of its destination's run,
// and a prefix sum of the keep flags for the compaction.
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>

#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

namespace atlas {
namespace {

constexpr int kBlock = 256;

__global__ __launch_bounds__(kBlock) void k_sample_keys(const int32_t *__restrict__ col, const uint32_t *__restrict__ key,
                                                       int64_t e, uint64_t *keys, uint32_t *pos) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= e) return;
    keys[i] = (static_cast<uint64_t>(static_cast<uint32_t>(col[i])) << 32) | key[i];
    pos[i] = static_cast<uint32_t>(i);
}

// run_start[p] = p where a destination's run begins in the sorted order, 0 elsewhere
__global__ __launch_bounds__(kBlock) void k_sample_heads(const uint64_t *__restrict__ keys_sorted, int64_t e,
                                                        uint32_t *run_start) {
    const int64_t p = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (p >= e) return;
    const bool head = p == 0 || (keys_sorted[p - 1] >> 32) != (keys_sorted[p] >> 32);
    run_start[p] = head ? static_cast<uint32_t>(p) : 0u;
}

// keep[original position] = rank within the destination's run < fanout
__global__ __launch_bounds__(kBlock) void k_sample_flag(const uint32_t *__restrict__ run_start,
                                                       const uint32_t *__restrict__ pos_sorted, int64_t e,
                                                       uint32_t fanout, uint32_t *keep) {
    const int64_t p = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (p >= e) return;
    keep[pos_sorted[p]] = (static_cast<uint32_t>(p) - run_start[p]) < fanout ? 1u : 0u;
}

// prefix = exclusive prefix sum of keep
__global__ __launch_bounds__(kBlock) void k_sample_emit(const int32_t *__restrict__ col, const uint32_t *__restrict__ keep,
                                                       const uint32_t *__restrict__ prefix, int64_t e, int32_t *out_col) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= e) return;
    if (keep[i]) out_col[prefix[i]] = col[i];
}

__global__ __launch_bounds__(kBlock) void k_sample_offsets(const int64_t *__restrict__ off, const uint32_t *__restrict__ keep,
                                                          const uint32_t *__restrict__ prefix, int64_t n, int64_t e,
                                                          int64_t *out_off) {
    const int64_t u = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (u > n) return;
    const int64_t b = off[u];
    // kept edges before edge b; for b == e that is all of them
    out_off[u] = b < e ? prefix[b] : (e > 0 ? static_cast<int64_t>(prefix[e - 1]) + keep[e - 1] : 0);
}

struct MaxU32 {
    __host__ __device__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; }
};

}  // namespace

hipError_t sample_in_edges(const int64_t *off, const int32_t *col, int64_t n, int64_t e, const uint32_t *key,
                           int32_t fanout, int64_t *out_off, int32_t *out_col) {
    hipError_t err = hipSuccess;
    uint64_t *keys = nullptr, *keys_sorted = nullptr;
    uint32_t *pos = nullptr, *pos_sorted = nullptr, *run = nullptr, *keep = nullptr, *prefix = nullptr;
    void *temp = nullptr;
    size_t t_sort = 0, t_max = 0, t_sum = 0, temp_bytes = 0;
    const size_t E = static_cast<size_t>(e);
    const unsigned eb = static_cast<unsigned>((e + kBlock - 1) / kBlock);
    const unsigned nb = static_cast<unsigned>((n + 1 + kBlock - 1) / kBlock);
    if (e == 0) {
        hipLaunchKernelGGL(k_sample_offsets, dim3(nb), dim3(kBlock), 0, nullptr, off, keep, prefix, n, e, out_off);
        if ((err = hipGetLastError()) != hipSuccess) return err;
        return hipStreamSynchronize(nullptr);
    }
    if ((err = hipMalloc(&keys, E * 8)) != hipSuccess) goto done;
    if ((err = hipMalloc(&keys_sorted, E * 8)) != hipSuccess) goto done;
    if ((err = hipMalloc(&pos, E * 4)) != hipSuccess) goto done;
    if ((err = hipMalloc(&pos_sorted, E * 4)) != hipSuccess) goto done;
    if ((err = hipMalloc(&run, E * 4)) != hipSuccess) goto done;
    if ((err = hipMalloc(&keep, E * 4)) != hipSuccess) goto done;
    if ((err = hipMalloc(&prefix, E * 4)) != hipSuccess) goto done;
    if ((err = rocprim::radix_sort_pairs(nullptr, t_sort, keys, keys_sorted, pos, pos_sorted, E, 0, 64, nullptr)) != hipSuccess) goto done;
    if ((err = rocprim::inclusive_scan(nullptr, t_max, run, prefix, E, MaxU32(), nullptr)) != hipSuccess) goto done;
    if ((err = rocprim::exclusive_scan(nullptr, t_sum, keep, prefix, 0u, E, rocprim::plus<uint32_t>(), nullptr)) != hipSuccess) goto done;
    temp_bytes = std::max(std::max(t_sort, t_max), std::max(t_sum, static_cast<size_t>(16)));
    if ((err = hipMalloc(&temp, temp_bytes)) != hipSuccess) goto done;

    hipLaunchKernelGGL(k_sample_keys, dim3(eb), dim3(kBlock), 0, nullptr, col, key, e, keys, pos);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    // stable: equal (destination, key) pairs stay in CSR order
    if ((err = rocprim::radix_sort_pairs(temp, t_sort, keys, keys_sorted, pos, pos_sorted, E, 0, 64, nullptr)) != hipSuccess) goto done;
    hipLaunchKernelGGL(k_sample_heads, dim3(eb), dim3(kBlock), 0, nullptr, keys_sorted, e, run);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    // running maximum of the run heads = start of every position's run (into `prefix`, free until the sum below)
    if ((err = rocprim::inclusive_scan(temp, t_max, run, prefix, E, MaxU32(), nullptr)) != hipSuccess) goto done;
    hipLaunchKernelGGL(k_sample_flag, dim3(eb), dim3(kBlock), 0, nullptr, prefix, pos_sorted, e,
                       static_cast<uint32_t>(fanout), keep);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    if ((err = rocprim::exclusive_scan(temp, t_sum, keep, prefix, 0u, E, rocprim::plus<uint32_t>(), nullptr)) != hipSuccess) goto done;
    hipLaunchKernelGGL(k_sample_emit, dim3(eb), dim3(kBlock), 0, nullptr, col, keep, prefix, e, out_col);
    hipLaunchKernelGGL(k_sample_offsets, dim3(nb), dim3(kBlock), 0, nullptr, off, keep, prefix, n, e, out_off);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    err = hipStreamSynchronize(nullptr);
done:
    for (void *p : {static_cast<void *>(temp), static_cast<void *>(prefix), static_cast<void *>(keep),
                    static_cast<void *>(run), static_cast<void *>(pos_sorted), static_cast<void *>(pos),
                    static_cast<void *>(keys_sorted), static_cast<void *>(keys)})
        if (p) (void)hipFree(p);
    return err;
}

}  // namespace atlas
