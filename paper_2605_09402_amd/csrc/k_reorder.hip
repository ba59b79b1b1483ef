// In-degree-descending vertex order with ties broken by the smaller old id:
// a stable descending radix sort of (in-degree, id) pairs, then the inverse
// map.  The paper reorders vertices before inference so that destinations
// complete early (Sec. 3.8); the degree ordering used here is the simple
// integer-exact variant of that idea.
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>

#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

namespace atlas {
namespace {

__global__ void k_iota(int32_t *p, int64_t n) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = static_cast<int32_t>(i);
}

__global__ void k_invert(const int32_t *old_of_new, int32_t *new_of_old, int64_t n) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) new_of_old[old_of_new[i]] = static_cast<int32_t>(i);
}

// Score(u) = (sum over out-edges (u,v) of 1/d_in(v)) / d_out(u), 0 without
// out-edges (paper Sec. 3.8).  One thread walks a source's out-edges in CSR
// order in fp64, the same order a sequential host loop uses, so the values
// (and the ordering derived from them) are reproducible bit for bit.
__global__ void k_order_score(const int64_t *__restrict__ off, const int32_t *__restrict__ col,
                              const int32_t *__restrict__ indeg, int64_t n, uint64_t *key) {
    const int64_t u = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (u >= n) return;
    const int64_t b = off[u], e = off[u + 1];
    double s = 0.0;
    for (int64_t i = b; i < e; ++i) s += 1.0 / static_cast<double>(indeg[col[i]]);
    const double score = e > b ? s / static_cast<double>(e - b) : 0.0;
    key[u] = static_cast<uint64_t>(__double_as_longlong(score));  // scores are >= 0: bit order = value order
}

}  // namespace

hipError_t reorder_score_desc(const int64_t *off, const int32_t *col, const int32_t *indeg, int64_t n,
                              int32_t *new_of_old, int32_t *old_of_new) {
    if (n == 0) return hipSuccess;
    hipError_t err;
    uint64_t *keys = nullptr, *keys_out = nullptr;
    int32_t *ids = nullptr;
    void *temp = nullptr;
    size_t temp_bytes = 0;
    const unsigned blocks = static_cast<unsigned>((n + 255) / 256);
    if ((err = hipMalloc(&keys, n * sizeof(uint64_t))) != hipSuccess) goto done;
    if ((err = hipMalloc(&keys_out, n * sizeof(uint64_t))) != hipSuccess) goto done;
    if ((err = hipMalloc(&ids, n * sizeof(int32_t))) != hipSuccess) goto done;
    hipLaunchKernelGGL(k_iota, dim3(blocks), dim3(256), 0, nullptr, ids, n);
    hipLaunchKernelGGL(k_order_score, dim3(blocks), dim3(256), 0, nullptr, off, col, indeg, n, keys);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    // stable descending sort: equal scores keep ascending id order
    err = rocprim::radix_sort_pairs_desc(nullptr, temp_bytes, keys, keys_out, ids, old_of_new,
                                         static_cast<size_t>(n), 0, 64, nullptr);
    if (err != hipSuccess) goto done;
    if ((err = hipMalloc(&temp, temp_bytes > 0 ? temp_bytes : 16)) != hipSuccess) goto done;
    err = rocprim::radix_sort_pairs_desc(temp, temp_bytes, keys, keys_out, ids, old_of_new,
                                         static_cast<size_t>(n), 0, 64, nullptr);
    if (err != hipSuccess) goto done;
    hipLaunchKernelGGL(k_invert, dim3(blocks), dim3(256), 0, nullptr, old_of_new, new_of_old, n);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    err = hipStreamSynchronize(nullptr);
done:
    if (temp) (void)hipFree(temp);
    if (ids) (void)hipFree(ids);
    if (keys_out) (void)hipFree(keys_out);
    if (keys) (void)hipFree(keys);
    return err;
}

hipError_t reorder_indegree_desc(const int32_t *indeg, int64_t n, int32_t *new_of_old,
                                 int32_t *old_of_new) {
    if (n == 0) return hipSuccess;
    hipError_t err;
    uint32_t *keys_out = nullptr;
    int32_t *ids = nullptr;
    void *temp = nullptr;
    size_t temp_bytes = 0;
    const unsigned blocks = static_cast<unsigned>((n + 255) / 256);
    const uint32_t *keys_in = reinterpret_cast<const uint32_t *>(indeg);
    if ((err = hipMalloc(&keys_out, n * sizeof(uint32_t))) != hipSuccess) goto done;
    if ((err = hipMalloc(&ids, n * sizeof(int32_t))) != hipSuccess) goto done;
    hipLaunchKernelGGL(k_iota, dim3(blocks), dim3(256), 0, nullptr, ids, n);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    // radix sort is stable: equal degrees keep ascending id order
    err = rocprim::radix_sort_pairs_desc(nullptr, temp_bytes, keys_in, keys_out, ids, old_of_new,
                                         static_cast<size_t>(n), 0, 32, nullptr);
    if (err != hipSuccess) goto done;
    if ((err = hipMalloc(&temp, temp_bytes > 0 ? temp_bytes : 16)) != hipSuccess) goto done;
    err = rocprim::radix_sort_pairs_desc(temp, temp_bytes, keys_in, keys_out, ids, old_of_new,
                                         static_cast<size_t>(n), 0, 32, nullptr);
    if (err != hipSuccess) goto done;
    hipLaunchKernelGGL(k_invert, dim3(blocks), dim3(256), 0, nullptr, old_of_new, new_of_old, n);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    err = hipStreamSynchronize(nullptr);
done:
    if (temp) (void)hipFree(temp);
    if (ids) (void)hipFree(ids);
    if (keys_out) (void)hipFree(keys_out);
    return err;
}

}  // namespace atlas
