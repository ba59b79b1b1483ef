// In-degree-descending vertex order with ties broken by the smaller old id:
// a stable descending radix sort of (in-degree, id) pairs, then the inverse
// map.  The paper reorders vertices before inference so that destinations
// complete early (Sec. 3.8); the degree ordering used here is the simple
// integer-exact variant of that idea.
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

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

// ---- the same ordering without any allocation --------------------------------
//
// Scratch of the no-allocation variant: sorted keys, the identity ids and the
// library sort's own workspace live in one fixed array in device memory.  Every
// GPU the library runs on holds its own copy of the array, at its own address,
// until the process ends.  In host code the array's name is only a stand-in:
// the address that kernels, copies and the sort may use is the one
// hipGetSymbolAddress returns for the device that is current, looked up once
// per device and kept.
namespace {

constexpr size_t kScratchBytes = size_t(24) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

hipError_t scratch_of_current_device(unsigned char **out) {
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<unsigned char *>(g_scratch_ptr[dev]);
    return hipSuccess;
}

size_t up256(size_t v) { return (v + 255) / 256 * 256; }

}  // namespace

hipError_t reorder_indegree_desc_noalloc(const int32_t *indeg, int64_t n, int32_t *new_of_old, int32_t *old_of_new,
                                         hipStream_t s, bool *too_large) {
    *too_large = false;
    if (n == 0) return hipSuccess;
    if (n > kNoAllocMaxVertices) {
        *too_large = true;
        return hipSuccess;
    }
    unsigned char *base = nullptr;
    hipError_t err = scratch_of_current_device(&base);
    if (err != hipSuccess) return err;
    const size_t count = static_cast<size_t>(n);
    const size_t keys_off = 0, ids_off = up256(count * sizeof(uint32_t)), temp_off = ids_off + up256(count * sizeof(int32_t));
    uint32_t *keys_out = reinterpret_cast<uint32_t *>(base + keys_off);
    int32_t *ids = reinterpret_cast<int32_t *>(base + ids_off);
    const uint32_t *keys_in = reinterpret_cast<const uint32_t *>(indeg);
    size_t temp_bytes = 0;   // a size query: nothing is allocated or launched
    err = rocprim::radix_sort_pairs_desc(nullptr, temp_bytes, keys_in, keys_out, ids, old_of_new, count, 0, 32, s);
    if (err != hipSuccess) return err;
    if (temp_off + temp_bytes > kScratchBytes) {
        *too_large = true;
        return hipSuccess;
    }
    const unsigned blocks = static_cast<unsigned>((n + 255) / 256);
    // every word of the scratch that is read below is written first: the ids here, the sorted keys
    // and the workspace by the sort itself, so nothing of an earlier call's contents is ever used
    hipLaunchKernelGGL(k_iota, dim3(blocks), dim3(256), 0, s, ids, n);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    err = rocprim::radix_sort_pairs_desc(base + temp_off, temp_bytes, keys_in, keys_out, ids, old_of_new, count, 0, 32, s);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(k_invert, dim3(blocks), dim3(256), 0, s, old_of_new, new_of_old, n);
    return hipGetLastError();
}

}  // namespace atlas
