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

// In-degree by one atomic per edge: for small graphs, and for edge arrays that
// are read over the host link (one pass over them is all that link allows).
__global__ __launch_bounds__(kBlock) void k_in_degree(const int32_t *__restrict__ col, int64_t num_edges,
                                                      int32_t *indeg) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; e < num_edges; e += stride)
        atomicAdd(&indeg[col[e]], 1);
}

// ---- in-degree of a large graph in device memory ----------------------------
//
// One global atomic per edge on a counter array far larger than the caches
// costs a memory line read and written back per edge (2^31 edges, 2^26
// counters: 180 ms).  Here the destinations are first split into buckets of
// 2^15 consecutive vertex ids -- two bytes per edge, the id within its bucket --
// and every bucket is then counted in LDS, where an increment costs nothing:
//   1. bucket sizes (a histogram in LDS per workgroup, merged with one atomic
//      per workgroup and non-empty bucket);
//   2. an exclusive scan of the bucket sizes, and the number of slices (of at
//      most kDegSlice entries) every bucket will be counted in;
//   3. scatter: a workgroup takes 2^16 consecutive edges, counts them per
//      bucket, claims room in every bucket with one atomic, and writes each
//      edge's low 15 bits to its place (ranks from LDS atomics);
//   4. count: a workgroup histograms one slice of one bucket in LDS (32 K
//      counters = 128 KiB) and writes the counts out -- plain stores where the
//      bucket has one slice, atomics on the non-zero counts otherwise.
constexpr int kDegBinBits = 15;
constexpr int kDegBins = 1 << kDegBinBits;
constexpr int kDegMaxBuckets = 8192;          // bucket histogram in LDS: graphs below 2^28 vertices
constexpr int kDegTile = 1 << 16;             // edges per workgroup and round of the scatter
constexpr int64_t kDegSlice = int64_t(1) << 19;   // entries per workgroup and round of the count
constexpr int kDegBlock = 1024;
typedef unsigned long long u64;

struct DegScratch {           // carved out of one caller-provided buffer
    u64 *count;               // [kDegMaxBuckets] entries per bucket
    u64 *base;                // [kDegMaxBuckets] first entry of the bucket in `part`
    u64 *cursor;              // [kDegMaxBuckets] next free entry while scattering
    uint32_t *slice_base;     // [kDegMaxBuckets + 1] slices of all earlier buckets
    uint16_t *part;           // [num_edges] id within the bucket, bucket by bucket
};

__global__ __launch_bounds__(kDegBlock) void k_deg_bucket_sizes(const int32_t *__restrict__ col, int64_t num_edges,
                                                                int n_buckets, u64 *count) {
    __shared__ uint32_t h[kDegMaxBuckets];
    for (int b = threadIdx.x; b < n_buckets; b += kDegBlock) h[b] = 0;
    __syncthreads();
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kDegBlock;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * kDegBlock + threadIdx.x; e < num_edges; e += stride)
        atomicAdd(&h[col[e] >> kDegBinBits], 1u);
    __syncthreads();
    for (int b = threadIdx.x; b < n_buckets; b += kDegBlock)
        if (h[b]) atomicAdd(&count[b], static_cast<u64>(h[b]));
}

__global__ void k_deg_scan(DegScratch sc, int n_buckets) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    u64 at = 0;
    uint32_t slices = 0;
    for (int b = 0; b < n_buckets; ++b) {
        const u64 c = sc.count[b];
        sc.base[b] = at;
        sc.cursor[b] = at;
        sc.slice_base[b] = slices;
        at += c;
        slices += static_cast<uint32_t>((c + kDegSlice - 1) / kDegSlice);
    }
    sc.slice_base[n_buckets] = slices;
}

__global__ __launch_bounds__(kDegBlock) void k_deg_scatter(const int32_t *__restrict__ col, int64_t num_edges,
                                                           int n_buckets, DegScratch sc) {
    __shared__ uint32_t cnt[kDegMaxBuckets];
    __shared__ u64 where[kDegMaxBuckets];
    const int64_t ntiles = (num_edges + kDegTile - 1) / kDegTile;
    for (int b = threadIdx.x; b < n_buckets; b += kDegBlock) cnt[b] = 0;
    __syncthreads();
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t e0 = tile * kDegTile;
        const int64_t e1 = e0 + kDegTile < num_edges ? e0 + kDegTile : num_edges;
        for (int64_t e = e0 + threadIdx.x; e < e1; e += kDegBlock) atomicAdd(&cnt[col[e] >> kDegBinBits], 1u);
        __syncthreads();
        for (int b = threadIdx.x; b < n_buckets; b += kDegBlock) {
            const uint32_t c = cnt[b];
            if (c) where[b] = atomicAdd(&sc.cursor[b], static_cast<u64>(c));
            cnt[b] = 0;
        }
        __syncthreads();
        for (int64_t e = e0 + threadIdx.x; e < e1; e += kDegBlock) {   // the tile is still in L2
            const int32_t v = col[e];
            const int b = v >> kDegBinBits;
            const uint32_t pos = atomicAdd(&cnt[b], 1u);
            sc.part[where[b] + pos] = static_cast<uint16_t>(v & (kDegBins - 1));
        }
        __syncthreads();
        for (int b = threadIdx.x; b < n_buckets; b += kDegBlock) cnt[b] = 0;
        __syncthreads();
    }
}

__global__ __launch_bounds__(kDegBlock) void k_deg_count(DegScratch sc, int n_buckets, int64_t n, int32_t *indeg) {
    extern __shared__ uint32_t hist[];   // [kDegBins]
    const uint32_t total = sc.slice_base[n_buckets];
    for (uint32_t s = blockIdx.x; s < total; s += gridDim.x) {
        // the bucket this slice belongs to: the last one whose first slice is <= s
        int lo = 0, hi = n_buckets;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (sc.slice_base[mid] <= s) lo = mid;
            else hi = mid;
        }
        const int b = lo;
        const uint32_t k = s - sc.slice_base[b];
        const uint32_t nsl = sc.slice_base[b + 1] - sc.slice_base[b];
        const u64 first = sc.base[b] + static_cast<u64>(k) * kDegSlice;
        const u64 end_b = sc.base[b] + sc.count[b];
        const u64 last = first + kDegSlice < end_b ? first + kDegSlice : end_b;
        for (int j = threadIdx.x; j < kDegBins; j += kDegBlock) hist[j] = 0;
        __syncthreads();
        for (u64 i = first + threadIdx.x; i < last; i += kDegBlock) atomicAdd(&hist[sc.part[i]], 1u);
        __syncthreads();
        const int64_t v0 = static_cast<int64_t>(b) << kDegBinBits;
        for (int j = threadIdx.x; j < kDegBins; j += kDegBlock) {
            const int64_t v = v0 + j;
            const uint32_t c = hist[j];
            if (v < n) {
                if (nsl == 1) indeg[v] = static_cast<int32_t>(c);
                else if (c) atomicAdd(&indeg[v], static_cast<int32_t>(c));
            }
        }
        __syncthreads();
    }
}

DegScratch carve_deg_scratch(void *scratch) {
    DegScratch sc;
    char *p = static_cast<char *>(scratch);
    sc.count = reinterpret_cast<u64 *>(p);
    sc.base = sc.count + kDegMaxBuckets;
    sc.cursor = sc.base + kDegMaxBuckets;
    sc.slice_base = reinterpret_cast<uint32_t *>(sc.cursor + kDegMaxBuckets);
    sc.part = reinterpret_cast<uint16_t *>(sc.slice_base + kDegMaxBuckets + 64);
    return sc;
}
constexpr size_t kDegHeaderBytes = 3 * kDegMaxBuckets * sizeof(u64) + (kDegMaxBuckets + 64) * sizeof(uint32_t);

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

// Graphs worth the bucketed count: more vertices than one LDS histogram holds, enough edges to pay for
// three passes, and few enough vertices for the bucket histogram.
bool in_degree_by_buckets(int64_t n, int64_t num_edges) {
    return n > kDegBins && num_edges >= (int64_t(1) << 22) && (n + kDegBins - 1) / kDegBins <= kDegMaxBuckets;
}

size_t in_degree_scratch_bytes(int64_t n, int64_t num_edges) {
    if (!in_degree_by_buckets(n, num_edges)) return 0;
    return kDegHeaderBytes + static_cast<size_t>(num_edges) * sizeof(uint16_t) + 256;
}

hipError_t launch_in_degree(const int32_t *col, int64_t num_edges, int32_t *indeg, int64_t n, void *scratch,
                            size_t scratch_bytes, hipStream_t s) {
    hipError_t err = launch_fill_zero(indeg, static_cast<size_t>(n) * sizeof(int32_t), s);
    if (err != hipSuccess) return err;
    if (num_edges == 0) return hipSuccess;
    const size_t need = in_degree_scratch_bytes(n, num_edges);
    if (need == 0 || !scratch || scratch_bytes < need) {
        hipLaunchKernelGGL(k_in_degree, dim3(grid_for(num_edges, 16)), dim3(kBlock), 0, s, col, num_edges, indeg);
        return hipGetLastError();
    }
    static bool configured = false;
    if (!configured) {
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_deg_count),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kDegBins * sizeof(uint32_t));
        if (err != hipSuccess) return err;
        configured = true;
    }
    const int n_buckets = static_cast<int>((n + kDegBins - 1) / kDegBins);
    const DegScratch sc = carve_deg_scratch(scratch);
    if ((err = launch_fill_zero(scratch, kDegHeaderBytes, s)) != hipSuccess) return err;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus <= 0) cus = 256;
    const int64_t ntiles = (num_edges + kDegTile - 1) / kDegTile;
    const int64_t max_slices = n_buckets + num_edges / kDegSlice;   // sum of ceil(count / slice) over the buckets
    auto grid_of = [&](int64_t items, int per_cu) {
        const int64_t cap = static_cast<int64_t>(cus) * per_cu;
        return dim3(static_cast<unsigned>(items < cap ? (items < 1 ? 1 : items) : cap));
    };
    hipLaunchKernelGGL(k_deg_bucket_sizes, grid_of((num_edges + kDegBlock - 1) / kDegBlock, 2), dim3(kDegBlock), 0, s, col,
                       num_edges, n_buckets, sc.count);
    hipLaunchKernelGGL(k_deg_scan, dim3(1), dim3(64), 0, s, sc, n_buckets);
    hipLaunchKernelGGL(k_deg_scatter, grid_of(ntiles, 1), dim3(kDegBlock), 0, s, col, num_edges, n_buckets, sc);
    hipLaunchKernelGGL(k_deg_count, grid_of(max_slices, 1), dim3(kDegBlock), kDegBins * sizeof(uint32_t), s, sc,
                       n_buckets, n, indeg);
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
