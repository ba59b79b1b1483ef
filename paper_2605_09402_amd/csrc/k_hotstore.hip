// Bounded accumulator store: the paper's memory manager (Sec. 3.5) with HBM as
// the hot tier and pinned host memory as the cold tier.
//
// A fixed number of slots holds the partial aggregates of the vertices that are
// currently being aggregated; `slot_of` maps a vertex to its slot.  Before a
// chunk is pushed, every vertex the chunk addresses gets a slot (a fresh one for
// its first message, its evicted state back from the cold tier otherwise).  If
// the free slots do not suffice, the shortfall is evicted from the resident
// vertices the chunk does not address, fewest pending messages first (the
// paper's minimum-pending policy), ties by vertex id.  The paper keeps the
// resident vertices in pending-indexed bucket lists on the CPU; here the
// ordered view is one radix sort of (pending, vertex) keys over the slots in the
// chunks that have to evict.  Rows move between the tiers inside kernels, which
// read and write the pinned host buffer directly (sizes are device-side values).
// Slots are released when a completed vertex has been flushed.
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>

#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

namespace atlas {
namespace {

constexpr int kBlock = 256;
constexpr int kWave = 64;

__global__ __launch_bounds__(kBlock) void k_hot_init(HotStore h, int64_t n) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n) {
        h.slot_of[i] = -1;
        h.stamp[i] = 0;
    }
    if (i < h.slots) {
        h.slot_owner[i] = -1;
        h.free_list[i] = static_cast<int32_t>(h.slots - 1 - i);   // slot 0 is handed out first
    }
    if (i < HS_COUNT) h.ctr[i] = i == HS_FREE_TOP ? static_cast<int32_t>(h.slots) : 0;
}

// append `v` of the lanes with `want` to list[] with one atomic per wave
__device__ __forceinline__ void wave_append(bool want, int32_t v, int32_t *list, int32_t *count, int64_t cap,
                                            int32_t *overflow) {
    const uint64_t m = __ballot(want);
    if (!m) return;
    const int lane = threadIdx.x & (kWave - 1);
    int32_t base = 0;
    if (lane == __ffsll(static_cast<unsigned long long>(m)) - 1) base = atomicAdd(count, __popcll(m));
    base = __shfl(base, __ffsll(static_cast<unsigned long long>(m)) - 1);
    if (want) {
        const int64_t idx = base + __popcll(m & ((1ull << lane) - 1ull));
        if (idx < cap) list[idx] = v;
        else *overflow = 1;
    }
}

// Item i < n_groups: the destination of group i.  Further items: the chunk's own
// sources, whose self message needs an existing state to be resident (it never
// starts one).  Every addressed vertex is stamped with the chunk; those without
// a slot are listed once.
__global__ __launch_bounds__(kBlock) void k_hot_mark(HotStore h, const int32_t *__restrict__ grp_dst, int32_t dst_mask,
                                                    int64_t n_groups, int64_t src_begin, int64_t n_self,
                                                    int32_t chunk_stamp) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    bool want = false;
    int32_t v = 0;
    if (i < n_groups + n_self) {
        const bool self = i >= n_groups;
        v = self ? static_cast<int32_t>(src_begin + (i - n_groups)) : (grp_dst[i] & dst_mask);
        const int32_t st = h.slot_of[v];
        if (!(self && st == -1)) {
            const int32_t old = atomicExch(&h.stamp[v], chunk_stamp);
            want = old != chunk_stamp && st < 0;
        }
    }
    wave_append(want, v, h.need_list, &h.ctr[HS_NEED], h.slots, &h.ctr[HS_OVERFLOW]);
}

// Eviction key of every slot: (pending, vertex) for resident vertices that the
// chunk does not address and that are incomplete, all-ones otherwise.
__global__ __launch_bounds__(kBlock) void k_hot_keys(HotStore h, const int32_t *__restrict__ pending,
                                                    int32_t chunk_stamp, int policy) {
    const int64_t s = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    bool cand = false;
    if (s < h.slots) {
        const int32_t v = h.slot_owner[s];
        uint64_t key = ~0ull;
        if (v >= 0) {
            const int32_t p = pending[v];
            if (h.stamp[v] != chunk_stamp && p > 0) {
                cand = true;
                const uint32_t rank = policy == 0 ? static_cast<uint32_t>(p) : 0x7fffffffu - static_cast<uint32_t>(p);
                key = (static_cast<uint64_t>(rank) << 32) | static_cast<uint32_t>(v);
            }
        }
        h.keys[s] = key;
    }
    const uint64_t m = __ballot(cand);
    if (m && (threadIdx.x & (kWave - 1)) == 0) atomicAdd(&h.ctr[HS_CANDIDATES], __popcll(m));
}

__device__ __forceinline__ void copy_row(float *__restrict__ dst, const float *__restrict__ src, int d, int lane) {
    for (int c = lane * 4; c < d; c += kWave * 4)
        *reinterpret_cast<float4 *>(dst + c) = *reinterpret_cast<const float4 *>(src + c);
}

// One wave per victim: the first n_evict keys of the sorted list.
__global__ __launch_bounds__(kBlock) void k_hot_evict(HotStore h, int64_t n_evict) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / kWave);
    const int32_t top = h.ctr[HS_FREE_TOP];   // not changed by this kernel
    for (int64_t i = wave; i < n_evict; i += nwaves) {
        const int64_t v = static_cast<int64_t>(h.keys_sorted[i] & 0xffffffffull);
        const int32_t s = h.slot_of[v];
        copy_row(h.cold + v * h.d, h.hot + static_cast<int64_t>(s) * h.d, h.d, lane);
        if (lane == 0) {
            h.slot_of[v] = -2;
            h.slot_owner[s] = -1;
            h.free_list[top + i] = s;
        }
    }
}

// One wave per listed vertex: take a free slot; bring an evicted state back.
__global__ __launch_bounds__(kBlock) void k_hot_assign(HotStore h, int64_t need) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / kWave);
    const int32_t top = h.ctr[HS_FREE_TOP];   // not changed by this kernel
    for (int64_t i = wave; i < need; i += nwaves) {
        const int64_t v = h.need_list[i];
        const int32_t s = h.free_list[top - 1 - i];
        const bool evicted = h.slot_of[v] == -2;
        if (evicted) copy_row(h.hot + static_cast<int64_t>(s) * h.d, h.cold + v * h.d, h.d, lane);
        if (lane == 0) {
            if (evicted) atomicAdd(&h.ctr[HS_RELOADS], 1);
            h.slot_of[v] = s;
            h.slot_owner[s] = static_cast<int32_t>(v);
        }
    }
}

__global__ void k_hot_after_evict(HotStore h, int32_t n_evict) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        h.ctr[HS_FREE_TOP] += n_evict;
        h.ctr[HS_EVICTIONS] += n_evict;
        h.ctr[HS_CANDIDATES] = 0;
    }
}
__global__ void k_hot_after_assign(HotStore h, int32_t need) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        h.ctr[HS_FREE_TOP] -= need;
        h.ctr[HS_NEED] = 0;
        const int32_t used = static_cast<int32_t>(h.slots) - h.ctr[HS_FREE_TOP];
        if (used > h.ctr[HS_PEAK]) h.ctr[HS_PEAK] = used;
    }
}

// The vertices flushed by the update that has just run give their slots back.
__global__ __launch_bounds__(kBlock) void k_hot_release(HotStore h, const int32_t *__restrict__ ready,
                                                       const int32_t *__restrict__ counters) {
    const int head = counters[CTR_READY_HEAD], tail = counters[CTR_READY_TAIL];
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    // all lanes of a wave run the same number of rounds
    for (int64_t i0 = head + static_cast<int64_t>(blockIdx.x) * kBlock + (threadIdx.x & ~(kWave - 1)); i0 < tail;
         i0 += stride) {
        const int64_t i = i0 + (threadIdx.x & (kWave - 1));
        int32_t s = -1, v = 0;
        if (i < tail) {
            v = ready[i];
            s = h.slot_of[v];
        }
        if (s >= 0) {
            h.slot_of[v] = -1;
            h.slot_owner[s] = -1;
        }
        wave_append(s >= 0, s, h.free_list, &h.ctr[HS_FREE_TOP], h.slots, &h.ctr[HS_OVERFLOW]);
    }
}

int grid_for(int64_t items, int per_block) {
    int64_t b = (items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > 256 * 16) b = 256 * 16;
    return static_cast<int>(b);
}

}  // namespace

hipError_t hot_init(const HotStore &h, int64_t n, hipStream_t s) {
    const int64_t items = std::max<int64_t>(std::max<int64_t>(n, h.slots), HS_COUNT);
    hipLaunchKernelGGL(k_hot_init, dim3(static_cast<unsigned>((items + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, h, n);
    return hipGetLastError();
}

hipError_t hot_mark(const HotStore &h, const int32_t *grp_dst, int32_t dst_mask, int64_t n_groups, int64_t src_begin,
                    int64_t n_self, int32_t chunk_stamp, hipStream_t s) {
    const int64_t items = n_groups + n_self;
    if (items <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_hot_mark, dim3(static_cast<unsigned>((items + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, h,
                       grp_dst, dst_mask, n_groups, src_begin, n_self, chunk_stamp);
    return hipGetLastError();
}

hipError_t hot_build_keys(const HotStore &h, const int32_t *pending, int32_t chunk_stamp, int policy, hipStream_t s) {
    hipLaunchKernelGGL(k_hot_keys, dim3(static_cast<unsigned>((h.slots + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, h,
                       pending, chunk_stamp, policy);
    return hipGetLastError();
}

size_t hot_sort_temp_bytes(int64_t slots) {
    size_t bytes = 0;
    uint64_t *null = nullptr;
    (void)rocprim::radix_sort_keys(nullptr, bytes, null, null, static_cast<size_t>(slots), 0, 64, nullptr);
    return bytes;
}

hipError_t hot_evict(const HotStore &h, int64_t n_evict, void *sort_temp, size_t sort_temp_bytes, hipStream_t s) {
    hipError_t e = rocprim::radix_sort_keys(sort_temp, sort_temp_bytes, h.keys, h.keys_sorted,
                                            static_cast<size_t>(h.slots), 0, 64, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_hot_evict, dim3(grid_for(n_evict, kBlock / kWave)), dim3(kBlock), 0, s, h, n_evict);
    hipLaunchKernelGGL(k_hot_after_evict, dim3(1), dim3(64), 0, s, h, static_cast<int32_t>(n_evict));
    return hipGetLastError();
}

hipError_t hot_assign(const HotStore &h, int64_t need, hipStream_t s) {
    if (need > 0) hipLaunchKernelGGL(k_hot_assign, dim3(grid_for(need, kBlock / kWave)), dim3(kBlock), 0, s, h, need);
    hipLaunchKernelGGL(k_hot_after_assign, dim3(1), dim3(64), 0, s, h, static_cast<int32_t>(need));
    return hipGetLastError();
}

hipError_t hot_release(const HotStore &h, const int32_t *ready, const int32_t *counters, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_hot_release, dim3(grid_for(n, kBlock)), dim3(kBlock), 0, s, h, ready, counters);
    return hipGetLastError();
}

}  // namespace atlas
