// Per-graph plan: for every aligned source chunk, the chunk's out-edges
// regrouped by destination.  The chunk is still what is streamed (paper
// Sec. 3.3: contiguous source range with its topology); only the order in
// which its edges are visited changes, so that all messages a chunk sends to
// one destination are adjacent.  Integer-only, done once per graph like the
// paper's offline reordering (Sec. 3.8).
//
// Steps for a chunk with edges [E0, E1):
//   1. source id of every edge (row starts scattered, then a running maximum);
//   2. stable radix sort of (destination, source) pairs by destination;
//   3. group heads / tails: bit 31 of the stored source id marks the last edge
//      of a destination's group, a prefix sum of the heads numbers the groups;
//   4. grp_dst[g] = destination of group g (bit 31: the destination's first group in
//      the whole stream), tile_grp[t] = group of edge 64 t.
//
// Source-blocked variant (block_sources > 0), between steps 2 and 3.  In
// destination order a hub's group walks the whole chunk's rows once, far more
// than an L2 holds, and the next hub walks them again: nothing is reused.  So
// the edges of destinations that receive at least hot_min_edges messages from
// the chunk are reordered by (source block, destination), a block being
// block_sources consecutive sources whose rows fit an L2: while the kernel
// sweeps one block's edges its rows stay cache resident and are gathered many
// times.  Such a destination then has one group per source block (bit 30 of
// grp_dst: several groups of this chunk address the destination, so all of them
// add with atomics); all other edges keep the destination order and follow.
#include "atlas_kernels.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <vector>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

namespace atlas {
namespace {

constexpr int kBlock = 256;

unsigned blocks_for(int64_t n) { return static_cast<unsigned>((n + kBlock - 1) / kBlock); }

// tmp[off[u] - E0] = u for every source of the chunk that has out-edges.
__global__ void k_mark_row_starts(const int64_t *__restrict__ off, int64_t src_begin, int64_t src_end,
                                  int64_t e0, int32_t *tmp) {
    const int64_t u = src_begin + static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (u >= src_end) return;
    const int64_t a = off[u], b = off[u + 1];
    if (b > a) tmp[a - e0] = static_cast<int32_t>(u);
}

// heads[i] = 1 where a destination's group starts; the source id of the last
// edge of a group gets bit 31.
__global__ void k_mark_groups(const uint32_t *__restrict__ dst_sorted, int64_t n_edges, int32_t *src_sorted,
                              uint32_t *heads) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n_edges) return;
    const uint32_t d = dst_sorted[i];
    heads[i] = (i == 0 || dst_sorted[i - 1] != d) ? 1u : 0u;
    if (i + 1 == n_edges || dst_sorted[i + 1] != d)
        src_sorted[i] = static_cast<int32_t>(static_cast<uint32_t>(src_sorted[i]) | 0x80000000u);
}

// gidx = inclusive prefix sum of heads (group number + 1).
// `seen[v]` says whether an earlier chunk of the plan already sends to v; a
// group that is its destination's first gets bit 31 of grp_dst (chunks are
// planned in streaming order and a destination has one group per chunk).
__global__ void k_emit_groups(const uint32_t *__restrict__ dst_sorted, const uint32_t *__restrict__ gidx,
                              int64_t n_edges, int32_t *grp_dst, int32_t *tile_grp, uint8_t *seen,
                              const uint32_t *__restrict__ block_key, uint32_t n_blocks) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n_edges) return;
    const uint32_t g = gidx[i] - 1u;
    if (i == 0 || gidx[i - 1] != gidx[i]) {
        const uint32_t v = dst_sorted[i];
        // without a first-touch map (a chunk regrouped on its own) no group claims to be its destination's first
        const bool first = seen && seen[v] == 0;
        if (seen) seen[v] = 1;
        // source-blocked chunks: the destination has a group in every source block
        const uint32_t multi = (block_key && block_key[i] < n_blocks) ? 0x40000000u : 0u;
        grp_dst[g] = static_cast<int32_t>((first ? (v | 0x80000000u) : v) | multi);
    }
    if ((i & 63) == 0) tile_grp[i >> 6] = static_cast<int32_t>(g);
}

// gstart[g] = position of the first edge of group g (gidx = group number + 1 per edge)
__global__ void k_group_starts(const uint32_t *__restrict__ heads, const uint32_t *__restrict__ gidx, int64_t n_edges,
                               uint32_t *gstart) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n_edges) return;
    if (heads[i]) gstart[gidx[i] - 1u] = static_cast<uint32_t>(i);
    if (i + 1 == n_edges) gstart[gidx[i]] = static_cast<uint32_t>(n_edges);
}

// key[i] = source block of edge i if its destination's group has at least hot_min edges, n_blocks otherwise
__global__ void k_block_keys(const int32_t *__restrict__ src_sorted, const uint32_t *__restrict__ gidx,
                             const uint32_t *__restrict__ gstart, int64_t n_edges, int64_t src_begin,
                             int64_t block_sources, uint32_t n_blocks, uint32_t hot_min, uint32_t *key, uint32_t *pos) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n_edges) return;
    const uint32_t g = gidx[i] - 1u;
    const uint32_t len = gstart[g + 1] - gstart[g];
    const int64_t u = src_sorted[i] & 0x7fffffff;
    key[i] = len >= hot_min ? static_cast<uint32_t>((u - src_begin) / block_sources) : n_blocks;
    pos[i] = static_cast<uint32_t>(i);
}

__global__ void k_apply_order(const uint32_t *__restrict__ pos, const uint32_t *__restrict__ dst_in,
                              const int32_t *__restrict__ src_in, int64_t n_edges, uint32_t *dst_out, int32_t *src_out) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n_edges) return;
    const uint32_t p = pos[i];
    dst_out[i] = dst_in[p];
    src_out[i] = src_in[p] & 0x7fffffff;   // group tails are marked again for the new order
}

// gstart[g] = position of group g's first edge, from the per-edge group numbers (gidx = group + 1)
__global__ void k_group_starts_only(const uint32_t *__restrict__ gidx, int64_t n_edges, uint32_t *gstart) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n_edges) return;
    if (i == 0 || gidx[i - 1] != gidx[i]) gstart[gidx[i] - 1u] = static_cast<uint32_t>(i);
}

// The rows a planned-only layer must clear before this chunk runs: destinations whose FIRST group of the
// layer is added to with atomics by more than one wave -- it is cut by a 64-edge tile boundary, or the
// destination has one group per source block.  One thread per group; duplicates are harmless.
__global__ void k_collect_zero_rows(const int32_t *__restrict__ grp_dst, const uint32_t *__restrict__ gstart_of_group,
                                    int64_t n_groups, int64_t n_edges, int32_t *rows, int32_t *spans,
                                    unsigned int *count) {
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (g >= n_groups) return;
    const int32_t gd = grp_dst[g];
    if (gd >= 0) return;                                    // not a first group
    const int64_t b = gstart_of_group[g];
    const int64_t e = g + 1 < n_groups ? gstart_of_group[g + 1] : n_edges;   // one past the group's last edge
    const bool cut = (b >> 6) != ((e - 1) >> 6);
    if (cut || (gd & 0x40000000)) {
        const unsigned int k = atomicAdd(count, 1u);
        rows[k] = gd & 0x3fffffff;
        // first and last tile of the group; a destination with one group per source block: always cleared
        const bool multi = (gd & 0x40000000) != 0;
        spans[2 * k] = multi ? -1 : static_cast<int32_t>(b >> 6);
        spans[2 * k + 1] = multi ? -1 : static_cast<int32_t>((e - 1) >> 6);
    }
}

// number of non-zero bytes (the destinations the first-touch map has seen)
__global__ __launch_bounds__(kBlock) void k_count_nonzero(const uint8_t *__restrict__ p, int64_t n,
                                                          unsigned long long *count) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    unsigned int mine = 0;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n; i += stride) mine += p[i] != 0;
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_down(mine, o);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(count, static_cast<unsigned long long>(mine));
}

struct MaxOp {
    __host__ __device__ int32_t operator()(int32_t a, int32_t b) const { return a > b ? a : b; }
};

}  // namespace

PlanWork::~PlanWork() {
    for (GrowBuf *b : {&tmp_src, &dst_sorted, &heads, &temp, &bkey, &bkey_sorted, &bpos, &bpos_sorted, &gstart, &src_new,
                       &rows, &cnt, &part_flags, &part_pos, &part_dst, &part_src})
        b->release();
}

hipError_t GrowBuf::need(size_t bytes) {
    if (bytes <= cap && p) return hipSuccess;
    release();
    const hipError_t e = hipMalloc(&p, bytes > 0 ? bytes : 16);
    if (e != hipSuccess) { p = nullptr; return e; }
    cap = bytes;
    return hipSuccess;
}
void GrowBuf::release() {
    if (p) (void)hipFree(p);
    p = nullptr;
    cap = 0;
}

hipError_t build_plan_chunk(const int64_t *off_dev, const int32_t *col_dev, int64_t n, int64_t src_begin,
                            int64_t src_end, int64_t edge_begin, int64_t edge_end, int32_t *src_sorted,
                            uint8_t *seen, int64_t block_sources, int64_t hot_min_edges, bool want_zero_rows,
                            PlanWork &w, PlanChunk *out, const EdgePairs *pairs) {
    *out = PlanChunk{};
    out->edge_base = edge_begin;
    out->n_edges = pairs ? pairs->count : edge_end - edge_begin;
    const int64_t ne = out->n_edges;
    if (ne <= 0) return hipSuccess;
    if (ne >= (int64_t(1) << 32)) return hipErrorInvalidValue;

    hipError_t err = hipSuccess;
    // source-blocked order: only for chunks of more than one block
    const int64_t n_blocks64 = block_sources > 0 ? (src_end - src_begin + block_sources - 1) / block_sources : 0;
    const bool blocked = n_blocks64 > 1;
    const uint32_t n_blocks = static_cast<uint32_t>(n_blocks64);
    size_t temp_bsort = 0;
    int bkey_bits = 1;
    size_t temp_sort = 0, temp_scan_max = 0, temp_scan_sum = 0, temp_bytes = 0;
    const uint32_t *keys_in = pairs ? pairs->dst : reinterpret_cast<const uint32_t *>(col_dev + edge_begin);
    uint32_t last = 0;
    int end_bit = 1;
    while (end_bit < 32 && (int64_t(1) << end_bit) < n) ++end_bit;
    const size_t count = static_cast<size_t>(ne);

    // work arrays: kept from chunk to chunk, grown when a chunk is larger than any before it
    if (!pairs && (err = w.tmp_src.need(count * 4)) != hipSuccess) return err;
    if ((err = w.dst_sorted.need(count * 4)) != hipSuccess) return err;
    if ((err = w.heads.need(count * 4)) != hipSuccess) return err;
    // source per edge (CSR order); reused for the group prefix sum
    int32_t *tmp_src = pairs ? pairs->src : static_cast<int32_t *>(w.tmp_src.p);
    uint32_t *dst_sorted = static_cast<uint32_t *>(w.dst_sorted.p);
    uint32_t *heads = static_cast<uint32_t *>(w.heads.p);
    uint32_t *bkey = nullptr, *bkey_sorted = nullptr, *bpos = nullptr, *bpos_sorted = nullptr, *gstart = nullptr;
    int32_t *src_new = nullptr;
    if ((err = rocprim::radix_sort_pairs(nullptr, temp_sort, keys_in, dst_sorted, tmp_src, src_sorted, count, 0,
                                         end_bit, nullptr)) != hipSuccess) return err;
    if ((err = rocprim::inclusive_scan(nullptr, temp_scan_max, tmp_src, tmp_src, count, MaxOp(), nullptr)) != hipSuccess) return err;
    if ((err = rocprim::inclusive_scan(nullptr, temp_scan_sum, heads, reinterpret_cast<uint32_t *>(tmp_src), count,
                                       rocprim::plus<uint32_t>(), nullptr)) != hipSuccess) return err;
    temp_bytes = temp_sort > temp_scan_max ? temp_sort : temp_scan_max;
    if (temp_scan_sum > temp_bytes) temp_bytes = temp_scan_sum;
    if (blocked) {
        while (bkey_bits < 32 && (uint64_t(1) << bkey_bits) <= n_blocks) ++bkey_bits;   // keys 0 .. n_blocks
        if ((err = w.bkey.need(count * 4)) != hipSuccess) return err;
        if ((err = w.bkey_sorted.need(count * 4)) != hipSuccess) return err;
        if ((err = w.bpos.need(count * 4)) != hipSuccess) return err;
        if ((err = w.bpos_sorted.need(count * 4)) != hipSuccess) return err;
        if ((err = w.gstart.need((count + 1) * 4)) != hipSuccess) return err;
        if ((err = w.src_new.need(count * 4)) != hipSuccess) return err;
        bkey = static_cast<uint32_t *>(w.bkey.p);
        bkey_sorted = static_cast<uint32_t *>(w.bkey_sorted.p);
        bpos = static_cast<uint32_t *>(w.bpos.p);
        bpos_sorted = static_cast<uint32_t *>(w.bpos_sorted.p);
        gstart = static_cast<uint32_t *>(w.gstart.p);
        src_new = static_cast<int32_t *>(w.src_new.p);
        if ((err = rocprim::radix_sort_pairs(nullptr, temp_bsort, bkey, bkey_sorted, bpos, bpos_sorted, count, 0,
                                             bkey_bits, nullptr)) != hipSuccess) return err;
        if (temp_bsort > temp_bytes) temp_bytes = temp_bsort;
    }
    if ((err = w.temp.need(temp_bytes > 0 ? temp_bytes : 16)) != hipSuccess) return err;
    void *temp = w.temp.p;

    // 1. source of every edge
    if (!pairs) {
        if ((err = hipMemsetAsync(tmp_src, 0, count * 4, nullptr)) != hipSuccess) goto done;
        hipLaunchKernelGGL(k_mark_row_starts, dim3(blocks_for(src_end - src_begin)), dim3(kBlock), 0, nullptr, off_dev,
                           src_begin, src_end, edge_begin, tmp_src);
        if ((err = hipGetLastError()) != hipSuccess) goto done;
        if ((err = rocprim::inclusive_scan(temp, temp_scan_max, tmp_src, tmp_src, count, MaxOp(), nullptr)) != hipSuccess) goto done;
    }
    // 2. stable sort by destination
    if ((err = rocprim::radix_sort_pairs(temp, temp_sort, keys_in, dst_sorted, tmp_src, src_sorted, count, 0, end_bit,
                                         nullptr)) != hipSuccess) goto done;
    if (blocked) {
        // groups of the destination order and their sizes, then the stable sort by source block (edges of
        // small groups all get the key n_blocks and stay behind, in destination order)
        hipLaunchKernelGGL(k_mark_groups, dim3(blocks_for(ne)), dim3(kBlock), 0, nullptr, dst_sorted, ne, src_sorted, heads);
        if ((err = hipGetLastError()) != hipSuccess) goto done;
        if ((err = rocprim::inclusive_scan(temp, temp_scan_sum, heads, reinterpret_cast<uint32_t *>(tmp_src), count,
                                           rocprim::plus<uint32_t>(), nullptr)) != hipSuccess) goto done;
        hipLaunchKernelGGL(k_group_starts, dim3(blocks_for(ne)), dim3(kBlock), 0, nullptr, heads,
                           reinterpret_cast<const uint32_t *>(tmp_src), ne, gstart);
        hipLaunchKernelGGL(k_block_keys, dim3(blocks_for(ne)), dim3(kBlock), 0, nullptr, src_sorted,
                           reinterpret_cast<const uint32_t *>(tmp_src), gstart, ne, src_begin, block_sources, n_blocks,
                           static_cast<uint32_t>(std::min<int64_t>(std::max<int64_t>(hot_min_edges, 1), 0xffffffffll)),
                           bkey, bpos);
        if ((err = hipGetLastError()) != hipSuccess) goto done;
        if ((err = rocprim::radix_sort_pairs(temp, temp_bsort, bkey, bkey_sorted, bpos, bpos_sorted, count, 0, bkey_bits,
                                             nullptr)) != hipSuccess) goto done;
        // heads is free again: it receives the destinations in the new order
        hipLaunchKernelGGL(k_apply_order, dim3(blocks_for(ne)), dim3(kBlock), 0, nullptr, bpos_sorted, dst_sorted,
                           src_sorted, ne, heads, src_new);
        if ((err = hipGetLastError()) != hipSuccess) goto done;
        if ((err = hipMemcpyAsync(dst_sorted, heads, count * 4, hipMemcpyDeviceToDevice, nullptr)) != hipSuccess) goto done;
        if ((err = hipMemcpyAsync(src_sorted, src_new, count * 4, hipMemcpyDeviceToDevice, nullptr)) != hipSuccess) goto done;
        out->blocked = true;
    }
    // 3. group heads, tail flags, group numbering
    hipLaunchKernelGGL(k_mark_groups, dim3(blocks_for(ne)), dim3(kBlock), 0, nullptr, dst_sorted, ne, src_sorted, heads);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    if ((err = rocprim::inclusive_scan(temp, temp_scan_sum, heads, reinterpret_cast<uint32_t *>(tmp_src), count,
                                       rocprim::plus<uint32_t>(), nullptr)) != hipSuccess) goto done;
    if ((err = hipMemcpy(&last, reinterpret_cast<uint32_t *>(tmp_src) + (count - 1), 4, hipMemcpyDeviceToHost)) != hipSuccess) goto done;
    out->n_groups = last;
    // 4. per-group destination and per-tile first group
    if ((err = hipMalloc(&out->grp_dst, static_cast<size_t>(last) * 4)) != hipSuccess) goto done;
    if ((err = hipMalloc(&out->tile_grp, static_cast<size_t>((ne + 63) / 64) * 4)) != hipSuccess) goto done;
    hipLaunchKernelGGL(k_emit_groups, dim3(blocks_for(ne)), dim3(kBlock), 0, nullptr, dst_sorted,
                       reinterpret_cast<const uint32_t *>(tmp_src), ne, out->grp_dst, out->tile_grp, seen,
                       blocked ? bkey_sorted : nullptr, n_blocks);
    if ((err = hipGetLastError()) != hipSuccess) goto done;
    if (want_zero_rows && n < (int64_t(1) << 30)) {
        // rows to clear for planned-only layers (first groups that several waves add to)
        uint32_t *gs = heads;   // free again: start position of every group
        unsigned int n_zero = 0;
        hipLaunchKernelGGL(k_group_starts_only, dim3(blocks_for(ne)), dim3(kBlock), 0, nullptr,
                           reinterpret_cast<const uint32_t *>(tmp_src), ne, gs);
        if ((err = w.cnt.need(sizeof(unsigned int))) != hipSuccess) goto done;
        unsigned int *cnt = static_cast<unsigned int *>(w.cnt.p);
        if ((err = hipMemsetAsync(cnt, 0, sizeof(unsigned int), nullptr)) != hipSuccess) goto done;
        // worst case one row per group; the list is trimmed below
        if ((err = w.rows.need(static_cast<size_t>(last) * 12)) != hipSuccess) goto done;
        int32_t *rows = static_cast<int32_t *>(w.rows.p);   // [last] rows, then [last][2] spans
        int32_t *spans = rows + last;
        hipLaunchKernelGGL(k_collect_zero_rows, dim3(blocks_for(last)), dim3(kBlock), 0, nullptr, out->grp_dst, gs,
                           static_cast<int64_t>(last), ne, rows, spans, cnt);
        if ((err = hipMemcpy(&n_zero, cnt, sizeof(unsigned int), hipMemcpyDeviceToHost)) != hipSuccess) goto done;
        if (n_zero > 0) {
            err = hipMalloc(&out->zero_rows, static_cast<size_t>(n_zero) * 4);
            if (err == hipSuccess)
                err = hipMemcpy(out->zero_rows, rows, static_cast<size_t>(n_zero) * 4, hipMemcpyDeviceToDevice);
            if (err == hipSuccess) err = hipMalloc(&out->zero_span, static_cast<size_t>(n_zero) * 8);
            if (err == hipSuccess)
                err = hipMemcpy(out->zero_span, spans, static_cast<size_t>(n_zero) * 8, hipMemcpyDeviceToDevice);
        }
        if (err != hipSuccess) goto done;
        out->n_zero_rows = n_zero;
        out->has_zero_rows = true;
    }
    err = hipStreamSynchronize(nullptr);
done:
    if (err != hipSuccess) {
        (void)hipStreamSynchronize(nullptr);
        if (out->grp_dst) (void)hipFree(out->grp_dst);
        if (out->tile_grp) (void)hipFree(out->tile_grp);
        if (out->zero_rows) (void)hipFree(out->zero_rows);
        if (out->zero_span) (void)hipFree(out->zero_span);
        out->grp_dst = nullptr;
        out->tile_grp = nullptr;
        out->zero_rows = nullptr;
        out->zero_span = nullptr;
    }
    return err;
}

void DensePart::release() {
    for (void *q : {static_cast<void *>(band_ksteps), static_cast<void *>(band_off), static_cast<void *>(cells),
                    static_cast<void *>(msgs), static_cast<void *>(items), static_cast<void *>(list_src),
                    static_cast<void *>(list.grp_dst),
                    static_cast<void *>(list.tile_grp), static_cast<void *>(list.zero_rows),
                    static_cast<void *>(list.zero_span)})
        if (q) (void)hipFree(q);
    *this = DensePart{};
}

namespace {
// The staircase: per destination bucket, how many sources (in k-steps of 64) its bands
// take.  A (source bucket, destination bucket) block belongs to the region when it spends at most
// cells_per_edge cells per edge it holds and so do all blocks before it in its row and column of buckets,
// which keeps the extents non-increasing from one destination bucket to the next.
int64_t bucket_begin(int k) { return k == 0 ? 0 : int64_t(1) << (7 + k); }
int64_t bucket_end(int k) { return int64_t(1) << (8 + k); }
void choose_staircase(const unsigned long long *hist, int64_t n, int64_t chunk_sources, int64_t cells_per_edge,
                      int32_t (&ksteps)[kDenseBuckets]) {
    const int64_t src_cap = (chunk_sources + 255) / 256 * 256;
    int prev = kDenseBuckets;   // source buckets the previous destination bucket took
    for (int j = 0; j < kDenseBuckets; ++j) {
        ksteps[j] = 0;
        if (bucket_begin(j) >= n) { prev = 0; continue; }
        const double dsts = static_cast<double>(std::min(bucket_end(j), n) - bucket_begin(j));
        int take = 0;
        while (take < prev && bucket_begin(take) < chunk_sources) {
            const double srcs = static_cast<double>(std::min(bucket_end(take), chunk_sources) - bucket_begin(take));
            const double edges = static_cast<double>(hist[take * kDenseBuckets + j]);
            if (edges * static_cast<double>(cells_per_edge) < srcs * dsts) break;
            ++take;
        }
        prev = take;
        // (a multiple of kDenseKstepUnit k-steps: the contraction's loop is unrolled that far; sources past the
        // chunk's end are zero rows to it)
        if (take > 0)
            ksteps[j] = static_cast<int32_t>((std::min(bucket_end(take - 1), src_cap) / 64 + kDenseKstepUnit - 1) /
                                             kDenseKstepUnit * kDenseKstepUnit);
    }
}
}  // namespace

hipError_t build_first_chunk_with_dense_part(const int64_t *off_dev, const int32_t *col_dev, int64_t n,
                                             int64_t src_begin, int64_t src_end, int64_t edge_begin,
                                             int64_t edge_end, int32_t *src_sorted, uint8_t *seen,
                                             int64_t block_sources, int64_t hot_min_edges, bool want_zero_rows,
                                             size_t max_bytes, int64_t cells_per_edge, PlanWork &w, PlanChunk *rest,
                                             DensePart *dense) {
    *dense = DensePart{};
    const int64_t ne = edge_end - edge_begin;
    auto plain = [&]() {
        return build_plan_chunk(off_dev, col_dev, n, src_begin, src_end, edge_begin, edge_end, src_sorted, seen,
                                block_sources, hot_min_edges, want_zero_rows, w, rest);
    };
    if (ne <= 0 || ne >= (int64_t(1) << 32) || n >= (int64_t(1) << 30) || cells_per_edge <= 0) return plain();
    const size_t count = static_cast<size_t>(ne);
    const int32_t *col = col_dev + edge_begin;
    hipError_t err = hipSuccess;
    unsigned long long *hist_dev = nullptr;
    unsigned long long hist[kDenseBuckets * kDenseBuckets];
    int32_t ksteps[kDenseBuckets];
    std::vector<int32_t> band_ksteps, items;
    std::vector<int64_t> band_off;
    size_t total = 0, temp_max = 0, temp_sum = 0;
    uint32_t flagged_last = 0;
    uint8_t flag_last = 0;
    int64_t n_dense = 0, n_rest = 0;
    EdgePairs pr{};

    // source of every edge, as in build_plan_chunk
    if ((err = w.tmp_src.need(count * 4)) != hipSuccess) return err;
    int32_t *src_of_edge = static_cast<int32_t *>(w.tmp_src.p);
    if ((err = rocprim::inclusive_scan(nullptr, temp_max, src_of_edge, src_of_edge, count, MaxOp(), nullptr)) != hipSuccess) return err;
    if ((err = w.part_flags.need(count)) != hipSuccess) return err;
    if ((err = w.part_pos.need(count * 4)) != hipSuccess) return err;
    uint8_t *flags = static_cast<uint8_t *>(w.part_flags.p);
    uint32_t *pos = static_cast<uint32_t *>(w.part_pos.p);
    if ((err = rocprim::exclusive_scan(nullptr, temp_sum, flags, pos, uint32_t(0), count, rocprim::plus<uint32_t>(),
                                       nullptr)) != hipSuccess) return err;
    if ((err = w.temp.need(std::max<size_t>(std::max(temp_max, temp_sum), 16))) != hipSuccess) return err;
    if ((err = hipMemsetAsync(src_of_edge, 0, count * 4, nullptr)) != hipSuccess) return err;
    hipLaunchKernelGGL(k_mark_row_starts, dim3(blocks_for(src_end - src_begin)), dim3(kBlock), 0, nullptr, off_dev,
                       src_begin, src_end, edge_begin, src_of_edge);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    if ((err = rocprim::inclusive_scan(w.temp.p, temp_max, src_of_edge, src_of_edge, count, MaxOp(), nullptr)) != hipSuccess) return err;

    // where the chunk is dense
    if ((err = hipMalloc(&hist_dev, sizeof(hist))) != hipSuccess) return err;
    err = launch_dense_histogram(src_of_edge, col, ne, src_begin, hist_dev, nullptr);
    if (err == hipSuccess) err = hipMemcpy(hist, hist_dev, sizeof(hist), hipMemcpyDeviceToHost);
    (void)hipFree(hist_dev);
    if (err != hipSuccess) return err;
    for (int64_t cpe = cells_per_edge; cpe > 0; cpe /= 2) {
        choose_staircase(hist, n, src_end - src_begin, cpe, ksteps);
        band_ksteps.clear();
        band_off.clear();
        total = 0;
        for (int j = 0; j < kDenseBuckets && ksteps[j] > 0; ++j) {
            const int64_t end = std::min(bucket_end(j), (n + 255) / 256 * 256);
            for (int64_t r = bucket_begin(j); r < end; r += 256) {
                band_ksteps.push_back(ksteps[j]);
                band_off.push_back(static_cast<int64_t>(total));
                total += static_cast<size_t>(ksteps[j]) * kDenseKstepBytes;
            }
        }
        if (total <= max_bytes) break;
        band_ksteps.clear();
    }
    if (band_ksteps.empty()) return plain();

    dense->n_bands = static_cast<int32_t>(band_ksteps.size());
    dense->rows = static_cast<int64_t>(dense->n_bands) * 256;
    dense->max_ksteps = band_ksteps[0];
    dense->cell_bytes = total;
    // work items in (source slice, band) order: the workgroups in flight at one time then read the same slice of
    // the repacked rows, which stays in the L2 caches, while each streams its own cells.  Last slice first: only
    // the longest bands reach it and all its items are full length; the first slice, with the thousands of short
    // bands of the staircase's lower steps, then fills the end of the launch evenly.
    for (int32_t k = (dense->max_ksteps - 1) / kDenseItemKsteps * kDenseItemKsteps; k >= 0; k -= kDenseItemKsteps)
        for (int32_t b = 0; b < dense->n_bands && band_ksteps[b] > k; ++b) {
            items.push_back(b);
            items.push_back(k);
            // bits 16..: the band's only item (its sums are stored, not added)
            items.push_back(std::min<int32_t>(kDenseItemKsteps, band_ksteps[b] - k) |
                            (band_ksteps[b] <= kDenseItemKsteps ? 1 << 16 : 0));
        }
    dense->n_items = static_cast<int64_t>(items.size() / 3);
    if ((err = hipMalloc(&dense->band_ksteps, band_ksteps.size() * 4)) != hipSuccess) goto fail;
    if ((err = hipMalloc(&dense->band_off, band_off.size() * 8)) != hipSuccess) goto fail;
    if ((err = hipMalloc(&dense->items, items.size() * 4)) != hipSuccess) goto fail;
    if ((err = hipMalloc(&dense->msgs, static_cast<size_t>(dense->rows) * 4)) != hipSuccess) goto fail;
    if ((err = hipMalloc(&dense->cells, total)) != hipSuccess) goto fail;
    if ((err = hipMemcpy(dense->band_ksteps, band_ksteps.data(), band_ksteps.size() * 4, hipMemcpyHostToDevice)) != hipSuccess) goto fail;
    if ((err = hipMemcpy(dense->band_off, band_off.data(), band_off.size() * 8, hipMemcpyHostToDevice)) != hipSuccess) goto fail;
    if ((err = hipMemcpy(dense->items, items.data(), items.size() * 4, hipMemcpyHostToDevice)) != hipSuccess) goto fail;
    if ((err = hipMemsetAsync(dense->cells, 0, total, nullptr)) != hipSuccess) goto fail;
    if ((err = hipMemsetAsync(dense->msgs, 0, static_cast<size_t>(dense->rows) * 4, nullptr)) != hipSuccess) goto fail;

    // the edges the cells take over, and the two halves of the chunk in CSR order
    if ((err = launch_dense_divert(src_of_edge, col, ne, src_begin, *dense, flags, nullptr)) != hipSuccess) goto fail;
    if ((err = rocprim::exclusive_scan(w.temp.p, temp_sum, flags, pos, uint32_t(0), count, rocprim::plus<uint32_t>(),
                                       nullptr)) != hipSuccess) goto fail;
    if ((err = hipMemcpy(&flagged_last, pos + (count - 1), 4, hipMemcpyDeviceToHost)) != hipSuccess) goto fail;
    if ((err = hipMemcpy(&flag_last, flags + (count - 1), 1, hipMemcpyDeviceToHost)) != hipSuccess) goto fail;
    n_dense = static_cast<int64_t>(flagged_last) + (flag_last ? 1 : 0);
    n_rest = ne - n_dense;
    if (n_dense == 0) {
        dense->release();
        return plain();
    }
    if ((err = w.part_dst.need(count * 4)) != hipSuccess) goto fail;
    if ((err = w.part_src.need(count * 4)) != hipSuccess) goto fail;
    if ((err = launch_dense_split(src_of_edge, col, flags, pos, ne, n_rest, static_cast<uint32_t *>(w.part_dst.p),
                                  static_cast<int32_t *>(w.part_src.p), nullptr)) != hipSuccess) goto fail;
    // the dense part is pushed first: its groups are the first touch of their destinations
    pr.dst = static_cast<const uint32_t *>(w.part_dst.p) + n_rest;
    pr.src = static_cast<int32_t *>(w.part_src.p) + n_rest;
    pr.count = n_dense;
    if ((err = build_plan_chunk(off_dev, col_dev, n, src_begin, src_end, edge_begin + n_rest, edge_end,
                                src_sorted + n_rest, seen, 0, 0, want_zero_rows, w, &dense->list, &pr)) != hipSuccess) goto fail;
    if ((err = launch_plan_chunk_in_degree(dense->list, src_sorted + n_rest, dense->msgs, nullptr)) != hipSuccess) goto fail;
    pr.dst = static_cast<const uint32_t *>(w.part_dst.p);
    pr.src = static_cast<int32_t *>(w.part_src.p);
    pr.count = n_rest;
    if ((err = build_plan_chunk(off_dev, col_dev, n, src_begin, src_end, edge_begin, edge_begin + n_rest, src_sorted,
                                seen, block_sources, hot_min_edges, want_zero_rows, w, rest, &pr)) != hipSuccess) goto fail;
    if ((err = hipStreamSynchronize(nullptr)) != hipSuccess) goto fail;
    return hipSuccess;
fail:
    (void)hipStreamSynchronize(nullptr);
    dense->release();
    return err;
}

// In-degree from a planned chunk: a group's size is the number of messages its destination
// receives from the chunk.  One wave per 64-edge tile; every piece of a group inside the tile
// (its last edge, or the tile's last edge) adds its length.
namespace {
__global__ __launch_bounds__(kBlock) void k_plan_chunk_in_degree(const int32_t *__restrict__ src_sorted,
                                                                 const int32_t *__restrict__ grp_dst,
                                                                 const int32_t *__restrict__ tile_grp, int64_t n_edges,
                                                                 int32_t id_mask, int32_t *indeg) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kBlock / 64) + (threadIdx.x >> 6);
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kBlock / 64);
    const int64_t ntiles = (n_edges + 63) / 64;
    for (int64_t t = wave; t < ntiles; t += nwaves) {
        const int64_t e0 = t * 64;
        const int64_t left = n_edges - e0;
        const int cnt = left < 64 ? static_cast<int>(left) : 64;
        int32_t s = 0;
        if (lane < cnt) s = src_sorted[e0 + lane];
        const bool is_end = lane < cnt && s < 0;
        const uint64_t below = __ballot(is_end) & ((1ull << lane) - 1ull);
        if (is_end || lane == cnt - 1) {
            const int32_t v = grp_dst[tile_grp[t] + __popcll(below)] & id_mask;
            const int prev_end = below ? 63 - __clzll(static_cast<long long>(below)) : -1;
            atomicAdd(&indeg[v], lane - prev_end);
        }
    }
}
}  // namespace

hipError_t launch_plan_chunk_in_degree(const PlanChunk &c, const int32_t *src_sorted, int32_t *indeg, hipStream_t s) {
    if (c.n_edges <= 0) return hipSuccess;
    const int64_t ntiles = (c.n_edges + 63) / 64;
    int64_t blocks = (ntiles + (kBlock / 64) - 1) / (kBlock / 64);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_plan_chunk_in_degree, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, src_sorted,
                       c.grp_dst, c.tile_grp, c.n_edges, c.blocked ? 0x3fffffff : 0x7fffffff, indeg);
    return hipGetLastError();
}

hipError_t count_nonzero_bytes(const uint8_t *p, int64_t n, int64_t *out) {
    *out = 0;
    if (n <= 0) return hipSuccess;
    unsigned long long *cnt = nullptr, host = 0;
    hipError_t err = hipMalloc(&cnt, sizeof(unsigned long long));
    if (err != hipSuccess) return err;
    err = hipMemset(cnt, 0, sizeof(unsigned long long));
    if (err == hipSuccess) {
        int64_t blocks = (n + kBlock - 1) / kBlock;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_count_nonzero, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, nullptr, p, n, cnt);
        err = hipGetLastError();
    }
    if (err == hipSuccess) err = hipMemcpy(&host, cnt, sizeof(host), hipMemcpyDeviceToHost);
    (void)hipFree(cnt);
    *out = static_cast<int64_t>(host);
    return err;
}

// ---- 24-bit edge words for plans that travel over the host link ------------
//
// A plan of a pinned-host graph is copied to the device chunk by chunk in every
// layer, so its edge words are stored in 3 bytes: the source as an offset from
// the chunk's first source (chunks of at most 2^23 sources) and the group-end
// flag in bit 23.  Four words make three dwords; a chunk's array is padded to
// a multiple of four words.

namespace {
__global__ __launch_bounds__(256) void k_pack24(const int32_t *__restrict__ src_sorted, int64_t n_edges,
                                                int32_t src_begin, uint32_t *__restrict__ packed) {
    const int64_t q = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;   // four edges
    if (q * 4 >= n_edges) return;
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t i = q * 4 + j;
        const int32_t v = i < n_edges ? src_sorted[i] : 0;
        w[j] = static_cast<uint32_t>((v & 0x7fffffff) - (i < n_edges ? src_begin : 0)) | (v < 0 ? 0x800000u : 0u);
    }
    packed[q * 3] = w[0] | (w[1] << 24);
    packed[q * 3 + 1] = (w[1] >> 8) | (w[2] << 16);
    packed[q * 3 + 2] = (w[2] >> 16) | (w[3] << 8);
}

__global__ __launch_bounds__(256) void k_unpack24(const uint32_t *__restrict__ packed, int64_t n_edges,
                                                  int32_t src_begin, int4 *__restrict__ src_sorted) {
    const int64_t q = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;   // four edges
    if (q * 4 >= n_edges) return;
    const uint32_t d0 = packed[q * 3], d1 = packed[q * 3 + 1], d2 = packed[q * 3 + 2];
    const uint32_t w[4] = {d0 & 0xffffffu, (d0 >> 24) | ((d1 & 0xffffu) << 8), (d1 >> 16) | ((d2 & 0xffu) << 16), d2 >> 8};
    int32_t v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        v[j] = static_cast<int32_t>(((w[j] & 0x7fffffu) + static_cast<uint32_t>(src_begin)) | ((w[j] & 0x800000u) << 8));
    src_sorted[q] = make_int4(v[0], v[1], v[2], v[3]);
}
}  // namespace

size_t packed24_bytes(int64_t n_edges) { return static_cast<size_t>((n_edges + 3) / 4) * 12; }

hipError_t launch_pack24(const int32_t *src_sorted, int64_t n_edges, int64_t src_begin, void *packed, hipStream_t s) {
    if (n_edges <= 0) return hipSuccess;
    const int64_t quads = (n_edges + 3) / 4;
    hipLaunchKernelGGL(k_pack24, dim3(static_cast<unsigned>((quads + 255) / 256)), dim3(256), 0, s, src_sorted, n_edges,
                       static_cast<int32_t>(src_begin), static_cast<uint32_t *>(packed));
    return hipGetLastError();
}

// `src_sorted` has room for n_edges rounded up to a multiple of four words.
hipError_t launch_unpack24(const void *packed, int64_t n_edges, int64_t src_begin, int32_t *src_sorted, hipStream_t s) {
    if (n_edges <= 0) return hipSuccess;
    const int64_t quads = (n_edges + 3) / 4;
    hipLaunchKernelGGL(k_unpack24, dim3(static_cast<unsigned>((quads + 255) / 256)), dim3(256), 0, s,
                       static_cast<const uint32_t *>(packed), n_edges, static_cast<int32_t>(src_begin),
                       reinterpret_cast<int4 *>(src_sorted));
    return hipGetLastError();
}

}  // namespace atlas
