// Dense part of a plan's first chunk.
//
// With ids in in-degree-descending order (paper Sec. 3.8) the first chunk's
// edges between the hottest sources and the hottest destinations are so many
// that the corresponding corner of the adjacency matrix is denser than one
// edge per hundred cells.  There the per-edge row gather (a 256-byte random
// read per edge) costs more than multiplying the corner as a dense matrix:
// the plan keeps the corner's multiplicities as 4-bit counts (`cells`), and the
// layer adds  cells x X[sources]  to the accumulator rows on the matrix cores
// (multiplicities up to 15 are exact 16-bit floats, products are exact, sums
// are fp32: the same sums as the edge stream in another order).  The region is
// a staircase: 256 destinations form a band, and each band has its own number
// of sources.  Half a byte per cell because the contraction is bound by the
// stream of cells out of HBM, not by the matrix pipeline; the few pairs that
// occur more than 15 times leave the surplus in the chunk's edge list.
//
// Cell layout.  A band's cells are stored in the order the kernel's wavefronts
// consume them, so that every load is a contiguous kilobyte: per k-step of 64
// sources 8 KB = [wave 0..3][row block 0..1][lane 0..63][16 bytes]; lane l of
// wave w holds destination row 64 w + 32 rb + (l & 31) of the band, and dword u
// of its 16 bytes holds the multiplicities of sources 16 u + 8 (l >> 5) + j,
// j = 0..7: j < 4 in the low half of byte j, j >= 4 in the high half of byte
// j - 4 -- the lane's 8-element operand for the matrix instruction's k-step u.
#include "atlas_kernels.h"

namespace atlas {
namespace {

constexpr int kBlock = 256;

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// Log-spaced bucket of a rank: 0 for ranks below 256, then one bucket per power of two.
__device__ __forceinline__ int rank_bucket(uint32_t x) { return x < 256u ? 0 : 24 - __clz(x); }

// Edge counts by (source bucket, destination bucket) of one chunk.
__global__ __launch_bounds__(kBlock) void k_dense_histogram(const int32_t *src_of_edge, const int32_t *col,
                                                             int64_t ne, int64_t src_begin,
                                                             unsigned long long *hist) {
    __shared__ unsigned int h[kDenseBuckets * kDenseBuckets];
    for (int i = threadIdx.x; i < kDenseBuckets * kDenseBuckets; i += kBlock) h[i] = 0;
    __syncthreads();
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < ne; i += stride) {
        const int bs = rank_bucket(static_cast<uint32_t>(src_of_edge[i] - src_begin));
        const int bd = rank_bucket(static_cast<uint32_t>(col[i]));
        atomicAdd(&h[bs * kDenseBuckets + bd], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kDenseBuckets * kDenseBuckets; i += kBlock)
        if (h[i]) atomicAdd(&hist[i], static_cast<unsigned long long>(h[i]));
}

// byte offset of the cell of (destination d, source s) and, in *high, which half of the byte it is
__device__ __forceinline__ int64_t cell_offset(const int64_t *band_off, uint32_t d, uint32_t s, uint32_t *high) {
    const uint32_t r = d & 255u, k = s & 63u;
    const uint32_t w = r >> 6, rb = (r >> 5) & 1u, row = r & 31u;
    const uint32_t u = k >> 4, kg = (k >> 3) & 1u, j = k & 7u;
    const uint32_t lane = kg * 32u + row;
    *high = j >> 2;
    return band_off[d >> 8] + static_cast<int64_t>(s >> 6) * kDenseKstepBytes + ((w * 2u + rb) * 64u + lane) * 16u +
           u * 4u + (j & 3u);
}

// Every edge of the chunk that falls into the region raises its cell by one
// and is flagged; a cell that is full (15) leaves the edge to the edge list.
__global__ __launch_bounds__(kBlock) void k_dense_divert(const int32_t *src_of_edge, const int32_t *col, int64_t ne,
                                                          int64_t src_begin, int64_t rows, const int32_t *band_ksteps,
                                                          const int64_t *band_off, uint8_t *cells, uint8_t *flags) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < ne; i += stride) {
        const uint32_t s = static_cast<uint32_t>(src_of_edge[i] - src_begin);
        const uint32_t d = static_cast<uint32_t>(col[i]);
        bool taken = false;
        if (static_cast<int64_t>(d) < rows && s < static_cast<uint32_t>(band_ksteps[d >> 8]) * 64u) {
            uint32_t high = 0;
            const int64_t off = cell_offset(band_off, d, s, &high);
            unsigned int *word = reinterpret_cast<unsigned int *>(cells) + (off >> 2);
            const unsigned int sh = static_cast<unsigned int>(off & 3) * 8u + high * 4u;
            unsigned int old = __atomic_load_n(word, __ATOMIC_RELAXED);
            while (((old >> sh) & 0xfu) != 0xfu) {
                const unsigned int seen = atomicCAS(word, old, old + (1u << sh));
                if (seen == old) {
                    taken = true;
                    break;
                }
                old = seen;
            }
        }
        flags[i] = taken ? 1 : 0;
    }
}

// The two halves of the chunk, each in CSR order: flagged edges to the back.
__global__ __launch_bounds__(kBlock) void k_dense_split(const int32_t *src_of_edge, const int32_t *col,
                                                         const uint8_t *flags, const uint32_t *flagged_before,
                                                         int64_t ne, int64_t n_rest, uint32_t *dst_out,
                                                         int32_t *src_out) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < ne; i += stride) {
        const int64_t fb = flagged_before[i];
        const int64_t pos = flags[i] ? n_rest + fb : i - fb;
        dst_out[pos] = static_cast<uint32_t>(col[i]);
        src_out[pos] = src_of_edge[i];
    }
}

// Rows of the chunk in the layout the contraction reads: per k-step of 64
// sources, N features x 128 bytes; the 16-byte piece of 8 sources that a lane
// of the matrix instruction takes at once sits at slot (piece ^ (feature & 7))
// of the feature's 128 bytes, which spreads the lanes' reads over the banks.
// Sources past the chunk's end are zeros.
template <int N>
__global__ __launch_bounds__(kBlock) void k_dense_pack_rows(const uint16_t *x, int64_t n_rows, int64_t n_ksteps,
                                                             uint16_t *xt) {
    __shared__ uint16_t tile[64][N + 2];
    for (int64_t ks = blockIdx.x; ks < n_ksteps; ks += gridDim.x) {
        for (int i = threadIdx.x; i < 64 * (N / 2); i += kBlock) {
            const int r = i / (N / 2), c2 = i % (N / 2);
            const int64_t row = ks * 64 + r;
            uint32_t v = 0;
            if (row < n_rows) v = *reinterpret_cast<const uint32_t *>(x + row * N + c2 * 2);
            tile[r][c2 * 2] = static_cast<uint16_t>(v & 0xffffu);
            tile[r][c2 * 2 + 1] = static_cast<uint16_t>(v >> 16);
        }
        __syncthreads();
        for (int i = threadIdx.x; i < N * 8; i += kBlock) {
            const int n = i >> 3, piece = i & 7;
            uint32_t q[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                q[j] = static_cast<uint32_t>(tile[piece * 8 + 2 * j][n]) |
                       (static_cast<uint32_t>(tile[piece * 8 + 2 * j + 1][n]) << 16);
            uint16_t *o = xt + (ks * N + n) * 64 + ((piece ^ (n & 7)) * 8);
            *reinterpret_cast<uint4 *>(o) = make_uint4(q[0], q[1], q[2], q[3]);
        }
        __syncthreads();
    }
}

template <int CT> struct Operand;
template <> struct Operand<1> { using type = bf16x8_t; };
template <> struct Operand<2> { using type = f16x8_t; };

// eight multiplicities (bytes of lo, then of hi) as the lane's operand
template <int CT>
__device__ __forceinline__ typename Operand<CT>::type bytes_to_operand(uint32_t lo, uint32_t hi) {
    const float f0 = static_cast<float>(lo & 0xffu), f1 = static_cast<float>((lo >> 8) & 0xffu);
    const float f2 = static_cast<float>((lo >> 16) & 0xffu), f3 = static_cast<float>(lo >> 24);
    const float f4 = static_cast<float>(hi & 0xffu), f5 = static_cast<float>((hi >> 8) & 0xffu);
    const float f6 = static_cast<float>((hi >> 16) & 0xffu), f7 = static_cast<float>(hi >> 24);
    uint4 q;
    if constexpr (CT == 1) {
        // an integer below 256 has at most 8 significant bits: the upper half of its float is its bf16, exactly
        q.x = __builtin_amdgcn_perm(__float_as_uint(f1), __float_as_uint(f0), 0x07060302u);
        q.y = __builtin_amdgcn_perm(__float_as_uint(f3), __float_as_uint(f2), 0x07060302u);
        q.z = __builtin_amdgcn_perm(__float_as_uint(f5), __float_as_uint(f4), 0x07060302u);
        q.w = __builtin_amdgcn_perm(__float_as_uint(f7), __float_as_uint(f6), 0x07060302u);
    } else {
        typedef __fp16 h2 __attribute__((ext_vector_type(2)));
        const h2 a = __builtin_amdgcn_cvt_pkrtz(f0, f1), b = __builtin_amdgcn_cvt_pkrtz(f2, f3);
        const h2 c = __builtin_amdgcn_cvt_pkrtz(f4, f5), d = __builtin_amdgcn_cvt_pkrtz(f6, f7);
        q.x = __builtin_bit_cast(uint32_t, a);
        q.y = __builtin_bit_cast(uint32_t, b);
        q.z = __builtin_bit_cast(uint32_t, c);
        q.w = __builtin_bit_cast(uint32_t, d);
    }
    return __builtin_bit_cast(typename Operand<CT>::type, q);
}

// eight 4-bit multiplicities: elements 0..3 in the low halves of the dword's bytes, 4..7 in the high halves
template <int CT>
__device__ __forceinline__ typename Operand<CT>::type nibbles_to_operand(uint32_t q) {
    return bytes_to_operand<CT>(q & 0x0f0f0f0fu, (q >> 4) & 0x0f0f0f0fu);
}

template <int CT>
__device__ __forceinline__ f32x16_t mfma(typename Operand<CT>::type a, typename Operand<CT>::type b, f32x16_t c) {
    if constexpr (CT == 1) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

struct CellRegs { uint4 q[2]; };   // [row block]: dword u = the lane's eight cells of the matrix instruction's k-step u

// acc[band rows][N] += cells[band rows][sources of the item] x X[sources][N].
// One workgroup (4 waves) per work item = 256 destinations x up to
// kDenseItemKsteps k-steps of 64 sources; wave w owns rows 64 w .. 64 w + 63
// (two 32-row blocks) and all N features (NB blocks of 32).  The
// multiplicities go from HBM straight into the registers of the lane that
// needs them (see the layout above), two k-steps ahead; the rows' tile
// (N x 64, 16-bit) is shared by the four waves through a double-buffered LDS
// tile, its loads two k-steps ahead too.  With the cells as the FIRST operand
// a lane holds 16 destinations of ONE feature, so the 32 lanes of a half-wave
// write 128 consecutive bytes of one row.  A band that is one item stores its
// sums; the partial sums of a longer band's items meet in the accumulator
// through fp32 atomics (64-byte atomic requests are what the chip retires
// slowest, some 20 G a second, so items are long and short bands avoid them).
template <int CT, int NB>
__global__ __launch_bounds__(kBlock, 2) void k_dense_contract(DenseArgs a) {
    constexpr int N = NB * 32;
    constexpr int kTileBytes = N * 128;
    constexpr int kPieces = kTileBytes / 16 / kBlock;   // 16-byte pieces of the tile per thread
    using op_t = typename Operand<CT>::type;
    __shared__ __align__(16) unsigned char tile[2][kTileBytes];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int32_t band = a.items[blockIdx.x * 3], ks0 = a.items[blockIdx.x * 3 + 1];
    const int32_t nks = a.items[blockIdx.x * 3 + 2] & 0xffff;
    const bool sole = (a.items[blockIdx.x * 3 + 2] >> 16) != 0;   // the band's only item: its rows are this workgroup's alone
    const unsigned char *cells = a.cells + a.band_off[band] + static_cast<int64_t>(ks0) * kDenseKstepBytes + (w * 2 * 64 + lane) * 16;
    const unsigned char *xt = static_cast<const unsigned char *>(a.xt) + static_cast<int64_t>(ks0) * kTileBytes + threadIdx.x * 16;

    auto load_cells = [&](int s, CellRegs &r) __attribute__((always_inline)) {
        const unsigned char *p = cells + static_cast<int64_t>(s) * kDenseKstepBytes;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            // read once: a streaming load, so that the cells do not push the shared row tiles out of the caches
            typedef unsigned int u4 __attribute__((ext_vector_type(4)));
            const u4 v = __builtin_nontemporal_load(reinterpret_cast<const u4 *>(p + rb * 1024));
            r.q[rb] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    // The tile registers are plain variables handled by macros: as arrays or structs passed to helper
    // closures they were kept in scratch memory across the loop's back edge.
    static_assert(kPieces == 2 || kPieces == 4, "tile pieces per thread");
#define ATLAS_TILE_LOAD(S, T)                                                                         \
    {                                                                                                 \
        const unsigned char *tp_ = xt + static_cast<int64_t>(S) * kTileBytes;                         \
        T##0 = *reinterpret_cast<const uint4 *>(tp_);                                                 \
        T##1 = *reinterpret_cast<const uint4 *>(tp_ + kBlock * 16);                                   \
        if constexpr (kPieces == 4) {                                                                 \
            T##2 = *reinterpret_cast<const uint4 *>(tp_ + 2 * kBlock * 16);                           \
            T##3 = *reinterpret_cast<const uint4 *>(tp_ + 3 * kBlock * 16);                           \
        }                                                                                             \
    }
#define ATLAS_TILE_STORE(BUF, T)                                                                      \
    {                                                                                                 \
        unsigned char *tp_ = &tile[BUF][threadIdx.x * 16];                                            \
        *reinterpret_cast<uint4 *>(tp_) = T##0;                                                       \
        *reinterpret_cast<uint4 *>(tp_ + kBlock * 16) = T##1;                                         \
        if constexpr (kPieces == 4) {                                                                 \
            *reinterpret_cast<uint4 *>(tp_ + 2 * kBlock * 16) = T##2;                                 \
            *reinterpret_cast<uint4 *>(tp_ + 3 * kBlock * 16) = T##3;                                 \
        }                                                                                             \
    }

    f32x16_t c[2][NB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) c[rb][nb][i] = 0.f;

    // the lane's read offset in a tile: feature (lane & 31) of block nb, piece 2 u + (lane >> 5), swizzled
    const int roff_row = (lane & 31) * 128, roff_half = lane >> 5, roff_swz = lane & 7;

    // Loads of a wave return in issue order, so a wait for one load also waits for every load issued before
    // it.  Each step issues the tile of step s + 2 and then the cells of step s + 2, nothing else; the waits
    // (for the tile of step s + 1 before it goes to LDS, for the cells of step s + 1 at the next step) then
    // leave the younger loads in flight, and both kinds of load have two full steps to arrive.
    CellRegs m0, m1, m2;
    uint4 ta0, ta1, ta2 = make_uint4(0, 0, 0, 0), ta3 = ta2, tb0, tb1, tb2 = ta2, tb3 = ta2;
    ATLAS_TILE_LOAD(0, ta)
    load_cells(0, m0);
    ATLAS_TILE_STORE(0, ta)
    ATLAS_TILE_LOAD(nks > 1 ? 1 : 0, ta)
    load_cells(nks > 1 ? 1 : 0, m1);
    __syncthreads();
    // one step: HELD carries the tile of step S + 1 (stored to LDS at the end), FRESH receives that of S + 2
    // (loads past the item's end repeat its last k-step: in bounds, unused)
#define ATLAS_DENSE_STEP(S, HELD, FRESH, MC, MF)                                                      \
    {                                                                                                 \
        ATLAS_TILE_LOAD((S) + 2 < nks ? (S) + 2 : nks - 1, FRESH)                                     \
        __builtin_amdgcn_sched_barrier(0);                                                            \
        load_cells((S) + 2 < nks ? (S) + 2 : nks - 1, MF);                                            \
        __builtin_amdgcn_sched_barrier(0);                                                            \
        const unsigned char *t = tile[(S) & 1] + roff_row;                                            \
        op_t xb[NB], xn[NB], ma[2], mn[2];                                                            \
        _Pragma("unroll") for (int nb = 0; nb < NB; ++nb)                                             \
            xb[nb] = *reinterpret_cast<const op_t *>(t + nb * 4096 + ((roff_half ^ roff_swz) * 16));  \
        _Pragma("unroll") for (int rb = 0; rb < 2; ++rb)                                              \
            ma[rb] = nibbles_to_operand<CT>(MC.q[rb].x);                                              \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) {                                               \
            /* operands of the matrix instruction's next k-step: rows from LDS, cells converted */    \
            if (u < 3) {                                                                              \
                _Pragma("unroll") for (int nb = 0; nb < NB; ++nb)                                     \
                    xn[nb] = *reinterpret_cast<const op_t *>(                                         \
                        t + nb * 4096 + (((2 * (u + 1) + roff_half) ^ roff_swz) * 16));               \
                _Pragma("unroll") for (int rb = 0; rb < 2; ++rb) {                                    \
                    const uint4 q = MC.q[rb];                                                         \
                    mn[rb] = nibbles_to_operand<CT>(u == 0 ? q.y : u == 1 ? q.z : q.w);               \
                }                                                                                     \
            }                                                                                         \
            _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) {                                       \
                _Pragma("unroll") for (int rb = 0; rb < 2; ++rb)                                      \
                    c[rb][nb] = mfma<CT>(ma[rb], xb[nb], c[rb][nb]);                                  \
            }                                                                                         \
            if (u < 3) {                                                                              \
                _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) xb[nb] = xn[nb];                    \
                ma[0] = mn[0];                                                                        \
                ma[1] = mn[1];                                                                        \
            }                                                                                         \
        }                                                                                             \
        /* issue order within the step: after the first operands, every product is followed by */     \
        /* some of the next operands' conversion instructions and every second one by a read */      \
        /* of a row operand, so that the matrix pipeline works while the vector ALU converts */       \
        __builtin_amdgcn_sched_group_barrier(0x100, NB, 0);                                           \
        __builtin_amdgcn_sched_group_barrier(0x002, 30, 0);                                           \
        _Pragma("unroll") for (int g = 0; g < 3 * 2 * NB; ++g) {                                      \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                        \
            __builtin_amdgcn_sched_group_barrier(0x002, (30 + 2 * NB - 1) / (2 * NB), 0);             \
            if ((g & 1) == 0) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                      \
        }                                                                                             \
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * NB, 0);                                       \
        __builtin_amdgcn_sched_barrier(0);                                                            \
        if ((S) + 1 < nks) ATLAS_TILE_STORE(((S) + 1) & 1, HELD)                                      \
        __syncthreads();                                                                              \
    }
    // Six steps per round: the two tile register sets and the three cell register sets return to their roles
    // without a single register copy -- a copy of a set whose loads are still in flight would wait for them
    // and expose the whole memory latency in every step.  An item has a multiple of twelve k-steps.
    for (int s = 0; s < nks; s += 6) {
        ATLAS_DENSE_STEP(s, ta, tb, m0, m2)
        ATLAS_DENSE_STEP(s + 1, tb, ta, m1, m0)
        ATLAS_DENSE_STEP(s + 2, ta, tb, m2, m1)
        ATLAS_DENSE_STEP(s + 3, tb, ta, m0, m2)
        ATLAS_DENSE_STEP(s + 4, ta, tb, m1, m0)
        ATLAS_DENSE_STEP(s + 5, tb, ta, m2, m1)
    }
#undef ATLAS_DENSE_STEP
#undef ATLAS_TILE_LOAD
#undef ATLAS_TILE_STORE

    // value 4 q + t of a lane: destination 8 q + 4 (lane >> 5) + t of the row block, feature 32 nb + (lane & 31)
    const int64_t row0 = static_cast<int64_t>(band) * 256 + w * 64;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t row = row0 + rb * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
            if (row < a.n) {
                float *o = a.acc + row * N + (lane & 31);
                if (sole) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) o[nb * 32] = c[rb][nb][i];
                } else {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) unsafeAtomicAdd(o + nb * 32, c[rb][nb][i]);
                }
            }
        }
}

// Pending counts of the region's destinations minus their dense messages; the
// vertices that complete go to the ready list.  Nothing else runs on the
// stream, every thread owns its vertex: plain read-modify-write.
__global__ __launch_bounds__(kBlock) void k_dense_pending(const int32_t *msgs, int64_t rows, int64_t n_edges,
                                                           int32_t *pending, int32_t *ready, int32_t *counters,
                                                           unsigned long long *counters64) {
    const int64_t v = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (v == 0) atomicAdd(&counters64[CTR64_EDGES], static_cast<unsigned long long>(n_edges));
    bool done = false;
    if (v < rows) {
        const int32_t c = msgs[v];
        if (c > 0) {
            const int32_t old = pending[v];
            pending[v] = old - c;
            done = old == c;
        }
    }
    const uint64_t m = __ballot(done);
    if (m == 0) return;
    const int lane = threadIdx.x & 63;
    int base = 0;
    if (lane == 0) base = atomicAdd(&counters[CTR_READY_TAIL], __popcll(m));
    base = __builtin_amdgcn_readfirstlane(base);
    if (done) ready[base + __popcll(m & ((1ull << lane) - 1ull))] = static_cast<int32_t>(v);
}

unsigned grid_for(int64_t items, int per_block) {
    int64_t b = (items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > 256 * 16) b = 256 * 16;
    return static_cast<unsigned>(b);
}

}  // namespace

hipError_t launch_dense_histogram(const int32_t *src_of_edge, const int32_t *col, int64_t ne, int64_t src_begin,
                                  unsigned long long *hist, hipStream_t s) {
    hipError_t err = hipMemsetAsync(hist, 0, sizeof(unsigned long long) * kDenseBuckets * kDenseBuckets, s);
    if (err != hipSuccess || ne <= 0) return err;
    hipLaunchKernelGGL(k_dense_histogram, dim3(grid_for(ne, kBlock * 16)), dim3(kBlock), 0, s, src_of_edge, col, ne,
                       src_begin, hist);
    return hipGetLastError();
}

hipError_t launch_dense_divert(const int32_t *src_of_edge, const int32_t *col, int64_t ne, int64_t src_begin,
                               const DensePart &p, uint8_t *flags, hipStream_t s) {
    if (ne <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_dense_divert, dim3(grid_for(ne, kBlock * 4)), dim3(kBlock), 0, s, src_of_edge, col, ne,
                       src_begin, p.rows, p.band_ksteps, p.band_off, p.cells, flags);
    return hipGetLastError();
}

hipError_t launch_dense_split(const int32_t *src_of_edge, const int32_t *col, const uint8_t *flags,
                              const uint32_t *flagged_before, int64_t ne, int64_t n_rest, uint32_t *dst_out,
                              int32_t *src_out, hipStream_t s) {
    if (ne <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_dense_split, dim3(grid_for(ne, kBlock * 4)), dim3(kBlock), 0, s, src_of_edge, col, flags,
                       flagged_before, ne, n_rest, dst_out, src_out);
    return hipGetLastError();
}

bool dense_contract_takes(int d, int in_dt) { return (d == 64 || d == 128) && (in_dt == 1 || in_dt == 2); }

size_t dense_packed_rows_bytes(const DensePart &p, int d) {
    return static_cast<size_t>(p.max_ksteps) * static_cast<size_t>(d) * 128;
}

hipError_t launch_dense_prepare(const DensePart &p, const void *emb, int64_t chunk_rows, int d, int in_dt, void *xt,
                                float *acc, int64_t n, hipStream_t s) {
    if (!dense_contract_takes(d, in_dt) || p.n_items <= 0) return hipErrorInvalidValue;
    const int64_t rows = p.rows < n ? p.rows : n;
    hipError_t err = launch_fill_zero(acc, static_cast<size_t>(rows) * d * sizeof(float), s);
    if (err != hipSuccess) return err;
    const unsigned pg = grid_for(p.max_ksteps, 1);
    const uint16_t *x = static_cast<const uint16_t *>(emb);
    if (d == 128) hipLaunchKernelGGL((k_dense_pack_rows<128>), dim3(pg), dim3(kBlock), 0, s, x, chunk_rows,
                                     static_cast<int64_t>(p.max_ksteps), static_cast<uint16_t *>(xt));
    else hipLaunchKernelGGL((k_dense_pack_rows<64>), dim3(pg), dim3(kBlock), 0, s, x, chunk_rows,
                            static_cast<int64_t>(p.max_ksteps), static_cast<uint16_t *>(xt));
    return hipGetLastError();
}

hipError_t launch_dense_contract(const DensePart &p, int d, int in_dt, const void *xt, float *acc, int64_t n,
                                 hipStream_t s) {
    if (!dense_contract_takes(d, in_dt) || p.n_items <= 0) return hipErrorInvalidValue;
    DenseArgs a{};
    a.cells = p.cells;
    a.band_off = p.band_off;
    a.items = p.items;
    a.xt = xt;
    a.acc = acc;
    a.n = n;
    const dim3 g(static_cast<unsigned>(p.n_items)), b(kBlock);
    if (d == 128) {
        if (in_dt == 1) hipLaunchKernelGGL((k_dense_contract<1, 4>), g, b, 0, s, a);
        else hipLaunchKernelGGL((k_dense_contract<2, 4>), g, b, 0, s, a);
    } else {
        if (in_dt == 1) hipLaunchKernelGGL((k_dense_contract<1, 2>), g, b, 0, s, a);
        else hipLaunchKernelGGL((k_dense_contract<2, 2>), g, b, 0, s, a);
    }
    return hipGetLastError();
}

hipError_t launch_dense_pending(const DensePart &p, int64_t n, int32_t *pending, int32_t *ready, int32_t *counters,
                                unsigned long long *counters64, hipStream_t s) {
    const int64_t rows = p.rows < n ? p.rows : n;
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_dense_pending, dim3(static_cast<unsigned>((rows + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                       p.msgs, rows, p.list.n_edges, pending, ready, counters, counters64);
    return hipGetLastError();
}

}  // namespace atlas
