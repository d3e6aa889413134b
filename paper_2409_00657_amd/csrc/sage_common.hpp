// Pieces of the GraphSAGE-mean layer shared by the forward (sage.hip) and backward
// (sage_bwd.hip) translation units: element types, the segmented-mean kernels and their launcher.
#pragma once
#include "common.hpp"

namespace hopgnn {

// Workgroup barrier that waits for this wave's LDS operations only.  __syncthreads()
// would also wait for every outstanding global load and drain the prefetch queue.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}


typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

// ----------------------------------------------------------- element types --

struct TrF32 {
    using store_t = float;
    static constexpr int kPer16 = 4;
    static constexpr hopgnn_dtype kDt = HOPGNN_F32;
    __device__ static __forceinline__ float to_f(float x) { return x; }
    __device__ static __forceinline__ float from_f(float x) { return x; }
};

struct TrBF16 {
    using store_t = uint16_t;
    static constexpr int kPer16 = 8;
    static constexpr hopgnn_dtype kDt = HOPGNN_BF16;
    __device__ static __forceinline__ float to_f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
    __device__ static __forceinline__ uint16_t from_f(float x) {   // round to nearest even
        uint32_t u = __float_as_uint(x);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);   // quiet NaN
        u += 0x7FFFu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
    // two values rounded to nearest even and packed (a in the low half): the hardware's packed
    // conversion, same bits as from_f for every finite value and infinity
    __device__ static __forceinline__ uint32_t pack2(float a, float b) {
        union {
            bf16x2 v;
            uint32_t u;
        } r;
        r.v = __builtin_convertvector(floatx2{a, b}, bf16x2);
        return r.u;
    }
};

struct TrF16 {
    using store_t = _Float16;
    static constexpr int kPer16 = 8;
    static constexpr hopgnn_dtype kDt = HOPGNN_F16;
    __device__ static __forceinline__ float to_f(_Float16 h) { return (float)h; }
    __device__ static __forceinline__ _Float16 from_f(float x) { return (_Float16)x; }
    __device__ static __forceinline__ uint32_t pack2(float a, float b) {
        union {
            halfx2 v;
            uint32_t u;
        } r;
        r.v = __builtin_convertvector(floatx2{a, b}, halfx2);
        return r.u;
    }
};

template <typename Tr>
union Pack16 {
    uint4 v;
    typename Tr::store_t e[Tr::kPer16];
};

// One v_mfma_f32_32x32x16_{bf16,f16}: lane l holds 8 consecutive contraction values of row (A) or
// column (B) l%32, group l/32; the accumulators are fp32.
template <typename Tr>
__device__ __forceinline__ floatx16 mfma16(const uint4& a, const uint4& b, floatx16 c);
template <>
__device__ __forceinline__ floatx16 mfma16<TrBF16>(const uint4& a, const uint4& b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(&a),
                                                   *reinterpret_cast<const bf16x8*>(&b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ floatx16 mfma16<TrF16>(const uint4& a, const uint4& b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const halfx8*>(&a),
                                                  *reinterpret_cast<const halfx8*>(&b), c, 0, 0, 0);
}

// ------------------------------------------------------------ segmented mean --

// Side job of the mean kernels for 2-byte types: the projection wants the weights with k
// contiguous, Wt[n][k] = (k < d_in ? W_self[k][n] : W_neigh[k - d_in][n]), zero outside
// [0, k_total) x [0, d_out); k_total is 2*d_in for the two-matrix layer and d_in for a layer
// with one weight matrix (then W_neigh is never read).  The workgroups after the last mean workgroup each transpose one
// 32 x 32 tile through LDS (coalesced reads and writes), which saves a launch per layer.
struct TransposeJob {
    const uint16_t* Wself;
    const uint16_t* Wneigh;
    uint16_t* Wt;
    int32_t d_in, d_out, KP, NP;
    uint32_t first_block;   // workgroups >= first_block transpose; n_tiles_k = KP / 32
    int32_t k_total;
};

// What the segmented aggregation combines and how:  op 0 = sum divided by the number of terms
// (mean), 1 = plain sum, 2 = element-wise maximum; with_self adds the destination's own source
// row as a term (self_idx, or row r when self_idx is NULL; a negative entry is no term).
// GraphSAGE-mean is {nullptr, 0, 0}.  No terms gives 0 for every op.
struct AggSpec {
    const int32_t* self_idx;
    int32_t with_self;
    int32_t op;
};
constexpr int kAggOpMean = 0, kAggOpSum = 1, kAggOpMax = 2;
constexpr AggSpec kAggMean{nullptr, 0, kAggOpMean};

__device__ __forceinline__ void transpose_w_tile(const TransposeJob& J, uint32_t tile_id) {
    __shared__ uint16_t tile[32][33];
    const uint32_t tiles_k = J.KP / 32;
    const int k0 = (tile_id % tiles_k) * 32, n0 = (tile_id / tiles_k) * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int j = ty; j < 32; j += 8) {
        const int k = k0 + j, n = n0 + tx;
        uint16_t v = 0;
        if (k < J.k_total && n < J.d_out)
            v = k < J.d_in ? J.Wself[(int64_t)k * J.d_out + n] : J.Wneigh[(int64_t)(k - J.d_in) * J.d_out + n];
        tile[j][tx] = v;
    }
    __syncthreads();
    for (int j = ty; j < 32; j += 8) {
        const int n = n0 + j, k = k0 + tx;
        if (n < J.NP && k < J.KP) J.Wt[(int64_t)n * J.KP + k] = tile[tx][j];
    }
}


constexpr int kMeanThreads = 256;
// Neighbour rows a lane has in flight per round.  Fanouts are mostly multiples of 5 (5, 10, 15, 25), so 5
// rows per round leaves no short last round; 2-byte rows (8 values, 8 running sums per word) stay
// at 4, where the extra registers cost more than the round saves.  First-layer aggregation, one
// stream, 4 / 5 / 8 rows: fp32, fanouts 15,10,5: 46.8 / 41.8 / 41.7 us; bf16, fanouts 25,10: 41.4 / 43.3 / 68 us;
// fp16, fanouts 10,10,10: 145 / 150 / 190 us.
template <typename Tr>
struct MeanUnroll {
    static constexpr int value = sizeof(typename Tr::store_t) == 4 ? 5 : 4;
};
constexpr int kMeanUnrollElem = 4;       // the element-wise path

// Vector path: d_in * sizeof(elem) is a multiple of 16.  `group` lanes (a power of
// two <= 64) share one destination row; lane g of the group owns 16-byte word
// g, g+group, ... of the row.  Four neighbour rows are fetched per step; absent
// entries (negative index) are skipped by predication, which measured faster than
// reading a stand-in row and masking it out (whole dead micrographs are common on
// graphs with isolated vertices).  The sum runs in entry order.
// Consecutive workgroups' rows that one XCD takes in a row.  Aggregation of the first layer, one
// stream, 1 (plain round robin) / 4 / 16 / 64 / 256: 56.3 / 52.1 / 46.8 / 46.9 / 46.6 us on 170 k rows of
// 400 bytes with fanouts 15, 10, 5; 43.4 / 41.9 / 41.4 / 41.5 / 48.9 us on 106 k rows of 512 bytes (fanouts
// 25, 10: long runs leave the XCDs with unequal levels); 149 / 147 / 145 / 146 / 146 us on 455 k rows of 256 bytes.
constexpr int kMeanXcdRun = 16;

template <typename Tr, int OP>
__global__ void __launch_bounds__(kMeanThreads)
sage_mean_vec(const uint4* __restrict__ Hsrc, const int32_t* __restrict__ indptr,
              const int32_t* __restrict__ idx, int64_t n_dst, int32_t words_per_row, int32_t group,
              uint4* __restrict__ Mean, uint32_t* __restrict__ zero_row, int32_t zero_words, TransposeJob job,
              AggSpec agg, const int64_t* __restrict__ n_rows_dev, uint32_t xcd_run) {
    if (blockIdx.x >= job.first_block) {
        transpose_w_tile(job, blockIdx.x - job.first_block);
        return;
    }
    if (blockIdx.x == 0)   // the projection reads absent rows and the K padding from this row
        for (int32_t i = threadIdx.x; i < zero_words; i += kMeanThreads) zero_row[i] = 0u;
    if (n_rows_dev != nullptr) {      // the row count lives on the device: rows past it do not exist
        const int64_t live = *n_rows_dev;
        n_dst = live < n_dst ? live : n_dst;
    }
    // Workgroup b runs on XCD b % 8, each with an L2 of its own.  Rows that are near each other in slot
    // order (one micrograph's) read many of the same source rows, so the XCDs take turns at runs of
    // kMeanXcdRun consecutive workgroups' worth of rows instead of single ones: a source row a
    // micrograph reads several times is then fetched into one L2 instead of eight, while every XCD
    // still sees every level of the tree.  (first_block is a multiple of 8 * kMeanXcdRun.)
    const uint32_t seq = blockIdx.x >> 3;
    const int64_t lb = ((int64_t)(seq / xcd_run) * 8 + (blockIdx.x & 7u)) * xcd_run + seq % xcd_run;
    const int64_t gid = (lb * kMeanThreads + threadIdx.x);
    const int64_t r = gid / group;
    const int32_t g = (int32_t)(gid - r * group);
    if (r >= n_dst) return;
    const int32_t beg = indptr[r], end = indptr[r + 1];
    int64_t self_row = -1;
    if (agg.with_self) self_row = agg.self_idx != nullptr ? (int64_t)agg.self_idx[r] : r;
    for (int32_t c = g; c < words_per_row; c += group) {
        float acc[Tr::kPer16];
#pragma unroll
        for (int i = 0; i < Tr::kPer16; ++i) acc[i] = 0.f;
        int32_t cnt = 0;
        constexpr bool is_max = OP == kAggOpMax;
        if (self_row >= 0) {     // first term: the sum starts from 0, the maximum from this row
            Pack16<Tr> v;
            v.v = Hsrc[self_row * words_per_row + c];
#pragma unroll
            for (int i = 0; i < Tr::kPer16; ++i) acc[i] = Tr::to_f(v.e[i]);
            ++cnt;
        }
        for (int32_t e = beg; e < end; e += MeanUnroll<Tr>::value) {
            int32_t u[MeanUnroll<Tr>::value];
            Pack16<Tr> v[MeanUnroll<Tr>::value];
#pragma unroll
            for (int k = 0; k < MeanUnroll<Tr>::value; ++k) u[k] = (e + k < end) ? idx[e + k] : -1;
#pragma unroll
            for (int k = 0; k < MeanUnroll<Tr>::value; ++k)
                if (u[k] >= 0) v[k].v = Hsrc[(int64_t)u[k] * words_per_row + c];
#pragma unroll
            for (int k = 0; k < MeanUnroll<Tr>::value; ++k)
                if (u[k] >= 0) {
#pragma unroll
                    for (int i = 0; i < Tr::kPer16; ++i) {
                        const float x = Tr::to_f(v[k].e[i]);
                        acc[i] = is_max ? (cnt == 0 ? x : fmaxf(acc[i], x)) : acc[i] + x;
                    }
                    ++cnt;
                }
        }
        Pack16<Tr> o;
        const float fc = OP == kAggOpMean ? (float)cnt : 1.f;
#pragma unroll
        for (int i = 0; i < Tr::kPer16; ++i) o.e[i] = Tr::from_f(cnt > 0 ? acc[i] / fc : 0.f);
        Mean[r * words_per_row + c] = o.v;
    }
}

// Element path for rows that are not a whole number of 16-byte words.
template <typename Tr, int OP>
__global__ void __launch_bounds__(kMeanThreads)
sage_mean_elem(const typename Tr::store_t* __restrict__ Hsrc, const int32_t* __restrict__ indptr,
               const int32_t* __restrict__ idx, int64_t n_dst, int32_t d_in, int32_t group,
               typename Tr::store_t* __restrict__ Mean, uint32_t* __restrict__ zero_row, int32_t zero_words,
               TransposeJob job, AggSpec agg, const int64_t* __restrict__ n_rows_dev) {
    if (blockIdx.x >= job.first_block) {
        transpose_w_tile(job, blockIdx.x - job.first_block);
        return;
    }
    if (blockIdx.x == 0)
        for (int32_t i = threadIdx.x; i < zero_words; i += kMeanThreads) zero_row[i] = 0u;
    if (n_rows_dev != nullptr) {      // the row count lives on the device: rows past it do not exist
        const int64_t live = *n_rows_dev;
        n_dst = live < n_dst ? live : n_dst;
    }
    const int64_t gid = ((int64_t)blockIdx.x * kMeanThreads + threadIdx.x);
    const int64_t r = gid / group;
    const int32_t g = (int32_t)(gid - r * group);
    if (r >= n_dst) return;
    const int32_t beg = indptr[r], end = indptr[r + 1];
    int64_t self_row = -1;
    if (agg.with_self) self_row = agg.self_idx != nullptr ? (int64_t)agg.self_idx[r] : r;
    for (int32_t c = g; c < d_in; c += group) {
        float acc = 0.f;
        int32_t cnt = 0;
        constexpr bool is_max = OP == kAggOpMax;
        if (self_row >= 0) {
            acc = Tr::to_f(Hsrc[self_row * d_in + c]);
            ++cnt;
        }
        for (int32_t e = beg; e < end; ++e) {
            const int32_t u = idx[e];
            if (u >= 0) {
                const float x = Tr::to_f(Hsrc[(int64_t)u * d_in + c]);
                acc = is_max ? (cnt == 0 ? x : fmaxf(acc, x)) : acc + x;
                ++cnt;
            }
        }
        Mean[r * d_in + c] = Tr::from_f(cnt > 0 ? (OP == kAggOpMean ? acc / (float)cnt : acc) : 0.f);
    }
}

// ------------------------------------------------------------------ launch --

static inline int mean_group(int units) {   // lanes per destination row: power of two, 1..64
    int g = 1;
    while (g < units && g < 64) g *= 2;
    return g;
}

template <typename Tr>
static hopgnn_status launch_mean(const void* Hsrc, const int32_t* indptr, const int32_t* idx,
                                 int64_t n_dst, int32_t d_in, void* mean, void* zero_row,
                                 size_t zero_bytes, TransposeJob job, uint32_t n_transpose_tiles, hipStream_t s,
                                 AggSpec agg = kAggMean, const int64_t* n_rows_dev = nullptr) {
    using T = typename Tr::store_t;
    const bool vec = (d_in % Tr::kPer16 == 0) && aligned(Hsrc, 16) && aligned(mean, 16);
    const int units = vec ? d_in / Tr::kPer16 : d_in;
    // lanes per destination row: one per 16-byte word (no lane idles on rows that are not a power of two
    // words long: 25 words of a 400-byte row on 32 lanes left 7 of them without work), at most a wavefront
    const int group = vec ? (units < 64 ? units : 64) : mean_group(units);
    constexpr int xcd_run = kMeanXcdRun;
    const int64_t mean_blocks = ceil_div(ceil_div(n_dst * group, kMeanThreads), 8 * xcd_run) * (8 * xcd_run);
    if (mean_blocks + n_transpose_tiles >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    job.first_block = (uint32_t)mean_blocks;
    const int64_t blocks = mean_blocks + n_transpose_tiles;
    auto kv = agg.op == kAggOpMean ? sage_mean_vec<Tr, kAggOpMean>
              : agg.op == kAggOpSum ? sage_mean_vec<Tr, kAggOpSum> : sage_mean_vec<Tr, kAggOpMax>;
    auto ke = agg.op == kAggOpMean ? sage_mean_elem<Tr, kAggOpMean>
              : agg.op == kAggOpSum ? sage_mean_elem<Tr, kAggOpSum> : sage_mean_elem<Tr, kAggOpMax>;
    if (vec)
        hipLaunchKernelGGL(kv, dim3((unsigned)blocks), dim3(kMeanThreads), 0, s,
                           static_cast<const uint4*>(Hsrc), indptr, idx, n_dst, units, group,
                           static_cast<uint4*>(mean), static_cast<uint32_t*>(zero_row), (int32_t)(zero_bytes / 4), job,
                           agg, n_rows_dev, (uint32_t)xcd_run);
    else
        hipLaunchKernelGGL(ke, dim3((unsigned)blocks), dim3(kMeanThreads), 0, s,
                           static_cast<const T*>(Hsrc), indptr, idx, n_dst, d_in, group,
                           static_cast<T*>(mean), static_cast<uint32_t*>(zero_row), (int32_t)(zero_bytes / 4), job,
                           agg, n_rows_dev);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

// Workspace of a projection: [ aggregate : n_rows x d_in ][ Wt : NP x KP, 2-byte types only ][ zero row ]
struct ProjWs {
    size_t agg_bytes, wt_bytes, zero_bytes, total;
    int32_t KP, NP;
};
ProjWs proj_ws_layout(hopgnn_dtype dt, int64_t n_rows, int32_t d_in, int32_t k_total, int32_t d_out);

// Workspace of the attention layer's forward call: [ z : n_src x d_out fp32 ][ scores : n_src x 2*n_heads
// fp32, s_src heads then s_dst heads per row ][ score weights ][ the projection's Wt and zero row ].
// The backward call reads z and the scores from it.
struct GatWs {
    size_t z_bytes, score_bytes, wscore_bytes;   // then the projection's [Wt][zero row]
    ProjWs P;
    size_t total;
};
static inline GatWs gat_ws_layout(hopgnn_dtype dt, int64_t n_src, int32_t d_in, int32_t d_out, int32_t n_heads) {
    GatWs L{};
    const int64_t ns = n_src > 0 ? n_src : 1;
    L.z_bytes = align_up((size_t)ns * d_out * 4, 256);
    L.score_bytes = align_up((size_t)ns * 2 * n_heads * 4, 256);     // [n_src][s_src heads | s_dst heads]
    L.wscore_bytes = align_up((size_t)d_in * 2 * n_heads * 4, 256);
    L.P = proj_ws_layout(dt, 0, d_in, d_in, d_out);     // no aggregate buffer: the rows are Hsrc itself
    L.total = L.z_bytes + L.score_bytes + L.wscore_bytes + L.P.wt_bytes + L.P.zero_bytes;
    return L;
}


// Row tiling of one layer over a slot tree (level-major rows: level 0 = the roots, the children
// of a level-(h-1) slot are f[h] consecutive level-h slots).  Tiles do not cross levels, and on
// levels >= 1 a tile holds whole groups of siblings (g[h] groups of f[h] rows), so that the
// projection's epilogue can also form the NEXT layer's neighbour means - the mean over a
// parent's children of the rows this layer has just produced - and rows of the deepest level,
// which the next layer reads through those means only, need not be written at all.
struct TreeTiles {
    int32_t n_levels;                    // this layer's destination rows are the slots of levels 0 .. n_levels-1
    int32_t store_levels;                // rows of levels < store_levels are written to `out`
    uint32_t tile0[kMaxLayers + 2];      // first row tile of level h; tile0[n_levels] = number of row tiles
    int64_t row0[kMaxLayers + 1];        // first slot of level h
    int64_t rows[kMaxLayers + 1];        // slots on level h
    int32_t f[kMaxLayers + 1];           // siblings per group on level h (level 0: unused)
    int32_t g[kMaxLayers + 1];           // groups per tile on level h
    const int32_t* ids;                  // DEVICE: vertex of every slot (negative = invalid slot, no term of a mean)
    void* mean_next;                     // DEVICE out [slots of levels 0 .. n_levels-2][d_out]; NULL: no means
};

// Host description of the same, before a tile height is chosen.
struct TreeLayer {
    int32_t n_levels;
    int64_t level_rows[kMaxLayers + 1];
    int32_t fan[kMaxLayers + 1];         // fan[h] = children per level-(h-1) slot, h >= 1
    const int32_t* ids;
    void* mean_next;
    int64_t n_src;                       // rows of the layer's source array (bounds what self_idx may name)
};
constexpr int kTreeMaxFan = 64;          // a group of siblings must fit the smallest row tile

// out = act( [x_self | agg][:, :k_total] * [W_self ; W_neigh][:k_total] + bias ) on MFMA (defined with
// the projection kernels).  k_total = 2*d_in is the two-matrix GraphSAGE layer, k_total = d_in a
// plain rows-times-W product over the rows Hsrc[self_idx[r]].  For 2-byte types Wt (row stride KP)
// must already hold the transposed weights; `zero` is a zeroed row of at least 2*d_in+64 elements.
// out_f32 != 0: `out` is a float array and receives the unrounded result whatever dt is.
// n_rows_dev (DEVICE, may be NULL): when given, only the first min(n_dst, *n_rows_dev) rows exist.
// tree (may be NULL): the rows are the slots of a slot tree; rows are tiled level by level in whole
// groups of siblings, the deepest level's rows are not written when tree->mean_next is given, and
// that array receives the next layer's neighbour means (same bits as the segmented-mean kernel
// would give over the stored rows).  Needs rows of whole 16-byte words, every fan <= kTreeMaxFan, no n_rows_dev.
hopgnn_status project_dispatch(hopgnn_dtype dt, hipStream_t s, const void* Hsrc, const int32_t* self_idx,
                               const void* agg, const void* W_self, const void* W_neigh, const uint16_t* Wt,
                               int32_t KP, const void* bias, int64_t n_dst, int32_t d_in, int32_t k_total,
                               int32_t d_out, int relu, const void* zero, void* out, int out_f32,
                               const int64_t* n_rows_dev, const TreeLayer* tree = nullptr);

// Writes the transposed, zero-padded weights of one 2-byte layer (job.Wt, see TransposeJob) and
// clears `zero_row` (zero_bytes, may be 0): what the segmented-mean kernel does as a side job, as
// a launch of its own for layers that run without that kernel.  job.Wt == NULL: only the clearing.
hopgnn_status launch_prep_weights(TransposeJob job, void* zero_row, size_t zero_bytes, hipStream_t s);

// Optional event pairs around the two kernels of a layer (a harness timing them inside its
// timed region); any handle may be NULL.
struct LayerMarks {
    hipEvent_t agg_begin, agg_end, proj_begin, proj_end;
};

// hopgnn_sage_fwd_dev with optional markers (marks may be NULL).
hopgnn_status sage_fwd_marked(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in, const int32_t* self_idx,
                              const int32_t* indptr, const int32_t* idx, int64_t n_dst, const int64_t* n_dst_dev,
                              const void* W_self, const void* W_neigh, const void* bias, int32_t d_out, int32_t agg,
                              int32_t relu, void* out, void* ws, size_t ws_bytes, void* stream,
                              const LayerMarks* marks);

}  // namespace hopgnn
