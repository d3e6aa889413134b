// hopgnn_sage_bwd: backward of one GraphSAGE-mean layer with in-place accumulation of
// the weight gradients (paper section 5.1, steps 3-4: every micrograph batch runs forward
// and backward where it sits and the gradients are accumulated until the subgraph is done;
// the discussion section: accumulated partial gradients are updated in place).
//
//   dZ        = dOut masked by the stored forward output (ReLU)          bwd_mask
//   G         = [x_self | mean]^T dZ      (2*d_in x d_out)               bwd_weight_grad (MFMA)
//   gW_self  += G[:d_in], gW_neigh += G[d_in:], gbias += colsum(dZ)      bwd_weight_reduce
//   [dXs|dM]  = dZ [W_self ; W_neigh]^T   (n_dst x 2*d_in)               bwd_input_grad (MFMA)
//   dHsrc[self_idx[r]] += dXs[r];  dHsrc[idx[e]] += dM[r] / c_r          bwd_scatter
//
// Hsrc, the weights and the stored forward output are in the activation type (fp32, bf16 or
// fp16); gradients (dOut, gW, gbias, dHsrc) are always fp32 in memory.  For fp32 activations the
// contractions run on the fp32 MFMA.  For 2-byte activations they run on the 2-byte MFMA with fp32
// accumulators, dZ rounded to the activation type on its way into LDS (shapes whose rows are not
// whole 16-byte runs take the fp32 MFMA with the 2-byte operands widened instead); the bias gradient
// always sums fp32 values.  The weight gradient contracts over the destination
// rows, which are split over workgroups; the partial tiles are summed in split order by a
// second kernel, so gW/gbias are bit-stable from run to run.  dHsrc uses float atomic adds:
// bit-stable when a source row receives at most two contributions (always the case for the
// slot-tree layout of hopgnn_sample: one self term, one parent), otherwise the rounding
// depends on arrival order.
#include <type_traits>

#include "sage_common.hpp"

namespace hopgnn {

constexpr int kBwdThreads = 256;

// Four consecutive stored elements as they sit in memory (16 bytes of fp32, 8 bytes of a 2-byte
// type); widened to fp32 only where the values are consumed, so that a prefetched load is not
// waited for at its issue point.
template <typename Tr>
struct Raw4 {
    using type = uint2;
    __device__ static __forceinline__ float4 widen(uint2 v) {
        union { uint2 v; typename Tr::store_t e[4]; } u;
        u.v = v;
        return make_float4(Tr::to_f(u.e[0]), Tr::to_f(u.e[1]), Tr::to_f(u.e[2]), Tr::to_f(u.e[3]));
    }
};
template <>
struct Raw4<TrF32> {
    using type = float4;
    __device__ static __forceinline__ float4 widen(float4 v) { return v; }
};

// ---------------------------------------------------------------- dZ mask --

template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
bwd_mask4(const typename Raw4<Tr>::type* __restrict__ out_fwd, const float4* __restrict__ dOut, int64_t n4,
          float4* __restrict__ dZ, const int64_t* __restrict__ n_rows_dev, int32_t row4) {
    const int64_t i = (int64_t)blockIdx.x * kBwdThreads + threadIdx.x;
    if (i >= n4 || (n_rows_dev != nullptr && i >= *n_rows_dev * row4)) return;     // row4 = 16-byte items per row
    const float4 o = Raw4<Tr>::widen(out_fwd[i]);
    float4 g = dOut[i];
    g.x = o.x > 0.f ? g.x : 0.f;
    g.y = o.y > 0.f ? g.y : 0.f;
    g.z = o.z > 0.f ? g.z : 0.f;
    g.w = o.w > 0.f ? g.w : 0.f;
    dZ[i] = g;
}

template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
bwd_mask_elem(const typename Tr::store_t* __restrict__ out_fwd, const float* __restrict__ dOut, int64_t n,
              float* __restrict__ dZ, const int64_t* __restrict__ n_rows_dev, int32_t d_out) {
    const int64_t i = (int64_t)blockIdx.x * kBwdThreads + threadIdx.x;
    if (n_rows_dev != nullptr && i >= *n_rows_dev * d_out) return;
    if (i < n) dZ[i] = Tr::to_f(out_fwd[i]) > 0.f ? dOut[i] : 0.f;
}

__global__ void __launch_bounds__(kBwdThreads)
bwd_zero_elem(float* __restrict__ p, int64_t n, const int64_t* __restrict__ n_rows_dev, int32_t row_items) {
    const int64_t i = (int64_t)blockIdx.x * kBwdThreads + threadIdx.x;
    if (n_rows_dev != nullptr && i >= *n_rows_dev * row_items) return;
    if (i < n) p[i] = 0.f;
}

__global__ void __launch_bounds__(kBwdThreads)
bwd_zero(float4* __restrict__ p, int64_t n4, const int64_t* __restrict__ n_rows_dev, int32_t row_items) {
    const int64_t i = (int64_t)blockIdx.x * kBwdThreads + threadIdx.x;
    if (n_rows_dev != nullptr && i >= *n_rows_dev * row_items) return;
    if (i < n4) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// ---------------------------------------------------------- weight gradient --
//
// G[k][n] = sum_r A[r][k] dZ[r][n] with A = [x_self | mean].  The contraction index r is the
// MFMA's K dimension: for v_mfma_f32_32x32x2_f32 lane l feeds A[r + l/32][k0 + l%32] and
// dZ[r + l/32][n0 + l%32], i.e. both operands are 32 consecutive floats of a row - no
// transposition anywhere.  A workgroup (4 waves, 2 x 2) owns a 128 x 128 tile of G for the rows
// [split*rows_per_split, ...), a wave a 64 x 64 piece (2 x 2 MFMA tiles: two A values and two
// dZ values feed four MFMAs).  Rows are staged 16 at a time through LDS, so that every element
// leaves global memory once per workgroup in a 128-bit load; the next chunk's loads (and the
// self indices of the chunk after it) are in flight while the current chunk is multiplied.
// Every load is unconditional from a clamped, in-bounds address and masked when it is written
// to LDS, which keeps the loop free of branches.  The tile goes to partial[split]; workgroups
// of the first k-tile row also produce the column sums of dZ.
// The host sizes the row splits for the capacity; when only the device knows how many rows exist,
// the rows that do are dealt out evenly over the same number of splits (multiples of 32 rows, never
// more than the host's figure), so that no split idles while another works through the whole input.
__device__ __forceinline__ int32_t balanced_split(int32_t rows_per_split, int64_t n_rows, bool device_count,
                                                  int32_t n_splits) {
    if (!device_count) return rows_per_split;
    int64_t need = (n_rows + n_splits - 1) / n_splits;
    need = (need + 31) / 32 * 32;
    need = need > 32 ? need : 32;
    return need < rows_per_split ? (int32_t)need : rows_per_split;
}

constexpr int kGradTile = 128;
constexpr int kGradRows = 16;               // contraction rows per LDS chunk
constexpr int kGradLd = kGradTile + 32;     // LDS row stride: the two rows of one MFMA step sit 32 banks apart

// One thread's share of a chunk: two rows (lr, lr + 8), four consecutive columns, of each operand.
template <typename Tr>
struct GradFrag {
    typename Raw4<Tr>::type a[2];
    float4 b[2];
    typename Raw4<Tr>::type o[2];      // MASK: the stored forward outputs that decide the ReLU mask
};

// MASK: dZ is the incoming gradient itself and OutFwd the stored forward output; the ReLU mask is
// applied on the way into LDS (a layer whose input gradient is not needed has no other reader of
// the masked gradient, so the separate masking pass and its array are saved).
template <typename Tr, bool VEC, bool MASK>
__global__ void __launch_bounds__(kBwdThreads)
bwd_weight_grad(const typename Tr::store_t* __restrict__ Hsrc, const int32_t* __restrict__ self_idx,
                const typename Tr::store_t* __restrict__ Mean, const float* __restrict__ dZ,
                const typename Tr::store_t* __restrict__ OutFwd, int64_t n_dst, int32_t d_in,
                int32_t d_out, int32_t rows_per_split, uint32_t tiles_n, float* __restrict__ partial,
                float* __restrict__ bias_partial, const int64_t* __restrict__ n_rows_dev, int32_t k_self) {
    __shared__ __attribute__((aligned(16))) float As[2][kGradRows][kGradLd];
    __shared__ __attribute__((aligned(16))) float Bs[2][kGradRows][kGradLd];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, l32 = lane & 31;
    const int wk = wave >> 1, wn = wave & 1;
    const int K = k_self + d_in;      // k_self = d_in: A = [x_self | aggregate]; 0: the aggregate alone
    const uint32_t tk = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
    // rows that exist (n_dst is the capacity: addresses are clamped to it, rows past n_rows are masked)
    const int64_t n_rows = n_rows_dev != nullptr && *n_rows_dev < n_dst ? *n_rows_dev : n_dst;
    rows_per_split = balanced_split(rows_per_split, n_rows, n_rows_dev != nullptr, (int32_t)gridDim.y);
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_split;
    int64_t r1 = r0 + rows_per_split < n_rows ? r0 + rows_per_split : n_rows;
    r1 = r1 > r0 ? r1 : r0;                    // a split past the last row: no chunk, a zero tile
    const int n_chunks = (int)((r1 - r0 + kGradRows - 1) / kGradRows);

    // this thread's part of every chunk
    const int lr = tid >> 5, lc = (tid & 31) * 4;
    const int ka = (int)tk * kGradTile + lc;      // column of A = row of G
    const int nb = (int)tn * kGradTile + lc;      // column of dZ and of G

    auto self_of = [&](int chunk, int i) -> int32_t {   // self index of row lr + 8 i of a chunk (clamped rows)
        int64_t r = r0 + (int64_t)chunk * kGradRows + lr + 8 * i;
        r = r < n_dst ? r : n_dst - 1;
        return self_idx != nullptr ? self_idx[r] : (int32_t)r;
    };
    using T = typename Tr::store_t;
    using R4 = typename Raw4<Tr>::type;
    auto load = [&](int chunk, const int32_t (&sidx)[2], GradFrag<Tr>& f) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int64_t r = r0 + (int64_t)chunk * kGradRows + lr + 8 * i;
            r = r < n_dst ? r : n_dst - 1;
            const int64_t srow = sidx[i] > 0 ? sidx[i] : 0;
            if (VEC) {
                const T* pa = ka < k_self ? Hsrc + srow * d_in + ka : Mean + r * d_in + (ka < K ? ka - k_self : 0);
                f.a[i] = *reinterpret_cast<const R4*>(pa);
                f.b[i] = *reinterpret_cast<const float4*>(dZ + r * d_out + (nb < d_out ? nb : 0));
                if (MASK) f.o[i] = *reinterpret_cast<const R4*>(OutFwd + r * d_out + (nb < d_out ? nb : 0));
            } else {
                union { R4 v; T e[4]; } av, ov;
                float bv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = ka + e, n = nb + e;
                    av.e[e] = k < k_self ? Hsrc[srow * d_in + k] : Mean[r * d_in + (k < K ? k - k_self : 0)];
                    bv[e] = dZ[r * d_out + (n < d_out ? n : 0)];
                    if (MASK) ov.e[e] = OutFwd[r * d_out + (n < d_out ? n : 0)];
                }
                f.a[i] = av.v;
                f.b[i] = make_float4(bv[0], bv[1], bv[2], bv[3]);
                if (MASK) f.o[i] = ov.v;
            }
        }
    };
    auto store = [&](int chunk, const int32_t (&sidx)[2], const GradFrag<Tr>& f, int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const bool row_ok = r0 + (int64_t)chunk * kGradRows + lr + 8 * i < r1;
            const float4 aw = Raw4<Tr>::widen(f.a[i]);
            float av[4] = {aw.x, aw.y, aw.z, aw.w};
            float bv[4] = {f.b[i].x, f.b[i].y, f.b[i].z, f.b[i].w};
            float ov[4] = {1.f, 1.f, 1.f, 1.f};
            if (MASK) {
                const float4 ow = Raw4<Tr>::widen(f.o[i]);
                ov[0] = ow.x;
                ov[1] = ow.y;
                ov[2] = ow.z;
                ov[3] = ow.w;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = ka + e, n = nb + e;
                const bool a_ok = row_ok && k < K && (k >= k_self || sidx[i] >= 0);
                av[e] = a_ok ? av[e] : 0.f;
                bv[e] = row_ok && n < d_out && ov[e] > 0.f ? bv[e] : 0.f;
            }
            *reinterpret_cast<float4*>(&As[buf][lr + 8 * i][lc]) = make_float4(av[0], av[1], av[2], av[3]);
            *reinterpret_cast<float4*>(&Bs[buf][lr + 8 * i][lc]) = make_float4(bv[0], bv[1], bv[2], bv[3]);
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    float colsum[2] = {0.f, 0.f};

    int32_t s_cur[2] = {self_of(0, 0), self_of(0, 1)};
    int32_t s_nxt[2] = {self_of(1, 0), self_of(1, 1)};
    GradFrag<Tr> f;
    load(0, s_cur, f);
    store(0, s_cur, f, 0);
    lds_barrier();
    for (int c = 0; c < n_chunks; ++c) {
        const int buf = c & 1;
        // chunk c+1 (past the end: clamped rows, masked, never multiplied) and the indices of chunk c+2
        load(c + 1, s_nxt, f);
        s_cur[0] = s_nxt[0];
        s_cur[1] = s_nxt[1];
        s_nxt[0] = self_of(c + 2, 0);
        s_nxt[1] = self_of(c + 2, 1);
#pragma unroll
        for (int st = 0; st < kGradRows / 2; ++st) {
            const int row = 2 * st + g;
            const float a0 = As[buf][row][wk * 64 + l32], a1 = As[buf][row][wk * 64 + 32 + l32];
            const float b0 = Bs[buf][row][wn * 64 + l32], b1 = Bs[buf][row][wn * 64 + 32 + l32];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
            colsum[0] += b0;
            colsum[1] += b1;
        }
        store(c + 1, s_cur, f, buf ^ 1);
        lds_barrier();
    }

    // partial[split][k][n]; accumulator register e of lane l holds G row 8*(e/4)+4*(l/32)+e%4, col l%32
    const int k0 = (int)tk * kGradTile + wk * 64, n0 = (int)tn * kGradTile + wn * 64;
    float* P = partial + (int64_t)blockIdx.y * K * d_out;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + j * 32 + l32;
            if (n >= d_out) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int kk = k0 + i * 32 + 8 * (e / 4) + 4 * g + (e & 3);
                if (kk < K) P[(int64_t)kk * d_out + n] = acc[i][j][e];
            }
        }
    if (bias_partial != nullptr && tk == 0 && wk == 0) {   // one wave per 64-column block
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float cs = colsum[j] + __shfl_xor(colsum[j], 32, kWave);   // even rows + odd rows
            const int n = n0 + j * 32 + l32;
            if (g == 0 && n < d_out) bias_partial[(int64_t)blockIdx.y * d_out + n] = cs;
        }
    }
}

// The same tile for 2-byte activations on v_mfma_f32_32x32x16_{bf16,f16} (fp32 accumulators).  Both
// operands of that instruction hold 8 consecutive values of the contraction index per lane, and
// the contraction index here is the row: the operands are columns of the staged chunk.  The chunk
// (32 rows: two MFMA steps) sits in LDS row-major as 2-byte values - A as stored, dZ rounded to the
// activation type on its way in (the mixed-precision convention: products of two 2-byte values,
// fp32 sums) - and a lane assembles its operand from 8 two-byte reads down a column; lanes of a
// half-wave read 32 consecutive columns of one row, the two halves rows 8 apart, whose banks the
// row stride of 128 + 4 elements keeps apart.  The column sums of dZ (the bias gradient) are taken
// from the fp32 values before rounding.  Workgroups are numbered so that the tiles of one row
// split run on one XCD at about the same time (workgroup b goes to XCD b % 8): the split's rows
// then come out of that XCD's L2 for every tile but the first.
// Requires d_in % 8 == 0 and d_out % 4 == 0 and 16-byte aligned operands (the caller checks).
//
// The workgroup's shape is a template parameter: WK x WN waves, each a (32 TM) x (32 TN) piece of G,
// so a tile of KT = 32 WK TM rows of G (feature columns of A) by NTL = 32 WN TN columns.  Every
// operand an MFMA consumes costs the same LDS reads and packing whatever it is multiplied with,
// and every staged element the same loads, masks and conversions, so the instruction count per
// MFMA falls with the piece a wave owns; and dZ (fp32, plus the 2-byte mask source: 6 of every 8
// operand bytes) is re-read once per tile row of G.  Wide layers therefore take all of K in one
// workgroup (4 x 2 waves of 128 x 64: dZ is read once), narrower ones 256 or 128 rows of G.
constexpr int kG16Rows = 32;

template <typename Tr, bool MASK, int WK, int WN, int TM, int TN>
__global__ void __launch_bounds__(64 * WK * WN)
bwd_weight_grad16(const typename Tr::store_t* __restrict__ Hsrc, const int32_t* __restrict__ self_idx,
                  const typename Tr::store_t* __restrict__ Mean, const float* __restrict__ dZ,
                  const typename Tr::store_t* __restrict__ OutFwd, int64_t n_dst, int32_t d_in, int32_t d_out,
                  int32_t rows_per_split, uint32_t tiles_n, uint32_t n_tiles, int32_t n_splits,
                  float* __restrict__ partial, float* __restrict__ bias_partial,
                  const int64_t* __restrict__ n_rows_dev, int32_t k_self) {
    using T = typename Tr::store_t;
    constexpr int NT = 64 * WK * WN;                 // threads
    constexpr int KT = 32 * WK * TM, NTL = 32 * WN * TN;
    // 2-byte elements; a row pitch of 16 banks past a multiple of 64 keeps the four rows and two column
    // halves that one transposing read touches on different banks
    constexpr int LDA = KT + 32, LDB = NTL + 32;
    static_assert(KT % 128 == 0 && NTL % 128 == 0, "row pitch");
    constexpr int A_PER_ROW = KT / 8, B_PER_ROW = NTL / 4;
    constexpr int A_ITEMS = kG16Rows * A_PER_ROW / NT, B_ITEMS = kG16Rows * B_PER_ROW / NT;
    constexpr int A_ROWS = NT / A_PER_ROW, B_ROWS = NT / B_PER_ROW;     // rows one round of the threads covers
    static_assert(NT % A_PER_ROW == 0 && NT % B_PER_ROW == 0 && A_ITEMS >= 1 && B_ITEMS >= 1, "chunk shares");
    static_assert(A_ITEMS * A_ROWS == kG16Rows && B_ITEMS * B_ROWS == kG16Rows, "chunk shares");
    static_assert(B_ROWS * NTL * 4 <= 2 * kG16Rows * LDA * 2, "column sums fit the A stage");
    __shared__ __attribute__((aligned(16))) uint16_t As[2][kG16Rows][LDA];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][kG16Rows][LDB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, l32 = lane & 31;
    const int wk = wave / WN, wn = wave % WN;
    const int K = k_self + d_in;
    // workgroup -> (tile, split): XCD x takes the splits x, x + 8, ... and runs each split's tiles back to back
    const uint32_t xcd = blockIdx.x & 7u, seq = blockIdx.x >> 3;
    const uint32_t tile = seq % n_tiles;
    const int32_t split = (int32_t)((seq / n_tiles) * 8u + xcd);
    if (split >= n_splits) return;             // uniform over the workgroup
    const uint32_t tk = tile / tiles_n, tn = tile % tiles_n;
    const int64_t n_rows = n_rows_dev != nullptr && *n_rows_dev < n_dst ? *n_rows_dev : n_dst;
    rows_per_split = balanced_split(rows_per_split, n_rows, n_rows_dev != nullptr, n_splits);
    const int64_t r0 = (int64_t)split * rows_per_split;
    int64_t r1 = r0 + rows_per_split < n_rows ? r0 + rows_per_split : n_rows;
    r1 = r1 > r0 ? r1 : r0;
    const int n_chunks = (int)((r1 - r0 + kG16Rows - 1) / kG16Rows);

    // this thread's part of every chunk: A rows ar + A_ROWS i (8 elements each), dZ rows br + B_ROWS i (4 each)
    const int ar = tid / A_PER_ROW, ac = (tid % A_PER_ROW) * 8;
    const int br = tid / B_PER_ROW, bc = (tid % B_PER_ROW) * 4;
    const int ka = (int)tk * KT + ac;
    const int nb = (int)tn * NTL + bc;
    const bool ka_ok = ka < K, nb_ok = nb < d_out;
    const int nbc = nb_ok ? nb : 0;
    // this thread's A columns come from the self rows or from the means, the same for every chunk
    const bool a_self = ka < k_self;
    const T* a_base = a_self ? Hsrc + ka : Mean + (ka_ok ? ka - k_self : 0);

    auto self_of = [&](int chunk, int i) -> int32_t {
        int64_t r = r0 + (int64_t)chunk * kG16Rows + ar + A_ROWS * i;
        r = r < n_dst ? r : n_dst - 1;
        return self_idx != nullptr && a_self ? self_idx[r] : (int32_t)r;
    };
    // One chunk's loads in flight.  Every load is unconditional from a clamped, in-bounds address;
    // what must not count is zeroed when the chunk goes to LDS.
    struct Frag {
        uint4 a[A_ITEMS];
        float4 b[B_ITEMS];
        uint2 o[B_ITEMS];
        bool a_ok[A_ITEMS];
    };
    auto load = [&](int chunk, const int32_t (&sidx)[A_ITEMS], Frag& f) {
        const int64_t base = r0 + (int64_t)chunk * kG16Rows;
#pragma unroll
        for (int i = 0; i < A_ITEMS; ++i) {
            int64_t r = base + ar + A_ROWS * i;
            f.a_ok[i] = r < r1 && ka_ok && (!a_self || sidx[i] >= 0);
            r = r < n_dst ? r : n_dst - 1;
            const int64_t srow = sidx[i] > 0 ? sidx[i] : 0;
            f.a[i] = *reinterpret_cast<const uint4*>(a_base + (a_self ? srow : r) * d_in);
        }
#pragma unroll
        for (int i = 0; i < B_ITEMS; ++i) {
            int64_t r = base + br + B_ROWS * i;
            r = r < n_dst ? r : n_dst - 1;
            f.b[i] = *reinterpret_cast<const float4*>(dZ + r * d_out + nbc);
            if (MASK) f.o[i] = *reinterpret_cast<const uint2*>(OutFwd + r * d_out + nbc);
        }
    };
    float colsum[4] = {0.f, 0.f, 0.f, 0.f};
    auto store = [&](int chunk, const Frag& f, int buf) {
        const int64_t base = r0 + (int64_t)chunk * kG16Rows;
#pragma unroll
        for (int i = 0; i < A_ITEMS; ++i) {
            const uint4 v = f.a_ok[i] ? f.a[i] : make_uint4(0u, 0u, 0u, 0u);
            uint2* dst = reinterpret_cast<uint2*>(&As[buf][ar + A_ROWS * i][ac]);
            dst[0] = make_uint2(v.x, v.y);
            dst[1] = make_uint2(v.z, v.w);
        }
#pragma unroll
        for (int i = 0; i < B_ITEMS; ++i) {
            const bool ok = base + br + B_ROWS * i < r1 && nb_ok;
            float bv[4] = {f.b[i].x, f.b[i].y, f.b[i].z, f.b[i].w};
            if (MASK) {
                union { uint2 v; T e[4]; } o;
                o.v = f.o[i];
#pragma unroll
                for (int e = 0; e < 4; ++e) bv[e] = Tr::to_f(o.e[e]) > 0.f ? bv[e] : 0.f;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                bv[e] = ok ? bv[e] : 0.f;
                colsum[e] += bv[e];
            }
            *reinterpret_cast<uint2*>(&Bs[buf][br + B_ROWS * i][bc]) = make_uint2(Tr::pack2(bv[0], bv[1]), Tr::pack2(bv[2], bv[3]));
        }
    };
    // 8 values down a column, rows row0 .. row0 + 7 of column col0 + lane % 32, as one MFMA operand: two
    // transposing LDS reads (ds_read_b64_tr_b16).  Within 16 lanes, lanes 4j .. 4j+3 name the four 8-byte
    // words of a 16-element piece of row j (j = 0..3), and lane i receives element i of each of the four
    // rows: four consecutive rows of ONE column, with no vector instruction spent on it.
    typedef short v4i16 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) v4i16 lds_v4i16;
    const int tr_row = (lane & 15) >> 2, tr_col = ((lane >> 4) & 1) * 16 + 4 * (lane & 3);
    auto column8 = [&](const uint16_t* S, int ld, int row0, int col0) -> uint4 {
        const uint16_t* p = S + (row0 + tr_row) * ld + col0 + tr_col;
        union { uint4 v; v4i16 h[2]; } u;
        u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)p);
        u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(p + 4 * ld));
        return u.v;
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // The next chunk's loads are in flight while one is multiplied, into the registers the current chunk
    // left when it went to LDS (chunks past the end: clamped rows, masked, never multiplied); the self
    // indices run one chunk ahead of the loads.  (Two chunks in flight cost a resident workgroup per
    // CU in registers and measured slower.)
    Frag f;
    int32_t s_nxt[A_ITEMS];
    {
        int32_t s_cur[A_ITEMS];
#pragma unroll
        for (int i = 0; i < A_ITEMS; ++i) s_cur[i] = self_of(0, i);
        load(0, s_cur, f);
#pragma unroll
        for (int i = 0; i < A_ITEMS; ++i) s_nxt[i] = self_of(1, i);
    }
    store(0, f, 0);
    lds_barrier();
    for (int c = 0; c < n_chunks; ++c) {
        const int buf = c & 1;
        int32_t s_cur[A_ITEMS];
#pragma unroll
        for (int i = 0; i < A_ITEMS; ++i) s_cur[i] = s_nxt[i];
        load(c + 1, s_cur, f);
#pragma unroll
        for (int i = 0; i < A_ITEMS; ++i) s_nxt[i] = self_of(c + 2, i);
#pragma unroll
        for (int kk = 0; kk < kG16Rows; kk += 16) {
            uint4 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = column8(&As[buf][0][0], LDA, kk + 8 * g, (wk * TM + i) * 32);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = column8(&Bs[buf][0][0], LDB, kk + 8 * g, (wn * TN + j) * 32);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = mfma16<Tr>(a[i], b[j], acc[i][j]);
        }
        store(c + 1, f, buf ^ 1);
        lds_barrier();
    }

    const int k0 = (int)tk * KT + wk * TM * 32, n0 = (int)tn * NTL + wn * TN * 32;
    float* P = partial + (int64_t)split * K * d_out;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + j * 32 + l32;
            if (n >= d_out) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int kk = k0 + i * 32 + 8 * (e / 4) + 4 * g + (e & 3);
                if (kk < K) P[(int64_t)kk * d_out + n] = acc[i][j][e];
            }
        }
    if (bias_partial != nullptr && tk == 0) {
        // the row groups' sums of every column, added in a fixed order (the staging tiles are free:
        // the loop's last barrier is behind every read of them)
        float* cs = reinterpret_cast<float*>(&As[0][0][0]);      // [B_ROWS][NTL]
#pragma unroll
        for (int e = 0; e < 4; ++e) cs[br * NTL + bc + e] = colsum[e];
        lds_barrier();
        if (tid < NTL) {
            float t = 0.f;
#pragma unroll
            for (int q = 0; q < B_ROWS; ++q) t += cs[q * NTL + tid];
            const int n = (int)tn * NTL + tid;
            if (n < d_out) bias_partial[(int64_t)split * d_out + n] = t;
        }
    }
}

// Shape of the 2-byte weight-gradient workgroup for K rows of G: rows of G per tile.
static inline int grad16_tile_k(int64_t K) { return K > 256 ? 512 : K > 128 ? 256 : 128; }

// gW += sum over the splits of the partial tiles; same for the bias.  A workgroup owns 64
// consecutive elements; wave q sums the splits q, q+4, q+8, ... in that order and the four
// sums are combined as (s0 + s1) + (s2 + s3): a fixed order, so the result is bit-stable.
__global__ void __launch_bounds__(kBwdThreads)
bwd_weight_reduce(const float* __restrict__ partial, const float* __restrict__ bias_partial, int32_t n_splits,
                  int32_t d_in, int32_t d_out, float* __restrict__ gW_self, float* __restrict__ gW_neigh,
                  float* __restrict__ gbias, int32_t k_self) {
    __shared__ float part[4][kWave];
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * kWave + lane;
    const int64_t per = ((int64_t)k_self + d_in) * d_out;     // rows of G: k_self for gW_self, then d_in for gW_neigh
    // elements [0, per) are the weights, [per, per + d_out) the bias
    const float* src = i < per ? partial + i : bias_partial + (i - per);
    const int64_t stride = i < per ? per : d_out;
    const bool live = i < per || (gbias != nullptr && i < per + d_out);
    float s = 0.f;
    if (live) {
        int32_t p = q;
        for (; p + 12 < n_splits; p += 16) {      // four independent loads in flight
            const float v0 = src[(int64_t)p * stride], v1 = src[(int64_t)(p + 4) * stride];
            const float v2 = src[(int64_t)(p + 8) * stride], v3 = src[(int64_t)(p + 12) * stride];
            s = (((s + v0) + v1) + v2) + v3;
        }
        for (; p < n_splits; p += 4) s += src[(int64_t)p * stride];
    }
    part[q][lane] = s;
    __syncthreads();
    if (q == 0 && live) {
        const float t = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
        const int64_t half = (int64_t)k_self * d_out;
        if (i < half) gW_self[i] += t;
        else if (i < per) gW_neigh[i - half] += t;
        else gbias[i - per] += t;
    }
}

// ----------------------------------------------------------- input gradient --
//
// D[r][j] = sum_n dZ[r][n] Wcat[j][n], j over the 2*d_in rows of [W_self ; W_neigh].  Both
// operands have the contraction index contiguous, so both sit in LDS row-major [64][BK+4] and
// are read as 128-bit words: lane group g = l/32 takes the four n values 4g..4g+3 of an 8-wide
// block and the block's four MFMAs pair the i-th values (a permutation of the summation order).
template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
bwd_input_grad(const float* __restrict__ dZ, const typename Tr::store_t* __restrict__ Wself,
               const typename Tr::store_t* __restrict__ Wneigh, int64_t n_dst_cap, int32_t d_in, int32_t d_out,
               float* __restrict__ D, const int64_t* __restrict__ n_rows_dev, int32_t k_self) {
    using T = typename Tr::store_t;
    using R4 = typename Raw4<Tr>::type;
    constexpr int BM = 64, BN = 64, BK = 16, LD = BK + 4;
    __shared__ __attribute__((aligned(16))) float As[BM][LD];
    __shared__ __attribute__((aligned(16))) float Bs[BN][LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, l32 = lane & 31;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t n_dst = n_rows_dev != nullptr && *n_rows_dev < n_dst_cap ? *n_rows_dev : n_dst_cap;
    const int64_t row0 = (int64_t)blockIdx.x * BM;
    if (row0 >= n_dst) return;                 // uniform over the workgroup
    const int col0 = blockIdx.y * BN;
    const int N = k_self + d_in;        // rows of [W_self ; W_neigh], or of the one matrix (k_self = 0)
    const bool vec = (d_out & 3) == 0;

    // one 16-byte item of each tile per thread: row tid/4, words (tid%4)*4 .. +3
    const int lr = tid >> 2, lk = (tid & 3) * 4;
    const int64_t ar = row0 + lr;
    const int bj = col0 + lr;
    const float* arow = ar < n_dst ? dZ + ar * d_out : nullptr;
    const T* brow = bj < N ? (bj < k_self ? Wself + (int64_t)bj * d_out : Wneigh + (int64_t)(bj - k_self) * d_out)
                           : nullptr;
    auto load4w = [&](const T* row, int kq) {      // raw weight elements, widened when they go to LDS
        union { R4 v; T e[4]; } u;
#pragma unroll
        for (int e = 0; e < 4; ++e) u.e[e] = Tr::from_f(0.f);
        if (row != nullptr) {
            if (vec && kq + 3 < d_out) {
                u.v = *reinterpret_cast<const R4*>(row + kq);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (kq + e < d_out) u.e[e] = row[kq + e];
            }
        }
        return u.v;
    };
    auto load4 = [&](const float* row, int kq) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row != nullptr) {
            if (vec && kq + 3 < d_out) {
                v = *reinterpret_cast<const float4*>(row + kq);
            } else {
                if (kq + 0 < d_out) v.x = row[kq + 0];
                if (kq + 1 < d_out) v.y = row[kq + 1];
                if (kq + 2 < d_out) v.z = row[kq + 2];
                if (kq + 3 < d_out) v.w = row[kq + 3];
            }
        }
        return v;
    };

    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    const int n_tiles = (d_out + BK - 1) / BK;
    float4 ra = load4(arow, lk);
    R4 rb = load4w(brow, lk);
    for (int t = 0; t < n_tiles; ++t) {
        __syncthreads();
        *reinterpret_cast<float4*>(&As[lr][lk]) = ra;
        *reinterpret_cast<float4*>(&Bs[lr][lk]) = Raw4<Tr>::widen(rb);
        __syncthreads();
        if (t + 1 < n_tiles) {
            ra = load4(arow, (t + 1) * BK + lk);
            rb = load4w(brow, (t + 1) * BK + lk);
        }
#pragma unroll
        for (int kk = 0; kk < BK; kk += 8) {
            const float4 a = *reinterpret_cast<const float4*>(&As[wm * 32 + l32][kk + 4 * g]);
            const float4 b = *reinterpret_cast<const float4*>(&Bs[wn * 32 + l32][kk + 4 * g]);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
        }
    }
    const int col = col0 + wn * 32 + l32;
    if (col < N) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t row = row0 + wm * 32 + 8 * (i / 4) + 4 * g + (i & 3);
            if (row < n_dst) D[row * N + col] = acc[i];
        }
    }
}

// The same product for 2-byte activations on v_mfma_f32_32x32x16_{bf16,f16}: the weights as stored,
// dZ rounded to the activation type on its way into LDS; both tiles [64][32 + 8] 2-byte values with
// the contraction index contiguous, read as 128-bit words.
template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
bwd_input_grad16(const float* __restrict__ dZ, const typename Tr::store_t* __restrict__ Wself,
                 const typename Tr::store_t* __restrict__ Wneigh, int64_t n_dst_cap, int32_t d_in, int32_t d_out,
                 float* __restrict__ D, const int64_t* __restrict__ n_rows_dev, int32_t k_self) {
    using T = typename Tr::store_t;
    constexpr int BM = 64, BN = 64, BK = 32, LD = BK + 8;
    __shared__ __attribute__((aligned(16))) uint16_t As[BM][LD];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[BN][LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, l32 = lane & 31;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t n_dst = n_rows_dev != nullptr && *n_rows_dev < n_dst_cap ? *n_rows_dev : n_dst_cap;
    const int64_t row0 = (int64_t)blockIdx.x * BM;
    if (row0 >= n_dst) return;                 // uniform over the workgroup
    const int col0 = blockIdx.y * BN;
    const int N = k_self + d_in;        // rows of [W_self ; W_neigh], or of the one matrix (k_self = 0)
    const bool vec = (d_out & 7) == 0;

    // one 8-element item of each tile per thread: row tid/4, k (tid%4)*8 .. +7
    const int lr = tid >> 2, lk = (tid & 3) * 8;
    const int64_t ar = row0 + lr;
    const int bj = col0 + lr;
    const float* arow = ar < n_dst ? dZ + ar * d_out : nullptr;
    const T* brow = bj < N ? (bj < k_self ? Wself + (int64_t)bj * d_out : Wneigh + (int64_t)(bj - k_self) * d_out)
                           : nullptr;
    struct Item {
        float4 a[2];
        uint4 b;
    };
    auto load = [&](int kq, Item& it) {
        it.a[0] = it.a[1] = make_float4(0.f, 0.f, 0.f, 0.f);
        it.b = make_uint4(0u, 0u, 0u, 0u);
        if (vec && kq + 7 < d_out) {
            if (arow != nullptr) {
                it.a[0] = *reinterpret_cast<const float4*>(arow + kq);
                it.a[1] = *reinterpret_cast<const float4*>(arow + kq + 4);
            }
            if (brow != nullptr) it.b = *reinterpret_cast<const uint4*>(brow + kq);
        } else {
            float av[8];
            union { uint4 v; T e[8]; } u;
            u.v = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                av[e] = arow != nullptr && kq + e < d_out ? arow[kq + e] : 0.f;
                if (brow != nullptr && kq + e < d_out) u.e[e] = brow[kq + e];
            }
            it.a[0] = make_float4(av[0], av[1], av[2], av[3]);
            it.a[1] = make_float4(av[4], av[5], av[6], av[7]);
            it.b = u.v;
        }
    };

    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    const int n_tiles = (d_out + BK - 1) / BK;
    Item it;
    load(lk, it);
    for (int t = 0; t < n_tiles; ++t) {
        __syncthreads();
        *reinterpret_cast<uint4*>(&As[lr][lk]) = make_uint4(Tr::pack2(it.a[0].x, it.a[0].y), Tr::pack2(it.a[0].z, it.a[0].w),
                                                            Tr::pack2(it.a[1].x, it.a[1].y), Tr::pack2(it.a[1].z, it.a[1].w));
        *reinterpret_cast<uint4*>(&Bs[lr][lk]) = it.b;
        __syncthreads();
        if (t + 1 < n_tiles) load((t + 1) * BK + lk, it);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            const uint4 a = *reinterpret_cast<const uint4*>(&As[wm * 32 + l32][kk + 8 * g]);
            const uint4 b = *reinterpret_cast<const uint4*>(&Bs[wn * 32 + l32][kk + 8 * g]);
            acc = mfma16<Tr>(a, b, acc);
        }
    }
    const int col = col0 + wn * 32 + l32;
    if (col < N) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t row = row0 + wm * 32 + 8 * (i / 4) + 4 * g + (i & 3);
            if (row < n_dst) D[row * N + col] = acc[i];
        }
    }
}

// dHsrc[self_idx[r]] += D[r][:d_in];  dHsrc[idx[e]] += D[r][d_in:] / c_r for the valid entries e.
// `group` lanes (power of two) per destination row, lane j owns columns j, j+group, ...
__global__ void __launch_bounds__(kBwdThreads)
bwd_scatter(const float* __restrict__ D, const int32_t* __restrict__ self_idx, const int32_t* __restrict__ indptr,
            const int32_t* __restrict__ idx, int64_t n_dst, int32_t d_in, int32_t group, float* __restrict__ dHsrc,
            const int64_t* __restrict__ n_rows_dev) {
    const int64_t gid = (int64_t)blockIdx.x * kBwdThreads + threadIdx.x;
    const int64_t r = gid / group;
    const int32_t j = (int32_t)(gid - r * group);
    if (r >= n_dst || (n_rows_dev != nullptr && r >= *n_rows_dev)) return;
    const int64_t s = self_idx != nullptr ? (int64_t)self_idx[r] : r;
    const int32_t beg = indptr[r], end = indptr[r + 1];
    int32_t cnt = 0;
    for (int32_t e = beg; e < end; ++e) cnt += idx[e] >= 0 ? 1 : 0;
    const float inv = cnt > 0 ? 1.f / (float)cnt : 0.f;
    const float* Dr = D + r * (2 * (int64_t)d_in);
    for (int32_t c = j; c < d_in; c += group) {
        if (s >= 0) atomicAdd(&dHsrc[s * d_in + c], Dr[c]);
        if (cnt > 0) {
            const float m = Dr[d_in + c] * inv;
            for (int32_t e = beg; e < end; ++e) {
                const int32_t u = idx[e];
                if (u >= 0) atomicAdd(&dHsrc[(int64_t)u * d_in + c], m);
            }
        }
    }
}

// The input gradient of the other layer kinds, from D = dZ [W_self ; W_neigh]^T (or dZ W^T):
//   kScatterSum   GraphSAGE, sum aggregator:  self term as above; every valid entry receives D[r][d_in:]
//   kScatterMax   GraphSAGE, max aggregator:  per column the entry that supplied the maximum receives it -
//                 the first one in entry order among equals, as the forward pass keeps it (a larger
//                 value replaces the running maximum, an equal one does not)
//   kScatterGcn   GCN-style: the self row and every valid entry receive D[r] / t, t = number of
//                 terms (norm = 1) or 1 (norm = 0)
constexpr int kScatterMean = 0, kScatterSum = 1, kScatterMax = 2, kScatterGcn = 3;

template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
bwd_scatter_kind(const float* __restrict__ D, const typename Tr::store_t* __restrict__ Hsrc,
                 const int32_t* __restrict__ self_idx, const int32_t* __restrict__ indptr,
                 const int32_t* __restrict__ idx, int64_t n_dst, int32_t d_in, int32_t group, int32_t mode,
                 int32_t norm, float* __restrict__ dHsrc, const int64_t* __restrict__ n_rows_dev) {
    const int64_t gid = (int64_t)blockIdx.x * kBwdThreads + threadIdx.x;
    const int64_t r = gid / group;
    const int32_t j = (int32_t)(gid - r * group);
    if (r >= n_dst || (n_rows_dev != nullptr && r >= *n_rows_dev)) return;
    const int64_t s = self_idx != nullptr ? (int64_t)self_idx[r] : r;
    const int32_t beg = indptr[r], end = indptr[r + 1];
    if (mode == kScatterGcn) {
        int32_t terms = s >= 0 ? 1 : 0;
        for (int32_t e = beg; e < end; ++e) terms += idx[e] >= 0 ? 1 : 0;
        const float scale = norm && terms > 0 ? 1.f / (float)terms : 1.f;
        const float* Dr = D + r * (int64_t)d_in;
        for (int32_t c = j; c < d_in; c += group) {
            const float g = Dr[c] * scale;
            if (s >= 0) atomicAdd(&dHsrc[s * d_in + c], g);
            for (int32_t e = beg; e < end; ++e) {
                const int32_t u = idx[e];
                if (u >= 0) atomicAdd(&dHsrc[(int64_t)u * d_in + c], g);
            }
        }
        return;
    }
    const float* Dr = D + r * (2 * (int64_t)d_in);
    for (int32_t c = j; c < d_in; c += group) {
        if (s >= 0) atomicAdd(&dHsrc[s * d_in + c], Dr[c]);
        const float g = Dr[d_in + c];
        if (mode == kScatterSum) {
            for (int32_t e = beg; e < end; ++e) {
                const int32_t u = idx[e];
                if (u >= 0) atomicAdd(&dHsrc[(int64_t)u * d_in + c], g);
            }
        } else {
            int32_t best = -1;
            float bv = 0.f;
            for (int32_t e = beg; e < end; ++e) {
                const int32_t u = idx[e];
                if (u < 0) continue;
                const float v = Tr::to_f(Hsrc[(int64_t)u * d_in + c]);
                if (best < 0 || v > bv) {
                    bv = v;
                    best = u;
                }
            }
            if (best >= 0) atomicAdd(&dHsrc[(int64_t)best * d_in + c], g);
        }
    }
}

// The same sums without atomics for neighbour lists in slot order: entry e of the segments is source
// row first + e (or -1), self rows are the rows themselves, so every source row has one parent and is
// written exactly once - by its parent's lanes, or by its own when it has none (rows below `first`).
// One group of lanes per source row u < n_src; the group of u < n_dst also serves u as a parent.
// Rows past the last entry are zeroed.  Nothing is read-modified: bit-stable, no zero pass before.
template <int W>      // W = 4: 16-byte pieces (d_in % 4 == 0, 16-byte aligned arrays), else single floats
__global__ void __launch_bounds__(kBwdThreads)
bwd_pull_slots(const float* __restrict__ D, const int32_t* __restrict__ indptr, const int32_t* __restrict__ idx,
               int64_t n_dst, int64_t n_src, int64_t first, int32_t d_in, int32_t group, float* __restrict__ dHsrc) {
    const int64_t gid = (int64_t)blockIdx.x * kBwdThreads + threadIdx.x;
    const int64_t r = gid / group;
    const int32_t j = (int32_t)(gid - r * group);
    if (r >= n_src) return;
    const int64_t two_d = 2 * (int64_t)d_in;
    using V = typename std::conditional<W == 4, float4, float>::type;
    auto ld = [](const float* p) -> V { return *reinterpret_cast<const V*>(p); };
    auto st = [](float* p, V v) { *reinterpret_cast<V*>(p) = v; };
    auto scaled = [](V v, float a) -> V {
        if constexpr (W == 4) return make_float4(v.x * a, v.y * a, v.z * a, v.w * a);
        else return v * a;
    };
    auto sum = [](V a, V b) -> V {
        if constexpr (W == 4) return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
        else return a + b;
    };
    V zero_v;
    if constexpr (W == 4) zero_v = make_float4(0.f, 0.f, 0.f, 0.f);
    else zero_v = 0.f;
    if (r < first || r >= first + (int64_t)indptr[n_dst])      // a row without a parent: its own self term, if any
        for (int32_t c = j * W; c < d_in; c += group * W) st(dHsrc + r * d_in + c, r < n_dst ? ld(D + r * two_d + c) : zero_v);
    if (r >= n_dst) return;
    const int32_t beg = indptr[r], end = indptr[r + 1];
    int32_t cnt = 0;
    for (int32_t e = beg; e < end; ++e) cnt += idx[e] >= 0 ? 1 : 0;
    const float inv = cnt > 0 ? 1.f / (float)cnt : 0.f;
    const float* Dr = D + r * two_d + d_in;
    for (int32_t e = beg; e < end; ++e) {
        const int64_t u = first + e;
        if (u >= n_src) break;                        // fewer source rows than entries: not this call's layout
        const bool fed = idx[e] >= 0;                 // an invalid slot takes no part in the mean
        const bool is_dst = u < n_dst;                // ... but a destination row still has its self term
        for (int32_t c = j * W; c < d_in; c += group * W) {
            V v = fed ? scaled(ld(Dr + c), inv) : zero_v;
            if (is_dst) v = sum(v, ld(D + u * two_d + c));
            st(dHsrc + u * d_in + c, v);
        }
    }
}

// ---------------------------------------------------------------- update --

// W <- W - lr * grad (fp32 arithmetic, one rounding to the stored type), optionally grad <- 0.
template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
sgd_update(typename Tr::store_t* __restrict__ W, float* __restrict__ grad, int64_t n, float lr, int zero_grad) {
    const int64_t stride = (int64_t)gridDim.x * kBwdThreads;
    for (int64_t i = (int64_t)blockIdx.x * kBwdThreads + threadIdx.x; i < n; i += stride) {
        W[i] = Tr::from_f(Tr::to_f(W[i]) - lr * grad[i]);
        if (zero_grad) grad[i] = 0.f;
    }
}

// The same update for up to kSgdMaxTensors tensors in one launch (a model's weight matrices and
// biases are a handful of small arrays: one launch each would cost more than the arithmetic).
constexpr int kSgdMaxTensors = 32;
struct SgdBatch {
    void* W[kSgdMaxTensors];
    float* grad[kSgdMaxTensors];
    int64_t first_block[kSgdMaxTensors + 1];     // blocks [first_block[t], first_block[t+1]) work on tensor t
    int64_t n[kSgdMaxTensors];
    int32_t n_tensors;
};
constexpr int kSgdPerBlock = 4 * kBwdThreads;    // elements per workgroup

template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
sgd_update_multi(SgdBatch b, float lr, int zero_grad) {
    int t = 0;
    while (t + 1 < b.n_tensors && (int64_t)blockIdx.x >= b.first_block[t + 1]) ++t;
    typename Tr::store_t* W = static_cast<typename Tr::store_t*>(b.W[t]);
    float* grad = b.grad[t];
    const int64_t i0 = ((int64_t)blockIdx.x - b.first_block[t]) * kSgdPerBlock;
    for (int k = 0; k < 4; ++k) {
        const int64_t i = i0 + k * kBwdThreads + threadIdx.x;
        if (i < b.n[t]) {
            W[i] = Tr::from_f(Tr::to_f(W[i]) - lr * grad[i]);
            if (zero_grad) grad[i] = 0.f;
        }
    }
}

// ------------------------------------------------------------------ host --

struct BwdWs {
    size_t mean_bytes, zero_bytes, dz_bytes, partial_bytes, bias_bytes, d_bytes, total;
    int32_t rows_per_split, n_splits;
};

static BwdWs bwd_ws_layout(int64_t n_dst, int32_t d_in, int32_t d_out, int want_dh, bool two_byte = false) {
    BwdWs L{};
    const int64_t nd = n_dst > 0 ? n_dst : 1;
    L.mean_bytes = align_up((size_t)nd * d_in * 4, 256);
    L.zero_bytes = align_up(((size_t)2 * d_in + 64) * 4, 256);
    L.dz_bytes = align_up((size_t)nd * d_out * 4, 256);
    // enough splits to fill the chip (about 2048 waves), at least 128 rows each so that the
    // partial tiles stay small next to the operands
    int64_t tiles = ceil_div(2 * (int64_t)d_in, kGradTile) * ceil_div(d_out, kGradTile);
    int64_t splits = ceil_div(512, tiles);
    if (two_byte && d_in % 8 == 0 && d_out % 4 == 0) {
        // the 2-byte kernel's tiles are taller; its 8-wave workgroups fill a CU alone (256 of them), the
        // 4-wave ones two to a CU
        const int kt = grad16_tile_k(2 * (int64_t)d_in);
        tiles = ceil_div(2 * (int64_t)d_in, kt) * ceil_div(d_out, kGradTile);
        splits = ceil_div(kt == 512 ? 256 : 512, tiles);
    }
    int64_t rows = ceil_div(nd, splits);
    if (rows < 128) rows = 128;
    rows = (rows + kGradRows - 1) / kGradRows * kGradRows;
    L.rows_per_split = (int32_t)rows;
    L.n_splits = (int32_t)ceil_div(nd, rows);
    L.partial_bytes = align_up((size_t)L.n_splits * 2 * d_in * d_out * 4, 256);
    L.bias_bytes = align_up((size_t)L.n_splits * d_out * 4, 256);
    L.d_bytes = want_dh ? align_up((size_t)nd * 2 * d_in * 4, 256) : 0;
    L.total = L.mean_bytes + L.zero_bytes + L.dz_bytes + L.partial_bytes + L.bias_bytes + L.d_bytes;
    return L;
}

}  // namespace hopgnn

using namespace hopgnn;

extern "C" size_t hopgnn_sage_bwd_ws_bytes(hopgnn_dtype dt, int64_t n_dst, int32_t d_in, int32_t d_out,
                                           int32_t want_dh) {
    if ((dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) || n_dst < 0 || d_in < 1 || d_out < 1) return 0;
    return bwd_ws_layout(n_dst, d_in, d_out, want_dh, dt != HOPGNN_F32).total;
}

namespace hopgnn {

// Which layer the backward pass is for: the GraphSAGE layer with one of its aggregators (two weight
// matrices, A = [x_self | aggregate]) or the GCN-style layer (one matrix on the aggregate that
// includes the self row).
struct BwdKind {
    int32_t k_self;      // d_in (two matrices) or 0 (one)
    int32_t scatter;     // kScatter*
    int32_t norm;        // GCN-style: divide by the number of terms
};

// Launch of the 2-byte weight-gradient kernel in the shape that fits K rows of G.
template <typename Tr, bool MASK>
static void launch_weight_grad16(hipStream_t s, const typename Tr::store_t* Hsrc, const int32_t* self_idx,
                                 const typename Tr::store_t* mean, const float* dZ, const typename Tr::store_t* out_fwd,
                                 int64_t n_rows, int32_t d_in, int32_t d_out, const BwdWs& L, float* partial,
                                 float* bias_partial, const int64_t* n_rows_dev, int32_t k_self) {
    const int64_t K = (int64_t)k_self + d_in;
    const int kt = grad16_tile_k(K);
    const uint32_t tiles_n = (uint32_t)ceil_div(d_out, kGradTile);
    const uint32_t n_tiles = (uint32_t)ceil_div(K, kt) * tiles_n;
    const uint32_t splits8 = (uint32_t)ceil_div(L.n_splits, 8) * 8u;
    const dim3 grid(n_tiles * splits8);
    if (kt == 512)
        hipLaunchKernelGGL((bwd_weight_grad16<Tr, MASK, 4, 2, 4, 2>), grid, dim3(512), 0, s, Hsrc, self_idx, mean, dZ, out_fwd,
                           n_rows, d_in, d_out, L.rows_per_split, tiles_n, n_tiles, L.n_splits, partial, bias_partial,
                           n_rows_dev, k_self);
    else if (kt == 256)
        hipLaunchKernelGGL((bwd_weight_grad16<Tr, MASK, 2, 2, 4, 2>), grid, dim3(256), 0, s, Hsrc, self_idx, mean, dZ, out_fwd,
                           n_rows, d_in, d_out, L.rows_per_split, tiles_n, n_tiles, L.n_splits, partial, bias_partial,
                           n_rows_dev, k_self);
    else
        hipLaunchKernelGGL((bwd_weight_grad16<Tr, MASK, 2, 2, 2, 2>), grid, dim3(256), 0, s, Hsrc, self_idx, mean, dZ, out_fwd,
                           n_rows, d_in, d_out, L.rows_per_split, tiles_n, n_tiles, L.n_splits, partial, bias_partial,
                           n_rows_dev, k_self);
}

template <typename Tr>
static hopgnn_status sage_bwd_typed(const void* Hsrc, int64_t n_src, int32_t d_in, const int32_t* self_idx,
                                    const int32_t* indptr, const int32_t* idx, int64_t n_dst, const void* W_self,
                                    const void* W_neigh, const void* out_fwd, int32_t relu, const float* dOut,
                                    int32_t d_out, float* gW_self, float* gW_neigh, float* gbias, float* dHsrc,
                                    void* ws, const BwdWs& L, const int64_t* n_dst_dev, int64_t slot_first,
                                    const void* mean_fwd, hipStream_t s, const BwdKind& kind) {
    const int32_t k_self = kind.k_self;
    using T = typename Tr::store_t;
    using R4 = typename Raw4<Tr>::type;
    char* p = static_cast<char*>(ws);
    T* mean = reinterpret_cast<T*>(p);
    void* zero = p + L.mean_bytes;
    float* dz_buf = reinterpret_cast<float*>(p + L.mean_bytes + L.zero_bytes);
    float* partial = reinterpret_cast<float*>(p + L.mean_bytes + L.zero_bytes + L.dz_bytes);
    float* bias_partial = reinterpret_cast<float*>(reinterpret_cast<char*>(partial) + L.partial_bytes);
    float* D = reinterpret_cast<float*>(reinterpret_cast<char*>(bias_partial) + L.bias_bytes);
    if (n_src == 0) Hsrc = zero;   // nothing is read from it unmasked

    // the means: the forward call's, if the caller kept them, else computed again (same kernel as the
    // forward pass, same rounding to the activation type)
    if (mean_fwd != nullptr) {
        mean = const_cast<T*>(static_cast<const T*>(mean_fwd));
    } else {
        const AggSpec spec = kind.scatter == kScatterGcn ? AggSpec{self_idx, 1, kind.norm ? kAggOpMean : kAggOpSum}
                             : kind.scatter == kScatterSum ? AggSpec{nullptr, 0, kAggOpSum}
                             : kind.scatter == kScatterMax ? AggSpec{nullptr, 0, kAggOpMax} : kAggMean;
        hopgnn_status st = launch_mean<Tr>(Hsrc, indptr, idx, n_dst, d_in, mean, zero, L.zero_bytes, TransposeJob{}, 0, s,
                                           spec, n_dst_dev);
        if (st != HOPGNN_OK) return st;
    }

    const float* dZ = dOut;
    // the masked gradient has a second reader only when the input gradient is wanted
    const bool fuse_mask = relu && !(dHsrc != nullptr && n_src > 0);
    if (relu && !fuse_mask) {
        const int64_t n = n_dst * d_out;
        // four elements per thread when the total allows it (and, with a device row count, every row does)
        if (n % 4 == 0 && (n_dst_dev == nullptr || d_out % 4 == 0) && aligned(out_fwd, 16) && aligned(dOut, 16))
            hipLaunchKernelGGL(bwd_mask4<Tr>, dim3((unsigned)ceil_div(n / 4, kBwdThreads)), dim3(kBwdThreads), 0, s,
                               static_cast<const R4*>(out_fwd), reinterpret_cast<const float4*>(dOut), n / 4,
                               reinterpret_cast<float4*>(dz_buf), n_dst_dev, d_out / 4);
        else
            hipLaunchKernelGGL(bwd_mask_elem<Tr>, dim3((unsigned)ceil_div(n, kBwdThreads)), dim3(kBwdThreads), 0, s,
                               static_cast<const T*>(out_fwd), dOut, n, dz_buf, n_dst_dev, d_out);
        HOPGNN_LAUNCH_CHECK();
        dZ = dz_buf;
    }

    const uint32_t tiles_k = (uint32_t)ceil_div((int64_t)k_self + d_in, kGradTile), tiles_n = (uint32_t)ceil_div(d_out, kGradTile);
    const bool vec = d_in % 4 == 0 && d_out % 4 == 0 && aligned(Hsrc, 16) && aligned(dZ, 16) && aligned(mean, 16) &&
                     (!fuse_mask || aligned(out_fwd, 16));
    bool on16 = false;
    if constexpr (sizeof(T) == 2) {
        // the 2-byte matrix instructions, when every 8-element run of A and 4-element run of dZ is whole
        on16 = vec && d_in % 8 == 0;
        if (on16) {
            float* bp = gbias != nullptr ? bias_partial : nullptr;
            if (fuse_mask)
                launch_weight_grad16<Tr, true>(s, static_cast<const T*>(Hsrc), self_idx, mean, dZ,
                                               static_cast<const T*>(out_fwd), n_dst, d_in, d_out, L, partial, bp, n_dst_dev,
                                               k_self);
            else
                launch_weight_grad16<Tr, false>(s, static_cast<const T*>(Hsrc), self_idx, mean, dZ, nullptr, n_dst, d_in,
                                                d_out, L, partial, bp, n_dst_dev, k_self);
        }
    }
    if (!on16) {
        auto grad_kernel = fuse_mask ? (vec ? bwd_weight_grad<Tr, true, true> : bwd_weight_grad<Tr, false, true>)
                                     : (vec ? bwd_weight_grad<Tr, true, false> : bwd_weight_grad<Tr, false, false>);
        hipLaunchKernelGGL(grad_kernel, dim3(tiles_k * tiles_n, (unsigned)L.n_splits), dim3(kBwdThreads), 0, s,
                           static_cast<const T*>(Hsrc), self_idx, mean, dZ, static_cast<const T*>(out_fwd), n_dst, d_in, d_out,
                           L.rows_per_split, tiles_n, partial, gbias != nullptr ? bias_partial : nullptr, n_dst_dev, k_self);
    }
    HOPGNN_LAUNCH_CHECK();
    const int64_t red = ((int64_t)k_self + d_in) * d_out + d_out;
    hipLaunchKernelGGL(bwd_weight_reduce, dim3((unsigned)ceil_div(red, kWave)), dim3(kBwdThreads), 0, s, partial,
                       bias_partial, L.n_splits, d_in, d_out, gW_self, gW_neigh, gbias, k_self);
    HOPGNN_LAUNCH_CHECK();

    if (dHsrc != nullptr && n_src > 0) {
        const int64_t gy = ceil_div((int64_t)k_self + d_in, 64);
        if (gy > 65535) return HOPGNN_ERANGE;
        auto in_kernel = bwd_input_grad<Tr>;
        if constexpr (sizeof(T) == 2) {
            if (aligned(dZ, 16) && aligned(W_self, 16) && aligned(W_neigh, 16)) in_kernel = bwd_input_grad16<Tr>;
        }
        hipLaunchKernelGGL(in_kernel, dim3((unsigned)ceil_div(n_dst, 64), (unsigned)gy), dim3(kBwdThreads), 0, s, dZ,
                           static_cast<const T*>(W_self), static_cast<const T*>(W_neigh), n_dst, d_in, d_out, D, n_dst_dev,
                           k_self);
        HOPGNN_LAUNCH_CHECK();
        const int group = mean_group(d_in);
        if (kind.scatter != kScatterMean)
            hipLaunchKernelGGL(bwd_scatter_kind<Tr>, dim3((unsigned)ceil_div(n_dst * group, kBwdThreads)), dim3(kBwdThreads),
                               0, s, D, static_cast<const T*>(Hsrc), self_idx, indptr, idx, n_dst, d_in, group, kind.scatter,
                               kind.norm, dHsrc, n_dst_dev);
        else if (slot_first >= 0)
        {
            const bool v4 = d_in % 4 == 0 && aligned(D, 16) && aligned(dHsrc, 16);
            const int pull_group = mean_group(v4 ? d_in / 4 : d_in);
            auto pull = v4 ? bwd_pull_slots<4> : bwd_pull_slots<1>;
            hipLaunchKernelGGL(pull, dim3((unsigned)ceil_div(n_src * pull_group, kBwdThreads)), dim3(kBwdThreads), 0, s, D,
                               indptr, idx, n_dst, n_src, slot_first, d_in, pull_group, dHsrc);
        }
        else
            hipLaunchKernelGGL(bwd_scatter, dim3((unsigned)ceil_div(n_dst * group, kBwdThreads)), dim3(kBwdThreads), 0, s,
                               D, self_idx, indptr, idx, n_dst, d_in, group, dHsrc, n_dst_dev);
        HOPGNN_LAUNCH_CHECK();
    }
    return HOPGNN_OK;
}

}  // namespace hopgnn

extern "C" hopgnn_status hopgnn_sage_bwd(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                         const int32_t* self_idx, const int32_t* indptr, const int32_t* idx,
                                         int64_t n_dst, const void* W_self, const void* W_neigh,
                                         const void* out_fwd, int32_t relu, const float* dOut, int32_t d_out,
                                         float* gW_self, float* gW_neigh, float* gbias, float* dHsrc, void* ws,
                                         size_t ws_bytes, void* stream) {
    return hopgnn_sage_bwd_dev(Hsrc, dt, n_src, nullptr, d_in, self_idx, indptr, idx, n_dst, nullptr, W_self, W_neigh,
                               out_fwd, nullptr, relu, dOut, d_out, gW_self, gW_neigh, gbias, dHsrc, ws, ws_bytes, stream);
}

static hopgnn_status sage_bwd_any(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t* n_src_dev,
                                  int32_t d_in, const int32_t* self_idx, const int32_t* indptr, const int32_t* idx,
                                  int64_t n_dst, const int64_t* n_dst_dev, const void* W_self, const void* W_neigh,
                                  const void* out_fwd, int32_t relu, const float* dOut, int32_t d_out, float* gW_self,
                                  float* gW_neigh, float* gbias, float* dHsrc, void* ws, size_t ws_bytes,
                                  int64_t slot_first, const void* mean_fwd, void* stream,
                                  const hopgnn::BwdKind& kind = hopgnn::BwdKind{-1, hopgnn::kScatterMean, 0});

extern "C" hopgnn_status hopgnn_sage_bwd_dev(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t* n_src_dev,
                                             int32_t d_in, const int32_t* self_idx, const int32_t* indptr,
                                             const int32_t* idx, int64_t n_dst, const int64_t* n_dst_dev,
                                             const void* W_self, const void* W_neigh, const void* out_fwd,
                                             const void* mean_fwd, int32_t relu, const float* dOut, int32_t d_out,
                                             float* gW_self, float* gW_neigh, float* gbias, float* dHsrc, void* ws,
                                             size_t ws_bytes, void* stream) {
    return sage_bwd_any(Hsrc, dt, n_src, n_src_dev, d_in, self_idx, indptr, idx, n_dst, n_dst_dev, W_self, W_neigh, out_fwd,
                        relu, dOut, d_out, gW_self, gW_neigh, gbias, dHsrc, ws, ws_bytes, -1, mean_fwd, stream);
}

extern "C" hopgnn_status hopgnn_sage_bwd_slots(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                               const int32_t* indptr, const int32_t* idx, int64_t n_dst,
                                               int64_t first_child_row, const void* W_self, const void* W_neigh,
                                               const void* out_fwd, const void* mean_fwd, int32_t relu,
                                               const float* dOut, int32_t d_out,
                                               float* gW_self, float* gW_neigh, float* gbias, float* dHsrc, void* ws,
                                               size_t ws_bytes, void* stream) {
    if (first_child_row < 0 || first_child_row > n_dst) return HOPGNN_EINVAL;
    if (n_dst > 0 && idx == nullptr) return HOPGNN_EINVAL;
    return sage_bwd_any(Hsrc, dt, n_src, nullptr, d_in, nullptr, indptr, idx, n_dst, nullptr, W_self, W_neigh, out_fwd, relu,
                        dOut, d_out, gW_self, gW_neigh, gbias, dHsrc, ws, ws_bytes, first_child_row, mean_fwd, stream);
}

extern "C" hopgnn_status hopgnn_sage_bwd_agg(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                             const int32_t* self_idx, const int32_t* indptr, const int32_t* idx,
                                             int64_t n_dst, const void* W_self, const void* W_neigh,
                                             const void* out_fwd, int32_t agg, int32_t relu, const float* dOut,
                                             int32_t d_out, float* gW_self, float* gW_neigh, float* gbias,
                                             float* dHsrc, void* ws, size_t ws_bytes, void* stream) {
    if (agg != HOPGNN_AGG_MEAN && agg != HOPGNN_AGG_SUM && agg != HOPGNN_AGG_MAX) return HOPGNN_EINVAL;
    const BwdKind kind{d_in, agg == HOPGNN_AGG_MEAN ? kScatterMean : agg == HOPGNN_AGG_SUM ? kScatterSum : kScatterMax, 0};
    return sage_bwd_any(Hsrc, dt, n_src, nullptr, d_in, self_idx, indptr, idx, n_dst, nullptr, W_self, W_neigh, out_fwd, relu,
                        dOut, d_out, gW_self, gW_neigh, gbias, dHsrc, ws, ws_bytes, -1, nullptr, stream, kind);
}

extern "C" hopgnn_status hopgnn_gcn_bwd(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                        const int32_t* self_idx, const int32_t* indptr, const int32_t* idx,
                                        int64_t n_dst, const void* W, const void* out_fwd, int32_t norm, int32_t relu,
                                        const float* dOut, int32_t d_out, float* gW, float* gbias, float* dHsrc,
                                        void* ws, size_t ws_bytes, void* stream) {
    if (norm != 0 && norm != 1) return HOPGNN_EINVAL;
    const BwdKind kind{0, kScatterGcn, norm};
    return sage_bwd_any(Hsrc, dt, n_src, nullptr, d_in, self_idx, indptr, idx, n_dst, nullptr, W, W, out_fwd, relu, dOut,
                        d_out, gW, gW, gbias, dHsrc, ws, ws_bytes, -1, nullptr, stream, kind);
}

static hopgnn_status sage_bwd_any(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t* n_src_dev,
                                  int32_t d_in, const int32_t* self_idx, const int32_t* indptr, const int32_t* idx,
                                  int64_t n_dst, const int64_t* n_dst_dev, const void* W_self, const void* W_neigh,
                                  const void* out_fwd, int32_t relu, const float* dOut, int32_t d_out, float* gW_self,
                                  float* gW_neigh, float* gbias, float* dHsrc, void* ws, size_t ws_bytes,
                                  int64_t slot_first, const void* mean_fwd, void* stream, const hopgnn::BwdKind& kind_in) {
    BwdKind kind = kind_in;
    if (kind.k_self < 0) kind.k_self = d_in;      // the default: the GraphSAGE-mean layer
    if (dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) return HOPGNN_EINVAL;
    if (n_src < 0 || n_dst < 0 || d_in < 1 || d_out < 1) return HOPGNN_EINVAL;
    if (d_in > (1 << 20) || d_out > (1 << 20)) return HOPGNN_ERANGE;
    if (n_dst >= ((int64_t)1 << 31) || n_src >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dHsrc != nullptr && n_src > 0 && (slot_first < 0 || n_dst == 0)) {    // the slot-order pull writes every row itself
        // a fill kernel, never a memset node; with a device row count only the rows that exist
        if (!aligned(dHsrc, 16) || ((int64_t)n_src * d_in) % 4 != 0 || (n_src_dev != nullptr && d_in % 4 != 0)) {
            const int64_t n = (int64_t)n_src * d_in;
            hipLaunchKernelGGL(bwd_zero_elem, dim3((unsigned)ceil_div(n, kBwdThreads)), dim3(kBwdThreads), 0, s, dHsrc, n,
                               n_src_dev, d_in);
            HOPGNN_LAUNCH_CHECK();
        } else {
            const int64_t n4 = (int64_t)n_src * d_in / 4;
            hipLaunchKernelGGL(bwd_zero, dim3((unsigned)ceil_div(n4, kBwdThreads)), dim3(kBwdThreads), 0, s,
                               reinterpret_cast<float4*>(dHsrc), n4, n_src_dev, d_in / 4);
            HOPGNN_LAUNCH_CHECK();
        }
    }
    if (n_dst == 0) return HOPGNN_OK;
    if (indptr == nullptr || W_self == nullptr || W_neigh == nullptr || dOut == nullptr || gW_self == nullptr ||
        gW_neigh == nullptr || ws == nullptr || (relu && out_fwd == nullptr))
        return HOPGNN_EINVAL;
    if (n_src > 0 && Hsrc == nullptr) return HOPGNN_EINVAL;
    if (self_idx == nullptr && n_src < n_dst) return HOPGNN_EINVAL;   // identity self rows must exist
    if (!aligned(ws, 256)) return HOPGNN_EINVAL;
    const BwdWs L = bwd_ws_layout(n_dst, d_in, d_out, dHsrc != nullptr, dt != HOPGNN_F32);
    if (ws_bytes < L.total) return HOPGNN_ENOMEM_WS;
    if (dt == HOPGNN_F32)
        return sage_bwd_typed<TrF32>(Hsrc, n_src, d_in, self_idx, indptr, idx, n_dst, W_self, W_neigh, out_fwd, relu, dOut,
                                     d_out, gW_self, gW_neigh, gbias, dHsrc, ws, L, n_dst_dev, slot_first, mean_fwd, s, kind);
    if (dt == HOPGNN_BF16)
        return sage_bwd_typed<TrBF16>(Hsrc, n_src, d_in, self_idx, indptr, idx, n_dst, W_self, W_neigh, out_fwd, relu,
                                      dOut, d_out, gW_self, gW_neigh, gbias, dHsrc, ws, L, n_dst_dev, slot_first, mean_fwd, s, kind);
    return sage_bwd_typed<TrF16>(Hsrc, n_src, d_in, self_idx, indptr, idx, n_dst, W_self, W_neigh, out_fwd, relu, dOut,
                                 d_out, gW_self, gW_neigh, gbias, dHsrc, ws, L, n_dst_dev, slot_first, mean_fwd, s, kind);
}

// ------------------------------------------------------- attention layer --
//
// Backward of the graph-attention layer (the third model of the paper's evaluation; the chain rule
// through softmax and LeakyReLU_0.2 written out).  z = Hsrc W (fp32) and the scores s_src, s_dst are
// read from the forward call's workspace.  With dY = dOut masked by the stored forward output:
//
//   gbias += column sums of dY                                            col_sum_rows + reduce_parts_add
//   per destination row and head over its entries u_i (self first):       gat_bwd_rows
//     alpha_i as in the forward pass;  dalpha_i = <dY[r,h], z_{u_i}[h]>;  dz[u_i,h] += alpha_i dY[r,h]
//     de_i = alpha_i (dalpha_i - sum_j alpha_j dalpha_j) * (e_i > 0 ? 1 : 0.2)
//     ds_src[u_i,h] += de_i;  ds_dst[self,h] += sum_i de_i
//   per source row:  dz[u,h] += ds_src[u,h] a_src[h] + ds_dst[u,h] a_dst[h]   gat_bwd_src
//     ga_src[h] += ds_src[u,h] z_u[h];  ga_dst[h] += ds_dst[u,h] z_u[h]       (+ reduce_parts_add)
//   gW += Hsrc^T dz  (the weight-gradient kernels, one matrix, rows = source rows)
//   dHsrc = dz W^T   (the input-gradient kernels, written in place)

namespace hopgnn {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float leaky02(float x) { return x > 0.f ? x : 0.2f * x; }

constexpr int kColRows = 128;    // rows per workgroup of the column-sum kernels

// partial[b][n] = sum over the rows of block b of dOut[r][n] where the activation passes
template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
col_sum_rows(const float* __restrict__ dOut, const typename Tr::store_t* __restrict__ out_fwd, int relu,
             int64_t n_rows, int32_t d_out, float* __restrict__ partial) {
    const int64_t r0 = (int64_t)blockIdx.x * kColRows;
    const int64_t r1 = r0 + kColRows < n_rows ? r0 + kColRows : n_rows;
    for (int32_t n = threadIdx.x; n < d_out; n += kBwdThreads) {
        float acc = 0.f;
        for (int64_t r = r0; r < r1; ++r) {
            const float g = dOut[r * d_out + n];
            acc += !relu || Tr::to_f(out_fwd[r * d_out + n]) > 0.f ? g : 0.f;
        }
        partial[(int64_t)blockIdx.x * d_out + n] = acc;
    }
}

// out[i] += sum over p < n_parts of partial[p * part_stride + i], i < width, in a fixed order (wave q
// takes the parts q, q + 4, ...; the four sums are combined as (s0 + s1) + (s2 + s3)): bit-stable.
// With a device row count only the parts of the rows that exist are summed (rows_per_part rows each).
__global__ void __launch_bounds__(kBwdThreads)
reduce_parts_add(const float* __restrict__ partial, int64_t part_stride, int32_t n_parts, int32_t width,
                 float* __restrict__ out, const int64_t* __restrict__ n_rows_dev, int32_t rows_per_part) {
    __shared__ float part[4][kWave];
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int32_t i = blockIdx.x * kWave + lane;
    if (n_rows_dev != nullptr) {
        const int64_t live = (*n_rows_dev + rows_per_part - 1) / rows_per_part;
        n_parts = live < n_parts ? (int32_t)live : n_parts;
    }
    float s = 0.f;
    if (i < width)
        for (int32_t p = q; p < n_parts; p += 4) s += partial[(int64_t)p * part_stride + i];
    part[q][lane] = s;
    __syncthreads();
    if (q == 0 && i < width) out[i] += (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
}

// One wavefront per destination row; heads are taken kHeadBatch at a time, side by side: per entry
// the scores, the z rows, the dot products (their wavefront sums interleave) and the atomic adds of
// the batch's heads are independent chains, where one head after the other leaves the wavefront
// waiting on one chain at a time (170 k rows x 4 heads x 6 entries: 2.5 ms one by one).
// The lanes share a head's columns.  The dot products dalpha_i of the first 64 entries stay in
// registers (lane i keeps entry i's); a longer segment computes the later ones a second time.
constexpr int kHeadBatch = 4;

template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
gat_bwd_rows(const float* __restrict__ Z, const float* __restrict__ scores, const int32_t* __restrict__ self_idx,
             const int32_t* __restrict__ indptr, const int32_t* __restrict__ idx,
             const typename Tr::store_t* __restrict__ out_fwd, int relu, const float* __restrict__ dOut,
             int64_t n_dst, int32_t d_out, int32_t n_heads, float* __restrict__ dZ, float* __restrict__ ds) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (kBwdThreads / kWave) + (threadIdx.x >> 6);
    if (r >= n_dst) return;                       // the whole wavefront
    const int32_t dh = d_out / n_heads, stride = 2 * n_heads;
    const int64_t s = self_idx != nullptr ? (int64_t)self_idx[r] : r;
    const int32_t beg = indptr[r], end = indptr[r + 1];
    const float* gy_row = dOut + r * d_out;
    const typename Tr::store_t* of_row = out_fwd != nullptr ? out_fwd + r * d_out : nullptr;
    auto g_at = [&](int32_t col) -> float {       // dY of this row: dOut where the activation passes
        const float g = gy_row[col];
        return !relu || Tr::to_f(of_row[col]) > 0.f ? g : 0.f;
    };
    for (int32_t h0 = 0; h0 < n_heads; h0 += kHeadBatch) {
        const int nh = n_heads - h0 < kHeadBatch ? n_heads - h0 : kHeadBatch;      // heads of this batch
        float sd[kHeadBatch], mx[kHeadBatch], den[kHeadBatch], inv[kHeadBatch];
#pragma unroll
        for (int b = 0; b < kHeadBatch; ++b) {
            sd[b] = (b < nh && s >= 0) ? scores[s * stride + n_heads + h0 + b] : 0.f;
            mx[b] = -INFINITY;
            den[b] = 0.f;
        }
        auto e_of = [&](int64_t u, int b) -> float {      // pre-activation score of entry u for head h0 + b
            return sd[b] + scores[u * stride + h0 + (b < nh ? b : 0)];
        };
        // the softmax's maximum and denominator, as the forward pass takes them
        if (s >= 0) {
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) mx[b] = leaky02(e_of(s, b));
        }
        for (int32_t e = beg; e < end; ++e) {
            const int32_t u = idx[e];
            if (u < 0) continue;
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) mx[b] = fmaxf(mx[b], leaky02(e_of(u, b)));
        }
        if (mx[0] == -INFINITY) continue;         // no entries: the row's output is act(bias)
        if (s >= 0) {
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) den[b] += expf(leaky02(e_of(s, b)) - mx[b]);
        }
        for (int32_t e = beg; e < end; ++e) {
            const int32_t u = idx[e];
            if (u < 0) continue;
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) den[b] += expf(leaky02(e_of(u, b)) - mx[b]);
        }
#pragma unroll
        for (int b = 0; b < kHeadBatch; ++b) inv[b] = 1.f / den[b];

        // first pass: dz, the dot products, and S = sum alpha_i dalpha_i
        float S[kHeadBatch], mine[kHeadBatch];
#pragma unroll
        for (int b = 0; b < kHeadBatch; ++b) S[b] = mine[b] = 0.f;
        auto dots = [&](int64_t u, float (&d)[kHeadBatch], const float (&al)[kHeadBatch], bool add) {
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) {
                d[b] = 0.f;
                if (b < nh) {
                    const int32_t c0 = (h0 + b) * dh;
                    for (int32_t j = lane; j < dh; j += kWave) {
                        const float g = g_at(c0 + j);
                        d[b] += g * Z[u * d_out + c0 + j];
                        if (add) atomicAdd(&dZ[u * d_out + c0 + j], al[b] * g);
                    }
                }
            }
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) d[b] = wave_sum(d[b]);
        };
        int32_t i = 0;
        auto first = [&](int64_t u) {
            float al[kHeadBatch], d[kHeadBatch];
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) al[b] = expf(leaky02(e_of(u, b)) - mx[b]) * inv[b];
            dots(u, d, al, true);
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) {
                S[b] += al[b] * d[b];
                if (lane == i) mine[b] = d[b];    // entries past 63 match no lane
            }
            ++i;
        };
        if (s >= 0) first(s);
        for (int32_t e = beg; e < end; ++e)
            if (idx[e] >= 0) first(idx[e]);
        // second pass: the score gradients
        i = 0;
        float sum_de[kHeadBatch];
#pragma unroll
        for (int b = 0; b < kHeadBatch; ++b) sum_de[b] = 0.f;
        auto second = [&](int64_t u) {
            float al[kHeadBatch], d[kHeadBatch], ev[kHeadBatch];
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) {
                ev[b] = e_of(u, b);
                al[b] = expf(leaky02(ev[b]) - mx[b]) * inv[b];
            }
            if (i < kWave) {
#pragma unroll
                for (int b = 0; b < kHeadBatch; ++b) d[b] = __shfl(mine[b], i, kWave);
            } else {
                dots(u, d, al, false);
            }
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b) {
                const float de = al[b] * (d[b] - S[b]) * (ev[b] > 0.f ? 1.f : 0.2f);
                if (lane == b && b < nh) atomicAdd(&ds[u * stride + h0 + b], de);
                sum_de[b] += de;
            }
            ++i;
        };
        if (s >= 0) second(s);
        for (int32_t e = beg; e < end; ++e)
            if (idx[e] >= 0) second(idx[e]);
        if (s >= 0) {
#pragma unroll
            for (int b = 0; b < kHeadBatch; ++b)
                if (lane == b && b < nh) atomicAdd(&ds[s * stride + n_heads + h0 + b], sum_de[b]);
        }
    }
}

constexpr int kSrcRows = 256;    // source rows per workgroup of gat_bwd_src

// dz[u] += ds_src[u,h] a_src[h] + ds_dst[u,h] a_dst[h] in place (one thread owns a column of the
// block's rows), and the block's part of ga_src / ga_dst: partial[b][0][n], partial[b][1][n].
template <typename Tr>
__global__ void __launch_bounds__(kBwdThreads)
gat_bwd_src(const float* __restrict__ Z, const float* __restrict__ ds, const typename Tr::store_t* __restrict__ a_src,
            const typename Tr::store_t* __restrict__ a_dst, int64_t n_src_cap, const int64_t* __restrict__ n_rows_dev,
            int32_t d_out, int32_t n_heads, float* __restrict__ dZ, float* __restrict__ partial) {
    const int32_t dh = d_out / n_heads, stride = 2 * n_heads;
    const int64_t n_src = n_rows_dev != nullptr && *n_rows_dev < n_src_cap ? *n_rows_dev : n_src_cap;
    const int64_t u0 = (int64_t)blockIdx.x * kSrcRows;       // a block past the last row writes zero parts
    const int64_t u1 = u0 + kSrcRows < n_src ? u0 + kSrcRows : n_src;
    for (int32_t n = threadIdx.x; n < d_out; n += kBwdThreads) {
        const int32_t h = n / dh;
        const float as = Tr::to_f(a_src[n]), ad = Tr::to_f(a_dst[n]);
        float acc_s = 0.f, acc_d = 0.f;
        for (int64_t u = u0; u < u1; ++u) {
            const float dss = ds[u * stride + h], dsd = ds[u * stride + n_heads + h];
            const float z = Z[u * d_out + n];
            acc_s += dss * z;
            acc_d += dsd * z;
            dZ[u * d_out + n] += dss * as + dsd * ad;
        }
        partial[((int64_t)blockIdx.x * 2 + 0) * d_out + n] = acc_s;
        partial[((int64_t)blockIdx.x * 2 + 1) * d_out + n] = acc_d;
    }
}

struct GatBwdWs {
    size_t dz_bytes, ds_bytes, col_bytes, zero_bytes;
    BwdWs G;          // the weight gradient's partial tiles (rows = source rows)
    size_t total;
};
static GatBwdWs gat_bwd_ws_layout(int64_t n_src, int64_t n_dst, int32_t d_in, int32_t d_out, int32_t n_heads) {
    GatBwdWs L{};
    const int64_t ns = n_src > 0 ? n_src : 1, nd = n_dst > 0 ? n_dst : 1;
    L.dz_bytes = align_up((size_t)ns * d_out * 4, 256);
    L.ds_bytes = align_up((size_t)ns * 2 * n_heads * 4, 256);
    const int64_t parts = ceil_div(nd, kColRows) > 2 * ceil_div(ns, kSrcRows) ? ceil_div(nd, kColRows) : 2 * ceil_div(ns, kSrcRows);
    L.col_bytes = align_up((size_t)parts * d_out * 4, 256);
    L.G = bwd_ws_layout(ns, d_in, d_out, 0);      // (row splits as for fp32 operands: any count is valid)
    L.total = L.dz_bytes + L.ds_bytes + L.col_bytes + L.G.partial_bytes + L.G.bias_bytes;
    return L;
}

template <typename Tr>
static hopgnn_status gat_bwd_typed(const void* Hsrc, int64_t n_src, const int64_t* n_src_dev, int32_t d_in,
                                   const int32_t* self_idx,
                                   const int32_t* indptr, const int32_t* idx, int64_t n_dst, const void* W,
                                   const void* a_src, const void* a_dst, const void* out_fwd, const void* fwd_ws,
                                   int32_t relu, const float* dOut, int32_t d_out, int32_t n_heads, float* gW,
                                   float* ga_src, float* ga_dst, float* gbias, float* dHsrc, void* ws,
                                   const GatBwdWs& L, hipStream_t s) {
    using T = typename Tr::store_t;
    char* p = static_cast<char*>(ws);
    float* dZ = reinterpret_cast<float*>(p);
    float* ds = reinterpret_cast<float*>(p + L.dz_bytes);
    float* col = reinterpret_cast<float*>(p + L.dz_bytes + L.ds_bytes);
    float* partial = reinterpret_cast<float*>(p + L.dz_bytes + L.ds_bytes + L.col_bytes);
    float* bias_partial = reinterpret_cast<float*>(reinterpret_cast<char*>(partial) + L.G.partial_bytes);
    const GatWs F = gat_ws_layout(Tr::kDt, n_src, d_in, d_out, n_heads);
    const float* Z = static_cast<const float*>(fwd_ws);
    const float* scores = reinterpret_cast<const float*>(static_cast<const char*>(fwd_ws) + F.z_bytes);

    if (gbias != nullptr) {
        const int32_t parts = (int32_t)ceil_div(n_dst, kColRows);
        hipLaunchKernelGGL(col_sum_rows<Tr>, dim3((unsigned)parts), dim3(kBwdThreads), 0, s, dOut,
                           static_cast<const T*>(out_fwd), relu, n_dst, d_out, col);
        HOPGNN_LAUNCH_CHECK();
        hipLaunchKernelGGL(reduce_parts_add, dim3((unsigned)ceil_div(d_out, kWave)), dim3(kBwdThreads), 0, s, col,
                           (int64_t)d_out, parts, d_out, gbias, nullptr, 0);
        HOPGNN_LAUNCH_CHECK();
    }
    if (n_src == 0) return HOPGNN_OK;              // no entries anywhere: only the bias has a gradient

    // dz and ds start at zero (fill kernels, never a memset node): the source rows that exist
    if (d_out % 4 == 0)
        hipLaunchKernelGGL(bwd_zero, dim3((unsigned)ceil_div(n_src * (d_out / 4), kBwdThreads)), dim3(kBwdThreads), 0, s,
                           reinterpret_cast<float4*>(dZ), n_src * (d_out / 4), n_src_dev, d_out / 4);
    else
        hipLaunchKernelGGL(bwd_zero_elem, dim3((unsigned)ceil_div(n_src * d_out, kBwdThreads)), dim3(kBwdThreads), 0, s, dZ,
                           n_src * d_out, n_src_dev, d_out);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(bwd_zero_elem, dim3((unsigned)ceil_div(n_src * 2 * n_heads, kBwdThreads)), dim3(kBwdThreads), 0, s, ds,
                       n_src * 2 * n_heads, n_src_dev, 2 * n_heads);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(gat_bwd_rows<Tr>, dim3((unsigned)ceil_div(n_dst, kBwdThreads / kWave)), dim3(kBwdThreads), 0, s, Z,
                       scores, self_idx, indptr, idx, static_cast<const T*>(out_fwd), relu, dOut, n_dst, d_out, n_heads, dZ,
                       ds);
    HOPGNN_LAUNCH_CHECK();
    const int32_t src_blocks = (int32_t)ceil_div(n_src, kSrcRows);
    hipLaunchKernelGGL(gat_bwd_src<Tr>, dim3((unsigned)src_blocks), dim3(kBwdThreads), 0, s, Z, ds,
                       static_cast<const T*>(a_src), static_cast<const T*>(a_dst), n_src, n_src_dev, d_out, n_heads, dZ, col);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(reduce_parts_add, dim3((unsigned)ceil_div(d_out, kWave)), dim3(kBwdThreads), 0, s, col,
                       (int64_t)2 * d_out, src_blocks, d_out, ga_src, n_src_dev, kSrcRows);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(reduce_parts_add, dim3((unsigned)ceil_div(d_out, kWave)), dim3(kBwdThreads), 0, s, col + d_out,
                       (int64_t)2 * d_out, src_blocks, d_out, ga_dst, n_src_dev, kSrcRows);
    HOPGNN_LAUNCH_CHECK();

    // gW += Hsrc^T dz: one matrix (k_self = 0), the "aggregate" operand is Hsrc itself, rows = source rows
    const uint32_t tiles_k = (uint32_t)ceil_div(d_in, kGradTile), tiles_n = (uint32_t)ceil_div(d_out, kGradTile);
    const bool vec = d_in % 4 == 0 && d_out % 4 == 0 && aligned(Hsrc, 16);
    bool on16 = false;
    if constexpr (sizeof(T) == 2) {
        on16 = vec && d_in % 8 == 0;
        if (on16) {
            launch_weight_grad16<Tr, false>(s, static_cast<const T*>(Hsrc), nullptr, static_cast<const T*>(Hsrc), dZ, nullptr,
                                            n_src, d_in, d_out, L.G, partial, nullptr, n_src_dev, 0);
        }
    }
    if (!on16) {
        auto grad_kernel = vec ? bwd_weight_grad<Tr, true, false> : bwd_weight_grad<Tr, false, false>;
        hipLaunchKernelGGL(grad_kernel, dim3(tiles_k * tiles_n, (unsigned)L.G.n_splits), dim3(kBwdThreads), 0, s,
                           static_cast<const T*>(Hsrc), nullptr, static_cast<const T*>(Hsrc), dZ, nullptr, n_src, d_in, d_out,
                           L.G.rows_per_split, tiles_n, partial, nullptr, n_src_dev, 0);
    }
    HOPGNN_LAUNCH_CHECK();
    const int64_t red = (int64_t)d_in * d_out;
    hipLaunchKernelGGL(bwd_weight_reduce, dim3((unsigned)ceil_div(red, kWave)), dim3(kBwdThreads), 0, s, partial,
                       bias_partial, L.G.n_splits, d_in, d_out, gW, gW, nullptr, 0);
    HOPGNN_LAUNCH_CHECK();

    if (dHsrc != nullptr) {      // dHsrc = dz W^T, every element written
        const int64_t gy = ceil_div(d_in, 64);
        if (gy > 65535) return HOPGNN_ERANGE;
        auto in_kernel = bwd_input_grad<Tr>;
        if constexpr (sizeof(T) == 2) {
            if (aligned(W, 16)) in_kernel = bwd_input_grad16<Tr>;
        }
        hipLaunchKernelGGL(in_kernel, dim3((unsigned)ceil_div(n_src, 64), (unsigned)gy), dim3(kBwdThreads), 0, s, dZ,
                           static_cast<const T*>(W), static_cast<const T*>(W), n_src, d_in, d_out, dHsrc, n_src_dev, 0);
        HOPGNN_LAUNCH_CHECK();
    }
    return HOPGNN_OK;
}

}  // namespace hopgnn

extern "C" size_t hopgnn_gat_bwd_ws_bytes(hopgnn_dtype dt, int64_t n_src, int64_t n_dst, int32_t d_in, int32_t d_out,
                                          int32_t n_heads) {
    if ((dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) || n_src < 0 || n_dst < 0 || d_in < 1 || d_out < 1 ||
        n_heads < 1 || n_heads > 16 || d_out % n_heads != 0)
        return 0;
    return gat_bwd_ws_layout(n_src, n_dst, d_in, d_out, n_heads).total;
}

extern "C" hopgnn_status hopgnn_gat_bwd(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t* n_src_dev,
                                        int32_t d_in, const int32_t* self_idx, const int32_t* indptr, const int32_t* idx,
                                        int64_t n_dst, const void* W, const void* a_src, const void* a_dst,
                                        const void* out_fwd, const void* fwd_ws, int32_t relu, const float* dOut,
                                        int32_t d_out, int32_t n_heads, float* gW, float* ga_src, float* ga_dst,
                                        float* gbias, float* dHsrc, void* ws, size_t ws_bytes, void* stream) {
    if (dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) return HOPGNN_EINVAL;
    if (n_src < 0 || n_dst < 0 || d_in < 1 || d_out < 1) return HOPGNN_EINVAL;
    if (n_heads < 1 || n_heads > 16 || d_out % n_heads != 0) return HOPGNN_EINVAL;
    if (d_in > (1 << 20) || d_out > (1 << 20)) return HOPGNN_ERANGE;
    if (n_dst >= ((int64_t)1 << 31) || n_src >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if (n_dst == 0) {
        if (dHsrc != nullptr && n_src > 0) {       // no destination rows: the input gradient is zero
            const int64_t n = (int64_t)n_src * d_in;
            hipLaunchKernelGGL(bwd_zero_elem, dim3((unsigned)ceil_div(n, kBwdThreads)), dim3(kBwdThreads), 0,
                               static_cast<hipStream_t>(stream), dHsrc, n, nullptr, 0);
            HOPGNN_LAUNCH_CHECK();
        }
        return HOPGNN_OK;
    }
    if (indptr == nullptr || W == nullptr || a_src == nullptr || a_dst == nullptr || dOut == nullptr || gW == nullptr ||
        ga_src == nullptr || ga_dst == nullptr || ws == nullptr || fwd_ws == nullptr || (relu && out_fwd == nullptr))
        return HOPGNN_EINVAL;
    if (n_src > 0 && Hsrc == nullptr) return HOPGNN_EINVAL;
    if (self_idx == nullptr && n_src < n_dst) return HOPGNN_EINVAL;
    if (!aligned(ws, 256) || !aligned(fwd_ws, 256)) return HOPGNN_EINVAL;
    const GatBwdWs L = gat_bwd_ws_layout(n_src, n_dst, d_in, d_out, n_heads);
    if (ws_bytes < L.total) return HOPGNN_ENOMEM_WS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == HOPGNN_F32)
        return gat_bwd_typed<TrF32>(Hsrc, n_src, n_src_dev, d_in, self_idx, indptr, idx, n_dst, W, a_src, a_dst, out_fwd, fwd_ws, relu, dOut,
                                    d_out, n_heads, gW, ga_src, ga_dst, gbias, dHsrc, ws, L, s);
    if (dt == HOPGNN_BF16)
        return gat_bwd_typed<TrBF16>(Hsrc, n_src, n_src_dev, d_in, self_idx, indptr, idx, n_dst, W, a_src, a_dst, out_fwd, fwd_ws, relu,
                                     dOut, d_out, n_heads, gW, ga_src, ga_dst, gbias, dHsrc, ws, L, s);
    return gat_bwd_typed<TrF16>(Hsrc, n_src, n_src_dev, d_in, self_idx, indptr, idx, n_dst, W, a_src, a_dst, out_fwd, fwd_ws, relu, dOut,
                                d_out, n_heads, gW, ga_src, ga_dst, gbias, dHsrc, ws, L, s);
}

extern "C" hopgnn_status hopgnn_sgd_update(void* W, hopgnn_dtype dt, float* grad, int64_t n, float lr, int32_t zero_grad,
                                           void* stream) {
    if (dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) return HOPGNN_EINVAL;
    if (n < 0) return HOPGNN_EINVAL;
    if (n == 0) return HOPGNN_OK;
    if (W == nullptr || grad == nullptr) return HOPGNN_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t want = ceil_div(n, kBwdThreads);
    const dim3 grid((unsigned)(want < 4096 ? want : 4096));
    if (dt == HOPGNN_F32)
        hipLaunchKernelGGL(sgd_update<TrF32>, grid, dim3(kBwdThreads), 0, s, static_cast<float*>(W), grad, n, lr, zero_grad);
    else if (dt == HOPGNN_BF16)
        hipLaunchKernelGGL(sgd_update<TrBF16>, grid, dim3(kBwdThreads), 0, s, static_cast<uint16_t*>(W), grad, n, lr,
                           zero_grad);
    else
        hipLaunchKernelGGL(sgd_update<TrF16>, grid, dim3(kBwdThreads), 0, s, static_cast<_Float16*>(W), grad, n, lr,
                           zero_grad);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

extern "C" hopgnn_status hopgnn_sgd_update_multi(void* const* W, hopgnn_dtype dt, float* const* grad, const int64_t* n,
                                                 int32_t n_tensors, float lr, int32_t zero_grad, void* stream) {
    if (dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) return HOPGNN_EINVAL;
    if (n_tensors < 0 || n_tensors > kSgdMaxTensors) return HOPGNN_EINVAL;
    if (n_tensors == 0) return HOPGNN_OK;
    if (W == nullptr || grad == nullptr || n == nullptr) return HOPGNN_EINVAL;
    SgdBatch b{};
    int64_t blocks = 0;
    for (int32_t t = 0; t < n_tensors; ++t) {
        if (n[t] < 0 || (n[t] > 0 && (W[t] == nullptr || grad[t] == nullptr))) return HOPGNN_EINVAL;
        if (n[t] == 0) continue;                 // nothing to update: no blocks
        b.W[b.n_tensors] = W[t];
        b.grad[b.n_tensors] = grad[t];
        b.n[b.n_tensors] = n[t];
        b.first_block[b.n_tensors] = blocks;
        blocks += ceil_div(n[t], kSgdPerBlock);
        ++b.n_tensors;
    }
    b.first_block[b.n_tensors] = blocks;
    if (blocks == 0) return HOPGNN_OK;
    if (blocks >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)blocks);
    if (dt == HOPGNN_F32) hipLaunchKernelGGL(sgd_update_multi<TrF32>, grid, dim3(kBwdThreads), 0, s, b, lr, zero_grad);
    else if (dt == HOPGNN_BF16) hipLaunchKernelGGL(sgd_update_multi<TrBF16>, grid, dim3(kBwdThreads), 0, s, b, lr, zero_grad);
    else hipLaunchKernelGGL(sgd_update_multi<TrF16>, grid, dim3(kBwdThreads), 0, s, b, lr, zero_grad);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}
