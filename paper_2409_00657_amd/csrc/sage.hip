// hopgnn_sage_fwd: one GraphSAGE-mean layer (paper section 2 "computation":
// aggregate the neighbouring features of each vertex, then a neural-network
// transform).
//
//   out[r] = act( Hsrc[self_idx[r]] W_self + mean_{e in seg(r), idx[e]>=0} Hsrc[idx[e]] W_neigh + b )
//
// Two kernels.
//   sage_mean     CSR segmented mean.  HBM/L2 bound: nnz indirect row reads in
//                 128-bit words, one lane group per destination row, fp32 running
//                 sum in entry order (deterministic), one rounding to the
//                 activation type.
//   sage_project  dense contraction [x_self | mean] (M x 2*d_in) times
//                 [W_self ; W_neigh] on the matrix cores (fp32 MFMA for fp32,
//                 bf16/fp16 MFMA with fp32 accumulate for 2-byte types).  The self
//                 half of the left operand is read straight from Hsrc through
//                 self_idx, so it is never copied.
#include "common.hpp"

namespace hopgnn {

typedef float floatx16 __attribute__((ext_vector_type(16)));
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
};

struct TrF16 {
    using store_t = _Float16;
    static constexpr int kPer16 = 8;
    static constexpr hopgnn_dtype kDt = HOPGNN_F16;
    __device__ static __forceinline__ float to_f(_Float16 h) { return (float)h; }
    __device__ static __forceinline__ _Float16 from_f(float x) { return (_Float16)x; }
};

template <typename Tr>
union Pack16 {
    uint4 v;
    typename Tr::store_t e[Tr::kPer16];
};

// ------------------------------------------------------------ segmented mean --

constexpr int kMeanThreads = 256;
constexpr int kMeanUnroll = 4;

// Vector path: d_in * sizeof(elem) is a multiple of 16.  `group` lanes (a power of
// two <= 64) share one destination row; lane g of the group owns 16-byte word
// g, g+group, ... of the row.
template <typename Tr>
__global__ void __launch_bounds__(kMeanThreads)
sage_mean_vec(const uint4* __restrict__ Hsrc, const int32_t* __restrict__ indptr,
              const int32_t* __restrict__ idx, int64_t n_dst, int32_t words_per_row, int32_t group,
              uint4* __restrict__ Mean) {
    const int64_t gid = ((int64_t)blockIdx.x * kMeanThreads + threadIdx.x);
    const int64_t r = gid / group;
    const int32_t g = (int32_t)(gid - r * group);
    if (r >= n_dst) return;
    const int32_t beg = indptr[r], end = indptr[r + 1];
    for (int32_t c = g; c < words_per_row; c += group) {
        float acc[Tr::kPer16];
#pragma unroll
        for (int i = 0; i < Tr::kPer16; ++i) acc[i] = 0.f;
        int32_t cnt = 0;
        for (int32_t e = beg; e < end; e += kMeanUnroll) {
            int32_t u[kMeanUnroll];
            Pack16<Tr> v[kMeanUnroll];
#pragma unroll
            for (int k = 0; k < kMeanUnroll; ++k) u[k] = (e + k < end) ? idx[e + k] : -1;
#pragma unroll
            for (int k = 0; k < kMeanUnroll; ++k)
                if (u[k] >= 0) v[k].v = Hsrc[(int64_t)u[k] * words_per_row + c];
#pragma unroll
            for (int k = 0; k < kMeanUnroll; ++k)
                if (u[k] >= 0) {
#pragma unroll
                    for (int i = 0; i < Tr::kPer16; ++i) acc[i] += Tr::to_f(v[k].e[i]);
                    ++cnt;
                }
        }
        Pack16<Tr> o;
        const float fc = (float)cnt;
#pragma unroll
        for (int i = 0; i < Tr::kPer16; ++i) o.e[i] = Tr::from_f(cnt > 0 ? acc[i] / fc : 0.f);
        Mean[r * words_per_row + c] = o.v;
    }
}

// Element path for rows that are not a whole number of 16-byte words.
template <typename Tr>
__global__ void __launch_bounds__(kMeanThreads)
sage_mean_elem(const typename Tr::store_t* __restrict__ Hsrc, const int32_t* __restrict__ indptr,
               const int32_t* __restrict__ idx, int64_t n_dst, int32_t d_in, int32_t group,
               typename Tr::store_t* __restrict__ Mean) {
    const int64_t gid = ((int64_t)blockIdx.x * kMeanThreads + threadIdx.x);
    const int64_t r = gid / group;
    const int32_t g = (int32_t)(gid - r * group);
    if (r >= n_dst) return;
    const int32_t beg = indptr[r], end = indptr[r + 1];
    for (int32_t c = g; c < d_in; c += group) {
        float acc = 0.f;
        int32_t cnt = 0;
        for (int32_t e = beg; e < end; ++e) {
            const int32_t u = idx[e];
            if (u >= 0) {
                acc += Tr::to_f(Hsrc[(int64_t)u * d_in + c]);
                ++cnt;
            }
        }
        Mean[r * d_in + c] = Tr::from_f(cnt > 0 ? acc / (float)cnt : 0.f);
    }
}

// -------------------------------------------------------------- projection --
//
// 256 threads = 4 waves in a 2 x 2 arrangement; each wave owns a (BM/2) x (BN/2)
// piece of the output as 32 x 32 MFMA tiles.  The K loop runs over two phases:
// phase 0 multiplies the self rows by W_self, phase 1 the means by W_neigh; each
// phase is zero-padded to a whole number of BK tiles.
//
// Accumulator layout of a 32x32 MFMA tile: register i of lane l holds
//   row = 8*(i/4) + 4*(l/32) + i%4,  col = l%32.

constexpr int kProjThreads = 256;

template <typename Tr, int BM, int BN>
__device__ __forceinline__ void project_epilogue(floatx16 (&acc)[BM / 64][BN / 64], int64_t row0,
                                                 int32_t col0, int wm, int wn, int lane, int64_t n_dst,
                                                 int32_t d_out, const typename Tr::store_t* bias,
                                                 int relu, typename Tr::store_t* out) {
#pragma unroll
    for (int tn = 0; tn < BN / 64; ++tn) {
        const int32_t col = col0 + wn * (BN / 2) + tn * 32 + (lane & 31);
        if (col >= d_out) continue;
        const float b = bias != nullptr ? Tr::to_f(bias[col]) : 0.f;
#pragma unroll
        for (int tm = 0; tm < BM / 64; ++tm) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t row = row0 + wm * (BM / 2) + tm * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
                if (row < n_dst) {
                    float x = acc[tm][tn][i] + b;
                    if (relu) x = fmaxf(x, 0.f);
                    out[row * d_out + col] = Tr::from_f(x);
                }
            }
        }
    }
}

// fp32: v_mfma_f32_32x32x2_f32.  LDS holds A transposed (k-major) so that the 32
// lanes of a half-wave read 32 consecutive floats.
template <int BM, int BN, bool VEC>
__global__ void __launch_bounds__(kProjThreads)
sage_project_f32(const float* __restrict__ Hsrc, const int32_t* __restrict__ self_idx,
                 const float* __restrict__ Mean, const float* __restrict__ Wself,
                 const float* __restrict__ Wneigh, const float* __restrict__ bias, int64_t n_dst,
                 int32_t d_in, int32_t d_out, int relu, float* __restrict__ out) {
    constexpr int BK = 16;
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int A_ITEMS = BM * BK / 4 / kProjThreads;   // float4 items per thread
    constexpr int B_ITEMS = BK * BN / 4 / kProjThreads;
    static_assert(A_ITEMS >= 1 && B_ITEMS >= 1, "tile too small for 256 threads");
    __shared__ float As[BK][BM + 4];
    __shared__ __attribute__((aligned(16))) float Bs[BK][BN + 4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t row0 = (int64_t)blockIdx.x * BM;
    const int32_t col0 = blockIdx.y * BN;

    // rows this thread stages, fixed for the whole K loop
    int64_t a_self[A_ITEMS], a_mean[A_ITEMS];
#pragma unroll
    for (int it = 0; it < A_ITEMS; ++it) {
        const int i = it * kProjThreads + tid;
        const int64_t r = row0 + i / (BK / 4);
        a_self[it] = -1;
        a_mean[it] = -1;
        if (r < n_dst) {
            const int64_t s = self_idx != nullptr ? (int64_t)self_idx[r] : r;
            a_self[it] = s >= 0 ? s * d_in : -1;
            a_mean[it] = r * d_in;
        }
    }

    floatx16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0.f;

    const int tiles_per_phase = (d_in + BK - 1) / BK;
    const int n_tiles = 2 * tiles_per_phase;

    float4 ra[A_ITEMS], rb[B_ITEMS];
    auto load_tile = [&](int t) {
        const int phase = t >= tiles_per_phase;
        const int k0 = (t - phase * tiles_per_phase) * BK;
        const float* Asrc = phase ? Mean : Hsrc;
        const float* W = phase ? Wneigh : Wself;
#pragma unroll
        for (int it = 0; it < A_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            const int k = k0 + (i % (BK / 4)) * 4;
            const int64_t base = phase ? a_mean[it] : a_self[it];
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (base >= 0) {
                if (VEC && k + 3 < d_in) {
                    v = *reinterpret_cast<const float4*>(Asrc + base + k);
                } else {
                    if (k + 0 < d_in) v.x = Asrc[base + k + 0];
                    if (k + 1 < d_in) v.y = Asrc[base + k + 1];
                    if (k + 2 < d_in) v.z = Asrc[base + k + 2];
                    if (k + 3 < d_in) v.w = Asrc[base + k + 3];
                }
            }
            ra[it] = v;
        }
#pragma unroll
        for (int it = 0; it < B_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            const int k = k0 + i / (BN / 4);
            const int n = col0 + (i % (BN / 4)) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k < d_in) {
                const float* p = W + (int64_t)k * d_out + n;
                if (VEC && n + 3 < d_out) {
                    v = *reinterpret_cast<const float4*>(p);
                } else {
                    if (n + 0 < d_out) v.x = p[0];
                    if (n + 1 < d_out) v.y = p[1];
                    if (n + 2 < d_out) v.z = p[2];
                    if (n + 3 < d_out) v.w = p[3];
                }
            }
            rb[it] = v;
        }
    };

    load_tile(0);
    for (int t = 0; t < n_tiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < A_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            const int r = i / (BK / 4), kq = (i % (BK / 4)) * 4;
            As[kq + 0][r] = ra[it].x;
            As[kq + 1][r] = ra[it].y;
            As[kq + 2][r] = ra[it].z;
            As[kq + 3][r] = ra[it].w;
        }
#pragma unroll
        for (int it = 0; it < B_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            *reinterpret_cast<float4*>(&Bs[i / (BN / 4)][(i % (BN / 4)) * 4]) = rb[it];
        }
        __syncthreads();
        if (t + 1 < n_tiles) load_tile(t + 1);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float a[TM], b[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) a[tm] = As[kk + (lane >> 5)][wm * (BM / 2) + tm * 32 + (lane & 31)];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) b[tn] = Bs[kk + (lane >> 5)][wn * (BN / 2) + tn * 32 + (lane & 31)];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
        }
    }
    project_epilogue<TrF32, BM, BN>(acc, row0, col0, wm, wn, lane, n_dst, d_out, bias, relu, out);
}

// bf16 / fp16: v_mfma_f32_32x32x16_{bf16,f16}.  Lane l feeds 8 consecutive k of
// row (or column) l%32, k-group l/32.  LDS: A row-major [BM][BK+8], B n-major
// [BN][BK+8] (W is transposed while it is staged), both read as 128-bit words.
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

template <typename Tr, int BM, int BN, bool VEC>
__global__ void __launch_bounds__(kProjThreads)
sage_project_16(const uint16_t* __restrict__ Hsrc, const int32_t* __restrict__ self_idx,
                const uint16_t* __restrict__ Mean, const uint16_t* __restrict__ Wself,
                const uint16_t* __restrict__ Wneigh, const typename Tr::store_t* __restrict__ bias,
                int64_t n_dst, int32_t d_in, int32_t d_out, int relu,
                typename Tr::store_t* __restrict__ out) {
    constexpr int BK = 32, LD = BK + 8;
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int A_ITEMS = BM * BK / 8 / kProjThreads;   // 16-byte items per thread
    constexpr int B_ITEMS = BK * BN / 8 / kProjThreads;
    static_assert(A_ITEMS >= 1 && B_ITEMS >= 1, "tile too small for 256 threads");
    __shared__ __attribute__((aligned(16))) uint16_t As[BM][LD];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[BN][LD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t row0 = (int64_t)blockIdx.x * BM;
    const int32_t col0 = blockIdx.y * BN;

    int64_t a_self[A_ITEMS], a_mean[A_ITEMS];
#pragma unroll
    for (int it = 0; it < A_ITEMS; ++it) {
        const int i = it * kProjThreads + tid;
        const int64_t r = row0 + i / (BK / 8);
        a_self[it] = -1;
        a_mean[it] = -1;
        if (r < n_dst) {
            const int64_t s = self_idx != nullptr ? (int64_t)self_idx[r] : r;
            a_self[it] = s >= 0 ? s * d_in : -1;
            a_mean[it] = r * d_in;
        }
    }

    floatx16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0.f;

    const int tiles_per_phase = (d_in + BK - 1) / BK;
    const int n_tiles = 2 * tiles_per_phase;

    union U16x8 {
        uint4 v;
        uint16_t e[8];
    };
    U16x8 ra[A_ITEMS], rb[B_ITEMS];
    auto load_tile = [&](int t) {
        const int phase = t >= tiles_per_phase;
        const int k0 = (t - phase * tiles_per_phase) * BK;
        const uint16_t* Asrc = phase ? Mean : Hsrc;
        const uint16_t* W = phase ? Wneigh : Wself;
#pragma unroll
        for (int it = 0; it < A_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            const int k = k0 + (i % (BK / 8)) * 8;
            const int64_t base = phase ? a_mean[it] : a_self[it];
            U16x8 v;
            v.v = make_uint4(0u, 0u, 0u, 0u);
            if (base >= 0) {
                if (VEC && k + 7 < d_in) {
                    v.v = *reinterpret_cast<const uint4*>(Asrc + base + k);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (k + j < d_in) v.e[j] = Asrc[base + k + j];
                }
            }
            ra[it] = v;
        }
        // B: lanes run along k so the transposed LDS stores of a wave are contiguous
#pragma unroll
        for (int it = 0; it < B_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            const int k = k0 + (i % BK);
            const int n = col0 + (i / BK) * 8;
            U16x8 v;
            v.v = make_uint4(0u, 0u, 0u, 0u);
            if (k < d_in) {
                const uint16_t* p = W + (int64_t)k * d_out + n;
                if (VEC && n + 7 < d_out) {
                    v.v = *reinterpret_cast<const uint4*>(p);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (n + j < d_out) v.e[j] = p[j];
                }
            }
            rb[it] = v;
        }
    };

    load_tile(0);
    for (int t = 0; t < n_tiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < A_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            *reinterpret_cast<uint4*>(&As[i / (BK / 8)][(i % (BK / 8)) * 8]) = ra[it].v;
        }
#pragma unroll
        for (int it = 0; it < B_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            const int k = i % BK, n = (i / BK) * 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) Bs[n + j][k] = rb[it].e[j];
        }
        __syncthreads();
        if (t + 1 < n_tiles) load_tile(t + 1);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            uint4 a[TM], b[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                a[tm] = *reinterpret_cast<const uint4*>(&As[wm * (BM / 2) + tm * 32 + (lane & 31)][kk + (lane >> 5) * 8]);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                b[tn] = *reinterpret_cast<const uint4*>(&Bs[wn * (BN / 2) + tn * 32 + (lane & 31)][kk + (lane >> 5) * 8]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = mfma16<Tr>(a[tm], b[tn], acc[tm][tn]);
        }
    }
    project_epilogue<Tr, BM, BN>(acc, row0, col0, wm, wn, lane, n_dst, d_out, bias, relu, out);
}

// ------------------------------------------------------------------ launch --

static int mean_group(int units) {   // lanes per destination row: power of two, 1..64
    int g = 1;
    while (g < units && g < 64) g *= 2;
    return g;
}

template <typename Tr>
static hopgnn_status launch_mean(const void* Hsrc, const int32_t* indptr, const int32_t* idx,
                                 int64_t n_dst, int32_t d_in, void* mean, hipStream_t s) {
    using T = typename Tr::store_t;
    const bool vec = (d_in % Tr::kPer16 == 0) && aligned(Hsrc, 16) && aligned(mean, 16);
    const int units = vec ? d_in / Tr::kPer16 : d_in;
    const int group = mean_group(units);
    const int64_t blocks = ceil_div(n_dst * group, kMeanThreads);
    if (vec)
        hipLaunchKernelGGL(sage_mean_vec<Tr>, dim3((unsigned)blocks), dim3(kMeanThreads), 0, s,
                           static_cast<const uint4*>(Hsrc), indptr, idx, n_dst, units, group,
                           static_cast<uint4*>(mean));
    else
        hipLaunchKernelGGL(sage_mean_elem<Tr>, dim3((unsigned)blocks), dim3(kMeanThreads), 0, s,
                           static_cast<const T*>(Hsrc), indptr, idx, n_dst, d_in, group,
                           static_cast<T*>(mean));
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

template <int BM, int BN>
static void launch_project_f32(bool vec, dim3 grid, hipStream_t s, const void* Hsrc,
                               const int32_t* self_idx, const void* mean, const void* Ws,
                               const void* Wn, const void* bias, int64_t n_dst, int32_t d_in,
                               int32_t d_out, int relu, void* out) {
    auto a = static_cast<const float*>(Hsrc);
    auto m = static_cast<const float*>(mean);
    auto ws = static_cast<const float*>(Ws);
    auto wn = static_cast<const float*>(Wn);
    auto b = static_cast<const float*>(bias);
    auto o = static_cast<float*>(out);
    if (vec)
        hipLaunchKernelGGL((sage_project_f32<BM, BN, true>), grid, dim3(kProjThreads), 0, s, a, self_idx,
                           m, ws, wn, b, n_dst, d_in, d_out, relu, o);
    else
        hipLaunchKernelGGL((sage_project_f32<BM, BN, false>), grid, dim3(kProjThreads), 0, s, a, self_idx,
                           m, ws, wn, b, n_dst, d_in, d_out, relu, o);
}

template <typename Tr, int BM, int BN>
static void launch_project_16(bool vec, dim3 grid, hipStream_t s, const void* Hsrc,
                              const int32_t* self_idx, const void* mean, const void* Ws,
                              const void* Wn, const void* bias, int64_t n_dst, int32_t d_in,
                              int32_t d_out, int relu, void* out) {
    using T = typename Tr::store_t;
    auto a = static_cast<const uint16_t*>(Hsrc);
    auto m = static_cast<const uint16_t*>(mean);
    auto ws = static_cast<const uint16_t*>(Ws);
    auto wn = static_cast<const uint16_t*>(Wn);
    auto b = static_cast<const T*>(bias);
    auto o = static_cast<T*>(out);
    if (vec)
        hipLaunchKernelGGL((sage_project_16<Tr, BM, BN, true>), grid, dim3(kProjThreads), 0, s, a,
                           self_idx, m, ws, wn, b, n_dst, d_in, d_out, relu, o);
    else
        hipLaunchKernelGGL((sage_project_16<Tr, BM, BN, false>), grid, dim3(kProjThreads), 0, s, a,
                           self_idx, m, ws, wn, b, n_dst, d_in, d_out, relu, o);
}

}  // namespace hopgnn

using namespace hopgnn;

extern "C" size_t hopgnn_sage_fwd_ws_bytes(hopgnn_dtype dt, int64_t n_dst, int32_t d_in, int32_t d_out) {
    (void)d_out;
    if (n_dst < 0 || d_in < 1) return 0;
    return align_up((size_t)n_dst * (size_t)d_in * dtype_size(dt), 256) + 256;
}

extern "C" hopgnn_status hopgnn_sage_fwd(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                         const int32_t* self_idx, const int32_t* indptr,
                                         const int32_t* idx, int64_t n_dst, const void* W_self,
                                         const void* W_neigh, const void* bias, int32_t d_out,
                                         int32_t relu, void* out, void* ws, size_t ws_bytes,
                                         void* stream) {
    if (dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) return HOPGNN_EINVAL;
    if (n_src < 0 || n_dst < 0 || d_in < 1 || d_out < 1) return HOPGNN_EINVAL;
    if (n_dst == 0) return HOPGNN_OK;
    if (indptr == nullptr || W_self == nullptr || W_neigh == nullptr || out == nullptr || ws == nullptr)
        return HOPGNN_EINVAL;
    if (n_src > 0 && Hsrc == nullptr) return HOPGNN_EINVAL;
    if (n_dst >= ((int64_t)1 << 31) || n_src >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if (!aligned(ws, 256)) return HOPGNN_EINVAL;
    if (ws_bytes < hopgnn_sage_fwd_ws_bytes(dt, n_dst, d_in, d_out)) return HOPGNN_ENOMEM_WS;
    hipStream_t s = static_cast<hipStream_t>(stream);

    hopgnn_status st;
    if (dt == HOPGNN_F32) st = launch_mean<TrF32>(Hsrc, indptr, idx, n_dst, d_in, ws, s);
    else if (dt == HOPGNN_BF16) st = launch_mean<TrBF16>(Hsrc, indptr, idx, n_dst, d_in, ws, s);
    else st = launch_mean<TrF16>(Hsrc, indptr, idx, n_dst, d_in, ws, s);
    if (st != HOPGNN_OK) return st;

    const int per16 = dt == HOPGNN_F32 ? 4 : 8;
    const bool vec = d_in % per16 == 0 && d_out % per16 == 0 && aligned(Hsrc, 16) &&
                     aligned(W_self, 16) && aligned(W_neigh, 16);
    // large tiles once there is enough work to fill 256 CUs twice over
    const bool big = d_out > 64 && ceil_div(n_dst, 128) * ceil_div(d_out, 128) >= 512;
    const int BM = big ? 128 : 64, BN = big ? 128 : 64;
    if (ceil_div(d_out, BN) > 65535) return HOPGNN_ERANGE;
    dim3 grid((unsigned)ceil_div(n_dst, BM), (unsigned)ceil_div(d_out, BN));
    if (dt == HOPGNN_F32) {
        if (big) launch_project_f32<128, 128>(vec, grid, s, Hsrc, self_idx, ws, W_self, W_neigh, bias, n_dst, d_in, d_out, relu, out);
        else launch_project_f32<64, 64>(vec, grid, s, Hsrc, self_idx, ws, W_self, W_neigh, bias, n_dst, d_in, d_out, relu, out);
    } else if (dt == HOPGNN_BF16) {
        if (big) launch_project_16<TrBF16, 128, 128>(vec, grid, s, Hsrc, self_idx, ws, W_self, W_neigh, bias, n_dst, d_in, d_out, relu, out);
        else launch_project_16<TrBF16, 64, 64>(vec, grid, s, Hsrc, self_idx, ws, W_self, W_neigh, bias, n_dst, d_in, d_out, relu, out);
    } else {
        if (big) launch_project_16<TrF16, 128, 128>(vec, grid, s, Hsrc, self_idx, ws, W_self, W_neigh, bias, n_dst, d_in, d_out, relu, out);
        else launch_project_16<TrF16, 64, 64>(vec, grid, s, Hsrc, self_idx, ws, W_self, W_neigh, bias, n_dst, d_in, d_out, relu, out);
    }
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}
