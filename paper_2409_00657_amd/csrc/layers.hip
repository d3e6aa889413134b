// The other two layer types of the paper's evaluation (section 7.1 trains GCN, GraphSAGE and
// GAT; section 2 describes a layer as an aggregation over the sampled neighbours followed by a
// neural transform), on the same slot-tree inputs as the GraphSAGE-mean layer:
//
//   GCN-style   out = act( agg W + b ),  agg = x_self + sum of the valid neighbour rows, divided by
//               the number of terms when norm = 1: (A+I) H W or D^-1 (A+I) H W on the sampled block
//   attention   z = Hsrc W once per SOURCE row (for the first layer these are the pre-gathered
//               unique rows, so no vertex is projected twice), kept in fp32 whatever the activation
//               type (a 2-byte z would be rounded a second time at the output, and where the
//               weighted rows cancel that exceeds the 2-byte tolerance); per destination row a softmax over
//               LeakyReLU_0.2(<z_self, a_dst> + <z_u, a_src>) for u in {self} + valid neighbours,
//               per head; out = act( sum alpha_u z_u + b )
//
// Both reuse the segmented-aggregation kernel and the MFMA projection of the GraphSAGE layer.
#include <type_traits>

#include "sage_common.hpp"

namespace hopgnn {

constexpr int kLayerThreads = 256;
constexpr int kMaxHeads = 16;

// Attention scores are linear in the source row: <Hsrc[u] W[:, head], a[head]> = Hsrc[u] (W[:, head] a[head]),
// so for fp32 they are 2 * n_heads extra output columns of a rows-times-matrix product with
// Wscore[k][h] = sum_j W[k][h*dh + j] a_src[h*dh + j] and Wscore[k][n_heads + h] likewise with a_dst.
struct ScoreWeightJob {
    const float* W;
    const float* a_src;
    const float* a_dst;
    float* Wscore;          // [d_in x 2*n_heads]; nullptr: no job
    int32_t d_in, d_out, n_heads;
    uint32_t n_blocks;
};

// Workgroup 0 zeroes the projection's zero row; the next n_blocks workgroups of the score-weight
// job compute one entry of Wscore per thread; the rest transpose one 32 x 32 weight tile each
// (2-byte types).
__global__ void __launch_bounds__(kLayerThreads)
layer_prep(uint32_t* __restrict__ zero_row, int32_t zero_words, TransposeJob job, ScoreWeightJob sw) {
    if (blockIdx.x == 0) {
        for (int32_t i = threadIdx.x; i < zero_words; i += kLayerThreads) zero_row[i] = 0u;
        return;
    }
    if (blockIdx.x - 1 < sw.n_blocks) {
        const int32_t cols = 2 * sw.n_heads, dh = sw.d_out / sw.n_heads;
        const int64_t i = (int64_t)(blockIdx.x - 1) * kLayerThreads + threadIdx.x;
        if (i >= (int64_t)sw.d_in * cols) return;
        const int32_t k = (int32_t)(i / cols), c = (int32_t)(i % cols);
        const int32_t h = c < sw.n_heads ? c : c - sw.n_heads;
        const float* a = (c < sw.n_heads ? sw.a_src : sw.a_dst) + h * dh;
        const float* w = sw.W + (int64_t)k * sw.d_out + h * dh;
        float acc = 0.f;
        for (int32_t j = 0; j < dh; ++j) acc += w[j] * a[j];
        sw.Wscore[i] = acc;
        return;
    }
    transpose_w_tile(job, blockIdx.x - 1 - sw.n_blocks);
}

// s_src[u][h] = <z_u[h], a_src[h]>, s_dst[u][h] = <z_u[h], a_dst[h]>.
//
// Vector form (d_head / 4 a power of two <= 64): a lane takes one 16-byte word of z, the lanes of
// a head form an aligned power-of-two segment and reduce with xor shuffles.  `lanes_row` lanes
// (a power of two) share a row, so narrow rows are packed several to a wavefront and wide rows
// are walked in strides of 64 words.
template <typename Tr>
__global__ void __launch_bounds__(kLayerThreads)
gat_scores_vec(const float4* __restrict__ Z, const typename Tr::store_t* __restrict__ a_src,
               const typename Tr::store_t* __restrict__ a_dst, int64_t n_src, const int64_t* __restrict__ n_src_dev,
               int32_t d_out, int32_t n_heads, int32_t lanes_row, int32_t seg, float* __restrict__ s_src,
               float* __restrict__ s_dst, int32_t score_stride) {
    if (n_src_dev != nullptr) {
        const int64_t live = *n_src_dev;
        n_src = live < n_src ? live : n_src;
    }
    const int lane = threadIdx.x & 63;
    const int rows_per_wave = 64 / lanes_row;
    const int64_t wave = (int64_t)blockIdx.x * (kLayerThreads / 64) + (threadIdx.x >> 6);
    const int64_t u = wave * rows_per_wave + lane / lanes_row;
    const int32_t lw = lane % lanes_row, wpr = d_out / 4;
    const bool live_row = u < n_src;
    for (int32_t w0 = 0; w0 < wpr; w0 += lanes_row) {      // the same trip count for every lane of the wave
        const int32_t w = w0 + lw;
        const bool ok = live_row && w < wpr;
        float ps = 0.f, pd = 0.f;
        if (ok) {
            const float4 z = Z[u * wpr + w];
            const typename Tr::store_t* as = a_src + 4 * w;
            const typename Tr::store_t* ad = a_dst + 4 * w;
            ps = z.x * Tr::to_f(as[0]) + z.y * Tr::to_f(as[1]) + z.z * Tr::to_f(as[2]) + z.w * Tr::to_f(as[3]);
            pd = z.x * Tr::to_f(ad[0]) + z.y * Tr::to_f(ad[1]) + z.z * Tr::to_f(ad[2]) + z.w * Tr::to_f(ad[3]);
        }
        for (int o = seg >> 1; o > 0; o >>= 1) {
            ps += __shfl_xor(ps, o, kWave);
            pd += __shfl_xor(pd, o, kWave);
        }
        if (ok && (w & (seg - 1)) == 0) {
            s_src[u * score_stride + w / seg] = ps;
            s_dst[u * score_stride + w / seg] = pd;
        }
    }
}

// General form: one wavefront per source row, one head after the other.
template <typename Tr>
__global__ void __launch_bounds__(kLayerThreads)
gat_scores(const float* __restrict__ Z, const typename Tr::store_t* __restrict__ a_src,
           const typename Tr::store_t* __restrict__ a_dst, int64_t n_src, const int64_t* __restrict__ n_src_dev,
           int32_t d_out, int32_t n_heads, float* __restrict__ s_src, float* __restrict__ s_dst,
           int32_t score_stride) {
    if (n_src_dev != nullptr) {
        const int64_t live = *n_src_dev;
        n_src = live < n_src ? live : n_src;
    }
    const int lane = threadIdx.x & 63;
    const int64_t u = (int64_t)blockIdx.x * (kLayerThreads / 64) + (threadIdx.x >> 6);
    if (u >= n_src) return;
    const int32_t dh = d_out / n_heads;
    for (int32_t h = 0; h < n_heads; ++h) {
        float ps = 0.f, pd = 0.f;
        for (int32_t j = lane; j < dh; j += 64) {
            const float z = Z[u * d_out + h * dh + j];
            ps += z * Tr::to_f(a_src[h * dh + j]);
            pd += z * Tr::to_f(a_dst[h * dh + j]);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            ps += __shfl_xor(ps, o, kWave);
            pd += __shfl_xor(pd, o, kWave);
        }
        if (lane == 0) {
            s_src[u * score_stride + h] = ps;
            s_dst[u * score_stride + h] = pd;
        }
    }
}

__device__ __forceinline__ float leaky(float x) { return x > 0.f ? x : 0.2f * x; }

// Softmax-weighted sum of z rows per destination row.  `group` lanes share a row; a lane owns
// units c, c+group, ... of it, a unit being W consecutive elements that lie in one head (four
// on the vector path - a 16-byte word of z - one otherwise).  Segments are short (a fanout), so
// each lane walks its row's entries twice: once for the largest score, once to accumulate
// exp(score - max) and the weighted rows.
template <typename Tr, int W>
__global__ void __launch_bounds__(kLayerThreads)
gat_aggregate(const float* __restrict__ Z, const float* __restrict__ s_src,
              const float* __restrict__ s_dst, const int32_t* __restrict__ self_idx,
              const int32_t* __restrict__ indptr, const int32_t* __restrict__ idx,
              const typename Tr::store_t* __restrict__ bias, int64_t n_dst, int32_t d_out, int32_t n_heads,
              int32_t score_stride, int32_t group, int relu, typename Tr::store_t* __restrict__ out,
              const int64_t* __restrict__ n_rows_dev) {
    using T = typename Tr::store_t;
    static_assert(W == 1 || W == 4, "one element or one 16-byte word of z per unit");
    const int64_t gid = (int64_t)blockIdx.x * kLayerThreads + threadIdx.x;
    const int64_t r = gid / group;
    const int32_t g = (int32_t)(gid - r * group);
    if (r >= n_dst || (n_rows_dev != nullptr && r >= *n_rows_dev)) return;
    const int32_t dh = d_out / n_heads, units = d_out / W;
    const int64_t s = self_idx != nullptr ? (int64_t)self_idx[r] : r;
    const int32_t beg = indptr[r], end = indptr[r + 1];
    for (int32_t c = g; c < units; c += group) {
        const int32_t h = (c * W) / dh;
        const float sd = s >= 0 ? s_dst[s * score_stride + h] : 0.f;
        constexpr int U = 4;     // entries in flight
        float mx = -INFINITY;
        if (s >= 0) mx = leaky(sd + s_src[s * score_stride + h]);
        for (int32_t e = beg; e < end; e += U) {
            int32_t u[U];
            float sc[U];
#pragma unroll
            for (int k = 0; k < U; ++k) u[k] = e + k < end ? idx[e + k] : -1;
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (u[k] >= 0) sc[k] = s_src[(int64_t)u[k] * score_stride + h];
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (u[k] >= 0) mx = fmaxf(mx, leaky(sd + sc[k]));
        }
        float acc[W];
#pragma unroll
        for (int i = 0; i < W; ++i) acc[i] = 0.f;
        float den = 0.f;
        auto fetch = [&](int64_t u, float4& v) {
            if (W == 1) v.x = Z[u * d_out + c];
            else v = *reinterpret_cast<const float4*>(Z + u * d_out + (int64_t)c * W);
        };
        auto add = [&](float score, const float4& v) {
            const float w = expf(leaky(sd + score) - mx);
            den += w;
            acc[0] += w * v.x;
            if (W > 1) {
                acc[1] += w * v.y;
                acc[2] += w * v.z;
                acc[3] += w * v.w;
            }
        };
        if (s >= 0) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            fetch(s, v);
            add(s_src[s * score_stride + h], v);
        }
        for (int32_t e = beg; e < end; e += U) {     // U rows in flight, accumulated in entry order
            int32_t u[U];
            float sc[U];
            float4 v[U];
#pragma unroll
            for (int k = 0; k < U; ++k) u[k] = e + k < end ? idx[e + k] : -1;
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (u[k] >= 0) {
                    sc[k] = s_src[(int64_t)u[k] * score_stride + h];
                    v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
                    fetch(u[k], v[k]);
                }
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (u[k] >= 0) add(sc[k], v[k]);
        }
        const float inv = den > 0.f ? 1.f / den : 0.f;
        T o[W];
#pragma unroll
        for (int i = 0; i < W; ++i) {
            float v = acc[i] * inv + (bias != nullptr ? Tr::to_f(bias[c * W + i]) : 0.f);
            if (relu) v = fmaxf(v, 0.f);
            o[i] = Tr::from_f(v);
        }
        if (W == 1) {
            out[r * d_out + c] = o[0];
        } else {     // four elements: 16 bytes of fp32, 8 bytes of a 2-byte type
            typename std::conditional<sizeof(T) == 4, uint4, uint2>::type p;
            __builtin_memcpy(&p, o, sizeof(p));
            *reinterpret_cast<decltype(p)*>(out + r * d_out + (int64_t)c * W) = p;
        }
    }
}

// -------------------------------------------------------------------- host --

static hopgnn_status launch_prep(hopgnn_dtype dt, const void* W, uint16_t* Wt, const ProjWs& P, int32_t d_in,
                                 int32_t d_out, void* zero, ScoreWeightJob sw, hipStream_t s) {
    TransposeJob job{};
    uint32_t n_tr = 0;
    if (dt != HOPGNN_F32) {
        job = TransposeJob{static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(W), Wt, d_in, d_out, P.KP,
                           P.NP, 0u, d_in};
        n_tr = (uint32_t)(P.KP / 32) * (uint32_t)(P.NP / 32);
    }
    sw.n_blocks = sw.Wscore != nullptr ? (uint32_t)ceil_div((int64_t)sw.d_in * 2 * sw.n_heads, kLayerThreads) : 0u;
    hipLaunchKernelGGL(layer_prep, dim3(1 + sw.n_blocks + n_tr), dim3(kLayerThreads), 0, s, static_cast<uint32_t*>(zero),
                       (int32_t)(P.zero_bytes / 4), job, sw);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

template <typename Tr>
static hopgnn_status gat_tail(const void* Z, const void* a_src, const void* a_dst, float* s_src, float* s_dst,
                              int64_t n_src, const int64_t* n_src_dev, const int32_t* self_idx, const int32_t* indptr,
                              const int32_t* idx, const void* bias, int64_t n_dst, int32_t d_out, int32_t n_heads,
                              int relu, void* out, bool scores_done, const int64_t* n_dst_dev, hipStream_t s) {
    using T = typename Tr::store_t;
    const int32_t dh = d_out / n_heads, stride = 2 * n_heads;
    if (n_src > 0 && !scores_done) {
        const int32_t seg = dh / 4;
        if (dh % 4 == 0 && seg <= 64 && (seg & (seg - 1)) == 0) {
            int32_t lanes_row = 1;
            while (lanes_row < d_out / 4 && lanes_row < 64) lanes_row *= 2;
            const int64_t waves = ceil_div(n_src, 64 / lanes_row);
            hipLaunchKernelGGL(gat_scores_vec<Tr>, dim3((unsigned)ceil_div(waves, kLayerThreads / 64)),
                               dim3(kLayerThreads), 0, s, static_cast<const float4*>(Z), static_cast<const T*>(a_src),
                               static_cast<const T*>(a_dst), n_src, n_src_dev, d_out, n_heads, lanes_row, seg, s_src,
                               s_dst, stride);
        } else {
            hipLaunchKernelGGL(gat_scores<Tr>, dim3((unsigned)ceil_div(n_src, kLayerThreads / 64)), dim3(kLayerThreads),
                               0, s, static_cast<const float*>(Z), static_cast<const T*>(a_src),
                               static_cast<const T*>(a_dst), n_src, n_src_dev, d_out, n_heads, s_src, s_dst, stride);
        }
        HOPGNN_LAUNCH_CHECK();
    }
    const bool vec = dh % 4 == 0 && aligned(out, 16);
    const int units = vec ? d_out / 4 : d_out;
    const int group = mean_group(units);
    const int64_t blocks = ceil_div(n_dst * group, kLayerThreads);
    if (blocks >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if (vec)
        hipLaunchKernelGGL((gat_aggregate<Tr, 4>), dim3((unsigned)blocks), dim3(kLayerThreads), 0, s,
                           static_cast<const float*>(Z), s_src, s_dst, self_idx, indptr, idx, static_cast<const T*>(bias),
                           n_dst, d_out, n_heads, stride, group, relu, static_cast<T*>(out), n_dst_dev);
    else
        hipLaunchKernelGGL((gat_aggregate<Tr, 1>), dim3((unsigned)blocks), dim3(kLayerThreads), 0, s,
                           static_cast<const float*>(Z), s_src, s_dst, self_idx, indptr, idx, static_cast<const T*>(bias),
                           n_dst, d_out, n_heads, stride, group, relu, static_cast<T*>(out), n_dst_dev);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

static hopgnn_status check_common(hopgnn_dtype dt, int64_t n_src, int32_t d_in, int64_t n_dst, int32_t d_out) {
    if (dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) return HOPGNN_EINVAL;
    if (n_src < 0 || n_dst < 0 || d_in < 1 || d_out < 1) return HOPGNN_EINVAL;
    if (n_dst >= ((int64_t)1 << 31) || n_src >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if (d_in > (1 << 20) || d_out > (1 << 20)) return HOPGNN_ERANGE;
    return HOPGNN_OK;
}

}  // namespace hopgnn

using namespace hopgnn;

extern "C" size_t hopgnn_gcn_fwd_ws_bytes(hopgnn_dtype dt, int64_t n_dst, int32_t d_in, int32_t d_out) {
    if (check_common(dt, 0, d_in, n_dst, d_out) != HOPGNN_OK) return 0;
    return proj_ws_layout(dt, n_dst, d_in, d_in, d_out).total;
}

extern "C" hopgnn_status hopgnn_gcn_fwd(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                        const int32_t* self_idx, const int32_t* indptr, const int32_t* idx,
                                        int64_t n_dst, const void* W, const void* bias, int32_t d_out, int32_t norm,
                                        int32_t relu, void* out, void* ws, size_t ws_bytes, void* stream) {
    return hopgnn_gcn_fwd_dev(Hsrc, dt, n_src, d_in, self_idx, indptr, idx, n_dst, nullptr, W, bias, d_out, norm, relu, out,
                              ws, ws_bytes, stream);
}

extern "C" hopgnn_status hopgnn_gcn_fwd_dev(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                            const int32_t* self_idx, const int32_t* indptr, const int32_t* idx,
                                            int64_t n_dst, const int64_t* n_dst_dev, const void* W, const void* bias,
                                            int32_t d_out, int32_t norm, int32_t relu, void* out, void* ws,
                                            size_t ws_bytes, void* stream) {
    const hopgnn_status chk = check_common(dt, n_src, d_in, n_dst, d_out);
    if (chk != HOPGNN_OK) return chk;
    if (norm != 0 && norm != 1) return HOPGNN_EINVAL;
    if (n_dst == 0) return HOPGNN_OK;
    if (indptr == nullptr || W == nullptr || out == nullptr || ws == nullptr) return HOPGNN_EINVAL;
    if (n_src > 0 && Hsrc == nullptr) return HOPGNN_EINVAL;
    if (self_idx == nullptr && n_src < n_dst) return HOPGNN_EINVAL;   // identity self rows must exist
    if (!aligned(ws, 256)) return HOPGNN_EINVAL;
    const ProjWs L = proj_ws_layout(dt, n_dst, d_in, d_in, d_out);
    if (ws_bytes < L.total) return HOPGNN_ENOMEM_WS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    void* agg = ws;
    uint16_t* Wt = reinterpret_cast<uint16_t*>(static_cast<char*>(ws) + L.agg_bytes);
    void* zero = static_cast<char*>(ws) + L.agg_bytes + L.wt_bytes;
    if (n_src == 0) Hsrc = zero;   // nothing is read from it unmasked

    TransposeJob job{};
    uint32_t n_tr = 0;
    if (dt != HOPGNN_F32) {
        job = TransposeJob{static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(W), Wt, d_in, d_out, L.KP, L.NP,
                           0u, d_in};
        n_tr = (uint32_t)(L.KP / 32) * (uint32_t)(L.NP / 32);
    }
    // with n_src == 0 every self index must be negative; identity self was rejected above
    const AggSpec spec{self_idx, 1, norm ? kAggOpMean : kAggOpSum};
    hopgnn_status st;
    if (dt == HOPGNN_F32)
        st = launch_mean<TrF32>(Hsrc, indptr, idx, n_dst, d_in, agg, zero, L.zero_bytes, job, n_tr, s, spec, n_dst_dev);
    else if (dt == HOPGNN_BF16)
        st = launch_mean<TrBF16>(Hsrc, indptr, idx, n_dst, d_in, agg, zero, L.zero_bytes, job, n_tr, s, spec, n_dst_dev);
    else
        st = launch_mean<TrF16>(Hsrc, indptr, idx, n_dst, d_in, agg, zero, L.zero_bytes, job, n_tr, s, spec, n_dst_dev);
    if (st != HOPGNN_OK) return st;
    // rows-times-W over the aggregate (identity row map, K = d_in)
    return project_dispatch(dt, s, agg, nullptr, agg, W, W, Wt, L.KP, bias, n_dst, d_in, d_in, d_out, relu, zero, out, 0,
                            n_dst_dev);
}

extern "C" size_t hopgnn_gat_fwd_ws_bytes(hopgnn_dtype dt, int64_t n_src, int32_t d_in, int32_t d_out,
                                          int32_t n_heads) {
    if (check_common(dt, n_src, d_in, 0, d_out) != HOPGNN_OK) return 0;
    if (n_heads < 1 || n_heads > kMaxHeads || d_out % n_heads != 0) return 0;
    return gat_ws_layout(dt, n_src, d_in, d_out, n_heads).total;
}

extern "C" hopgnn_status hopgnn_gat_fwd(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t* n_src_dev,
                                        int32_t d_in, const int32_t* self_idx, const int32_t* indptr, const int32_t* idx,
                                        int64_t n_dst, const void* W, const void* a_src, const void* a_dst,
                                        const void* bias, int32_t d_out, int32_t n_heads, int32_t relu, void* out,
                                        void* ws, size_t ws_bytes, void* stream) {
    return hopgnn_gat_fwd_dev(Hsrc, dt, n_src, n_src_dev, d_in, self_idx, indptr, idx, n_dst, nullptr, W, a_src, a_dst, bias,
                              d_out, n_heads, relu, out, ws, ws_bytes, stream);
}

extern "C" hopgnn_status hopgnn_gat_fwd_dev(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t* n_src_dev,
                                            int32_t d_in, const int32_t* self_idx, const int32_t* indptr,
                                            const int32_t* idx, int64_t n_dst, const int64_t* n_dst_dev, const void* W,
                                            const void* a_src, const void* a_dst, const void* bias, int32_t d_out,
                                            int32_t n_heads, int32_t relu, void* out, void* ws, size_t ws_bytes,
                                            void* stream) {
    const hopgnn_status chk = check_common(dt, n_src, d_in, n_dst, d_out);
    if (chk != HOPGNN_OK) return chk;
    if (n_heads < 1 || n_heads > kMaxHeads || d_out % n_heads != 0) return HOPGNN_EINVAL;
    if (n_dst == 0) return HOPGNN_OK;
    if (indptr == nullptr || W == nullptr || a_src == nullptr || a_dst == nullptr || out == nullptr || ws == nullptr)
        return HOPGNN_EINVAL;
    if (n_src > 0 && Hsrc == nullptr) return HOPGNN_EINVAL;
    if (self_idx == nullptr && n_src < n_dst) return HOPGNN_EINVAL;   // identity self rows must exist
    if (!aligned(ws, 256)) return HOPGNN_EINVAL;
    const GatWs L = gat_ws_layout(dt, n_src, d_in, d_out, n_heads);
    if (ws_bytes < L.total) return HOPGNN_ENOMEM_WS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* p = static_cast<char*>(ws);
    void* Z = p;
    float* s_src = reinterpret_cast<float*>(p + L.z_bytes);
    float* s_dst = s_src + n_heads;
    float* Wscore = reinterpret_cast<float*>(p + L.z_bytes + L.score_bytes);
    uint16_t* Wt = reinterpret_cast<uint16_t*>(p + L.z_bytes + L.score_bytes + L.wscore_bytes);
    void* zero = p + L.z_bytes + L.score_bytes + L.wscore_bytes + L.P.wt_bytes;

    // fp32 with many source rows: the scores come from a second, skinny rows-times-matrix product (it
    // reads the source rows once more instead of the wider z: 74 against 165 us on 0.47 M rows of
    // 100 -> 256); otherwise from z, which is kept in fp32 (a few microseconds on small inputs,
    // where the extra product's latency costs more)
    const bool score_gemm = dt == HOPGNN_F32 && n_src >= 131072;
    if (n_src > 0) {
        ScoreWeightJob sw{};
        if (score_gemm)
            sw = ScoreWeightJob{static_cast<const float*>(W), static_cast<const float*>(a_src),
                                static_cast<const float*>(a_dst), Wscore, d_in, d_out, n_heads, 0u};
        hopgnn_status st = launch_prep(dt, W, Wt, L.P, d_in, d_out, zero, sw, s);
        if (st != HOPGNN_OK) return st;
        if (score_gemm) {
            st = project_dispatch(dt, s, Hsrc, nullptr, Hsrc, Wscore, Wscore, nullptr, 0, nullptr, n_src, d_in, d_in,
                                  2 * n_heads, 0, zero, s_src, 0, n_src_dev);
            if (st != HOPGNN_OK) return st;
        }
        // z = Hsrc W for every source row: identity row map, K = d_in, no bias, no activation
        st = project_dispatch(dt, s, Hsrc, nullptr, Hsrc, W, W, Wt, L.P.KP, nullptr, n_src, d_in, d_in, d_out, 0, zero, Z, 1,
                              n_src_dev);
        if (st != HOPGNN_OK) return st;
    }
    if (dt == HOPGNN_F32)
        return gat_tail<TrF32>(Z, a_src, a_dst, s_src, s_dst, n_src, n_src_dev, self_idx, indptr, idx, bias, n_dst, d_out, n_heads,
                               relu, out, score_gemm, n_dst_dev, s);
    if (dt == HOPGNN_BF16)
        return gat_tail<TrBF16>(Z, a_src, a_dst, s_src, s_dst, n_src, n_src_dev, self_idx, indptr, idx, bias, n_dst, d_out, n_heads,
                                relu, out, false, n_dst_dev, s);
    return gat_tail<TrF16>(Z, a_src, a_dst, s_src, s_dst, n_src, n_src_dev, self_idx, indptr, idx, bias, n_dst, d_out, n_heads, relu,
                           out, false, n_dst_dev, s);
}
