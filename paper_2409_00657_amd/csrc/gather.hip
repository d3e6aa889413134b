// hopgnn_gather: Xu[i, :] = X[uniq[i], :], byte for byte (paper section 2
// "gathering"; section 3.1: the step that dominates training time).
//
// Pure HBM traffic: U random row reads + one dense write.  Rows are moved as
// 128-bit words; consecutive lanes take consecutive words of a row, so a 512-byte
// row is one fully coalesced request of 32 lanes, and every lane keeps several
// independent loads in flight before the first store.
#include "common.hpp"

namespace hopgnn {

constexpr int kGatherThreads = 256;
constexpr int kGatherUnroll = 4;

// VecT words per row = `vpr`; source rows `ld_vec` words apart; flat item t = (row i, word c).
template <typename VecT>
__global__ void __launch_bounds__(kGatherThreads)
gather_rows(const VecT* __restrict__ X, const int32_t* __restrict__ uniq, int64_t n_rows_host,
            const int64_t* __restrict__ n_rows_dev, uint32_t vpr, int64_t ld_vec,
            VecT* __restrict__ Xu) {
    const int64_t n_rows = n_rows_dev != nullptr ? min(*n_rows_dev, n_rows_host) : n_rows_host;
    const int64_t n_items = n_rows * vpr;
    const int64_t tile = (int64_t)kGatherThreads * kGatherUnroll;
    for (int64_t t0 = (int64_t)blockIdx.x * tile; t0 < n_items; t0 += (int64_t)gridDim.x * tile) {
        // one 64-bit division per tile (uniform), 32-bit arithmetic per item
        const int64_t row0 = t0 / vpr;
        const uint32_t c0 = (uint32_t)(t0 - row0 * vpr);
        VecT val[kGatherUnroll];
        int64_t dst[kGatherUnroll];
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u) {
            const uint32_t l = c0 + u * kGatherThreads + threadIdx.x;
            const int64_t t = t0 + u * kGatherThreads + threadIdx.x;
            dst[u] = t < n_items ? t : -1;
            if (t < n_items) {
                const uint32_t di = l / vpr;
                const uint32_t c = l - di * vpr;
                val[u] = X[(int64_t)uniq[row0 + di] * ld_vec + c];
            }
        }
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u)
            if (dst[u] >= 0) Xu[dst[u]] = val[u];
    }
}

template <typename VecT>
static hopgnn_status launch_gather(const void* X, const int32_t* uniq, int64_t n_uniq,
                                   const int64_t* n_uniq_dev, int64_t row_bytes, int64_t ld_bytes,
                                   void* Xu, hipStream_t s) {
    const uint32_t vpr = (uint32_t)(row_bytes / sizeof(VecT));
    const int64_t items = n_uniq * vpr;
    const int64_t tile = (int64_t)kGatherThreads * kGatherUnroll;
    int64_t grid = ceil_div(items, tile);
    const int64_t cap = 256 * 64;      // 64 workgroups per CU's worth of tiles, then grid-stride
    if (grid > cap) grid = cap;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(gather_rows<VecT>, dim3((unsigned)grid), dim3(kGatherThreads), 0, s,
                       static_cast<const VecT*>(X), uniq, n_uniq, n_uniq_dev, vpr,
                       ld_bytes / (int64_t)sizeof(VecT), static_cast<VecT*>(Xu));
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

}  // namespace hopgnn

using namespace hopgnn;

extern "C" hopgnn_status hopgnn_gather(const void* X, hopgnn_dtype dt, int64_t n_rows, int32_t dim,
                                       int64_t ld_elems, const int32_t* uniq, int64_t n_uniq,
                                       const int64_t* n_uniq_dev, void* Xu, void* stream) {
    if (dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) return HOPGNN_EINVAL;
    if (n_rows < 0 || dim < 1 || ld_elems < dim || n_uniq < 0) return HOPGNN_EINVAL;
    if (n_uniq == 0) return HOPGNN_OK;
    if (X == nullptr || uniq == nullptr || Xu == nullptr) return HOPGNN_EINVAL;
    if (n_uniq >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    const int64_t es = (int64_t)dtype_size(dt);
    const int64_t row_bytes = dim * es, ld_bytes = ld_elems * es;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (row_bytes % 16 == 0 && ld_bytes % 16 == 0 && aligned(X, 16) && aligned(Xu, 16))
        return launch_gather<uint4>(X, uniq, n_uniq, n_uniq_dev, row_bytes, ld_bytes, Xu, s);
    if (row_bytes % 4 == 0 && ld_bytes % 4 == 0 && aligned(X, 4) && aligned(Xu, 4))
        return launch_gather<uint32_t>(X, uniq, n_uniq, n_uniq_dev, row_bytes, ld_bytes, Xu, s);
    return launch_gather<uint8_t>(X, uniq, n_uniq, n_uniq_dev, row_bytes, ld_bytes, Xu, s);
}
