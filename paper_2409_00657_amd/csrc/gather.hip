// hopgnn_gather: Xu[i, :] = X[uniq[i], :], byte for byte (paper section 2
// "gathering"; section 3.1: the step that dominates training time).
//
// Pure HBM traffic: U random row reads + one dense write.  Rows are moved as
// 128-bit words, ONE word per thread: consecutive lanes take consecutive words of a
// row, so a 512-byte row is one fully coalesced request of 32 lanes.  Memory-level
// parallelism comes from occupancy (a grid of U * words-per-row threads), not from
// unrolling: a 4-deep unrolled variant measured 4-5x slower on 18 MB gathers and
// 20 % slower on 1 GB ones, a one-word-per-thread grid reaches the rate of a plain copy.
#include "common.hpp"

namespace hopgnn {

constexpr int kGatherThreads = 256;

// VecT words per row = `vpr`; source rows `ld_vec` words apart; thread t = (row t / vpr, word t % vpr).
// IdxT is uint32_t whenever U * vpr fits 32 bits (a 32-bit division per thread).
template <typename VecT, typename IdxT>
__global__ void __launch_bounds__(kGatherThreads)
gather_rows(const VecT* __restrict__ X, const int32_t* __restrict__ uniq, int64_t n_rows_host,
            const int64_t* __restrict__ n_rows_dev, uint32_t vpr, int64_t ld_vec,
            VecT* __restrict__ Xu) {
    int64_t n_rows = n_rows_host;
    if (n_rows_dev != nullptr) {   // U lives on the device: the grid was sized for the capacity
        const int64_t d = *n_rows_dev;
        n_rows = d < n_rows ? d : n_rows;
    }
    const IdxT n_items = (IdxT)n_rows * vpr;
    const IdxT stride = (IdxT)gridDim.x * kGatherThreads;
    for (IdxT t = (IdxT)blockIdx.x * kGatherThreads + threadIdx.x; t < n_items; t += stride) {
        const IdxT i = t / (IdxT)vpr;
        const uint32_t c = (uint32_t)(t - i * (IdxT)vpr);
        Xu[t] = X[(int64_t)uniq[i] * ld_vec + c];
    }
}

template <typename VecT>
static hopgnn_status launch_gather(const void* X, const int32_t* uniq, int64_t n_uniq,
                                   const int64_t* n_uniq_dev, int64_t row_bytes, int64_t ld_bytes,
                                   void* Xu, hipStream_t s) {
    const uint32_t vpr = (uint32_t)(row_bytes / sizeof(VecT));
    const int64_t items = n_uniq * vpr;
    // With U known on the host the grid covers it exactly (one word per thread).  With U
    // on the device only a capacity is known, so a resident-sized grid strides over the
    // real count instead of launching capacity-many workgroups that mostly exit at once.
    int64_t grid = ceil_div(items, kGatherThreads);
    const int64_t resident = 256 * 8;   // 256 CUs x 8 workgroups of 4 waves: all that can be resident
    if (n_uniq_dev != nullptr && grid > resident) grid = resident;
    if (grid >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    const int64_t ld_vec = ld_bytes / (int64_t)sizeof(VecT);
    // 32-bit item indices only where the loop's last step cannot wrap around: index + stride < 2^32
    if (items + grid * kGatherThreads < ((int64_t)1 << 32))
        hipLaunchKernelGGL((gather_rows<VecT, uint32_t>), dim3((unsigned)grid), dim3(kGatherThreads), 0, s,
                           static_cast<const VecT*>(X), uniq, n_uniq, n_uniq_dev, vpr, ld_vec,
                           static_cast<VecT*>(Xu));
    else
        hipLaunchKernelGGL((gather_rows<VecT, uint64_t>), dim3((unsigned)grid), dim3(kGatherThreads), 0, s,
                           static_cast<const VecT*>(X), uniq, n_uniq, n_uniq_dev, vpr, ld_vec,
                           static_cast<VecT*>(Xu));
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
