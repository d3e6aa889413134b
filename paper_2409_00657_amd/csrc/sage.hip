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
#include "sage_common.hpp"

namespace hopgnn {

// -------------------------------------------------------------- projection --
//
// out = act( [x_self | mean] (M x 2*d_in) * [W_self ; W_neigh] (2*d_in x d_out) + b )
//
// 256 threads = 4 waves in a 2 x 2 arrangement; each wave owns a (BM/2) x (BN/2)
// piece of the output as 32 x 32 MFMA tiles.  K runs over the concatenation of the
// self half (read from Hsrc through self_idx) and the mean half; the last K tile is
// zero padded.  Tiles are staged global -> registers -> LDS with two register sets
// and two LDS stages, so the loads of tiles t+2 and t+3 are in flight while tile t is
// multiplied; the per-tile barrier waits for LDS traffic only.
//
// Accumulator layout of a 32x32 MFMA tile: register i of lane l holds
//   row = 8*(i/4) + 4*(l/32) + i%4,  col = l%32.

constexpr int kProjThreads = 256;
constexpr int kXcds = 8;
// Scheduling barrier mask of the projection loops: vector/scalar ALU work and global memory
// operations may be moved across, MFMAs and LDS operations may not.
constexpr int kSchedPin = 0x2 | 0x4 | 0x10;

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Keep all N
// tiles of one M tile on one XCD so the left operand is fetched into one L2 only.
__device__ __forceinline__ void tile_of_block(uint32_t bid, uint32_t n_tiles, uint32_t& mt, uint32_t& nt) {
    const uint32_t xcd = bid % kXcds, j = bid / kXcds;
    nt = j % n_tiles;
    mt = (j / n_tiles) * kXcds + xcd;
}

// Writes one wave's TM x TN block of 32x32 tiles whose top-left element is (row0, col0).
template <typename Tr, int TM, int TN>
__device__ __forceinline__ void project_epilogue(floatx16 (&acc)[TM][TN], int64_t row0, int32_t col0,
                                                 int lane, int64_t n_dst, int32_t d_out,
                                                 const typename Tr::store_t* bias, int relu,
                                                 typename Tr::store_t* out) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int32_t col = col0 + tn * 32 + (lane & 31);
        if (col >= d_out) continue;
        const float b = bias != nullptr ? Tr::to_f(bias[col]) : 0.f;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t row = row0 + tm * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
                if (row < n_dst) {
                    float x = acc[tm][tn][i] + b;
                    if (relu) x = fmaxf(x, 0.f);
                    out[row * d_out + col] = Tr::from_f(x);
                }
            }
        }
    }
}

// fp32 output from a kernel whose inputs are 2-byte (the attention layer keeps its projected
// rows unrounded): 32 consecutive floats of a row per half wave.
template <typename Tr, int TM, int TN>
__device__ __forceinline__ void project_epilogue_f32out(floatx16 (&acc)[TM][TN], int64_t row0, int32_t col0,
                                                        int lane, int64_t n_dst, int32_t d_out,
                                                        const typename Tr::store_t* bias, int relu, float* out) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int32_t col = col0 + tn * 32 + (lane & 31);
        if (col >= d_out) continue;
        const float b = bias != nullptr ? Tr::to_f(bias[col]) : 0.f;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t row = row0 + tm * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
                if (row < n_dst) {
                    float x = acc[tm][tn][i] + b;
                    if (relu) x = fmaxf(x, 0.f);
                    out[row * d_out + col] = x;
                }
            }
        }
    }
}

// 2-byte outputs: a lane of an MFMA tile holds single elements of 16 different rows, so
// storing them directly issues 2-byte writes (64-byte pieces of two rows per instruction).
// Instead each wave passes one 32-row band of its tiles through a private piece of LDS
// ([32][32*TN + 8] elements) and writes it out as 128-bit words, whole rows at a time.
// Requires d_out % 8 == 0.  `band` points at this wave's LDS piece; waves do not share it,
// so only this wave's own LDS traffic has to be waited for.
template <typename Tr, int TM, int TN>
__device__ __forceinline__ void project_epilogue_staged(floatx16 (&acc)[TM][TN], int64_t row0, int32_t col0,
                                                        int lane, int64_t n_dst, int32_t d_out,
                                                        const typename Tr::store_t* bias, int relu,
                                                        typename Tr::store_t* out,
                                                        typename Tr::store_t* band) {
    using T = typename Tr::store_t;
    constexpr int W = 32 * TN, LDW = W + 8;          // band width in elements, padded row
    constexpr int WORDS = W / 8;                     // 16-byte words per band row
    float b[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int32_t col = col0 + tn * 32 + (lane & 31);
        b[tn] = (bias != nullptr && col < d_out) ? Tr::to_f(bias[col]) : 0.f;
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float x = acc[tm][tn][i] + b[tn];
                if (relu) x = fmaxf(x, 0.f);
                band[(8 * (i / 4) + 4 * (lane >> 5) + (i & 3)) * LDW + tn * 32 + (lane & 31)] = Tr::from_f(x);
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < 32 * WORDS / 64; ++j) {
            const int w = j * 64 + lane;
            const int r = w / WORDS, c = (w % WORDS) * 8;
            const int64_t row = row0 + tm * 32 + r;
            const uint4 v = *reinterpret_cast<const uint4*>(&band[r * LDW + c]);
            if (row < n_dst && col0 + c < d_out)
                *reinterpret_cast<uint4*>(&out[row * d_out + col0 + c]) = v;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // band is rewritten by the next tm
    }
    (void)sizeof(T);
}

// With SW the 2-byte kernel multiplies with its operands exchanged (weights as the MFMA's row operand,
// the activations as its column operand), so a lane of a 32x32 tile holds ONE output row (lane % 32)
// and 16 of its columns in four runs of four: register i is column 8*(i/4) + 4*(lane/32) + i%4.
// Four consecutive columns convert with two packed conversions and leave in one 8-byte store,
// instead of sixteen conversions and sixteen 2-byte stores per tile in the other orientation.

// Plain stores of one wave's TM x TN block (any d_out; OutT = the storage type or float for the
// unrounded result).
template <typename Tr, typename OutT, int TM, int TN>
__device__ __forceinline__ void epilogue16_direct(floatx16 (&acc)[TM][TN], int64_t row0, int32_t col0, int lane,
                                                  int64_t row_end, int32_t d_out, const typename Tr::store_t* bias,
                                                  int relu, OutT* out) {
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int64_t row = row0 + tm * 32 + (lane & 31);
        if (row >= row_end) continue;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int32_t col = col0 + tn * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
                if (col < d_out) {
                    float x = acc[tm][tn][i] + (bias != nullptr ? Tr::to_f(bias[col]) : 0.f);
                    if (relu) x = fmaxf(x, 0.f);
                    if constexpr (sizeof(OutT) == 4) out[row * d_out + col] = x;
                    else out[row * d_out + col] = Tr::from_f(x);
                }
            }
    }
}

// One run of four consecutive columns of a tile: bias, activation, rounding, packed.
template <typename Tr>
__device__ __forceinline__ uint2 pack_run(const floatx16& a, int q, const typename Tr::store_t* bias, int32_t col,
                                          int32_t d_out, int relu) {
    float x[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[e] = a[4 * q + e];
        if (bias != nullptr && col + e < d_out) x[e] += Tr::to_f(bias[col + e]);
        if (relu) x[e] = fmaxf(x[e], 0.f);
    }
    return make_uint2(Tr::pack2(x[0], x[1]), Tr::pack2(x[2], x[3]));
}

// 2-byte outputs through a per-wave band of LDS ([32][32*TN + 8] elements) so that rows leave as
// 128-bit words.  Requires d_out % 8 == 0.  Waves do not share a band, so only this wave's own
// LDS traffic has to be waited for.
template <typename Tr, int TM, int TN>
__device__ __forceinline__ void epilogue16_staged(floatx16 (&acc)[TM][TN], int64_t row0, int32_t col0, int lane,
                                                  int64_t row_end, int32_t d_out, const typename Tr::store_t* bias,
                                                  int relu, typename Tr::store_t* out, typename Tr::store_t* band) {
    constexpr int W = 32 * TN, LDW = W + 8;          // band width in elements, padded row
    constexpr int WORDS = W / 8;                     // 16-byte words per band row
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = tn * 32 + 8 * q + 4 * (lane >> 5);
                *reinterpret_cast<uint2*>(&band[(lane & 31) * LDW + c]) =
                    pack_run<Tr>(acc[tm][tn], q, bias, col0 + c, d_out, relu);
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < 32 * WORDS / 64; ++j) {
            const int w = j * 64 + lane;
            const int r = w / WORDS, c = (w % WORDS) * 8;
            const int64_t row = row0 + tm * 32 + r;
            const uint4 v = *reinterpret_cast<const uint4*>(&band[r * LDW + c]);
            if (row < row_end && col0 + c < d_out)
                *reinterpret_cast<uint4*>(&out[row * d_out + col0 + c]) = v;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // band is rewritten by the next tm
    }
}

// Slot-tree layers: which rows a row tile covers.  Returns false for a tile past the last one.
template <int BM>
__device__ __forceinline__ bool tree_tile_rows(const TreeTiles& tt, uint32_t mt, int& lvl, uint32_t& tile_in_level,
                                               int64_t& row0, int64_t& row_end) {
    if (mt >= tt.tile0[tt.n_levels]) return false;
    lvl = 0;
    while (mt >= tt.tile0[lvl + 1]) ++lvl;
    tile_in_level = mt - tt.tile0[lvl];
    const int64_t per_tile = lvl == 0 ? (int64_t)BM : (int64_t)tt.g[lvl] * tt.f[lvl];
    row0 = tt.row0[lvl] + (int64_t)tile_in_level * per_tile;
    const int64_t level_end = tt.row0[lvl] + tt.rows[lvl];
    row_end = row0 + per_tile < level_end ? row0 + per_tile : level_end;
    return true;
}

// Epilogue of a slot-tree layer, by the whole workgroup.  The tile's results (bias, activation,
// rounding to the storage type applied) are staged in LDS PW columns at a time; from there
//   - the rows of levels the next layer reads directly leave as 128-bit row pieces, and
//   - every group of siblings is averaged into its parent's row of the next layer's neighbour
//     means: fp32 running sum of the STORED values in child order over the valid children, one
//     division, one rounding - the arithmetic of the segmented-mean kernel, so the bits are the
//     ones that kernel would produce from the written rows.
// LDS: [BM][PW + 16 bytes] staged values, then BM validity bytes.  Needs d_out % (16 / sizeof(T)) == 0.
template <typename Tr, int BM, int BN, int PW, int TM, int TN, int NT, bool SW>
__device__ __forceinline__ void tree_epilogue(floatx16 (&acc)[TM][TN], void* lds, int wave_row0, int wave_col0, int tid,
                                              int lane, int64_t row0, int64_t row_end, int32_t col0, int32_t d_out,
                                              const typename Tr::store_t* bias, int relu, typename Tr::store_t* out,
                                              const TreeTiles& tt, int lvl, uint32_t tile_in_level, int32_t my_id) {
    using T = typename Tr::store_t;
    static_assert(BM <= NT, "one validity flag per thread");
    constexpr int EPW = 16 / (int)sizeof(T);      // elements per 16-byte word
    constexpr int LDT = PW + EPW;                 // padded row of the staged tile
    constexpr int WORDS = PW / EPW;
    static_assert(BN % PW == 0 && PW % 32 == 0, "column passes");
    T* tile = static_cast<T*>(lds);
    uint8_t* vld = reinterpret_cast<uint8_t*>(tile + BM * LDT);
    const int n_rows = (int)(row_end - row0);
    const bool make_means = lvl >= 1 && tt.mean_next != nullptr;
    const bool store_rows = lvl < tt.store_levels;
    if (make_means && tid < BM) vld[tid] = my_id >= 0 ? 1 : 0;
#pragma unroll 1
    for (int c_lo = 0; c_lo < BN; c_lo += PW) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int wc = wave_col0 + tn * 32;
            if (wc < c_lo || wc >= c_lo + PW) continue;
            // One 32 x 32 tile at a time, fetched into ordinary registers where it is used (the
            // accumulators may live in the accumulation registers, which no vector instruction reads)
            // and finished before the next: a few results in flight, not the whole block's.
            if constexpr (SW) {      // a lane holds runs of four columns of one row (operands exchanged)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    floatx16 av = acc[tm][tn];
                    asm volatile("" : "+v"(av));
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int c = wc + 8 * q + 4 * (lane >> 5);
                        T* dst = &tile[(wave_row0 + tm * 32 + (lane & 31)) * LDT + (c - c_lo)];
                        if constexpr (sizeof(T) == 4) {
                            float4 v;
                            float* x = &v.x;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                x[e] = av[4 * q + e];
                                if (bias != nullptr && col0 + c + e < d_out) x[e] += Tr::to_f(bias[col0 + c + e]);
                                if (relu) x[e] = fmaxf(x[e], 0.f);
                            }
                            *reinterpret_cast<float4*>(dst) = v;
                        } else {
                            *reinterpret_cast<uint2*>(dst) = pack_run<Tr>(av, q, bias, col0 + c, d_out, relu);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                const int32_t col = col0 + wc + (lane & 31);
                const float b = (bias != nullptr && col < d_out) ? Tr::to_f(bias[col]) : 0.f;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    floatx16 av = acc[tm][tn];
                    asm volatile("" : "+v"(av));
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float x = av[i] + b;
                        if (relu) x = fmaxf(x, 0.f);
                        const int row = wave_row0 + tm * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
                        tile[row * LDT + (wc - c_lo) + (lane & 31)] = Tr::from_f(x);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        lds_barrier();
        if (store_rows)
            for (int w = tid; w < n_rows * WORDS; w += NT) {
                const int r = w / WORDS, c = (w % WORDS) * EPW;
                const int32_t gc = col0 + c_lo + c;
                if (gc < d_out)
                    *reinterpret_cast<uint4*>(&out[(row0 + r) * d_out + gc]) =
                        *reinterpret_cast<const uint4*>(&tile[r * LDT + c]);
            }
        if (make_means) {
            const int f = tt.f[lvl];
            const int n_groups = n_rows / f;              // a level's rows are whole groups
            T* mean_next = static_cast<T*>(tt.mean_next);
            const int64_t parent0 = tt.row0[lvl - 1] + (int64_t)tile_in_level * tt.g[lvl];
            for (int w = tid; w < n_groups * WORDS; w += NT) {
                const int j = w / WORDS, c = (w % WORDS) * EPW;
                float a[EPW];
#pragma unroll
                for (int e = 0; e < EPW; ++e) a[e] = 0.f;
                int cnt = 0;
                for (int i = 0; i < f; ++i) {
                    const int row = j * f + i;
                    if (vld[row]) {
                        Pack16<Tr> v;
                        v.v = *reinterpret_cast<const uint4*>(&tile[row * LDT + c]);
#pragma unroll
                        for (int e = 0; e < EPW; ++e) a[e] = a[e] + Tr::to_f(v.e[e]);
                        ++cnt;
                    }
                }
                Pack16<Tr> o;
                const float fc = (float)cnt;
#pragma unroll
                for (int e = 0; e < EPW; ++e) o.e[e] = Tr::from_f(cnt > 0 ? a[e] / fc : 0.f);
                const int32_t gc = col0 + c_lo + c;
                if (gc < d_out) *reinterpret_cast<uint4*>(&mean_next[(parent0 + j) * d_out + gc]) = o.v;
            }
        }
        lds_barrier();        // the staged tile is rewritten by the next pass (its words are in registers by now)
    }
}

// fp32: v_mfma_f32_32x32x2_f32 (lane l feeds A[row l%32][k = l/32] and B[k = l/32][col l%32]).
// LDS: A row-major [BM][BK+4] read as 128-bit words - lane group g = l/32 takes the four
// k values 4g..4g+3 of an 8-wide K block and the four MFMAs of the block pair A's i-th
// value with B row 4g+i, which only permutes the order in which k is summed.
// B is [BK][BN+4], read as 32 consecutive floats per half wave.
template <int BM, int BN, int BK, int D, bool VEC, bool TREE>
__global__ void __launch_bounds__(kProjThreads)
sage_project_f32(const float* __restrict__ Hsrc, const int32_t* __restrict__ self_idx,
                 const float* __restrict__ Mean, const float* __restrict__ Wself,
                 const float* __restrict__ Wneigh, const float* __restrict__ bias, int64_t n_dst,
                 int32_t d_in, int32_t k_total, int32_t d_out, int relu, uint32_t n_tiles_n,
                 const float* __restrict__ Zero, float* __restrict__ out, const int64_t* __restrict__ n_rows_dev,
                 TreeTiles tt) {
    constexpr int LDA = BK + 4, LDB = BN + 4;   // LDA/4 odd: conflict-free 128-bit reads
    static_assert(BK % 8 == 0 && (LDA / 4) % 2 == 1, "K tile");
    static_assert(D >= 2 && D % 2 == 0, "ring depth");
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int A_ITEMS = BM * BK / 4 / kProjThreads;   // float4 items per thread
    constexpr int B_ITEMS = BK * BN / 4 / kProjThreads;
    static_assert(A_ITEMS >= 1 && B_ITEMS >= 1, "tile too small for 256 threads");
    extern __shared__ __attribute__((aligned(16))) float lds_f32[];
    float (*As)[BM][LDA] = reinterpret_cast<float (*)[BM][LDA]>(lds_f32);
    float (*Bs)[BK][LDB] = reinterpret_cast<float (*)[BK][LDB]>(lds_f32 + 2 * BM * LDA);

    uint32_t mt, nt;
    tile_of_block(blockIdx.x, n_tiles_n, mt, nt);
    int64_t row0 = (int64_t)mt * BM, row_end;
    int lvl = 0;
    uint32_t tile_in_level = 0;
    if (TREE) {
        if (!tree_tile_rows<BM>(tt, mt, lvl, tile_in_level, row0, row_end)) return;
    } else {
        if (n_rows_dev != nullptr) {      // the row count lives on the device: rows past it do not exist
            const int64_t live = *n_rows_dev;
            n_dst = live < n_dst ? live : n_dst;
        }
        if (row0 >= n_dst) return;
        row_end = n_dst;
    }
    const int32_t col0 = nt * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int K = k_total;
    // the slot id behind this thread's row of the tile (which siblings count in a mean): read here,
    // used after the K loop
    int32_t my_id = -1;
    if (TREE && lvl >= 1 && tt.mean_next != nullptr && row0 + tid < row_end) my_id = tt.ids[row0 + tid];

    // rows this thread stages, fixed for the whole K loop
    int64_t a_self[A_ITEMS], a_mean[A_ITEMS];
#pragma unroll
    for (int it = 0; it < A_ITEMS; ++it) {
        const int i = it * kProjThreads + tid;
        const int64_t r = row0 + i / (BK / 4);
        a_self[it] = -1;
        a_mean[it] = -1;
        if (r < row_end) {
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

    struct Regs {
        float4 a[A_ITEMS], b[B_ITEMS];
    };
    const int n_tiles = (K + BK - 1) / BK;

    // Branch-free addressing for the vector path: rows that do not exist and the K padding
    // are read from `Zero`, a row of zeros at least one padded K long, so the loop has no
    // control flow and nothing consumes a loaded value before it is stored to LDS.
    const float* p_self[A_ITEMS];
    const float* p_mean[A_ITEMS];
#pragma unroll
    for (int it = 0; it < A_ITEMS; ++it) {
        p_self[it] = a_self[it] >= 0 ? Hsrc + a_self[it] : Zero;
        p_mean[it] = a_mean[it] >= 0 ? Mean + a_mean[it] - d_in : Zero;   // indexed by the concatenated k
    }
    // weight rows by the concatenated k: row k of W_self for k < d_in, row k - d_in of W_neigh after
    const float* b_self[B_ITEMS];
    const float* b_neigh[B_ITEMS];
#pragma unroll
    for (int it = 0; it < B_ITEMS; ++it) {
        const int n = col0 + ((it * kProjThreads + tid) % (BN / 4)) * 4;
        b_self[it] = Wself + n;
        b_neigh[it] = Wneigh + n - (int64_t)d_in * d_out;
    }
    auto a_elem = [&](int it, int k) -> float {   // one element of the concatenated row
        if (k < d_in) return a_self[it] >= 0 ? Hsrc[a_self[it] + k] : 0.f;
        if (k < K) return a_mean[it] >= 0 ? Mean[a_mean[it] + (k - d_in)] : 0.f;
        return 0.f;
    };
    auto load_tile = [&](Regs& r, int t) {
        const int k0 = t * BK;
#pragma unroll
        for (int it = 0; it < A_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            const int k = k0 + (i % (BK / 4)) * 4;
            float4 v;
            if (VEC) {   // d_in % 4 == 0: a float4 never straddles the self/mean boundary
                const float* p = (k < d_in ? p_self[it] : p_mean[it]) + k;
                v = *reinterpret_cast<const float4*>(k < K ? p : Zero);
            } else {
                v = make_float4(a_elem(it, k), a_elem(it, k + 1), a_elem(it, k + 2), a_elem(it, k + 3));
            }
            r.a[it] = v;
        }
#pragma unroll
        for (int it = 0; it < B_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            const int k = k0 + i / (BN / 4);
            const int n = col0 + (i % (BN / 4)) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (VEC) {   // d_out % 4 == 0; one multiply-add and selects, no control flow
                const float* p = (k < d_in ? b_self[it] : b_neigh[it]) + (int64_t)k * d_out;
                v = *reinterpret_cast<const float4*>((k < K && n < d_out) ? p : Zero);
            } else if (k < K) {
                const float* p = (k < d_in ? Wself + (int64_t)k * d_out : Wneigh + (int64_t)(k - d_in) * d_out) + n;
                if (n + 0 < d_out) v.x = p[0];
                if (n + 1 < d_out) v.y = p[1];
                if (n + 2 < d_out) v.z = p[2];
                if (n + 3 < d_out) v.w = p[3];
            }
            r.b[it] = v;
        }
    };
    auto store_tile = [&](const Regs& r, int st) {
#pragma unroll
        for (int it = 0; it < A_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            *reinterpret_cast<float4*>(&As[st][i / (BK / 4)][(i % (BK / 4)) * 4]) = r.a[it];
        }
#pragma unroll
        for (int it = 0; it < B_ITEMS; ++it) {
            const int i = it * kProjThreads + tid;
            *reinterpret_cast<float4*>(&Bs[st][i / (BN / 4)][(i % (BN / 4)) * 4]) = r.b[it];
        }
    };
    // One 8-wide K block of a stage as this lane's MFMA operands: TM 128-bit words of A, 4 x TN
    // single values of B.  The fragments of block kk+8 are read from LDS while block kk is
    // multiplied (two fragment sets), and the scheduler is told not to move LDS operations or
    // MFMAs across the marked points: left alone it sinks every read to just before its first
    // use, and the matrix pipe then idles for an LDS round trip before every group of four MFMAs.
    struct Frag {
        float4 a[TM];
        float b[4][TN];
    };
    const int fg = lane >> 5, fl32 = lane & 31;
    auto load_frag = [&](Frag& f, int st, int kk) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
            f.a[tm] = *reinterpret_cast<const float4*>(&As[st][wm * (BM / 2) + tm * 32 + fl32][kk + 4 * fg]);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) f.b[i][tn] = Bs[st][kk + 4 * fg + i][wn * (BN / 2) + tn * 32 + fl32];
    };
    auto mma = [&](const Frag& f) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const float av = i == 0 ? f.a[tm].x : i == 1 ? f.a[tm].y : i == 2 ? f.a[tm].z : f.a[tm].w;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)   // slot-tree layers: operands exchanged, a lane then holds runs of one row
                    acc[tm][tn] = TREE ? __builtin_amdgcn_mfma_f32_32x32x2f32(f.b[i][tn], av, acc[tm][tn], 0, 0, 0)
                                       : __builtin_amdgcn_mfma_f32_32x32x2f32(av, f.b[i][tn], acc[tm][tn], 0, 0, 0);
            }
    };
    auto compute = [&](int st) {
        Frag f0, f1;
        load_frag(f0, st, 0);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            if (kk + 8 < BK) load_frag(f1, st, kk + 8);
            __builtin_amdgcn_sched_barrier(kSchedPin);
            mma(f0);
            if (kk + 16 < BK) load_frag(f0, st, kk + 16);
            __builtin_amdgcn_sched_barrier(kSchedPin);
            if (kk + 8 < BK) mma(f1);
        }
        __builtin_amdgcn_sched_barrier(kSchedPin);
    };

    // A ring of D register sets and two LDS stages.  Iteration t: the loads of tile t+D are issued
    // first (into the set tile t has left), tile t is multiplied from LDS stage t&1, and only then
    // is tile t+1 - loaded D-1 iterations ago - moved from its registers to the other stage, so
    // a load has D iterations to arrive before anything waits for it.  Exactly n_tiles tiles are
    // multiplied (tiles at or beyond n_tiles load as zeros and are never multiplied); D is even
    // so that the stage of an unrolled iteration is a constant.
    Regs r[D];
    load_tile(r[0], 0);
    store_tile(r[0], 0);
#pragma unroll
    for (int j = 1; j < D; ++j) load_tile(r[j], j);
    lds_barrier();
    auto iter = [&](int t, int i) {     // i = t % D, a constant after unrolling
        load_tile(r[i], t + D);
        compute(i & 1);
        store_tile(r[(i + 1) % D], (i + 1) & 1);
        lds_barrier();
    };
    int t = 0;
    for (; t + D <= n_tiles; t += D) {
#pragma unroll
        for (int i = 0; i < D; ++i) iter(t + i, i);
    }
#pragma unroll
    for (int i = 0; i < D - 1; ++i)
        if (t + i < n_tiles) iter(t + i, i);
    if (TREE)
        tree_epilogue<TrF32, BM, BN, BN, TM, TN, kProjThreads, true>(acc, lds_f32, wm * (BM / 2), wn * (BN / 2), tid, lane, row0,
                                                               row_end, col0, d_out, bias, relu, out, tt, lvl,
                                                               tile_in_level, my_id);
    else
        project_epilogue<TrF32, TM, TN>(acc, row0 + wm * (BM / 2), col0 + wn * (BN / 2), lane, row_end, d_out, bias, relu,
                                        out);
}

// bf16 / fp16: v_mfma_f32_32x32x16_{bf16,f16}.  Lane l feeds 8 consecutive k of row (or
// column) l%32, k-group l/32, so both operands sit in LDS with k contiguous and are read
// as 128-bit words: A [BM][BK+8], B [BN][BK+8] (row stride 80 bytes: conflict free).
// B comes from Wt, the transposed weights [NP][KP] (k contiguous, zero padded to whole
// tiles) that the mean kernel's side job writes into the workspace.
constexpr int kKPad16 = 64;   // Wt rows are zero padded to a multiple of this many k

template <typename Tr, int BM, int BN, int BK, int WM, int WN, int D, bool VEC, bool TREE, bool SW>
__global__ void __launch_bounds__(64 * WM * WN)
sage_project_16(const uint16_t* __restrict__ Hsrc, const int32_t* __restrict__ self_idx,
                const uint16_t* __restrict__ Mean, const uint16_t* __restrict__ Wt, int32_t KP,
                const typename Tr::store_t* __restrict__ bias, int64_t n_dst, int32_t d_in, int32_t k_total,
                int32_t d_out, int relu, uint32_t n_tiles_n, const uint16_t* __restrict__ Zero,
                typename Tr::store_t* __restrict__ out, int out_f32, const int64_t* __restrict__ n_rows_dev,
                TreeTiles tt) {
    constexpr int LD = BK + 8;
    static_assert(kKPad16 % BK == 0, "Wt padding must cover whole K tiles");
    static_assert(D >= 2 && D % 2 == 0, "ring depth");
    constexpr int NT = 64 * WM * WN;                      // threads: WM x WN waves
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // 32x32 MFMA tiles per wave
    constexpr int A_ITEMS = BM * BK / 8 / NT;             // 16-byte items per thread
    constexpr int B_ITEMS = BN * BK / 8 / NT;
    static_assert(A_ITEMS >= 1 && B_ITEMS >= 1, "tile too small for the workgroup");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds16[];
    uint16_t (*As)[BM][LD] = reinterpret_cast<uint16_t (*)[BM][LD]>(lds16);
    uint16_t (*Bs)[BN][LD] = reinterpret_cast<uint16_t (*)[BN][LD]>(lds16 + 2 * BM * LD);

    uint32_t mt, nt;
    tile_of_block(blockIdx.x, n_tiles_n, mt, nt);
    int64_t row0 = (int64_t)mt * BM, row_end;
    int lvl = 0;
    uint32_t tile_in_level = 0;
    if (TREE) {
        if (!tree_tile_rows<BM>(tt, mt, lvl, tile_in_level, row0, row_end)) return;
    } else {
        if (n_rows_dev != nullptr) {      // the row count lives on the device: rows past it do not exist
            const int64_t live = *n_rows_dev;
            n_dst = live < n_dst ? live : n_dst;
        }
        if (row0 >= n_dst) return;
        row_end = n_dst;
    }
    const int32_t col0 = nt * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int K = k_total;
    int32_t my_id = -1;      // see the fp32 kernel
    if (TREE && lvl >= 1 && tt.mean_next != nullptr && row0 + tid < row_end) my_id = tt.ids[row0 + tid];

    int64_t a_self[A_ITEMS], a_mean[A_ITEMS];
#pragma unroll
    for (int it = 0; it < A_ITEMS; ++it) {
        const int i = it * NT + tid;
        const int64_t r = row0 + i / (BK / 8);
        a_self[it] = -1;
        a_mean[it] = -1;
        if (r < row_end) {
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

    struct Regs {
        uint4 a[A_ITEMS], b[B_ITEMS];
    };
    union U16x8 {
        uint4 v;
        uint16_t e[8];
    };
    const int n_tiles = (K + BK - 1) / BK;

    const uint16_t* p_self[A_ITEMS];
    const uint16_t* p_mean[A_ITEMS];
#pragma unroll
    for (int it = 0; it < A_ITEMS; ++it) {
        p_self[it] = a_self[it] >= 0 ? Hsrc + a_self[it] : Zero;
        p_mean[it] = a_mean[it] >= 0 ? Mean + a_mean[it] - d_in : Zero;   // indexed by the concatenated k
    }
    auto a_elem = [&](int it, int k) -> uint16_t {
        if (k < d_in) return a_self[it] >= 0 ? Hsrc[a_self[it] + k] : (uint16_t)0;
        if (k < K) return a_mean[it] >= 0 ? Mean[a_mean[it] + (k - d_in)] : (uint16_t)0;
        return 0;
    };
    auto load_tile = [&](Regs& r, int t) {
        const int k0 = t * BK;
#pragma unroll
        for (int it = 0; it < A_ITEMS; ++it) {
            const int i = it * NT + tid;
            const int k = k0 + (i % (BK / 8)) * 8;
            U16x8 v;
            if (VEC) {   // d_in % 8 == 0: a 16-byte word never straddles the self/mean boundary
                const uint16_t* p = (k < d_in ? p_self[it] : p_mean[it]) + k;
                v.v = *reinterpret_cast<const uint4*>(k < K ? p : Zero);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) v.e[j] = a_elem(it, k + j);
            }
            r.a[it] = v.v;
        }
        // Wt is padded to whole tiles; tiles past the end re-read the last one (A is zero there)
        const int kb = k0 < KP ? k0 : KP - BK;
#pragma unroll
        for (int it = 0; it < B_ITEMS; ++it) {
            const int i = it * NT + tid;
            r.b[it] = *reinterpret_cast<const uint4*>(Wt + (int64_t)(col0 + i / (BK / 8)) * KP + kb + (i % (BK / 8)) * 8);
        }
    };
    auto store_tile = [&](const Regs& r, int st) {
#pragma unroll
        for (int it = 0; it < A_ITEMS; ++it) {
            const int i = it * NT + tid;
            *reinterpret_cast<uint4*>(&As[st][i / (BK / 8)][(i % (BK / 8)) * 8]) = r.a[it];
        }
#pragma unroll
        for (int it = 0; it < B_ITEMS; ++it) {
            const int i = it * NT + tid;
            *reinterpret_cast<uint4*>(&Bs[st][i / (BK / 8)][(i % (BK / 8)) * 8]) = r.b[it];
        }
    };
    // One 16-wide K block of a stage as this lane's MFMA operands (TM + TN 128-bit words); the
    // next block's are read from LDS while this one is multiplied, and the scheduler may not move
    // LDS operations or MFMAs across the marked points (see the fp32 kernel).
    struct Frag {
        uint4 a[TM], b[TN];
    };
    const int fg = lane >> 5, fl32 = lane & 31;
    auto load_frag = [&](Frag& f, int st, int kk) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
            f.a[tm] = *reinterpret_cast<const uint4*>(&As[st][wm * (BM / WM) + tm * 32 + fl32][kk + fg * 8]);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
            f.b[tn] = *reinterpret_cast<const uint4*>(&Bs[st][wn * (BN / WN) + tn * 32 + fl32][kk + fg * 8]);
    };
    auto mma = [&](const Frag& f) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                acc[tm][tn] = SW ? mfma16<Tr>(f.b[tn], f.a[tm], acc[tm][tn]) : mfma16<Tr>(f.a[tm], f.b[tn], acc[tm][tn]);
    };
    auto compute = [&](int st) {
        if constexpr (TM * TN <= 4) {
            Frag f0, f1;
            load_frag(f0, st, 0);
#pragma unroll
            for (int kk = 0; kk < BK; kk += 32) {
                if (kk + 16 < BK) load_frag(f1, st, kk + 16);
                __builtin_amdgcn_sched_barrier(kSchedPin);
                mma(f0);
                if (kk + 32 < BK) load_frag(f0, st, kk + 32);
                __builtin_amdgcn_sched_barrier(kSchedPin);
                if (kk + 16 < BK) mma(f1);
            }
            __builtin_amdgcn_sched_barrier(kSchedPin);
        } else {      // the largest tile has no registers for a second fragment set
#pragma unroll
            for (int kk = 0; kk < BK; kk += 16) {
                Frag f;
                load_frag(f, st, kk);
                mma(f);
            }
        }
    };

    // A ring of D register sets and two LDS stages.  Iteration t: the loads of tile t+D are issued
    // first (into the set tile t has left), tile t is multiplied from LDS stage t&1, and only then
    // is tile t+1 - loaded D-1 iterations ago - moved from its registers to the other stage, so
    // a load has D iterations to arrive before anything waits for it.  Exactly n_tiles tiles are
    // multiplied (tiles at or beyond n_tiles load as zeros and are never multiplied); D is even
    // so that the stage of an unrolled iteration is a constant.
    Regs r[D];
    load_tile(r[0], 0);
    store_tile(r[0], 0);
#pragma unroll
    for (int j = 1; j < D; ++j) load_tile(r[j], j);
    lds_barrier();
    auto iter = [&](int t, int i) {     // i = t % D, a constant after unrolling
        load_tile(r[i], t + D);
        compute(i & 1);
        store_tile(r[(i + 1) % D], (i + 1) & 1);
        lds_barrier();
    };
    int t = 0;
    for (; t + D <= n_tiles; t += D) {
#pragma unroll
        for (int i = 0; i < D; ++i) iter(t + i, i);
    }
#pragma unroll
    for (int i = 0; i < D - 1; ++i)
        if (t + i < n_tiles) iter(t + i, i);
    const int64_t wrow0 = row0 + wm * (BM / WM);
    const int32_t wcol0 = col0 + wn * (BN / WN);
    if (TREE) {
        tree_epilogue<Tr, BM, BN, BN, TM, TN, NT, SW>(acc, lds16, wm * (BM / WM), wn * (BN / WN), tid, lane, row0, row_end, col0,
                                                      d_out, bias, relu, out, tt, lvl, tile_in_level, my_id);
    } else if (out_f32) {     // `out` is a float array: unrounded result
        if constexpr (SW) epilogue16_direct<Tr, float, TM, TN>(acc, wrow0, wcol0, lane, row_end, d_out, bias, relu, reinterpret_cast<float*>(out));
        else project_epilogue_f32out<Tr, TM, TN>(acc, wrow0, wcol0, lane, row_end, d_out, bias, relu, reinterpret_cast<float*>(out));
    } else if (VEC && (d_out & 7) == 0) {
        // every wave is past its last LDS read of the tiles: reuse that LDS, one band per wave
        constexpr int BAND = 32 * (32 * TN + 8);
        static_assert((size_t)WM * WN * BAND <= (size_t)2 * (BM + BN) * LD, "epilogue bands exceed the tile LDS");
        typename Tr::store_t* band = reinterpret_cast<typename Tr::store_t*>(lds16) + wave * BAND;
        if constexpr (SW) epilogue16_staged<Tr, TM, TN>(acc, wrow0, wcol0, lane, row_end, d_out, bias, relu, out, band);
        else project_epilogue_staged<Tr, TM, TN>(acc, wrow0, wcol0, lane, row_end, d_out, bias, relu, out, band);
    } else {
        if constexpr (SW) epilogue16_direct<Tr, typename Tr::store_t, TM, TN>(acc, wrow0, wcol0, lane, row_end, d_out, bias, relu, out);
        else project_epilogue<Tr, TM, TN>(acc, wrow0, wcol0, lane, row_end, d_out, bias, relu, out);
    }
}

// Slot-tree layers on the largest 2-byte tile (256 x 256 x 64, 8 waves) by workgroups that WALK over
// their tiles (b, b + gridDim.x, ...; one workgroup per CU) instead of one workgroup per tile.
// With K as short as 4 tiles, a tile of the one-tile kernel spends as long waiting as multiplying: for
// the next workgroup to be started (2 us), then for its row indices, then for the rows behind them
// (3.8 us until the first K tile is in LDS, against 7.7 us of K loop and 6.1 us of epilogue).  Here
//   - the next tile's row indices are requested a whole K loop ahead,
//   - its first two K tiles are requested during the last two K steps of the current tile and wait in
//     the registers through the epilogue, so the next tile multiplies as soon as the epilogue's LDS is free,
//   - the weights (L2 resident) are requested one K tile ahead, the left operand two.
// LDS layout, summation order and the epilogue are those of sage_project_16: the same bits.
// Needs d_in % 64 == 0 and k_total = 2 * d_in or d_in with an even number of K tiles (a K tile lies in the
// self half or in the mean half as a whole; the ring's parity is the same for every tile), byte
// offsets within 32 bits (the host checks), and n_blocks >= 1 blocks of project_grid's numbering.
template <typename Tr, bool SW>
__global__ void __launch_bounds__(512)
sage_project_16_walk(const uint16_t* __restrict__ Hsrc, const int32_t* __restrict__ self_idx,
                     const uint16_t* __restrict__ Mean, const uint16_t* __restrict__ Wt, int32_t KP,
                     const typename Tr::store_t* __restrict__ bias, int32_t d_in, int32_t k_total, int32_t d_out,
                     int relu, uint32_t n_tiles_n, uint32_t n_blocks, typename Tr::store_t* __restrict__ out,
                     TreeTiles tt) {
    constexpr int BM = 256, BN = 256, BK = 64, WM = 2, WN = 4, LD = BK + 8, NT = 64 * WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int ITEMS = BM * BK / 8 / NT;          // 16-byte items per thread and operand (BM == BN)
    constexpr int SLICE = NT / (BK / 8);             // rows one item of every thread covers together
    static_assert(BM == BN && ITEMS * SLICE == BM, "items");
    // LDS: stage 0 (left operand's K tile [BM][LD], then the weights' [BN][LD]), then stage 1 the same
    constexpr int STAGE = (BM + BN) * LD;            // elements per stage
    static_assert((size_t)BM * (BN + 8) * 2 + BM <= (size_t)2 * STAGE * 2, "the staged tile must fit the K tiles' LDS");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds16[];
    auto As = [&](int st) { return reinterpret_cast<uint16_t (*)[LD]>(lds16 + st * STAGE); };
    auto Bs = [&](int st) { return reinterpret_cast<uint16_t (*)[LD]>(lds16 + st * STAGE + BM * LD); };
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int nk = (k_total + BK - 1) / BK;
    const int trow = tid / (BK / 8), tk = (tid % (BK / 8)) * 8;   // this thread's row of a slice, its k within a K tile

    struct Tile {
        int64_t row0, row_end;
        int32_t col0;
        int lvl;
        uint32_t til;
    };
    auto tile_at = [&](uint32_t bid, Tile& T) -> bool {
        uint32_t mt, nt;
        tile_of_block(bid, n_tiles_n, mt, nt);
        T.col0 = (int32_t)(nt * BN);
        return tree_tile_rows<BM>(tt, mt, T.lvl, T.til, T.row0, T.row_end);
    };
    // Addresses are a uniform base plus a 32-bit BYTE offset of the thread's.  Per tile a thread keeps,
    // for each of its ITEMS rows, the offset of the self row (row index * row bytes) and of the mean
    // row; rows past the tile's last one repeat that row (their results are never used); an absent
    // self row (negative index) reads row 0 and is zeroed on its way to LDS.
    const uint32_t row_bytes = (uint32_t)d_in * 2u, tk_bytes = (uint32_t)tk * 2u;
    struct Rows {
        uint32_t so[ITEMS];
        uint32_t absent;         // bit it: self row absent
        int32_t id;              // slot id behind row `tid` of the tile (see tree_epilogue)
    };
    // the indices are requested here and not touched: whoever turns them into offsets waits for them
    auto load_idx = [&](const Tile& T, int32_t (&sidx)[ITEMS], int32_t& id) {
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const int64_t r = T.row0 + it * SLICE + trow;
            const bool in = r < T.row_end;
            const int32_t v = self_idx != nullptr ? self_idx[in ? r : T.row0] : (int32_t)r;    // loads are unconditional
            sidx[it] = in ? v : -1;
        }
        const bool in = T.row0 + tid < T.row_end;
        const int32_t v = tt.ids[in ? T.row0 + tid : T.row0];
        id = (in && T.lvl >= 1 && tt.mean_next != nullptr) ? v : -1;
    };
    auto rows_of = [&](const Tile& T, const int32_t (&sidx)[ITEMS], int32_t id, Rows& R) {
        R.absent = 0u;
        R.id = id;
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            R.so[it] = (uint32_t)(sidx[it] >= 0 ? sidx[it] : 0) * row_bytes + tk_bytes;
            if (sidx[it] < 0) R.absent |= 1u << it;
        }
    };
    auto load_a = [&](uint4 (&ra)[ITEMS], const Tile& T, const Rows& R, int kt) {
        // one instruction stream for both halves (a branch here makes the waits for earlier loads conservative)
        const int k0 = kt * BK;
        const bool self_half = k0 < d_in;
        const char* base = self_half ? reinterpret_cast<const char*>(Hsrc + k0)
                                     : reinterpret_cast<const char*>(Mean + T.row0 * d_in + (k0 - d_in));
        const uint32_t last = (uint32_t)(T.row_end - T.row0 - 1);
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const uint32_t rr = (uint32_t)(it * SLICE + trow);
            const uint32_t mo = (rr <= last ? rr : last) * row_bytes + tk_bytes;
            ra[it] = *reinterpret_cast<const uint4*>(base + (self_half ? R.so[it] : mo));
        }
    };
    const uint32_t b_off = ((uint32_t)trow * (uint32_t)KP + (uint32_t)tk) * 2u;
    auto load_b = [&](uint4 (&rb)[ITEMS], int32_t col0, int kt) {
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const char* base = reinterpret_cast<const char*>(Wt + (int64_t)(col0 + it * SLICE) * KP + kt * BK);
            rb[it] = *reinterpret_cast<const uint4*>(base + b_off);
        }
    };
    // kt: the K tile the words belong to, R: the rows of the tile they belong to
    auto store_tile = [&](const uint4 (&ra)[ITEMS], const uint4 (&rb)[ITEMS], int st, int kt, const Rows& R) {
        const uint32_t absent = kt * BK < d_in ? R.absent : 0u;
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const uint32_t keep = ((absent >> it) & 1u) - 1u;      // all ones, or zero for an absent row: four ANDs, no branch
            *reinterpret_cast<uint4*>(&As(st)[it * SLICE + trow][tk]) =
                make_uint4(ra[it].x & keep, ra[it].y & keep, ra[it].z & keep, ra[it].w & keep);
            *reinterpret_cast<uint4*>(&Bs(st)[it * SLICE + trow][tk]) = rb[it];
        }
    };
    floatx16 acc[TM][TN];
    const int fg = lane >> 5, fl32 = lane & 31;
    // one 16-wide K block at a time (see sage_project_16: the largest tile has registers for one set of
    // operand words; the SIMD's other wave covers the wait for them)
    auto compute = [&](int st) {
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            uint4 fa[TM], fb[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                fa[tm] = *reinterpret_cast<const uint4*>(&As(st)[wm * (BM / WM) + tm * 32 + fl32][kk + fg * 8]);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                fb[tn] = *reinterpret_cast<const uint4*>(&Bs(st)[wn * (BN / WN) + tn * 32 + fl32][kk + fg * 8]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = SW ? mfma16<Tr>(fb[tn], fa[tm], acc[tm][tn]) : mfma16<Tr>(fa[tm], fb[tn], acc[tm][tn]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    uint32_t bid = blockIdx.x;
    Tile cur;
    if (bid >= n_blocks || !tile_at(bid, cur)) return;
    Rows R;
    {
        int32_t sidx[ITEMS], id;
        load_idx(cur, sidx, id);
        rows_of(cur, sidx, id, R);
    }
    // (one struct for everything under way: a weights array of its own ended up in scratch memory)
    struct Ring {
        uint4 a[2][ITEMS], b[ITEMS];
    };
    Ring rg;
    load_a(rg.a[0], cur, R, 0);
    load_b(rg.b, cur.col0, 0);
    store_tile(rg.a[0], rg.b, 0, 0, R);
    load_a(rg.a[1], cur, R, 1);
    lds_barrier();
    for (;;) {
        // Stage 0 holds this tile's first K tile.  The tile after this one (the last tile stands in for
        // its own successor: its first K tile is then re-read at the end and nothing uses it):
        uint32_t nbid = bid + gridDim.x;
        Tile nxt = cur;
        bool has_next = false;
        while (nbid < n_blocks && !(has_next = tile_at(nbid, nxt))) nbid += gridDim.x;
        if (!has_next) nxt = cur;
        int32_t nidx[ITEMS], nid;
        load_idx(nxt, nidx, nid);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0.f;
        // Step t multiplies K tile t from LDS stage t & 1 while the left operand's K tile t + 2 and the
        // weights' K tile t + 1 are on their way.
        int t = 0;
        for (; t + 2 < nk; t += 2) {
            load_b(rg.b, cur.col0, t + 1);      // wanted first: the younger load may stay under way past the hand-over
            load_a(rg.a[0], cur, R, t + 2);
            compute(0);
            store_tile(rg.a[1], rg.b, 1, t + 1, R);
            lds_barrier();
            load_b(rg.b, cur.col0, t + 2);
            load_a(rg.a[1], cur, R, t + 3);
            compute(1);
            store_tile(rg.a[0], rg.b, 0, t + 2, R);
            lds_barrier();
        }
        // The last two K tiles: what is requested now is the NEXT tile's first K tile (first use of its
        // row indices: requested at the top of this tile, waited for here).  It waits in the registers
        // until the epilogue has released the LDS.
        Rows N;
        rows_of(nxt, nidx, nid, N);
        load_b(rg.b, cur.col0, t + 1);
        load_a(rg.a[0], nxt, N, 0);
        compute(0);
        store_tile(rg.a[1], rg.b, 1, t + 1, R);
        lds_barrier();
        load_b(rg.b, nxt.col0, 0);
        load_a(rg.a[1], nxt, N, 1);      // and its second one, wanted at the end of the next tile's first step
        compute(1);
        // The next tile's words are waited for HERE, before the epilogue issues its stores: the counter of
        // outstanding memory operations is in order, so a wait for these loads placed after the epilogue
        // would also wait for every store of it.
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            asm volatile("" : "+v"(rg.a[0][it].x), "+v"(rg.a[0][it].y), "+v"(rg.a[0][it].z), "+v"(rg.a[0][it].w));
            asm volatile("" : "+v"(rg.b[it].x), "+v"(rg.b[it].y), "+v"(rg.b[it].z), "+v"(rg.b[it].w));
        }
        lds_barrier();     // every wave is past its last read of the K tiles: the epilogue reuses their LDS
        tree_epilogue<Tr, BM, BN, BN, TM, TN, NT, SW>(acc, lds16, wm * (BM / WM), wn * (BN / WN), tid, lane, cur.row0,
                                                      cur.row_end, cur.col0, d_out, bias, relu, out, tt, cur.lvl, cur.til,
                                                      R.id);
        store_tile(rg.a[0], rg.b, 0, 0, N);      // the next tile's first K tile, which waited in the registers
        lds_barrier();
        if (!has_next) break;
        cur = nxt;
        bid = nbid;
        R = N;
    }
}

// ------------------------------------------------------------------ launch --

static uint32_t project_grid(int64_t m_tiles, uint32_t n_tiles_n) {
    return (uint32_t)(ceil_div(m_tiles, kXcds) * kXcds * n_tiles_n);
}

// The row tiles of a slot-tree layer for tile height BM (see TreeTiles); returns their number.
static int64_t tree_tiles(const TreeLayer& t, int BM, TreeTiles& tt) {
    tt = TreeTiles{};
    tt.n_levels = t.n_levels;
    tt.store_levels = t.mean_next != nullptr ? t.n_levels - 1 : t.n_levels;
    tt.ids = t.ids;
    tt.mean_next = t.mean_next;
    int64_t row = 0, tiles = 0;
    for (int h = 0; h < t.n_levels; ++h) {
        tt.row0[h] = row;
        tt.rows[h] = t.level_rows[h];
        tt.f[h] = h ? t.fan[h] : 1;
        tt.g[h] = h ? BM / t.fan[h] : BM;
        const int64_t per_tile = h ? (int64_t)tt.g[h] * tt.f[h] : BM;
        tt.tile0[h] = (uint32_t)tiles;
        tiles += ceil_div(t.level_rows[h], per_tile);
        row += t.level_rows[h];
    }
    tt.tile0[t.n_levels] = (uint32_t)tiles;
    return tiles;
}

template <int BM, int BN, int BK, int D>
static hopgnn_status launch_project_f32(bool vec, hipStream_t s, const void* Hsrc, const int32_t* self_idx,
                                        const void* mean, const void* Ws, const void* Wn, const void* bias,
                                        int64_t n_dst, int32_t d_in, int32_t k_total, int32_t d_out, int relu,
                                        const void* zero, void* out, const int64_t* n_rows_dev, const TreeLayer* tree) {
    const uint32_t ntn = (uint32_t)ceil_div(d_out, BN);
    TreeTiles tt{};
    const int64_t m_tiles = tree != nullptr ? tree_tiles(*tree, BM, tt) : ceil_div(n_dst, BM);
    if (m_tiles * ntn + kXcds * ntn >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    const dim3 grid(project_grid(m_tiles, ntn));
    auto a = static_cast<const float*>(Hsrc);
    auto m = static_cast<const float*>(mean);
    auto ws = static_cast<const float*>(Ws);
    auto wn = static_cast<const float*>(Wn);
    auto b = static_cast<const float*>(bias);
    auto o = static_cast<float*>(out);
    auto z = static_cast<const float*>(zero);
    constexpr size_t lds_loop = (size_t)2 * (BM * (BK + 4) + BK * (BN + 4)) * sizeof(float);
    constexpr size_t lds_tree = (size_t)BM * (BN + 4) * sizeof(float) + BM;     // staged tile + validity bytes
    const size_t lds = tree != nullptr && lds_tree > lds_loop ? lds_tree : lds_loop;
    auto kern = tree != nullptr ? sage_project_f32<BM, BN, BK, D, true, true>
                : vec           ? sage_project_f32<BM, BN, BK, D, true, false>
                                : sage_project_f32<BM, BN, BK, D, false, false>;
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess)
        return HOPGNN_EHIP;
    hipLaunchKernelGGL(kern, grid, dim3(kProjThreads), lds, s, a, self_idx, m, ws, wn, b, n_dst, d_in, k_total, d_out,
                       relu, ntn, z, o, n_rows_dev, tt);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

template <typename Tr, int BM, int BN, int BK, int WM, int WN, int D = 2>
static hopgnn_status launch_project_16(bool vec, hipStream_t s, const void* Hsrc, const int32_t* self_idx,
                                       const void* mean, const uint16_t* Wt, int32_t KP, const void* bias,
                                       int64_t n_dst, int32_t d_in, int32_t k_total, int32_t d_out, int relu,
                                       const void* zero, void* out, int out_f32, const int64_t* n_rows_dev,
                                       const TreeLayer* tree) {
    using T = typename Tr::store_t;
    constexpr size_t lds = (size_t)2 * (BM + BN) * (BK + 8) * sizeof(uint16_t);
    static_assert((size_t)BM * (BN + 8) * 2 + BM <= lds, "the staged tile of a slot-tree layer must fit the loop's LDS");
    // Exchanged operands pay where rounding is expensive: bf16 (packed hardware conversion of two
    // values instead of an integer rounding sequence per value; measured -11 % on the 4096-seed bf16
    // workload's first layer).  fp16 converts in one instruction either way and measured 5 % slower.
    const bool sw = Tr::kDt == HOPGNN_BF16;
    auto kern = tree != nullptr ? (sw ? sage_project_16<Tr, BM, BN, BK, WM, WN, D, true, true, true> : sage_project_16<Tr, BM, BN, BK, WM, WN, D, true, true, false>)
                : vec           ? (sw ? sage_project_16<Tr, BM, BN, BK, WM, WN, D, true, false, true> : sage_project_16<Tr, BM, BN, BK, WM, WN, D, true, false, false>)
                                : (sw ? sage_project_16<Tr, BM, BN, BK, WM, WN, D, false, false, true> : sage_project_16<Tr, BM, BN, BK, WM, WN, D, false, false, false>);
    if (lds > 64 * 1024) {   // above the default limit the size has to be opted into
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return HOPGNN_EHIP;
    }
    const uint32_t ntn = (uint32_t)ceil_div(d_out, BN);
    TreeTiles tt{};
    const int64_t m_tiles = tree != nullptr ? tree_tiles(*tree, BM, tt) : ceil_div(n_dst, BM);
    if (m_tiles * ntn + kXcds * ntn >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if constexpr (BM == 256 && BN == 256 && BK == 64 && WM == 2 && WN == 4) {
        const int nk = (k_total + BK - 1) / BK;
        // the walking kernel's requirements: whole K tiles in each half, 32-bit byte offsets; it is for
        // short K (at 16 K tiles the fixed waits of a tile are a small share and the one-tile kernel's
        // deeper ring for the weights wins: 224 us against 235 us on the 100 M-vertex workload's second layer)
        const bool fits = tree != nullptr && vec && d_in % BK == 0 && (k_total == d_in || k_total == 2 * d_in) &&
                          nk % 2 == 0 && nk <= 8 && n_dst * (int64_t)d_in * 2 < ((int64_t)1 << 32) &&
                          tree->n_src * (int64_t)d_in * 2 < ((int64_t)1 << 32) && (int64_t)KP * 2 * BN < ((int64_t)1 << 32);
        if (fits) {
            int dev = 0, cus = 0;
            if (hipGetDevice(&dev) != hipSuccess ||
                hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
                return HOPGNN_EHIP;
            const uint32_t n_blocks = project_grid(m_tiles, ntn);
            uint32_t grid = (uint32_t)(cus / kXcds) * kXcds;      // a multiple of the XCD count: a walk stays on its XCD
            if (grid < kXcds) grid = kXcds;
            // Walking pays once a workgroup has several tiles to hide waits between; with one or two tiles
            // per CU the hardware's own placement of single-tile workgroups is as good or better
            // (measured on one machine: 426 tiles 48 us against 44 us; 3638 tiles of K = 256: 254-257 us
            // against 271 us, 7276 tiles 487-493 against 521 us, 14.5 k and 29 k tiles within 1 %).
            if (n_blocks >= 4 * grid) {
                auto walk = sw ? sage_project_16_walk<Tr, true> : sage_project_16_walk<Tr, false>;
                if (hipFuncSetAttribute(reinterpret_cast<const void*>(walk), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)lds) != hipSuccess)
                    return HOPGNN_EHIP;
                hipLaunchKernelGGL(walk, dim3(grid), dim3(512), lds, s, static_cast<const uint16_t*>(Hsrc), self_idx,
                                   static_cast<const uint16_t*>(mean), Wt, KP, static_cast<const T*>(bias), d_in, k_total,
                                   d_out, relu, ntn, n_blocks, static_cast<T*>(out), tt);
                HOPGNN_LAUNCH_CHECK();
                return HOPGNN_OK;
            }
        }
    }
    hipLaunchKernelGGL(kern, dim3(project_grid(m_tiles, ntn)), dim3(64 * WM * WN), lds, s,
                       static_cast<const uint16_t*>(Hsrc), self_idx, static_cast<const uint16_t*>(mean), Wt,
                       KP, static_cast<const T*>(bias), n_dst, d_in, k_total, d_out, relu, ntn,
                       static_cast<const uint16_t*>(zero), static_cast<T*>(out), out_f32, n_rows_dev, tt);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

ProjWs proj_ws_layout(hopgnn_dtype dt, int64_t n_rows, int32_t d_in, int32_t k_total, int32_t d_out) {
    ProjWs L{};
    L.agg_bytes = align_up((size_t)n_rows * (size_t)d_in * dtype_size(dt), 256);
    L.KP = (int32_t)(ceil_div((int64_t)k_total, kKPad16) * kKPad16);
    L.NP = (int32_t)(ceil_div(d_out, 256) * 256);
    L.wt_bytes = dt == HOPGNN_F32 ? 0 : align_up((size_t)L.KP * (size_t)L.NP * 2, 256);
    L.zero_bytes = align_up(((size_t)2 * d_in + 64) * dtype_size(dt), 256);
    L.total = L.agg_bytes + L.wt_bytes + L.zero_bytes;
    return L;
}

hopgnn_status project_dispatch(hopgnn_dtype dt, hipStream_t s, const void* Hsrc, const int32_t* self_idx,
                               const void* mean, const void* W_self, const void* W_neigh, const uint16_t* Wt,
                               int32_t KP, const void* bias, int64_t n_dst, int32_t d_in, int32_t k_total,
                               int32_t d_out, int relu, const void* zero, void* out, int out_f32,
                               const int64_t* n_rows_dev, const TreeLayer* tree) {
    const int per16 = dt == HOPGNN_F32 ? 4 : 8;
    const int64_t work = ceil_div(n_dst, 128) * ceil_div(d_out, 128);   // 128 x 128 output tiles
    bool vec = d_in % per16 == 0 && aligned(Hsrc, 16) && aligned(mean, 16);
    if (dt == HOPGNN_F32) vec = vec && d_out % per16 == 0 && aligned(W_self, 16) && aligned(W_neigh, 16);
    if (tree != nullptr) {      // the slot-tree kernels are built for the vector path only
        if (!vec || out_f32 || n_rows_dev != nullptr || d_out % per16 != 0 || !aligned(out, 16) ||
            (tree->mean_next != nullptr && !aligned(tree->mean_next, 16)) || tree->n_levels < 1 ||
            tree->n_levels > kMaxLayers + 1)
            return HOPGNN_EINVAL;
        for (int h = 1; h < tree->n_levels; ++h)
            if (tree->fan[h] < 1 || tree->fan[h] > kTreeMaxFan) return HOPGNN_EINVAL;
    }
    if (dt == HOPGNN_F32) {
        // large tiles once there is enough work to fill 256 CUs twice over
        if (d_out > 64 && work >= 512)
            return launch_project_f32<128, 128, 16, 2>(vec, s, Hsrc, self_idx, mean, W_self, W_neigh, bias, n_dst, d_in, k_total, d_out, relu, zero, out, n_rows_dev, tree);
        return launch_project_f32<64, 64, 32, 2>(vec, s, Hsrc, self_idx, mean, W_self, W_neigh, bias, n_dst, d_in, k_total, d_out, relu, zero, out, n_rows_dev, tree);
    }
    const bool huge = d_out > 128 && work >= 1024;   // 256 x 256 tiles once they still fill 256 CUs
    const bool big = d_out > 64 && work >= 512;
    if (dt == HOPGNN_BF16) {
        if (huge) return launch_project_16<TrBF16, 256, 256, 64, 2, 4>(vec, s, Hsrc, self_idx, mean, Wt, KP, bias, n_dst, d_in, k_total, d_out, relu, zero, out, out_f32, n_rows_dev, tree);
        if (big) return launch_project_16<TrBF16, 128, 128, 64, 2, 2>(vec, s, Hsrc, self_idx, mean, Wt, KP, bias, n_dst, d_in, k_total, d_out, relu, zero, out, out_f32, n_rows_dev, tree);
        return launch_project_16<TrBF16, 64, 64, 64, 2, 2>(vec, s, Hsrc, self_idx, mean, Wt, KP, bias, n_dst, d_in, k_total, d_out, relu, zero, out, out_f32, n_rows_dev, tree);
    }
    if (huge) return launch_project_16<TrF16, 256, 256, 64, 2, 4>(vec, s, Hsrc, self_idx, mean, Wt, KP, bias, n_dst, d_in, k_total, d_out, relu, zero, out, out_f32, n_rows_dev, tree);
    if (big) return launch_project_16<TrF16, 128, 128, 64, 2, 2>(vec, s, Hsrc, self_idx, mean, Wt, KP, bias, n_dst, d_in, k_total, d_out, relu, zero, out, out_f32, n_rows_dev, tree);
    return launch_project_16<TrF16, 64, 64, 64, 2, 2>(vec, s, Hsrc, self_idx, mean, Wt, KP, bias, n_dst, d_in, k_total, d_out, relu, zero, out, out_f32, n_rows_dev, tree);
}

__global__ void __launch_bounds__(kMeanThreads)
prep_weights(TransposeJob job, uint32_t n_tiles, uint32_t* __restrict__ zero_row, int32_t zero_words) {
    if (blockIdx.x < n_tiles) {
        transpose_w_tile(job, blockIdx.x);
        return;
    }
    for (int32_t i = (blockIdx.x - n_tiles) * kMeanThreads + threadIdx.x; i < zero_words; i += kMeanThreads * (gridDim.x - n_tiles))
        zero_row[i] = 0u;
}

hopgnn_status launch_prep_weights(TransposeJob job, void* zero_row, size_t zero_bytes, hipStream_t s) {
    const uint32_t n_tiles = job.Wt != nullptr ? (uint32_t)(job.KP / 32) * (uint32_t)(job.NP / 32) : 0u;
    const uint32_t n_zero = zero_bytes > 0 ? 1u : 0u;
    if (n_tiles + n_zero == 0) return HOPGNN_OK;
    hipLaunchKernelGGL(prep_weights, dim3(n_tiles + n_zero), dim3(kMeanThreads), 0, s, job, n_tiles,
                       static_cast<uint32_t*>(zero_row), (int32_t)(zero_bytes / 4));
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

}  // namespace hopgnn

using namespace hopgnn;

static_assert(HOPGNN_AGG_MEAN == kAggOpMean && HOPGNN_AGG_SUM == kAggOpSum && HOPGNN_AGG_MAX == kAggOpMax,
              "aggregator codes");

extern "C" size_t hopgnn_sage_fwd_ws_bytes(hopgnn_dtype dt, int64_t n_dst, int32_t d_in, int32_t d_out) {
    if (n_dst < 0 || d_in < 1 || d_out < 1) return 0;
    return proj_ws_layout(dt, n_dst, d_in, 2 * d_in, d_out).total;
}

extern "C" hopgnn_status hopgnn_sage_fwd(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                         const int32_t* self_idx, const int32_t* indptr,
                                         const int32_t* idx, int64_t n_dst, const void* W_self,
                                         const void* W_neigh, const void* bias, int32_t d_out,
                                         int32_t relu, void* out, void* ws, size_t ws_bytes,
                                         void* stream) {
    return hopgnn_sage_fwd_agg(Hsrc, dt, n_src, d_in, self_idx, indptr, idx, n_dst, W_self, W_neigh, bias, d_out,
                               HOPGNN_AGG_MEAN, relu, out, ws, ws_bytes, stream);
}

extern "C" hopgnn_status hopgnn_sage_fwd_agg(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                             const int32_t* self_idx, const int32_t* indptr,
                                             const int32_t* idx, int64_t n_dst, const void* W_self,
                                             const void* W_neigh, const void* bias, int32_t d_out, int32_t agg,
                                             int32_t relu, void* out, void* ws, size_t ws_bytes,
                                             void* stream) {
    return hopgnn_sage_fwd_dev(Hsrc, dt, n_src, d_in, self_idx, indptr, idx, n_dst, nullptr, W_self, W_neigh, bias, d_out,
                               agg, relu, out, ws, ws_bytes, stream);
}

extern "C" hopgnn_status hopgnn_sage_fwd_dev(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                             const int32_t* self_idx, const int32_t* indptr,
                                             const int32_t* idx, int64_t n_dst, const int64_t* n_dst_dev,
                                             const void* W_self, const void* W_neigh, const void* bias,
                                             int32_t d_out, int32_t agg, int32_t relu, void* out, void* ws,
                                             size_t ws_bytes, void* stream) {
    return sage_fwd_marked(Hsrc, dt, n_src, d_in, self_idx, indptr, idx, n_dst, n_dst_dev, W_self, W_neigh, bias, d_out,
                           agg, relu, out, ws, ws_bytes, stream, nullptr);
}

namespace hopgnn {

static inline bool mark(hipEvent_t ev, hipStream_t s) { return ev == nullptr || hipEventRecord(ev, s) == hipSuccess; }

hopgnn_status sage_fwd_marked(const void* Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in, const int32_t* self_idx,
                              const int32_t* indptr, const int32_t* idx, int64_t n_dst, const int64_t* n_dst_dev,
                              const void* W_self, const void* W_neigh, const void* bias, int32_t d_out, int32_t agg,
                              int32_t relu, void* out, void* ws, size_t ws_bytes, void* stream,
                              const LayerMarks* marks) {
    if (agg != HOPGNN_AGG_MEAN && agg != HOPGNN_AGG_SUM && agg != HOPGNN_AGG_MAX) return HOPGNN_EINVAL;
    if (dt != HOPGNN_F32 && dt != HOPGNN_BF16 && dt != HOPGNN_F16) return HOPGNN_EINVAL;
    if (n_src < 0 || n_dst < 0 || d_in < 1 || d_out < 1) return HOPGNN_EINVAL;
    if (n_dst == 0) return HOPGNN_OK;
    if (indptr == nullptr || W_self == nullptr || W_neigh == nullptr || out == nullptr || ws == nullptr)
        return HOPGNN_EINVAL;
    if (n_src > 0 && Hsrc == nullptr) return HOPGNN_EINVAL;
    if (self_idx == nullptr && n_src < n_dst) return HOPGNN_EINVAL;   // identity self rows must exist
    if (n_dst >= ((int64_t)1 << 31) || n_src >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if (d_in > (1 << 20) || d_out > (1 << 20)) return HOPGNN_ERANGE;
    if (!aligned(ws, 256)) return HOPGNN_EINVAL;
    const ProjWs L = proj_ws_layout(dt, n_dst, d_in, 2 * d_in, d_out);
    if (ws_bytes < L.total) return HOPGNN_ENOMEM_WS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    void* mean = ws;
    if (n_src == 0) Hsrc = static_cast<char*>(ws) + L.agg_bytes + L.wt_bytes;   // nothing is read from it unmasked
    uint16_t* Wt = reinterpret_cast<uint16_t*>(static_cast<char*>(ws) + L.agg_bytes);
    void* zero = static_cast<char*>(ws) + L.agg_bytes + L.wt_bytes;

    TransposeJob job{};
    uint32_t n_tr = 0;
    if (dt != HOPGNN_F32) {
        job = TransposeJob{static_cast<const uint16_t*>(W_self), static_cast<const uint16_t*>(W_neigh), Wt, d_in,
                           d_out, L.KP, L.NP, 0u, 2 * d_in};
        n_tr = (uint32_t)(L.KP / 32) * (uint32_t)(L.NP / 32);
    }
    hopgnn_status st;
    const AggSpec spec{nullptr, 0, agg};     // the C ABI's aggregator codes are the kernel's op codes
    if (marks != nullptr && !mark(marks->agg_begin, s)) return HOPGNN_EHIP;
    if (dt == HOPGNN_F32) st = launch_mean<TrF32>(Hsrc, indptr, idx, n_dst, d_in, mean, zero, L.zero_bytes, job, n_tr, s, spec, n_dst_dev);
    else if (dt == HOPGNN_BF16) st = launch_mean<TrBF16>(Hsrc, indptr, idx, n_dst, d_in, mean, zero, L.zero_bytes, job, n_tr, s, spec, n_dst_dev);
    else st = launch_mean<TrF16>(Hsrc, indptr, idx, n_dst, d_in, mean, zero, L.zero_bytes, job, n_tr, s, spec, n_dst_dev);
    if (st != HOPGNN_OK) return st;
    if (marks != nullptr && (!mark(marks->agg_end, s) || !mark(marks->proj_begin, s))) return HOPGNN_EHIP;

    st = project_dispatch(dt, s, Hsrc, self_idx, mean, W_self, W_neigh, Wt, L.KP, bias, n_dst, d_in, 2 * d_in, d_out, relu,
                          zero, out, 0, n_dst_dev);
    if (st != HOPGNN_OK) return st;
    if (marks != nullptr && !mark(marks->proj_end, s)) return HOPGNN_EHIP;
    return HOPGNN_OK;
}

}  // namespace hopgnn
