// cbench: a torch-free driver of the C ABI for timing one entry point under rocprofv3.
//
//   cbench sage   <n_src> <n_dst> <d_in> <d_out> <f32|bf16|f16> <fanout> <iters>
//   cbench gather <n_rows> <n_uniq> <dim> <f32|bf16|f16> <iters> [capacity]
//          with a capacity, U is passed on the device and the launch is sized for the
//          capacity, as in a batch where the pre-gather count never visits the host
//   cbench pregather <n_ids> <n_vertices> <iters> [algo: 0 auto, 1 bitmap, 2 radix]
//   cbench batch <scale> <avg_degree> <dim> <f32|bf16|f16> <n_seeds> <fanouts f1,f2,..> <hidden> <iters> [streams]
//          whole batches (sample -> pregather -> gather -> layers) on a row-conditional R-MAT
//          graph (0.57, 0.19, 0.19, 0.05) built on the host, fresh seeds and key per batch
//   cbench copy <bytes> <iters>      plain 128-bit copy kernel of known size, to calibrate
//                                    the profiler's FETCH_SIZE / WRITE_SIZE counters; also the
//                                    copy rate this machine reaches (bytes read + written per second)
//   cbench mfma <f32|bf16|f16> <iters>   register-resident MFMA loop (no memory traffic): the
//                                    matrix rate this machine reaches with the instruction the
//                                    projection kernels use, against the published peak
//
// Inputs are pseudo-random with the right shapes; results are not checked here (the
// parity tests do that).  Prints the mean time per call measured with HIP events.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <chrono>
#include <string>
#include <vector>

#include "hopgnn.h"

#define CK(x)                                                                      \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                \
            exit(1);                                                               \
        }                                                                          \
    } while (0)

typedef float cb_floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 cb_bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 cb_halfx8 __attribute__((ext_vector_type(8)));

// Four independent accumulators per wave, operands in registers: nothing but MFMA issue.
// kind 0: v_mfma_f32_32x32x2_f32, 1: v_mfma_f32_32x32x16_bf16, 2: v_mfma_f32_32x32x16_f16.
template <int KIND>
__global__ void __launch_bounds__(256) mfma_loop(float* __restrict__ sink, int n_rounds) {
    cb_floatx16 acc[4];
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    const float a32 = 1.0f + threadIdx.x * 1e-6f, b32 = 0.5f;
    cb_bf16x8 a16b, b16b;
    cb_halfx8 a16h, b16h;
    for (int i = 0; i < 8; ++i) {
        a16b[i] = (__bf16)(1.0f + i * 0.001f);
        b16b[i] = (__bf16)0.5f;
        a16h[i] = (_Float16)(1.0f + i * 0.001f);
        b16h[i] = (_Float16)0.5f;
    }
    for (int r = 0; r < n_rounds; ++r) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (KIND == 0) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a32, b32, acc[j], 0, 0, 0);
                else if (KIND == 1) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a16b, b16b, acc[j], 0, 0, 0);
                else acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a16h, b16h, acc[j], 0, 0, 0);
            }
    }
    float s = 0.f;
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    if (s == 123.456f) sink[threadIdx.x] = s;      // keeps the loop alive; never true for these operands
}

__global__ void __launch_bounds__(256) plain_copy(const uint4* __restrict__ a, uint4* __restrict__ b, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) b[i] = a[i];
}

static uint64_t rng_state = 0x1234567;
static uint64_t rnd() {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return rng_state;
}

static hopgnn_dtype parse_dt(const char* s) {
    if (!strcmp(s, "f32")) return HOPGNN_F32;
    if (!strcmp(s, "bf16")) return HOPGNN_BF16;
    return HOPGNN_F16;
}

template <typename T>
static T* upload(const std::vector<T>& h) {
    T* d;
    CK(hipMalloc(&d, h.size() * sizeof(T) + 256));
    CK(hipMemcpy(d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
    return d;
}

// small finite values of the given type
static std::vector<uint8_t> random_table(size_t n, hopgnn_dtype dt) {
    const size_t es = dt == HOPGNN_F32 ? 4 : 2;
    std::vector<uint8_t> h(n * es);
    for (size_t i = 0; i < n; ++i) {
        const float f = (float)((int64_t)(rnd() % 2001) - 1000) * 1e-3f;
        if (dt == HOPGNN_F32) {
            memcpy(&h[i * 4], &f, 4);
        } else if (dt == HOPGNN_BF16) {
            uint32_t u;
            memcpy(&u, &f, 4);
            const uint16_t b = (uint16_t)(u >> 16);
            memcpy(&h[i * 2], &b, 2);
        } else {
            const _Float16 hf = (_Float16)f;
            memcpy(&h[i * 2], &hf, 2);
        }
    }
    return h;
}

template <typename F>
static double time_it(const char* what, int iters, F&& f) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    for (int i = 0; i < 3; ++i) f();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0, 0));
    for (int i = 0; i < iters; ++i) f();
    CK(hipEventRecord(e1, 0));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    printf("%s: %.2f us per call (%d calls)\n", what, ms * 1e3f / iters, iters);
    return (double)ms * 1e3 / iters;
}

int main(int argc, char** argv) {
    if (argc < 2) return 1;
    const std::string mode = argv[1];
    if (mode == "sage" && argc >= 9) {
        const int64_t n_src = atoll(argv[2]), n_dst = atoll(argv[3]);
        const int d_in = atoi(argv[4]), d_out = atoi(argv[5]);
        const hopgnn_dtype dt = parse_dt(argv[6]);
        const int fan = atoi(argv[7]), iters = atoi(argv[8]);
        const size_t es = dt == HOPGNN_F32 ? 4 : 2;
        auto H = upload(random_table((size_t)n_src * d_in, dt));
        auto Ws = upload(random_table((size_t)d_in * d_out, dt));
        auto Wn = upload(random_table((size_t)d_in * d_out, dt));
        std::vector<int32_t> indptr(n_dst + 1), idx((size_t)n_dst * fan), self(n_dst);
        for (int64_t r = 0; r <= n_dst; ++r) indptr[r] = (int32_t)(r * fan);
        for (auto& x : idx) x = (int32_t)(rnd() % n_src);
        for (auto& x : self) x = (int32_t)(rnd() % n_src);
        auto d_indptr = upload(indptr);
        auto d_idx = upload(idx);
        auto d_self = upload(self);
        void *out, *ws;
        const size_t wsb = hopgnn_sage_fwd_ws_bytes(dt, n_dst, d_in, d_out);
        CK(hipMalloc(&out, (size_t)n_dst * d_out * es));
        CK(hipMalloc(&ws, wsb));
        time_it("hopgnn_sage_fwd", iters, [&] {
            hopgnn_status st = hopgnn_sage_fwd(H, dt, n_src, d_in, d_self, d_indptr, d_idx, n_dst, Ws, Wn, nullptr,
                                               d_out, 1, out, ws, wsb, nullptr);
            if (st != HOPGNN_OK) { fprintf(stderr, "sage_fwd: %s\n", hopgnn_status_str(st)); exit(1); }
        });
        const double flop = 2.0 * n_dst * 2.0 * d_in * d_out;
        printf("projection flop per call: %.3f GFLOP; aggregate bytes per call: %.1f MB\n", flop / 1e9,
               (double)(n_dst * (fan + 1)) * d_in * es / 1e6);
    } else if (mode == "gather" && argc >= 7) {
        const int64_t n_rows = atoll(argv[2]), n_uniq = atoll(argv[3]);
        const int dim = atoi(argv[4]);
        const hopgnn_dtype dt = parse_dt(argv[5]);
        const int iters = atoi(argv[6]);
        const size_t es = dt == HOPGNN_F32 ? 4 : 2;
        void *X, *Xu;
        CK(hipMalloc(&X, (size_t)n_rows * dim * es));
        CK(hipMemset(X, 1, (size_t)n_rows * dim * es));
        CK(hipMalloc(&Xu, (size_t)n_uniq * dim * es));
        std::vector<int32_t> uniq(n_uniq);   // ascending sample of the rows
        for (int64_t i = 0; i < n_uniq; ++i) {
            const int64_t lo = i * n_rows / n_uniq, hi = (i + 1) * n_rows / n_uniq;
            uniq[i] = (int32_t)(lo + (int64_t)(rnd() % (uint64_t)(hi > lo ? hi - lo : 1)));
        }
        const int64_t cap = argc >= 8 ? atoll(argv[7]) : 0;
        if (cap > 0) uniq.resize(cap, 0);
        auto d_uniq = upload(uniq);
        int64_t* d_count = nullptr;
        if (cap > 0) {
            CK(hipFree(Xu));
            CK(hipMalloc(&Xu, (size_t)cap * dim * es));
            CK(hipMalloc(&d_count, 8));
            CK(hipMemcpy(d_count, &n_uniq, 8, hipMemcpyHostToDevice));
        }
        time_it("hopgnn_gather", iters, [&] {
            hopgnn_status st = hopgnn_gather(X, dt, n_rows, dim, dim, d_uniq, cap > 0 ? cap : n_uniq, d_count, Xu, nullptr);
            if (st != HOPGNN_OK) { fprintf(stderr, "gather: %s\n", hopgnn_status_str(st)); exit(1); }
        });
        printf("algorithmic bytes per call: %.1f MB\n", (double)n_uniq * (2.0 * dim * es + 4) / 1e6);
    } else if (mode == "pregather" && argc >= 5) {
        const int64_t n_ids = atoll(argv[2]), n_vertices = atoll(argv[3]);
        const int iters = atoi(argv[4]);
        const int algo = argc >= 6 ? atoi(argv[5]) : 0;
        std::vector<int32_t> ids(n_ids);
        for (auto& x : ids) {   // skewed towards low IDs like a power-law graph
            const double u = (double)(rnd() >> 11) / 9007199254740992.0;
            x = (int32_t)((double)n_vertices * u * u * u);
        }
        auto d_ids = upload(ids);
        int32_t *uniq, *remap;
        int64_t* n_uniq;
        void* ws;
        const size_t wsb = hopgnn_pregather_ws_bytes(n_ids, n_vertices, algo);
        CK(hipMalloc(&uniq, (size_t)n_ids * 4));
        CK(hipMalloc(&remap, (size_t)n_ids * 4));
        CK(hipMalloc(&n_uniq, 8));
        CK(hipMalloc(&ws, wsb));
        time_it("hopgnn_pregather", iters, [&] {
            hopgnn_status st = hopgnn_pregather(d_ids, n_ids, n_vertices, algo, uniq, n_uniq, remap, ws, wsb, nullptr);
            if (st != HOPGNN_OK) { fprintf(stderr, "pregather: %s\n", hopgnn_status_str(st)); exit(1); }
        });
    } else if (mode == "batch" && argc >= 10) {
        const int scale = atoi(argv[2]);
        const double avg_deg = atof(argv[3]);
        const int dim = atoi(argv[4]);
        const hopgnn_dtype dt = parse_dt(argv[5]);
        const int B = atoi(argv[6]);
        std::vector<int32_t> fan;
        for (char* tok = strtok(argv[7], ","); tok; tok = strtok(nullptr, ",")) fan.push_back(atoi(tok));
        const int hidden = atoi(argv[8]), iters = atoi(argv[9]);
        const int L = (int)fan.size();
        const size_t es = dt == HOPGNN_F32 ? 4 : 2;
        const int64_t N = (int64_t)1 << scale;
        // row-conditional R-MAT: degree of i = round(E * 0.76^zeros(i) * 0.24^ones(i)), each target bit is 0
        // with probability 0.75 where the source bit is 0 and 0.79 where it is 1
        std::vector<int64_t> off(N + 1, 0);
        for (int64_t i = 0; i < N; ++i) {
            const int ones = __builtin_popcountll((unsigned long long)i);
            double w = avg_deg * (double)N;
            for (int b = 0; b < scale; ++b) w *= b < ones ? 0.24 : 0.76;
            const double fl = (double)(int64_t)w;
            off[i + 1] = off[i] + (int64_t)fl + (((double)(rnd() >> 11) / 9007199254740992.0) < (w - fl) ? 1 : 0);
        }
        const int64_t E = off[N];
        std::vector<int32_t> ind(E);
        for (int64_t i = 0; i < N; ++i)
            for (int64_t e = off[i]; e < off[i + 1]; ++e) {
                const uint64_t r = rnd();
                int64_t dst = 0;
                for (int b = 0; b < scale; ++b) {
                    const unsigned u = (unsigned)((r >> (b * 3 % 61)) ^ (r >> ((b * 7 + 13) % 59))) & 1023u;
                    const unsigned thr = ((i >> b) & 1) ? 811u : 768u;   // 0.79 and 0.75 of 1024
                    if (u >= thr) dst |= (int64_t)1 << b;
                }
                ind[e] = (int32_t)dst;
            }
        printf("graph: %lld vertices, %lld edges\n", (long long)N, (long long)E);
        auto d_off = upload(off);
        auto d_ind = upload(ind);
        void* X;
        CK(hipMalloc(&X, (size_t)N * dim * es));
        CK(hipMemset(X, 0x3c, (size_t)N * dim * es));     // finite, non-zero values in every type
        const int n_streams = argc >= 11 ? atoi(argv[10]) : 1;
        const int64_t t_seed = hopgnn_slots_per_seed(fan.data(), L);
        const int64_t T = t_seed * B;
        std::vector<int64_t> lv(L + 1);
        lv[0] = B;
        for (int h = 1; h <= L; ++h) lv[h] = lv[h - 1] * fan[h - 1];
        const int64_t S = T - lv[L];
        const int64_t cap = T < N ? T : N;
        int32_t* seeds;
        CK(hipMalloc(&seeds, (size_t)B * 4 * 64));
        std::vector<int32_t> hseeds((size_t)B * 64);
        for (auto& x : hseeds) x = (int32_t)(rnd() % (uint64_t)N);
        CK(hipMemcpy(seeds, hseeds.data(), hseeds.size() * 4, hipMemcpyHostToDevice));
        std::vector<void*> Wsv(L), Wnv(L);
        for (int k = 1; k <= L; ++k) {
            const int din = k == 1 ? dim : hidden;
            Wsv[k - 1] = upload(random_table((size_t)din * hidden, dt));
            Wnv[k - 1] = upload(random_table((size_t)din * hidden, dt));
        }
        // one plan (its own buffers) and one stream per concurrent batch
        std::vector<hopgnn_batch_plan> plans(n_streams);
        std::vector<hipStream_t> streams(n_streams);
        std::vector<void*> outs(n_streams);
        for (int s = 0; s < n_streams; ++s) {
            hopgnn_batch_plan& p = plans[s];
            memset(&p, 0, sizeof p);
            p.graph = hopgnn_csr{N, E, d_off, 1, d_ind};
            p.X = X; p.dt = dt; p.dim = dim; p.ld_elems = dim;
            p.n_seeds = B; p.n_layers = L;
            p.pg_algo = 0; p.group = 1;
            CK(hipMalloc(&p.ids, T * 4)); CK(hipMalloc(&p.indptr, (S + 1) * 4));
            CK(hipMalloc(&p.slot_idx, (S + 1) * 4));
            CK(hipMalloc(&p.uniq, cap * 4)); CK(hipMalloc(&p.remap, T * 4)); CK(hipMalloc(&p.n_uniq, 8));
            p.uniq_capacity = cap;
            CK(hipMalloc(&p.Xu, (size_t)cap * dim * es));
            p.pg_ws_bytes = hopgnn_pregather_ws_bytes(T, N, 0);
            CK(hipMalloc(&p.pg_ws, p.pg_ws_bytes));
            if (!getenv("CBENCH_NO_CLEAN_WS")) {
                if (hopgnn_pregather_ws_init(p.pg_ws, p.pg_ws_bytes, T, N, 0, nullptr) != HOPGNN_OK) return 1;
                p.pg_ws_clean = 1;
            }
            for (int k = 1; k <= L; ++k) {
                int64_t nd = 0;
                for (int h = 0; h <= L - k; ++h) nd += lv[h];
                const int din = k == 1 ? dim : hidden;
                p.fanouts[k - 1] = fan[k - 1];
                p.d_out[k - 1] = hidden;
                p.W_self[k - 1] = Wsv[k - 1];
                p.W_neigh[k - 1] = Wnv[k - 1];
                CK(hipMalloc(&p.H[k - 1], (size_t)nd * hidden * es));
                const size_t bytes = hopgnn_sage_fwd_ws_bytes(dt, nd, din, hidden);
                p.sage_ws_bytes = bytes > p.sage_ws_bytes ? bytes : p.sage_ws_bytes;
            }
            CK(hipMalloc(&p.sage_ws, p.sage_ws_bytes));
            CK(hipMalloc(&outs[s], (size_t)B * hidden * es));
            CK(hipStreamCreate(&streams[s]));
        }
        auto run = [&](int it) {
            const int s = it % n_streams;
            const uint64_t key = (uint64_t)it;
            const hopgnn_status st = hopgnn_batch_fwd(&plans[s], seeds + (size_t)(it % 64) * B, &key, 1, outs[s], streams[s]);
            if (st != HOPGNN_OK) { fprintf(stderr, "batch: %s\n", hopgnn_status_str(st)); exit(1); }
        };
        for (int it = 0; it < 8; ++it) run(it);
        CK(hipDeviceSynchronize());
        const auto t0 = std::chrono::steady_clock::now();
        for (int it = 0; it < iters; ++it) run(8 + it);
        const auto t1 = std::chrono::steady_clock::now();
        CK(hipDeviceSynchronize());
        const auto t2 = std::chrono::steady_clock::now();
        printf("whole batch on %d stream(s): %.2f us per batch (%.2f us to issue), %d batches\n", n_streams,
               std::chrono::duration<double, std::micro>(t2 - t0).count() / iters,
               std::chrono::duration<double, std::micro>(t1 - t0).count() / iters, iters);
        if (getenv("CBENCH_GRAPH")) {
            // the same sequence captured once per stream and replayed (fixed key and seeds: timing only)
            std::vector<hipGraphExec_t> execs(n_streams);
            for (int s = 0; s < n_streams; ++s) {
                hipGraph_t gr;
                CK(hipStreamBeginCapture(streams[s], hipStreamCaptureModeThreadLocal));
                run(s);
                CK(hipStreamEndCapture(streams[s], &gr));
                CK(hipGraphInstantiate(&execs[s], gr, nullptr, nullptr, 0));
            }
            for (int it = 0; it < 8; ++it) CK(hipGraphLaunch(execs[it % n_streams], streams[it % n_streams]));
            CK(hipDeviceSynchronize());
            const auto g0 = std::chrono::steady_clock::now();
            for (int it = 0; it < iters; ++it) CK(hipGraphLaunch(execs[it % n_streams], streams[it % n_streams]));
            const auto g1 = std::chrono::steady_clock::now();
            CK(hipDeviceSynchronize());
            const auto g2 = std::chrono::steady_clock::now();
            printf("graph replay on %d stream(s): %.2f us per batch (%.2f us to issue)\n", n_streams,
                   std::chrono::duration<double, std::micro>(g2 - g0).count() / iters,
                   std::chrono::duration<double, std::micro>(g1 - g0).count() / iters);
        }
        int64_t U;
        CK(hipMemcpy(&U, plans[0].n_uniq, 8, hipMemcpyDeviceToHost));
        printf("slots per batch %lld, unique rows in the last batch on stream 0: %lld\n", (long long)T, (long long)U);
    } else if (mode == "copy" && argc >= 4) {
        const int64_t bytes = atoll(argv[2]) / 16 * 16;
        const int iters = atoi(argv[3]);
        void *a, *b;
        CK(hipMalloc(&a, bytes));
        CK(hipMalloc(&b, bytes));
        CK(hipMemset(a, 1, bytes));
        const int64_t n = bytes / 16;
        const double us = time_it("plain_copy", iters, [&] {
            hipLaunchKernelGGL(plain_copy, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, 0,
                               static_cast<const uint4*>(a), static_cast<uint4*>(b), n);
        });
        printf("copy rate: %.1f GB/s read + written\n", 2.0 * bytes / us * 1e-3);
        printf("bytes read = bytes written = %lld\n", (long long)bytes);
    } else if (mode == "mfma" && argc >= 4) {
        const std::string dt = argv[2];
        const int iters = atoi(argv[3]);
        const int kind = dt == "f32" ? 0 : dt == "bf16" ? 1 : 2;
        const int n_rounds = 2048, blocks = 256 * 8;            // 8 workgroups of 4 waves per CU
        float* sink;
        CK(hipMalloc(&sink, 1024));
        auto launch = [&] {
            if (kind == 0) hipLaunchKernelGGL(mfma_loop<0>, dim3(blocks), dim3(256), 0, 0, sink, n_rounds);
            else if (kind == 1) hipLaunchKernelGGL(mfma_loop<1>, dim3(blocks), dim3(256), 0, 0, sink, n_rounds);
            else hipLaunchKernelGGL(mfma_loop<2>, dim3(blocks), dim3(256), 0, 0, sink, n_rounds);
        };
        const double us = time_it("mfma_loop", iters, launch);
        const double flops_per_mfma = kind == 0 ? 32.0 * 32 * 2 * 2 : 32.0 * 32 * 16 * 2;
        const double flops = (double)blocks * 4 /*waves*/ * n_rounds * 16 /*MFMAs per round*/ * flops_per_mfma;
        printf("%s MFMA loop: %.1f TFLOP/s (%.3g flop in %.1f us)\n", dt.c_str(), flops / us * 1e-6, flops, us);
    } else {
        fprintf(stderr, "see the header of cbench.cpp for usage\n");
        return 1;
    }
    return 0;
}
