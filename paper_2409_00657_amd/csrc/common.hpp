// Internal helpers shared by the HIP translation units of libhopgnn (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hopgnn.h"

#define HOPGNN_LAUNCH_CHECK()                                    \
    do {                                                         \
        if (hipGetLastError() != hipSuccess) return HOPGNN_EHIP; \
    } while (0)

namespace hopgnn {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kMaxLayers = 8;

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
static inline size_t dtype_size(hopgnn_dtype dt) { return dt == HOPGNN_F32 ? 4 : 2; }

}  // namespace hopgnn
