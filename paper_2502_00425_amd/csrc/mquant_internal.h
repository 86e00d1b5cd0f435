// Internal helpers shared by the HIP translation units of libmquant (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <stdint.h>

#include "mquant.h"

namespace mquant {

constexpr int kWave = 64;                 // CDNA wavefront width
constexpr int kNumCU = 256;               // compute units of an MI355X

static inline bool aligned_to(const void *p, uintptr_t a)
{
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

// Kernel launch that first drops whatever error an earlier, unrelated HIP call of
// this thread left behind (HIP keeps the last error per thread until it is read, so
// a failed query made by the caller's framework would otherwise be reported as ours).
#define MQ_LAUNCH(...)                      \
    do {                                    \
        (void)hipGetLastError();            \
        hipLaunchKernelGGL(__VA_ARGS__);    \
    } while (0)

// Status of the launch just made.  With MQUANT_DEBUG set in the environment the
// HIP error text goes to stderr as well (the C-ABI carries only the status code).
static inline int launch_status()
{
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return MQUANT_OK;
    if (getenv("MQUANT_DEBUG")) fprintf(stderr, "mquant: HIP error %d: %s\n", (int)e, hipGetErrorString(e));
    return MQUANT_ERR_HIP;
}

// Process-wide overrides of kernel choices (mquant_tune_set); -1 / 0 = cost model.
struct TuneState {
    std::atomic<int32_t> gemm_tile{-1};
    std::atomic<int32_t> gemm_nosplit{0};
    std::atomic<int32_t> g128_tile{-1};
    std::atomic<int32_t> gemv_variant{-1};
};
TuneState &tune_state();

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Geometry of the prepacked int4 weight layout (see w4a8_gemm.hip).
constexpr int kPackN = 32;                // output channels per packed tile (one MFMA N extent)
constexpr int kPackK = 64;                // input channels per packed tile (two 32x32x32 MFMAs)
constexpr int kPackTileBytes = kPackN * kPackK / 2;   // 1024: one 16-byte load per lane
constexpr int kMaxK = 65536;              // 16 * 128 * 8 * K < 2^31 must hold for the x16 unpack

}  // namespace mquant
