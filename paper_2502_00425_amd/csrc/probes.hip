// Measurement probes of the benchmark (not part of the method and not part of
// libmquant: built into their own shared object, libmquant_probes.so): what the
// chip attains on the resources the hot path is bound by, so that a kernel's rate
// can be set against the attainable figure as well as the published one.
//   - an MFMA-only loop of v_mfma_i32_32x32x32_i8 on caller-supplied operand data
//     (the matrix clock of this chip depends on the data: constant operands run at
//     the published rate, random int8 operands about 30 % below it);
//   - a read-only stream over a buffer (16 bytes per lane, non-temporal);
//   - an empty kernel (the launch-to-launch floor of back-to-back kernels).
#include "probes.h"

#include "mquant_internal.h"

using namespace mquant;

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// Eight independent accumulators per wave, operands rotating among eight register
// sets so that consecutive MFMAs see different data, as in a real product.
__global__ __launch_bounds__(256) void probe_mfma_kernel(int32_t iters, const v4i *__restrict__ data,
                                                         int32_t n_vec, int32_t *__restrict__ sink)
{
    v16i acc[8];
    v4i a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
        a[i] = data[(threadIdx.x * 8 + i) % n_vec];
        b[i] = data[(threadIdx.x * 8 + i + n_vec / 2 + blockIdx.x) % n_vec];
    }
    for (int32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[(i + 1) & 7], acc[i], 0, 0, 0);
    }
    int32_t s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 0x12345678) sink[0] = s;                 // keeps the loop alive, practically never taken
}

__global__ __launch_bounds__(256) void probe_read_kernel(const v4u *__restrict__ p, int64_t n_vec,
                                                         uint32_t *__restrict__ sink)
{
    v4u x = {0u, 0u, 0u, 0u};
    const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n_vec; i += stride) {
        const v4u t = __builtin_nontemporal_load(p + i);
        x ^= t;
    }
    if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x9e3779b9u) sink[0] = x[0];
}

__global__ void probe_empty_kernel() {}

constexpr int kProbeGroups = 1024;                    // 4 per CU, 4 waves each: 4 waves per SIMD

}  // namespace

extern "C" int64_t mqprobe_mfma_i8_ops(int32_t iters)
{
    if (iters < 0) return MQUANT_ERR_BAD_SHAPE;
    return static_cast<int64_t>(iters) * 8 * (2LL * 32 * 32 * 32) * 4 * kProbeGroups;
}

extern "C" int mqprobe_mfma_i8(int32_t iters, const void *data, int64_t data_bytes, int32_t *sink,
                                    mquant_stream_t stream)
{
    if (iters < 0 || data_bytes < 4096) return MQUANT_ERR_BAD_SHAPE;
    if (!data || !sink) return MQUANT_ERR_NULL;
    if (!aligned_to(data, 16)) return MQUANT_ERR_ALIGNMENT;
    const int64_t n_vec = data_bytes / 16;
    MQ_LAUNCH(probe_mfma_kernel, dim3(kProbeGroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters,
              static_cast<const v4i *>(data), static_cast<int32_t>(n_vec > (1 << 30) ? (1 << 30) : n_vec),
              sink);
    return launch_status();
}

extern "C" int mqprobe_hbm_read(const void *data, int64_t data_bytes, uint32_t *sink,
                                     mquant_stream_t stream)
{
    if (data_bytes < 0) return MQUANT_ERR_BAD_SHAPE;
    if (data_bytes == 0) return MQUANT_OK;
    if (!data || !sink) return MQUANT_ERR_NULL;
    if (!aligned_to(data, 16)) return MQUANT_ERR_ALIGNMENT;
    MQ_LAUNCH(probe_read_kernel, dim3(8 * 256), dim3(256), 0, static_cast<hipStream_t>(stream),
              static_cast<const v4u *>(data), data_bytes / 16, sink);
    return launch_status();
}

extern "C" int mqprobe_empty(int32_t groups, int32_t threads, mquant_stream_t stream)
{
    if (groups < 1 || threads < 64 || threads > 1024 || threads % 64 != 0) return MQUANT_ERR_BAD_SHAPE;
    MQ_LAUNCH(probe_empty_kernel, dim3(static_cast<unsigned>(groups)), dim3(static_cast<unsigned>(threads)), 0,
              static_cast<hipStream_t>(stream));
    return launch_status();
}
