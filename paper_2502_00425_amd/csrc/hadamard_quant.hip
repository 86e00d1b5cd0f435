// Online block-Hadamard rotation fused with the modality-specific static int8
// quantizer (MQuant Sec. 3.2; Eq. (2) with z = 0; Eq. (3)), plus the rotated
// absmax statistic used to calibrate the static scales (Algorithm 1).
//
// One wavefront owns 512 contiguous channels of one row (1024 when the block
// is 1024): lane l holds channels 8l..8l+7, so index bits 0-2 live in a lane's
// registers and bits 3-8 across the 64 lanes.  The butterflies run in the fixed
// stage order h = 1, 2, 4, ..., B/2, one fp32 add or subtract each, which is
// what makes the int8 codes reproducible bit for bit.  The kernel is bound by
// HBM traffic: 2 bytes read and 1 byte written per element.
#include <hip/hip_fp16.h>
#include <math.h>

#include "hadamard_segment.h"
#include "mquant_internal.h"

using namespace mquant;

namespace {

// Grid: x walks the 512-channel (1024 for B = 1024) segments of a row, four per work-group
// (one per wave), y walks the rows.  Row and segment come straight from the block index: an
// earlier form flattened (row, segment) into one 64-bit index and paid a 64-bit division per
// segment, half of the kernel's instructions.
template <int B, bool ABSMAX>
__global__ __launch_bounds__(256) void hadamard_quant_kernel(
    const __half *__restrict__ x, int64_t ldx, const int32_t *__restrict__ perm,
    int8_t *__restrict__ xq, int32_t T, int32_t K, int32_t n_vis, float c_vis, float c_txt,
    int32_t segs_per_row, float *__restrict__ absmax, float q_lo, float q_hi)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t sidx = static_cast<int32_t>(blockIdx.x) * 4 + static_cast<int32_t>(threadIdx.x >> 6);
    float wave_max = 0.0f;

    if (sidx < segs_per_row) {                            // wave-uniform
        for (int32_t i = blockIdx.y; i < T; i += gridDim.y) {
            int32_t src = i;
            if (perm != nullptr) {
                src = perm[i];
                src = (src < 0 || src >= T) ? 0 : src;
            }
            Segment<B> sg;
            sg.load_rotate(x + static_cast<int64_t>(src) * ldx, sidx, K, lane);
            if constexpr (ABSMAX) {
                wave_max = sg.absmax(wave_max);
            } else {
                sg.quant_store((i < n_vis) ? c_vis : c_txt, xq + static_cast<int64_t>(i) * K, sidx, lane,
                               q_lo, q_hi);
            }
        }
    }

    if constexpr (ABSMAX) {
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) wave_max = fmaxf(wave_max, __shfl_xor(wave_max, m, kWave));
        // non-negative floats order like their bit patterns
        if (lane == 0) atomicMax(reinterpret_cast<unsigned int *>(absmax), __float_as_uint(wave_max));
    }
}

// Per-token dynamic quantization (the baseline the paper's speed tables compare
// against; Sec. 2.2 and the appendix on quantization granularity): one
// work-group per token.  Its four waves rotate the token's segments and keep
// them in registers (NS segments per wave), the row maximum meets in LDS, the
// scale s_i = fp32(max / sqrt(B) / 127) and the multiplier fp32(1 / (s_i sqrt(B)))
// are formed in double, and the codes are written from the registers: the token
// is read once, like in the static kernel, but nothing can be stored before the
// whole token has been seen.  An all-zero token gets s_i = 1.
template <int B, int NS>
__global__ __launch_bounds__(256) void hadamard_dynquant_kernel(
    const __half *__restrict__ x, int64_t ldx, const int32_t *__restrict__ perm,
    int8_t *__restrict__ xq, float *__restrict__ row_scale, int32_t T, int32_t K,
    int32_t segs_per_row, double sqrt_b)
{
    __shared__ float wave_max[4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    for (int32_t i = blockIdx.x; i < T; i += gridDim.x) {
        int32_t src = i;
        if (perm != nullptr) {
            src = perm[i];
            src = (src < 0 || src >= T) ? 0 : src;
        }
        const __half *row = x + static_cast<int64_t>(src) * ldx;
        Segment<B> sg[NS];
        float m = 0.0f;
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            const int32_t sidx = wave + 4 * q;
            if (sidx < segs_per_row) {               // wave-uniform
                sg[q].load_rotate(row, sidx, K, lane);
                m = sg[q].absmax(m);
            }
        }
#pragma unroll
        for (int sh = 32; sh >= 1; sh >>= 1) m = fmaxf(m, __shfl_xor(m, sh, kWave));
        if (lane == 0) wave_max[wave] = m;
        __syncthreads();
        const float a = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
        __syncthreads();                              // wave_max is reused by the next token
        float s = 1.0f, cmul = 1.0f;
        if (a > 0.0f) {
            s = static_cast<float>(static_cast<double>(a) / sqrt_b / 127.0);
            cmul = static_cast<float>(1.0 / (static_cast<double>(s) * sqrt_b));
        }
        if (threadIdx.x == 0) row_scale[i] = s;
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            const int32_t sidx = wave + 4 * q;
            if (sidx < segs_per_row) sg[q].quant_store(cmul, xq + static_cast<int64_t>(i) * K, sidx, lane);
        }
    }
}

template <bool ABSMAX>
int launch(const void *x, int64_t ldx, const int32_t *perm, int8_t *xq, int32_t T, int32_t K,
           int32_t n_vis, float c_vis, float c_txt, int32_t B, float *absmax, hipStream_t stream,
           int32_t bits = 8)
{
    const int32_t seg = B > 512 ? B : 512;
    const int32_t segs_per_row = static_cast<int32_t>(ceil_div(K, seg));
    const dim3 grid(static_cast<unsigned>(ceil_div(segs_per_row, 4)), static_cast<unsigned>(T < 65535 ? T : 65535)),
        block(256);
    const __half *xh = static_cast<const __half *>(x);
    const float q_hi = static_cast<float>((1 << (bits - 1)) - 1), q_lo = -static_cast<float>(1 << (bits - 1));
#define MQ_CASE(BV)                                                                          \
    case BV:                                                                                 \
        MQ_LAUNCH((hadamard_quant_kernel<BV, ABSMAX>), grid, block, 0, stream, xh,  \
                           ldx, perm, xq, T, K, n_vis, c_vis, c_txt, segs_per_row, absmax,   \
                           q_lo, q_hi);                                                      \
        break;
    switch (B) {
        MQ_CASE(1) MQ_CASE(2) MQ_CASE(4) MQ_CASE(8) MQ_CASE(16) MQ_CASE(32) MQ_CASE(64)
        MQ_CASE(128) MQ_CASE(256) MQ_CASE(512) MQ_CASE(1024)
    default: return MQUANT_ERR_UNSUPPORTED;
    }
#undef MQ_CASE
    return launch_status();
}

int check_common(const void *x, int64_t ldx, int32_t T, int32_t K, int32_t B)
{
    if (T < 0 || K < 0) return MQUANT_ERR_BAD_SHAPE;
    if (B < 1 || B > 1024 || (B & (B - 1)) != 0) return MQUANT_ERR_UNSUPPORTED;
    if (K % B != 0 || K % 8 != 0) return MQUANT_ERR_UNSUPPORTED;
    if (T == 0 || K == 0) return MQUANT_OK;
    if (!x) return MQUANT_ERR_NULL;
    if (ldx < K) return MQUANT_ERR_BAD_SHAPE;
    if (ldx % 8 != 0 || !aligned_to(x, 16)) return MQUANT_ERR_ALIGNMENT;
    return MQUANT_OK;
}

}  // namespace

extern "C" int mquant_hadamard_quant_act(const void *x, int64_t ldx, const int32_t *perm,
                                         int8_t *xq, int32_t T, int32_t K, int32_t n_vis,
                                         float s_vis, float s_txt, int32_t had_block,
                                         mquant_stream_t stream)
{
    return mquant_hadamard_quant_act_bits(x, ldx, perm, xq, T, K, n_vis, s_vis, s_txt, had_block, 8,
                                          stream);
}

extern "C" int mquant_hadamard_quant_act_bits(const void *x, int64_t ldx, const int32_t *perm,
                                              int8_t *xq, int32_t T, int32_t K, int32_t n_vis,
                                              float s_vis, float s_txt, int32_t had_block,
                                              int32_t act_bits, mquant_stream_t stream)
{
    if (act_bits < 2 || act_bits > 8) return MQUANT_ERR_UNSUPPORTED;
    const int st = check_common(x, ldx, T, K, had_block);
    if (st != MQUANT_OK) return st;
    if (n_vis < 0 || n_vis > T) return MQUANT_ERR_BAD_SHAPE;
    if (!(s_vis > 0.0f) || !(s_txt > 0.0f) || !isfinite(s_vis) || !isfinite(s_txt))
        return MQUANT_ERR_BAD_SHAPE;
    if (T == 0 || K == 0) return MQUANT_OK;
    if (!xq) return MQUANT_ERR_NULL;
    if (!aligned_to(xq, 8)) return MQUANT_ERR_ALIGNMENT;
    // 1 / (s * sqrt(B)) in double, rounded once to fp32.
    const double rb = sqrt(static_cast<double>(had_block));
    const float c_vis = static_cast<float>(1.0 / (static_cast<double>(s_vis) * rb));
    const float c_txt = static_cast<float>(1.0 / (static_cast<double>(s_txt) * rb));
    return launch<false>(x, ldx, perm, xq, T, K, n_vis, c_vis, c_txt, had_block, nullptr,
                         static_cast<hipStream_t>(stream), act_bits);
}

// Eq. (2): s = max|x_rot| / (2^(b-1) - 1), x_rot = u / sqrt(B); double, one rounding.
extern "C" int mquant_static_scale_from_absmax(float absmax_u, int32_t had_block, int32_t act_bits,
                                               float *scale)
{
    if (!scale) return MQUANT_ERR_NULL;
    if (had_block < 1 || had_block > 1024 || (had_block & (had_block - 1)) != 0)
        return MQUANT_ERR_UNSUPPORTED;
    if (act_bits < 2 || act_bits > 8) return MQUANT_ERR_UNSUPPORTED;
    if (!(absmax_u >= 0.0f) || !isfinite(absmax_u)) return MQUANT_ERR_BAD_SHAPE;
    const double q_max = static_cast<double>((1 << (act_bits - 1)) - 1);
    *scale = static_cast<float>(static_cast<double>(absmax_u) / sqrt(static_cast<double>(had_block)) / q_max);
    return MQUANT_OK;
}

extern "C" int mquant_hadamard_absmax(const void *x, int64_t ldx, int32_t T, int32_t K,
                                      int32_t had_block, float *absmax, mquant_stream_t stream)
{
    const int st = check_common(x, ldx, T, K, had_block);
    if (st != MQUANT_OK) return st;
    if (T == 0 || K == 0) return MQUANT_OK;
    if (!absmax) return MQUANT_ERR_NULL;
    return launch<true>(x, ldx, nullptr, nullptr, T, K, 0, 0.0f, 0.0f, had_block, absmax,
                        static_cast<hipStream_t>(stream));
}

extern "C" int mquant_hadamard_dynquant_act(const void *x, int64_t ldx, const int32_t *perm,
                                            int8_t *xq, float *row_scale, int32_t T, int32_t K,
                                            int32_t had_block, mquant_stream_t stream)
{
    const int st = check_common(x, ldx, T, K, had_block);
    if (st != MQUANT_OK) return st;
    if (T == 0 || K == 0) return MQUANT_OK;
    if (!xq || !row_scale) return MQUANT_ERR_NULL;
    if (!aligned_to(xq, 8) || !aligned_to(row_scale, 4)) return MQUANT_ERR_ALIGNMENT;
    const int32_t seg = had_block > 512 ? had_block : 512;
    const int32_t segs_per_row = static_cast<int32_t>(ceil_div(K, seg));
    const int32_t per_wave = static_cast<int32_t>(ceil_div(segs_per_row, 4));
    if (per_wave > 16) return MQUANT_ERR_UNSUPPORTED;     // a token must fit the registers of a group
    const dim3 grid(static_cast<unsigned>(T < (1 << 20) ? T : (1 << 20))), block(256);
    const __half *xh = static_cast<const __half *>(x);
    const double sqrt_b = sqrt(static_cast<double>(had_block));
    hipStream_t hs = static_cast<hipStream_t>(stream);
#define MQ_CASE(BV)                                                                              \
    case BV:                                                                                     \
        if (per_wave <= 4)                                                                       \
            MQ_LAUNCH((hadamard_dynquant_kernel<BV, 4>), grid, block, 0, hs, xh, ldx, perm, xq,  \
                      row_scale, T, K, segs_per_row, sqrt_b);                                    \
        else                                                                                     \
            MQ_LAUNCH((hadamard_dynquant_kernel<BV, 16>), grid, block, 0, hs, xh, ldx, perm, xq, \
                      row_scale, T, K, segs_per_row, sqrt_b);                                    \
        break;
    switch (had_block) {
        MQ_CASE(1) MQ_CASE(2) MQ_CASE(4) MQ_CASE(8) MQ_CASE(16) MQ_CASE(32) MQ_CASE(64)
        MQ_CASE(128) MQ_CASE(256) MQ_CASE(512)
    case 1024:                       // two chunks per segment: half as many segments fit
        if (per_wave > 8) return MQUANT_ERR_UNSUPPORTED;
        if (per_wave <= 2)
            MQ_LAUNCH((hadamard_dynquant_kernel<1024, 2>), grid, block, 0, hs, xh, ldx, perm, xq,
                      row_scale, T, K, segs_per_row, sqrt_b);
        else
            MQ_LAUNCH((hadamard_dynquant_kernel<1024, 8>), grid, block, 0, hs, xh, ldx, perm, xq,
                      row_scale, T, K, segs_per_row, sqrt_b);
        break;
    default: return MQUANT_ERR_UNSUPPORTED;
    }
#undef MQ_CASE
    return launch_status();
}
