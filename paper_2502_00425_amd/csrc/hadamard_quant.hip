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

#include "mquant_internal.h"

using namespace mquant;

namespace {

template <int B>
__device__ __forceinline__ void register_stages(float (&v)[8])
{
    // h = 1, 2, 4 inside the lane's eight contiguous channels.
#pragma unroll
    for (int h = 1; h < 8 && h < B; h <<= 1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if ((j & h) == 0) {
                const float a = v[j], b = v[j + h];
                v[j] = a + b;
                v[j + h] = a - b;
            }
        }
    }
}

// Value of lane (l ^ M) for M in {1, 2, 4, 8, 16, 32}, without touching LDS
// memory: DPP quad/row permutes inside a row of 16 lanes, a swizzle across the
// two rows of a half-wave, the half-wave swap instruction across the halves.
template <int M>
__device__ __forceinline__ float lane_xor(float x, int lane)
{
    const int xi = __float_as_int(x);
    int r;
    if constexpr (M == 1) {
        r = __builtin_amdgcn_update_dpp(0, xi, 0xB1, 0xF, 0xF, true);       // quad_perm [1,0,3,2]
    } else if constexpr (M == 2) {
        r = __builtin_amdgcn_update_dpp(0, xi, 0x4E, 0xF, 0xF, true);       // quad_perm [2,3,0,1]
    } else if constexpr (M == 4) {
        // i -> 7 - i inside each group of 8, then reverse inside each quad: i -> i ^ 4
        const int t = __builtin_amdgcn_update_dpp(0, xi, 0x141, 0xF, 0xF, true);   // row_half_mirror
        r = __builtin_amdgcn_update_dpp(0, t, 0x1B, 0xF, 0xF, true);               // quad_perm [3,2,1,0]
    } else if constexpr (M == 8) {
        r = __builtin_amdgcn_update_dpp(0, xi, 0x128, 0xF, 0xF, true);      // row_ror:8
    } else if constexpr (M == 16) {
        r = __builtin_amdgcn_ds_swizzle(xi, 0x401F);                        // bit mode, xor 16
    } else {
        static_assert(M == 32, "lane_xor distance");
        // {x[0..31], x[0..31]} and {x[32..63], x[32..63]}
        const auto sw = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
        r = lane < 32 ? sw[1] : sw[0];
    }
    return __int_as_float(r);
}

template <int B, int M>
__device__ __forceinline__ void lane_stage(float (&v)[8], int lane)
{
    if constexpr (8 * M < B) {
        if constexpr (M < 16) {
            // The lane holding the lower index keeps a + b, the other one a - b with
            // a the lower-index value: other + (upper ? -mine : mine), one add each.
            const int sign = (lane & M) ? static_cast<int>(0x80000000u) : 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float other = lane_xor<M>(v[j], lane);
                const float mine = __int_as_float(__float_as_int(v[j]) ^ sign);
                v[j] = other + mine;
            }
        } else {
            // Partner lanes sit in different rows (M = 16) or wave halves (M = 32).
            // The row / half swap instructions exchange the odd rows (upper half)
            // of one register with the even rows (lower half) of another: applied to
            // (v[j], v[j+4]) it leaves every lane with a complete pair (a, b) -- the
            // lower-index lanes for register j, the upper-index lanes for j+4 --
            // so each lane does one add and one subtract, and the same swap puts the
            // results back where they belong.  No select, no LDS.
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int lo = __float_as_int(v[j]), hi = __float_as_int(v[j + 4]);
                float a, b;
                if constexpr (M == 16) {
                    const auto sw = __builtin_amdgcn_permlane16_swap(lo, hi, false, false);
                    a = __int_as_float(sw[0]);
                    b = __int_as_float(sw[1]);
                } else {
                    const auto sw = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
                    a = __int_as_float(sw[0]);
                    b = __int_as_float(sw[1]);
                }
                const int p = __float_as_int(a + b), q = __float_as_int(a - b);
                if constexpr (M == 16) {
                    const auto sw = __builtin_amdgcn_permlane16_swap(p, q, false, false);
                    v[j] = __int_as_float(sw[0]);
                    v[j + 4] = __int_as_float(sw[1]);
                } else {
                    const auto sw = __builtin_amdgcn_permlane32_swap(p, q, false, false);
                    v[j] = __int_as_float(sw[0]);
                    v[j + 4] = __int_as_float(sw[1]);
                }
            }
        }
    }
}

template <int B>
__device__ __forceinline__ void lane_stages(float (&v)[8], int lane)
{
    // h = 8, 16, ..., min(B, 512)/2: partner lane differs in bit h/8.
    lane_stage<B, 1>(v, lane);
    lane_stage<B, 2>(v, lane);
    lane_stage<B, 4>(v, lane);
    lane_stage<B, 8>(v, lane);
    lane_stage<B, 16>(v, lane);
    lane_stage<B, 32>(v, lane);
}

// One wave segment: SEG = max(B, 512) consecutive channels of one row, C = SEG/512
// chunks of 512, 8 channels per lane and chunk.  Loads fp16, rotates in fp32.
template <int B>
struct Segment {
    static constexpr int C = B > 512 ? B / 512 : 1;
    static constexpr int SEG = 512 * C;
    float v[C][8];
    bool valid[C];

    __device__ __forceinline__ void load_rotate(const __half *row, int32_t sidx, int32_t K, int lane)
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int32_t k0 = sidx * SEG + c * 512 + lane * 8;
            valid[c] = k0 < K;
            if (valid[c]) {
                const uint4 raw = *reinterpret_cast<const uint4 *>(row + k0);
                const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float2 f = __half22float2(h2[j]);
                    v[c][2 * j] = f.x;
                    v[c][2 * j + 1] = f.y;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[c][j] = 0.0f;
            }
        }
#pragma unroll
        for (int c = 0; c < C; ++c) {
            register_stages<B>(v[c]);
            lane_stages<B>(v[c], lane);
        }
        // h = 512, ...: across the wave segment's chunks.
#pragma unroll
        for (int hc = 1; hc < C; hc <<= 1) {
#pragma unroll
            for (int c = 0; c < C; ++c) {
                if ((c & hc) == 0) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float a = v[c][j], b = v[c + hc][j];
                        v[c][j] = a + b;
                        v[c + hc][j] = a - b;
                    }
                }
            }
        }
    }

    __device__ __forceinline__ float absmax(float m) const
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if (valid[c]) {
#pragma unroll
                for (int j = 0; j < 8; ++j) m = fmaxf(m, fabsf(v[c][j]));
            }
        }
        return m;
    }

    // int8 codes clamp(rne(v * cmul)) of this segment into row `xq_row`.
    __device__ __forceinline__ void quant_store(float cmul, int8_t *xq_row, int32_t sidx, int lane,
                                                float q_lo = -128.0f, float q_hi = 127.0f) const
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if (valid[c]) {
                // clamp(rint(t)) == rint(clamp(t)) for integer bounds; adding 1.5 * 2^23
                // rounds to an integer (ties to even) and leaves it in the low mantissa
                // bits, whose low byte is the two's-complement int8 code.
                uint32_t bits[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float t = __builtin_amdgcn_fmed3f(v[c][j] * cmul, q_lo, q_hi);
                    bits[j] = __float_as_uint(t + 12582912.0f);
                }
                uint32_t packed[2];
#pragma unroll
                for (int w = 0; w < 2; ++w) {
                    // byte 0 of four words -> one dword
                    const uint32_t p01 = __builtin_amdgcn_perm(bits[4 * w + 1], bits[4 * w], 0x0c0c0400u);
                    const uint32_t p23 = __builtin_amdgcn_perm(bits[4 * w + 3], bits[4 * w + 2], 0x04000c0cu);
                    packed[w] = p01 | p23;
                }
                const int64_t k0 = static_cast<int64_t>(sidx) * SEG + c * 512 + lane * 8;
                *reinterpret_cast<uint2 *>(xq_row + k0) = make_uint2(packed[0], packed[1]);
            }
        }
    }
};

template <int B, bool ABSMAX>
__global__ __launch_bounds__(256) void hadamard_quant_kernel(
    const __half *__restrict__ x, int64_t ldx, const int32_t *__restrict__ perm,
    int8_t *__restrict__ xq, int32_t T, int32_t K, int32_t n_vis, float c_vis, float c_txt,
    int32_t segs_per_row, float *__restrict__ absmax, float q_lo, float q_hi)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave0 = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    const int64_t total = static_cast<int64_t>(T) * segs_per_row;
    float wave_max = 0.0f;

    for (int64_t seg = wave0; seg < total; seg += static_cast<int64_t>(gridDim.x) * 4) {
        const int32_t i = static_cast<int32_t>(seg / segs_per_row);
        const int32_t sidx = static_cast<int32_t>(seg - static_cast<int64_t>(i) * segs_per_row);
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
    const int64_t total = static_cast<int64_t>(T) * segs_per_row;
    int64_t blocks = ceil_div(total, 4);
    if (blocks > (1 << 20)) blocks = 1 << 20;
    const dim3 grid(static_cast<unsigned>(blocks)), block(256);
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
