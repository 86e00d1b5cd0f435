// Wave-level building block of the online block-Hadamard rotation and the int8
// quantizer (MQuant Sec. 3.2; Eq. (2) with z = 0), shared by the front-end
// kernels and by the decode kernel that rotates and quantizes its own input.
//
// One wavefront owns 512 contiguous channels of one row (1024 when the block
// is 1024): lane l holds channels 8l..8l+7, so index bits 0-2 live in a lane's
// registers and bits 3-8 across the 64 lanes.  The butterflies run in the fixed
// stage order h = 1, 2, 4, ..., B/2, one fp32 add or subtract each, which is
// what makes the int8 codes reproducible bit for bit.  After load_rotate the registers
// of some lanes hold the exact negative of the rotated value (lane_sign_bit); absmax
// does not care and quant_store folds the sign into its multiplier.
#pragma once

#include <hip/hip_fp16.h>

#include "mquant_internal.h"

namespace mquant {

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

// Lanes whose values carry a minus sign after the in-row stages (see lane_stage): the
// parity of the lane-index bits those stages paired on.
template <int B>
__device__ __forceinline__ uint32_t lane_sign_bit(int lane)
{
    constexpr int bits = B >= 128 ? 15 : (B >= 64 ? 7 : (B >= 32 ? 3 : (B >= 16 ? 1 : 0)));
    return (__builtin_popcount(lane & bits) & 1) ? 0x80000000u : 0u;
}

// v[j] += c * (v[j] of lane ^ M) for the eight registers of a lane, one instruction per
// register: the DPP operand of v_fmac_f32 fetches the partner lane's value.  c is +-1, so
// the product is exact and the result is the correctly rounded sum or difference, as a
// separate add would give.  A DPP operand must not be read within two wait states of the
// VALU write that produced it, and the compiler does not see into the statement: the
// leading s_nop covers whatever wrote the registers last, and inside the block a register
// is read at least eight instructions after it was written.
#define MQ_FMAC8(CTRL)                                                                         \
    asm volatile("s_nop 1\n\t"                                                                 \
                 "v_fmac_f32_dpp %0, %0, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"            \
                 "v_fmac_f32_dpp %1, %1, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"            \
                 "v_fmac_f32_dpp %2, %2, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"            \
                 "v_fmac_f32_dpp %3, %3, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"            \
                 "v_fmac_f32_dpp %4, %4, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"            \
                 "v_fmac_f32_dpp %5, %5, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"            \
                 "v_fmac_f32_dpp %6, %6, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"            \
                 "v_fmac_f32_dpp %7, %7, %8 " CTRL " row_mask:0xf bank_mask:0xf"                \
                 : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]),     \
                   "+v"(v[6]), "+v"(v[7])                                                      \
                 : "v"(c))

template <int M>
__device__ __forceinline__ void fmac_lane_xor(float (&v)[8], float c)
{
    static_assert(M == 1 || M == 2 || M == 4 || M == 8, "in-row distance");
    if constexpr (M == 1) {
        MQ_FMAC8("quad_perm:[1,0,3,2]");
    } else if constexpr (M == 2) {
        MQ_FMAC8("quad_perm:[2,3,0,1]");
    } else if constexpr (M == 8) {
        MQ_FMAC8("row_ror:8");
    } else {
        // i -> 7 - i inside each group of 8 into temporaries, then the quad reversed as the
        // DPP operand of the multiply-add: i -> i ^ 4
        float t[8];
        asm volatile("s_nop 1\n\t"
                     "v_mov_b32_dpp %0, %8 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                     "v_mov_b32_dpp %1, %9 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                     "v_mov_b32_dpp %2, %10 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                     "v_mov_b32_dpp %3, %11 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                     "v_mov_b32_dpp %4, %12 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                     "v_mov_b32_dpp %5, %13 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                     "v_mov_b32_dpp %6, %14 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                     "v_mov_b32_dpp %7, %15 row_half_mirror row_mask:0xf bank_mask:0xf"
                     : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]),
                       "=&v"(t[6]), "=&v"(t[7])
                     : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]),
                       "v"(v[7]));
        asm volatile("s_nop 1\n\t"
                     "v_fmac_f32_dpp %0, %8, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
                     "v_fmac_f32_dpp %1, %9, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
                     "v_fmac_f32_dpp %2, %10, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
                     "v_fmac_f32_dpp %3, %11, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
                     "v_fmac_f32_dpp %4, %12, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
                     "v_fmac_f32_dpp %5, %13, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
                     "v_fmac_f32_dpp %6, %14, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
                     "v_fmac_f32_dpp %7, %15, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf"
                     : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]),
                       "+v"(v[6]), "+v"(v[7])
                     : "v"(t[0]), "v"(t[1]), "v"(t[2]), "v"(t[3]), "v"(t[4]), "v"(t[5]), "v"(t[6]),
                       "v"(t[7]), "v"(c));
    }
}
#undef MQ_FMAC8

template <int B, int M>
__device__ __forceinline__ void lane_stage(float (&v)[8], int lane)
{
    if constexpr (8 * M < B) {
        if constexpr (M < 16) {
            // Butterfly between lane l (lower index, bit M clear) and l ^ M: the lower lane
            // must end with a + b, the upper one with a - b, a being the lower lane's value.
            // Each lane computes mine + c * other with c = +1 (lower) or -1 (upper): the
            // lower lane gets a + b, the upper lane b - a = -(a - b).  The minus sign is
            // not repaired here: a value that is the exact negative of the true one stays
            // the exact negative through every later add and subtract (IEEE rounding is
            // symmetric), both partners of a later stage carry the same sign, and the
            // quantizer multiplies by a constant whose sign is flipped for those lanes
            // (lane_sign_bit).  One instruction per element and stage.
            const float c = (lane & M) ? -1.0f : 1.0f;
            fmac_lane_xor<M>(v, c);
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

    // The 16 bytes (8 fp16 channels) of chunk c of segment sidx that this lane owns; zeros past K.
    static __device__ __forceinline__ uint4 load_chunk(const __half *row, int32_t sidx, int c, int32_t K,
                                                       int lane, bool &in_range)
    {
        const int32_t k0 = sidx * SEG + c * 512 + lane * 8;
        in_range = k0 < K;
        return in_range ? *reinterpret_cast<const uint4 *>(row + k0) : make_uint4(0u, 0u, 0u, 0u);
    }

    __device__ __forceinline__ void set_chunk(int c, const uint4 raw, bool in_range)
    {
        valid[c] = in_range;
        const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 f = __half22float2(h2[j]);
            v[c][2 * j] = f.x;
            v[c][2 * j + 1] = f.y;
        }
    }

    // All stages h = 1 ... B/2 on the chunks set before.
    __device__ __forceinline__ void rotate(int lane)
    {
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

    __device__ __forceinline__ void load_rotate(const __half *row, int32_t sidx, int32_t K, int lane)
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            bool in_range;
            const uint4 raw = load_chunk(row, sidx, c, K, lane, in_range);
            set_chunk(c, raw, in_range);
        }
        rotate(lane);
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
                // lanes that hold the exact negative of the rotated value multiply by -cmul
                const float cm = __uint_as_float(__float_as_uint(cmul) ^ lane_sign_bit<B>(lane));
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float t = __builtin_amdgcn_fmed3f(v[c][j] * cm, q_lo, q_hi);
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

}  // namespace mquant
