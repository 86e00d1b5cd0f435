// Pieces shared by the W4A8 GEMM and GEMV translation units: the int4 -> int8 operand
// unpack of the prepacked weight layout and the dequantising epilogue (Eq. (3) scale choice,
// per-channel weight scale of Algorithm 1, the split terms of Rotation Magnitude Suppression).
#pragma once

#include <hip/hip_fp16.h>

#include <type_traits>

#include "mquant_internal.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

namespace mquant {

// 16 bytes of prepacked weights -> B operands of two MFMAs (values x16).
__device__ __forceinline__ void unpack_w4x16(const uint4 p, v4i &b0, v4i &b1)
{
    b0[0] = static_cast<int>((p.x << 4) & 0xF0F0F0F0u);
    b0[1] = static_cast<int>(p.x & 0xF0F0F0F0u);
    b0[2] = static_cast<int>((p.y << 4) & 0xF0F0F0F0u);
    b0[3] = static_cast<int>(p.y & 0xF0F0F0F0u);
    b1[0] = static_cast<int>((p.z << 4) & 0xF0F0F0F0u);
    b1[1] = static_cast<int>(p.z & 0xF0F0F0F0u);
    b1[2] = static_cast<int>((p.w << 4) & 0xF0F0F0F0u);
    b1[3] = static_cast<int>(p.w & 0xF0F0F0F0u);
}

__device__ __forceinline__ v4i as_v4i(const uint4 u)
{
    v4i r;
    r[0] = static_cast<int>(u.x);
    r[1] = static_cast<int>(u.y);
    r[2] = static_cast<int>(u.z);
    r[3] = static_cast<int>(u.w);
    return r;
}

// Row of the 32x32 MFMA result held in accumulator register r by k-group g.
__device__ __forceinline__ int acc_row(int r, int g) { return (r >> 2) * 8 + g * 4 + (r & 3); }

// fp16 round-to-nearest-even of an fp32 value that has ALREADY been rounded to fp32.  The
// empty asm keeps the compiler from merging the last fp32 multiply of the dequantisation
// with the conversion into one v_fma_mixlo_f16, which rounds the exact product once, straight
// to fp16: the defined result is the fp32 product rounded again (about 6 outputs in 10^5
// differ by one fp16 ulp otherwise).
__device__ __forceinline__ __half half_of_rounded_f32(float v)
{
    asm("" : "+v"(v));
    return __float2half_rn(v);
}

// Everything the dequantising epilogue needs besides the accumulator and the
// per-channel weight scale.  Activation scale of a row: the two static modality
// scales split at row n_vis (Eq. (3)), or, for the per-token dynamic baseline,
// one scale per row.  Rotation Magnitude Suppression (Sec. 3.2): n_split flagged
// input channels were zeroed in the main weight; each lives on as an int4 row
// split_w[j][0..N) (one byte per value) with one scale, and its product with the
// token's int8 code of that channel is added to the main path before the store.
constexpr int kEpiStatic = 0, kEpiRowScale = 1, kEpiSplit = 2;
constexpr int kMaxSplitChannels = 64;     // flagged channels per linear

struct Epilogue {
    int32_t n_vis;
    float s_vis, s_txt;
    const float *rows;          // nullptr: static scales
    int32_t n_split;            // 0: no split path
    int32_t K;
    const int8_t *xq;
    const int8_t *split_w;
    // Per-layer constants, passed by value so that a kernel reads them as scalars
    // instead of chasing two more pointers per output.
    int32_t split_idx[kMaxSplitChannels];
    float split_scale[kMaxSplitChannels];

    // EPI selects the code compiled into a kernel: the static path must not pay for
    // the pointer test and the split loop (measured: 10 % of the 1280 x 3584 x 37888 GEMM).
    template <int EPI>
    __device__ __forceinline__ float scale_of(int32_t row) const
    {
        if constexpr (EPI == kEpiRowScale) return rows[row];
        else return row < n_vis ? s_vis : s_txt;
    }
    // (float(acc) * s_row) * ws, plus the split terms in the order j = 0, 1, ...;
    // one rounding per operation.  row < T and n < N.
    template <int EPI>
    __device__ __forceinline__ float dequant(int32_t acc, float s_row, int32_t row, int32_t n,
                                             int32_t N, float ws) const
    {
        float v = (static_cast<float>(acc) * s_row) * ws;
        if constexpr (EPI == kEpiSplit) {
            for (int32_t j = 0; j < n_split; ++j) {
                const int32_t c = split_idx[j];           // validated on the host
                const int32_t p = static_cast<int32_t>(xq[static_cast<int64_t>(row) * K + c]) *
                                  static_cast<int32_t>(split_w[static_cast<int64_t>(j) * N + n]);
                v = v + (static_cast<float>(p) * s_row) * split_scale[j];
            }
        }
        return v;
    }
};

template <int EPI>
__device__ __forceinline__ void store_out(int32_t acc16, int32_t row, int32_t n, const Epilogue &ep,
                                          float ws, __half *y, int64_t ldy, int32_t *acc_out,
                                          int32_t N)
{
    const int32_t acc = acc16 >> 4;                       // exact: acc16 = 16 * acc
    const float s_row = ep.scale_of<EPI>(row);
    y[static_cast<int64_t>(row) * ldy + n] =
        half_of_rounded_f32(ep.dequant<EPI>(acc, s_row, row, n, N, ws));
    if (acc_out) acc_out[static_cast<int64_t>(row) * N + n] = acc;
}


// ---- the streaming GEMV of w4a8_gemv.hip (T <= kGemvStreamMaxT rows), also reached through
// the single-linear entry points
constexpr int kGemvStreamMaxT = 16;         // rows the streaming kernels take
constexpr int kGemvStreamLdsMaxT = 4;       // ... of which the form with xq resident in LDS
constexpr int kGemvMaxGroup = 4;            // linears per grouped launch

struct GemvProblem {
    const uint4 *wp;
    const __half *w_scale;
    __half *y;
    int32_t *acc_out;                       // optional raw accumulators [T, N]
    int64_t ldy;
    int32_t N;
    int32_t units;                          // work-groups of this linear (set by the dispatcher)
};

struct GemvGroup {
    GemvProblem p[kGemvMaxGroup];
    int32_t n;
};

// True when the streaming kernel handles this shape (else the callers use the tile kernel).
bool gemv_stream_takes(int32_t T, int32_t K, int64_t n_tiles);

// The linears of a group (one, or several sharing their input), front end (rotation with
// Hadamard block had_block in {1, 128, 512} + static quantizer) inside the launch.
// MQUANT_ERR_UNSUPPORTED when the shape is outside the kernel's range
// (gemv_stream_fused_takes): nothing was launched and the caller takes another path.
bool gemv_stream_fused_takes(int32_t T, int32_t K, int32_t had_block);
int gemv_stream_fused(const __half *x, int64_t ldx, int32_t T, int32_t K, int32_t had_block, const GemvGroup &grp,
                      const Epilogue &ep, float c_vis, float c_txt, hipStream_t stream);

template <int EPI>
int gemv_stream_dispatch(const int8_t *xq, int32_t T, int32_t K, GemvGroup grp, const Epilogue &ep,
                         hipStream_t stream);

// The tile GEMV kernel (every decode shape the streaming kernels do not take) for the same
// kind of group; defined next to the kernel in w4a8_gemm.hip.
template <int EPI>
int gemv_tile_dispatch(const int8_t *xq, int32_t T, int32_t K, GemvGroup grp, const Epilogue &ep,
                       hipStream_t stream);

}  // namespace mquant
