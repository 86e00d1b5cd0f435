// AIFS (Attention-Invariant Flexible Switching, MQuant Sec. 3.1): index vector,
// row gather and causal-mask remap.  All three are pure index/byte work.
#include "mquant_internal.h"

using namespace mquant;

extern "C" int mquant_version(void) { return 200; }

#ifndef MQUANT_BUILD_ID
#define MQUANT_BUILD_ID "unknown"
#endif
extern "C" const char *mquant_build_id(void) { return MQUANT_BUILD_ID; }

namespace mquant {
TuneState &tune_state()
{
    static TuneState st;
    return st;
}
}  // namespace mquant

extern "C" int mquant_tune_set(int32_t key, int32_t value)
{
    TuneState &t = tune_state();
    switch (key) {
    case MQUANT_TUNE_GEMM_TILE:
        if (value < -1 || value > 4) return MQUANT_ERR_BAD_SHAPE;
        t.gemm_tile.store(value, std::memory_order_relaxed);
        return MQUANT_OK;
    case MQUANT_TUNE_GEMM_NOSPLIT:
        if (value < 0 || value > 1) return MQUANT_ERR_BAD_SHAPE;
        t.gemm_nosplit.store(value, std::memory_order_relaxed);
        return MQUANT_OK;
    case MQUANT_TUNE_G128_TILE:
        if (value < -1 || value > 1) return MQUANT_ERR_BAD_SHAPE;
        t.g128_tile.store(value, std::memory_order_relaxed);
        return MQUANT_OK;
    case MQUANT_TUNE_GEMV_VARIANT:
        if (value < -1 || value > 3) return MQUANT_ERR_BAD_SHAPE;
        t.gemv_variant.store(value, std::memory_order_relaxed);
        return MQUANT_OK;
    default: return MQUANT_ERR_BAD_SHAPE;
    }
}

extern "C" const char *mquant_status_string(int status)
{
    switch (status) {
    case MQUANT_OK: return "ok";
    case MQUANT_ERR_NULL: return "required pointer is NULL";
    case MQUANT_ERR_BAD_SHAPE: return "bad shape, leading dimension, span or scale";
    case MQUANT_ERR_UNSUPPORTED: return "shape or block size not supported by these kernels";
    case MQUANT_ERR_WORKSPACE: return "workspace missing or too small";
    case MQUANT_ERR_HIP: return "HIP runtime error";
    case MQUANT_ERR_ALIGNMENT: return "pointer or leading dimension not sufficiently aligned";
    default: return "unknown status";
    }
}

// Stable partition of 0..T-1: visual rows first (Sec. 3.1, E^u; index form in
// the appendix on rotary position embedding).  Host code, O(T).
extern "C" int mquant_aifs_build_perm(int32_t T, const mquant_span_t *vis, int32_t n_spans,
                                      int32_t *perm, int32_t *inv_perm, int32_t *n_vis)
{
    if (n_vis == nullptr) return MQUANT_ERR_NULL;
    if (T < 0 || n_spans < 0) return MQUANT_ERR_BAD_SHAPE;
    if (n_spans > 0 && vis == nullptr) return MQUANT_ERR_NULL;
    int64_t V = 0;
    int64_t prev_end = 0;
    for (int32_t s = 0; s < n_spans; ++s) {
        const int64_t b = vis[s].start, l = vis[s].len;
        if (l < 0 || b < prev_end || b + l > T) return MQUANT_ERR_BAD_SHAPE;
        prev_end = b + l;
        V += l;
    }
    *n_vis = static_cast<int32_t>(V);
    if (perm == nullptr && inv_perm == nullptr) return MQUANT_OK;
    // Walk the sequence once; a visual row goes to the next visual slot, a
    // text row to the next text slot behind all V visual ones.
    int64_t next_vis = 0, next_txt = V;
    int32_t s = 0;
    for (int32_t i = 0; i < T; ++i) {
        while (s < n_spans && i >= vis[s].start + vis[s].len) ++s;
        const bool is_vis = s < n_spans && i >= vis[s].start;
        const int64_t slot = is_vis ? next_vis++ : next_txt++;
        if (perm) perm[slot] = i;
        if (inv_perm) inv_perm[i] = static_cast<int32_t>(slot);
    }
    return MQUANT_OK;
}

namespace {

// One 16-byte chunk per thread; grid.y walks rows.
__global__ __launch_bounds__(256) void permute_rows_kernel(
    const uint4 *__restrict__ x, int64_t ldx16, uint4 *__restrict__ xu, int64_t ldxu16,
    const int32_t *__restrict__ perm, int32_t T, int32_t chunks)
{
    const int32_t c = blockIdx.x * 256 + threadIdx.x;
    if (c >= chunks) return;
    for (int32_t i = blockIdx.y; i < T; i += gridDim.y) {
        int32_t src = perm[i];
        src = (src < 0 || src >= T) ? 0 : src;
        xu[static_cast<int64_t>(i) * ldxu16 + c] = x[static_cast<int64_t>(src) * ldx16 + c];
    }
}

// Four output bytes per thread: M^u[i, j..j+3] = M[perm[i], perm[j..j+3]].
__global__ __launch_bounds__(256) void remap_mask_kernel(
    const uint8_t *__restrict__ mask, uint8_t *__restrict__ mask_u,
    const int32_t *__restrict__ perm, int32_t T)
{
    const int32_t j0 = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (j0 >= T) return;
    for (int32_t i = blockIdx.y; i < T; i += gridDim.y) {
        int32_t pi = perm[i];
        pi = (pi < 0 || pi >= T) ? 0 : pi;
        const uint8_t *row = mask + static_cast<int64_t>(pi) * T;
        uint8_t *out = mask_u + static_cast<int64_t>(i) * T + j0;
        if (j0 + 4 <= T && (T & 3) == 0) {
            const int4 pj = *reinterpret_cast<const int4 *>(perm + j0);
            const int32_t p[4] = {pj.x, pj.y, pj.z, pj.w};
            uint32_t v = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int32_t pq = (p[q] < 0 || p[q] >= T) ? 0 : p[q];
                v |= static_cast<uint32_t>(row[pq] != 0) << (8 * q);
            }
            *reinterpret_cast<uint32_t *>(out) = v;
        } else {
            for (int q = 0; q < 4 && j0 + q < T; ++q) {
                int32_t pq = perm[j0 + q];
                pq = (pq < 0 || pq >= T) ? 0 : pq;
                out[q] = row[pq] != 0;
            }
        }
    }
}

// The same remap for T % 16 == 0 with R output rows per work-group: their R source rows
// M[perm[i], :] are copied into LDS with 16-byte loads, and every thread then gathers four
// consecutive output bytes of each row from there.  The index vector is read once per R rows
// instead of once per row (it is four times the size of a mask row), and the byte gathers hit
// LDS instead of the memory pipeline.
template <int R>
__global__ __launch_bounds__(1024) void remap_mask_rows_kernel(
    const uint8_t *__restrict__ mask, uint8_t *__restrict__ mask_u,
    const int32_t *__restrict__ perm, int32_t T)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t rows[];      // R rows of T bytes
    const int tid = threadIdx.x;
    for (int32_t i0 = blockIdx.x * R; i0 < T; i0 += gridDim.x * R) {
        __syncthreads();                                                 // the previous rows are consumed
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (i0 + r < T) {                                            // uniform
                int32_t pi = perm[i0 + r];
                pi = (pi < 0 || pi >= T) ? 0 : pi;
                const uint4 *src = reinterpret_cast<const uint4 *>(mask + static_cast<int64_t>(pi) * T);
                for (int32_t c = tid; c < T / 16; c += 1024)
                    *reinterpret_cast<uint4 *>(rows + r * T + c * 16) = src[c];
            }
        }
        __syncthreads();
        for (int32_t j0 = tid * 4; j0 < T; j0 += 4096) {
            const int4 pj = *reinterpret_cast<const int4 *>(perm + j0);
            int32_t p[4] = {pj.x, pj.y, pj.z, pj.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) p[q] = (p[q] < 0 || p[q] >= T) ? 0 : p[q];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (i0 + r < T) {
                    const uint8_t *row = rows + r * T;
                    const uint32_t x = static_cast<uint32_t>(row[p[0]]) | (static_cast<uint32_t>(row[p[1]]) << 8) |
                                       (static_cast<uint32_t>(row[p[2]]) << 16) | (static_cast<uint32_t>(row[p[3]]) << 24);
                    // every byte -> 1 if non-zero, else 0
                    const uint32_t nz = ((((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x) & 0x80808080u) >> 7;
                    *reinterpret_cast<uint32_t *>(mask_u + static_cast<int64_t>(i0 + r) * T + j0) = nz;
                }
            }
        }
    }
}

template <int R>
int launch_remap_rows(const uint8_t *mask, uint8_t *mask_u, const int32_t *perm, int32_t T, hipStream_t stream)
{
    const size_t lds = static_cast<size_t>(R) * T;
    auto kern = remap_mask_rows_kernel<R>;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                144 * 1024) != hipSuccess)
            return MQUANT_ERR_HIP;
        attr_set.store(true, std::memory_order_release);
    }
    int64_t blocks = ceil_div(T, R);
    if (blocks > 8 * kNumCU) blocks = 8 * kNumCU;
    MQ_LAUNCH(kern, dim3(static_cast<unsigned>(blocks)), dim3(1024), lds, stream, mask, mask_u, perm, T);
    return launch_status();
}

}  // namespace

extern "C" int mquant_aifs_permute(const void *x, int64_t ldx, void *x_u, int64_t ldxu,
                                   const int32_t *perm, int32_t T, int32_t K,
                                   mquant_stream_t stream)
{
    if (T < 0 || K < 0) return MQUANT_ERR_BAD_SHAPE;
    if (T == 0 || K == 0) return MQUANT_OK;
    if (!x || !x_u || !perm) return MQUANT_ERR_NULL;
    if (ldx < K || ldxu < K) return MQUANT_ERR_BAD_SHAPE;
    if (x == x_u) return MQUANT_ERR_BAD_SHAPE;            // a gather cannot run in place
    if (K % 8 != 0) return MQUANT_ERR_UNSUPPORTED;
    if (ldx % 8 != 0 || ldxu % 8 != 0 || !aligned_to(x, 16) || !aligned_to(x_u, 16))
        return MQUANT_ERR_ALIGNMENT;
    const int32_t chunks = K / 8;
    dim3 grid(static_cast<unsigned>(ceil_div(chunks, 256)),
              static_cast<unsigned>(T < 65535 ? T : 65535));
    MQ_LAUNCH(permute_rows_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(x), ldx / 8, static_cast<uint4 *>(x_u), ldxu / 8,
                       perm, T, chunks);
    return launch_status();
}

extern "C" int mquant_aifs_remap_mask(const uint8_t *mask, uint8_t *mask_u, const int32_t *perm,
                                      int32_t T, mquant_stream_t stream)
{
    if (T < 0) return MQUANT_ERR_BAD_SHAPE;
    if (T == 0) return MQUANT_OK;
    if (!mask || !mask_u || !perm) return MQUANT_ERR_NULL;
    if (!aligned_to(mask_u, 4) || !aligned_to(perm, 16)) return MQUANT_ERR_ALIGNMENT;
    if (T % 16 == 0 && aligned_to(mask, 16) && T <= 144 * 1024) {
        hipStream_t hs = static_cast<hipStream_t>(stream);
        if (8 * static_cast<int64_t>(T) <= 144 * 1024) return launch_remap_rows<8>(mask, mask_u, perm, T, hs);
        if (4 * static_cast<int64_t>(T) <= 144 * 1024) return launch_remap_rows<4>(mask, mask_u, perm, T, hs);
        return launch_remap_rows<1>(mask, mask_u, perm, T, hs);
    }
    dim3 grid(static_cast<unsigned>(ceil_div(ceil_div(T, 4), 256)),
              static_cast<unsigned>(T < 65535 ? T : 65535));
    MQ_LAUNCH(remap_mask_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                       mask, mask_u, perm, T);
    return launch_status();
}
