// Weight-only W4 linear with group-wise scales (the weight-only setting of
// Table 13: int4 weight, one fp16 scale per 128 input channels of an output
// channel, 16-bit activations; group-wise granularity as in the appendix on
// quantization granularity).
//
//   W~[n, k] = fp16(wq[n, k] * s[n, k / 128])          (one rounding)
//   y[i, n]  = fp16(sum_k x[i, k] * W~[n, k])           (fp32 accumulation)
//
// Matrix core: v_mfma_f32_32x32x16_f16.  A = fp16 activations (M = tokens), staged
// through LDS; B = weights, dequantised in registers on their way into the MFMA.
// Lane l supplies row/column l % 32 and the 8 consecutive k of slot group l / 32.
// The contraction order inside a 64-channel k-tile is free as long as A and B
// agree: MFMA step s of a tile contracts channels {s*8..s*8+7} (lanes 0..31) and
// {32+s*8..32+s*8+7} (lanes 32..63), so that the 16 bytes a lane fetches from the
// prepacked weight are its B operands of all four steps.
//
// Prepacked weights: [n_tile][k_tile][lane][16 bytes] as for the W4A8 kernels
// (tile = 32 output x 64 input channels, lane (n % 32) + 32 * g holds channels
// 64*k_tile + 32*g .. +31 of row n), but inside a dword of 8 channels nibble j
// holds channel 2j and nibble j + 4 channel 2j + 1 (j = 0..3), each stored as
// code + 8.  (v >> 4j) & 0x000F000F then is a pair of adjacent channels in the
// two halves of a dword; OR-ing 0x6400 into each half makes the fp16 number
// 1024 + code + 8, from which 1032 is subtracted exactly before the multiply by
// the scale -- two packed fp16 operations per pair and no integer->float convert.
// The scale table follows the weight tiles, transposed to [K/128][N padded to 32]
// so that the 32 lanes of a tile read consecutive halves.
#include <hip/hip_fp16.h>

#include <atomic>

#include "mquant_internal.h"

using namespace mquant;

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

namespace {

constexpr int kGroup = 128;               // input channels per weight scale
constexpr int kAPitch = 272;              // bytes per LDS row of the A tile: 128 halves + 16 pad

// 16-byte reads of 16 consecutive rows at pitch 272 B start at banks 68 r mod 64 = 4 r:
// the 64 banks exactly once.

__global__ __launch_bounds__(256) void g128_prepack_kernel(
    const uint8_t *__restrict__ w, const __half *__restrict__ scales, uint32_t *__restrict__ out_w,
    __half *__restrict__ out_s, int32_t N, int32_t K, int32_t n_tiles, int32_t k_tiles)
{
    const int64_t total = static_cast<int64_t>(n_tiles) * k_tiles * 64 * 4;     // dwords
    const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
    for (int64_t o = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; o < total; o += stride) {
        const int d = static_cast<int>(o & 3);
        const int lane = static_cast<int>((o >> 2) & 63);
        const int64_t tile = o >> 8;
        const int32_t kt = static_cast<int32_t>(tile % k_tiles);
        const int32_t nt = static_cast<int32_t>(tile / k_tiles);
        const int32_t n = nt * kPackN + (lane & 31);
        const int32_t k0 = kt * kPackK + (lane >> 5) * 32 + d * 8;
        uint32_t v = 0x88888888u;                                   // code 0 everywhere
        if (n < N) {
            const uint32_t src =
                *reinterpret_cast<const uint32_t *>(w + static_cast<int64_t>(n) * (K / 2) + k0 / 2) ^
                0x88888888u;                                        // nibble c of src = channel k0 + c
            v = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v |= ((src >> (4 * (2 * j))) & 0xFu) << (4 * j);
                v |= ((src >> (4 * (2 * j + 1))) & 0xFu) << (4 * (j + 4));
            }
        }
        out_w[o] = v;
    }
    const int32_t n_pad = n_tiles * kPackN;
    const int64_t total_s = static_cast<int64_t>(K / kGroup) * n_pad;
    for (int64_t o = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; o < total_s; o += stride) {
        const int32_t n = static_cast<int32_t>(o % n_pad);
        const int32_t kg = static_cast<int32_t>(o / n_pad);
        out_s[o] = n < N ? scales[static_cast<int64_t>(n) * (K / kGroup) + kg] : __float2half(1.0f);
    }
}

// (a & mask) | c in one VALU operation (the compiler emits an AND and an OR when both
// constants are literals: a VOP3 instruction of this ISA takes no literal operand).
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t c)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(c));
    return r;
}

// One dword of prepacked weights -> 8 fp16 weights (channels in ascending order),
// each fp16(code * scale); s2 holds the scale in both halves.
__device__ __forceinline__ v4u dequant8(uint32_t v, v2h s2, uint32_t mask, uint32_t magic)
{
    const v2h bias = {static_cast<_Float16>(1032.0f), static_cast<_Float16>(1032.0f)};
    v4u out;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        v2h h = __builtin_bit_cast(v2h, and_or(v >> (4 * j), mask, magic));
        h = (h - bias) * s2;                      // the difference is exact; one rounding
        out[j] = __builtin_bit_cast(uint32_t, h);
    }
    return out;
}

__device__ __forceinline__ int acc_row(int r, int g) { return (r >> 2) * 8 + g * 4 + (r & 3); }

// Work-group id -> (tm, tn): the eight XCDs (work-groups are dealt to them round
// robin) each get a contiguous run of a tile order that walks bands of `band`
// tile-rows, so the tiles an XCD holds at a time share few row and column panels.
__device__ __forceinline__ void tile_of_group(int32_t id, int32_t tiles_m, int32_t tiles_n,
                                              int32_t band, int32_t &tm, int32_t &tn)
{
    const int32_t total = tiles_m * tiles_n;
    const int32_t per = total / 8, rem = total % 8;
    const int32_t xcd = id % 8, local = id / 8;
    const int32_t t = xcd * per + (xcd < rem ? xcd : rem) + local;
    const int32_t band_tiles = band * tiles_n;
    const int32_t b = t / band_tiles;
    const int32_t in_band = t - b * band_tiles;
    const int32_t rows = (tiles_m - b * band) < band ? (tiles_m - b * band) : band;
    tm = b * band + in_band % rows;
    tn = in_band / rows;
}

// Work-group tile BM x BN, WM x WN wavefronts.  K advances one scale group (128
// channels, two k-tiles) at a time; the A tile of the next group is fetched into
// registers while the current one is multiplied, then written to the other LDS
// buffer: one barrier per group.
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64, 2) void w4g128_gemm_kernel(
    const __half *__restrict__ x, int64_t ldx, const v4u *__restrict__ wp,
    const __half *__restrict__ sT, __half *__restrict__ y, int64_t ldy, int32_t T, int32_t N,
    int32_t K, int32_t tiles_m, int32_t tiles_n, int32_t n_tiles32, int32_t wide_store,
    int32_t band)
{
    constexpr int NW = WM * WN, NTHR = NW * 64;
    constexpr int MT = BM / WM / 32, NT = BN / WN / 32;
    constexpr int A_BUF = BM * kAPitch;
    constexpr int A_LOADS = BM * 16 / NTHR;           // 16-byte chunks of the A tile per thread
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && (BM * 16) % NTHR == 0, "tile shape");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];   // g128_lds_bytes<...>()

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;
    int32_t tm, tn;
    tile_of_group(blockIdx.x, tiles_m, tiles_n, band, tm, tn);
    const int32_t row0 = tm * BM;
    const int32_t ntile0 = tn * (BN / 32);
    const int32_t k_tiles = K / kPackK;
    const int32_t trips = K / kGroup;
    const int32_t n_pad = n_tiles32 * kPackN;

    // n-tiles of this wave, clamped to the last real tile (columns beyond N are never stored)
    int32_t my_tile[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int32_t t = ntile0 + wn * NT + nt;
        my_tile[nt] = t < n_tiles32 ? t : n_tiles32 - 1;
    }

    // Rows past T read row T - 1 again: their results are never stored.
    v4u areg[A_LOADS];
    const __half *arow[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int c = tid + i * NTHR;
        const int32_t row = row0 + (c >> 4);
        arow[i] = x + static_cast<int64_t>(row < T ? row : T - 1) * ldx + (c & 15) * 8;
    }
    auto load_a = [&](int32_t trip) {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            areg[i] = *reinterpret_cast<const v4u *>(arow[i] + static_cast<int64_t>(trip) * kGroup);
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const int c = tid + i * NTHR;
            *reinterpret_cast<v4u *>(smem + buf * A_BUF + (c >> 4) * kAPitch + (c & 15) * 16) = areg[i];
        }
    };
    auto load_b = [&](int32_t trip, v4u (&b)[2][NT]) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                b[kk][nt] = wp[(static_cast<int64_t>(my_tile[nt]) * k_tiles + 2 * trip + kk) * 64 + lane];
    };
    auto load_s = [&](int32_t trip, uint16_t (&s)[NT]) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            s[nt] = __builtin_bit_cast(
                uint16_t, sT[static_cast<int64_t>(trip) * n_pad + my_tile[nt] * kPackN + l32]);
    };

    v16f acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;

    const uint32_t mask = 0x000F000Fu;
    uint32_t magic = 0x64006400u;
    asm volatile("" : "+v"(magic));           // keep it in a VGPR (third operand of v_and_or_b32)

    // One scale group (eight MFMA steps) on LDS buffer `buf` with weights b and scales s.
    auto compute = [&](int buf, const v4u (&b)[2][NT], const uint16_t (&s)[NT]) {
        const uint8_t *abase = smem + buf * A_BUF + (wm * MT * 32 + l32) * kAPitch + g * 64;
        v2h s2[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const _Float16 v = __builtin_bit_cast(_Float16, s[nt]);
            s2[nt] = v2h{v, v};
        }
        // Operands of MFMA step i + 1 (A fragments from LDS, dequantised weights) are produced
        // while the MFMAs of step i run: a fragment read just before its MFMA would expose
        // the LDS latency once per MFMA.
        v8h bfr[2][NT], afr[2][MT];
        auto fetch = [&](int i) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                afr[i & 1][mt] = *reinterpret_cast<const v8h *>(abase + mt * 32 * kAPitch +
                                                                (i >> 2) * 128 + (i & 3) * 16);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                bfr[i & 1][nt] =
                    __builtin_bit_cast(v8h, dequant8(b[i >> 2][nt][i & 3], s2[nt], mask, magic));
        };
        fetch(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i < 7) fetch(i + 1);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(afr[i & 1][mt], bfr[i & 1][nt],
                                                                        acc[mt][nt], 0, 0, 0);
            // order inside the step: the next step's fragment reads first, then its VALU work
            // dealt between this step's MFMAs
            if (i < 7) {
                __builtin_amdgcn_sched_group_barrier(0x100, MT, 0);
#pragma unroll
                for (int j = 0; j < MT * NT; ++j) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, (16 * NT + MT * NT - 1) / (MT * NT), 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);      // nothing moves across steps: bounds the live operands
        }
    };

    // Two groups per loop trip with two register sets for the weights, so that no set is
    // copied and every wait is for loads issued a whole group earlier.  The last fetch of
    // a tile repeats the final group instead of branching; it is not used.  The scheduling
    // fences keep the fetches of the next group ahead of this group's arithmetic (the
    // compiler would otherwise sink them next to their LDS stores and expose the whole
    // memory latency).
    v4u b0[2][NT], b1[2][NT];
    uint16_t s0[NT], s1[NT];
    load_a(0);
    load_b(0, b0);
    load_s(0, s0);
    store_a(0);
    __syncthreads();

    for (int32_t t = 0; t < trips; t += 2) {
        const int32_t t1 = t + 1 < trips ? t + 1 : trips - 1;
        load_a(t1);
        load_b(t1, b1);
        load_s(t1, s1);
        __builtin_amdgcn_sched_barrier(0);
        compute(0, b0, s0);
        __builtin_amdgcn_sched_barrier(0);
        store_a(1);
        __syncthreads();
        if (t + 1 >= trips) break;

        const int32_t t2 = t + 2 < trips ? t + 2 : trips - 1;
        load_a(t2);
        load_b(t2, b0);
        load_s(t2, s0);
        __builtin_amdgcn_sched_barrier(0);
        compute(1, b1, s1);
        __builtin_amdgcn_sched_barrier(0);
        store_a(0);
        __syncthreads();
    }

    const int32_t wave_row0 = row0 + wm * (BM / WM);
    const int32_t wave_n0 = (ntile0 + wn * NT) * 32;

    if (!wide_store) {
        // every lane stores its own 2-byte results
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int32_t n = wave_n0 + nt * 32 + l32;
            if (n >= N) continue;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int32_t row = wave_row0 + mt * 32 + acc_row(r, g);
                    if (row < T) y[static_cast<int64_t>(row) * ldy + n] = __float2half_rn(acc[mt][nt][r]);
                }
        }
        return;
    }

    // Wide stores: the MFMA result has a lane per column; each wave turns 32 rows x
    // NT*32 columns through its own LDS patch (the A buffers are free after the last
    // barrier) and stores 16 bytes per lane.
    constexpr int ROWB = NT * 64 + 16;
    constexpr int LPR = NT * 64 / 16;
    constexpr int RPI = 64 / LPR;
    uint8_t *patch = smem + wave * (32 * ROWB);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = acc_row(r, g);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                *reinterpret_cast<__half *>(patch + rl * ROWB + (nt * 32 + l32) * 2) =
                    __float2half_rn(acc[mt][nt][r]);
        }
#pragma unroll
        for (int q = 0; q < 32 / RPI; ++q) {
            const int rl = q * RPI + lane / LPR;
            const int c = lane % LPR;
            const v4u v = *reinterpret_cast<const v4u *>(patch + rl * ROWB + c * 16);
            const int32_t row = wave_row0 + mt * 32 + rl;
            const int32_t n = wave_n0 + c * 8;
            if (row < T && n < N)                                  // N % 8 == 0 on this path
                *reinterpret_cast<v4u *>(y + static_cast<int64_t>(row) * ldy + n) = v;
        }
    }
}

// Decode shape (T <= 32): the weights are streamed once and nothing is reused.  One
// work-group owns one 32-channel tile, its NWAVES waves split K, and every wave requests
// a batch of KT k-tiles (activation fragments first, they hit L2; then the weights, with
// the non-temporal hint, and their scales) before it touches the first one.  Loads are
// branch free: k-tiles past a wave's range are clamped and their weights replaced by
// code 0, lanes whose token row is >= T read row T - 1 (rows >= T of the MFMA result
// are never stored).  The fp32 partial sums of the waves meet in LDS and are added in
// wave order.
template <int NWAVES, int KT>
__global__ __launch_bounds__(NWAVES * 64) void w4g128_gemv_kernel(
    const __half *__restrict__ x, int64_t ldx, const v4u *__restrict__ wp,
    const __half *__restrict__ sT, __half *__restrict__ y, int64_t ldy, int32_t T, int32_t N,
    int32_t K, int32_t n_pad)
{
    __shared__ float red[NWAVES][16][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int32_t ntile = blockIdx.x;
    const int32_t k_tiles = K / kPackK;
    const int32_t per_wave = (k_tiles + NWAVES - 1) / NWAVES;
    const int32_t kt_begin = wave * per_wave;
    int32_t kt_end = kt_begin + per_wave;
    kt_end = kt_end < k_tiles ? kt_end : k_tiles;
    const int32_t n = ntile * kPackN + l32;

    v16f acc0, acc1;                                      // two chains: no back-to-back dependent MFMAs
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        acc0[r] = 0.0f;
        acc1[r] = 0.0f;
    }
    const v4u *wtile = wp + static_cast<int64_t>(ntile) * k_tiles * 64 + lane;
    const __half *xrow = x + static_cast<int64_t>(l32 < T ? l32 : T - 1) * ldx + g * 32;
    const __half *scol = sT + ntile * kPackN + l32;
    const uint32_t mask = 0x000F000Fu;
    uint32_t magic = 0x64006400u;
    asm volatile("" : "+v"(magic));

    for (int32_t base = kt_begin; base < kt_end; base += KT) {
        v4u a[KT][4], b[KT];
        uint16_t sc[KT];
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            int32_t kt = base + u;
            kt = kt < kt_end ? kt : kt_end - 1;
#pragma unroll
            for (int st = 0; st < 4; ++st)
                a[u][st] = *reinterpret_cast<const v4u *>(xrow + kt * kPackK + st * 8);
        }
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            int32_t kt = base + u;
            kt = kt < kt_end ? kt : kt_end - 1;
            b[u] = __builtin_nontemporal_load(wtile + static_cast<int64_t>(kt) * 64);
            sc[u] = __builtin_bit_cast(uint16_t, scol[static_cast<int64_t>(kt / 2) * n_pad]);
        }
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            const bool live = base + u < kt_end;                     // wave-uniform
            const _Float16 sv = __builtin_bit_cast(_Float16, sc[u]);
            const v2h s2 = {sv, sv};
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const uint32_t code = live ? b[u][st] : 0x88888888u;
                const v8h bf = __builtin_bit_cast(v8h, dequant8(code, s2, mask, magic));
                const v8h af = __builtin_bit_cast(v8h, a[u][st]);
                if (st & 1) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf, acc1, 0, 0, 0);
                else acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf, acc0, 0, 0, 0);
            }
        }
        // all memory reads of the batch first, then the arithmetic
        __builtin_amdgcn_sched_group_barrier(0x020, 6 * KT, 0);
        __builtin_amdgcn_sched_group_barrier(0x00A, 20 * 4 * KT, 0);
    }

    const int rmax = T <= 8 ? 4 : (T <= 16 ? 8 : 16);     // accumulator registers that can hold a row < T
#pragma unroll
    for (int r = 0; r < 16; ++r)
        if (r < rmax) red[wave][r][lane] = acc0[r] + acc1[r];
    __syncthreads();
    for (int r = wave; r < rmax; r += NWAVES) {
        const int32_t row = acc_row(r, g);
        if (row < T && n < N) {
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < NWAVES; ++w) sum += red[w][r][lane];
            y[static_cast<int64_t>(row) * ldy + n] = __float2half_rn(sum);
        }
    }
}

template <int BM, int BN, int WM, int WN>
constexpr int g128_lds_bytes()
{
    constexpr int a = 2 * BM * kAPitch;                                   // two A buffers
    constexpr int patch = WM * WN * 32 * (BN / WN / 32 * 64 + 16);        // epilogue patches
    return a > patch ? a : patch;
}

template <int BM, int BN, int WM, int WN>
int launch_g128(const __half *x, int64_t ldx, const uint8_t *wp, __half *y, int64_t ldy, int32_t T,
                int32_t N, int32_t K, hipStream_t stream)
{
    const int32_t n_tiles32 = static_cast<int32_t>(ceil_div(N, kPackN));
    const int32_t tiles_m = static_cast<int32_t>(ceil_div(T, BM));
    const int32_t tiles_n = static_cast<int32_t>(ceil_div(N, BN));
    const int64_t w_bytes = static_cast<int64_t>(n_tiles32) * (K / kPackK) * kPackTileBytes;
    const __half *sT = reinterpret_cast<const __half *>(wp + w_bytes);
    const int32_t wide = (N % 8 == 0 && ldy % 8 == 0 && aligned_to(y, 16)) ? 1 : 0;
    const int32_t band = tiles_m < 4 ? tiles_m : 4;
    constexpr int lds = g128_lds_bytes<BM, BN, WM, WN>();
    auto kern = w4g128_gemm_kernel<BM, BN, WM, WN>;
    // Raising the dynamic LDS limit is idempotent: threads racing here at most repeat it.
    static std::atomic<bool> attr_set{false};
    if (lds > 64 * 1024 && !attr_set.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return MQUANT_ERR_HIP;
        attr_set.store(true, std::memory_order_release);
    }
    MQ_LAUNCH(kern, dim3(tiles_m * tiles_n), dim3(WM * WN * 64), lds,
              stream, x, ldx, reinterpret_cast<const v4u *>(wp), sT, y, ldy, T, N, K, tiles_m,
              tiles_n, n_tiles32, wide, band);
    return launch_status();
}

}  // namespace

extern "C" int64_t mquant_w4g128_prepacked_bytes(int32_t N, int32_t K)
{
    if (N < 0 || K < 0) return MQUANT_ERR_BAD_SHAPE;
    if (K % kGroup != 0) return MQUANT_ERR_UNSUPPORTED;
    const int64_t n_tiles = ceil_div(N, kPackN);
    return n_tiles * (K / kPackK) * kPackTileBytes + static_cast<int64_t>(K / kGroup) * n_tiles * kPackN * 2;
}

extern "C" int mquant_w4g128_prepack(const uint8_t *w, const void *scales, uint8_t *out, int32_t N,
                                     int32_t K, mquant_stream_t stream)
{
    if (N < 0 || K < 0) return MQUANT_ERR_BAD_SHAPE;
    if (K % kGroup != 0) return MQUANT_ERR_UNSUPPORTED;
    if (N == 0 || K == 0) return MQUANT_OK;
    if (!w || !scales || !out) return MQUANT_ERR_NULL;
    if (!aligned_to(w, 4) || !aligned_to(out, 16) || !aligned_to(scales, 2)) return MQUANT_ERR_ALIGNMENT;
    const int32_t n_tiles = static_cast<int32_t>(ceil_div(N, kPackN));
    const int32_t k_tiles = K / kPackK;
    const int64_t w_bytes = static_cast<int64_t>(n_tiles) * k_tiles * kPackTileBytes;
    const int64_t dwords = w_bytes / 4;
    const int grid = static_cast<int>(dwords / 256 < 4096 ? (dwords / 256 > 0 ? dwords / 256 : 1) : 4096);
    MQ_LAUNCH(g128_prepack_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), w,
              static_cast<const __half *>(scales), reinterpret_cast<uint32_t *>(out),
              reinterpret_cast<__half *>(out + w_bytes), N, K, n_tiles, k_tiles);
    return launch_status();
}

extern "C" int mquant_w4g128_gemm(const void *x, int64_t ldx, const uint8_t *wp, void *y,
                                  int64_t ldy, int32_t T, int32_t N, int32_t K,
                                  mquant_stream_t stream)
{
    if (T < 0 || N < 0 || K < 0 || ldx < K || ldy < N) return MQUANT_ERR_BAD_SHAPE;
    if (K % kGroup != 0) return MQUANT_ERR_UNSUPPORTED;
    if (T == 0 || N == 0) return MQUANT_OK;
    if (K == 0) return MQUANT_ERR_UNSUPPORTED;
    if (!x || !wp || !y) return MQUANT_ERR_NULL;
    if (!aligned_to(x, 16) || ldx % 8 != 0 || !aligned_to(wp, 16) || !aligned_to(y, 2))
        return MQUANT_ERR_ALIGNMENT;
    const __half *xh = static_cast<const __half *>(x);
    __half *yh = static_cast<__half *>(y);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Decode shapes stream the weights through the GEMV.  In the GEMM every wave owns 32
    // output channels of the tile (WM = 1): a weight is dequantised once
    // per work-group.
    const int32_t n_tiles32 = static_cast<int32_t>(ceil_div(N, kPackN));
    if (T <= 32 || (T <= 64 && n_tiles32 < 512)) {
        const int64_t w_bytes = static_cast<int64_t>(n_tiles32) * (K / kPackK) * kPackTileBytes;
        const __half *sT = reinterpret_cast<const __half *>(wp + w_bytes);
        const v4u *wt = reinterpret_cast<const v4u *>(wp);
        const int32_t n_pad = n_tiles32 * kPackN;
        // The GEMV holds 32 token rows (one MFMA M extent).  With few output tiles, up to 64
        // rows take two launches: that still beats a GEMM whose few tiles would each walk all
        // of K alone (18944 x 3584 at T = 64: 91 us against 129 us).
        for (int32_t t0 = 0; t0 < T; t0 += 32) {
            const int32_t tc = T - t0 < 32 ? T - t0 : 32;
            const __half *xc = xh + static_cast<int64_t>(t0) * ldx;
            __half *yc = yh + static_cast<int64_t>(t0) * ldy;
            // Many tiles: small work-groups with one k-tile in flight per wave keep the register
            // count low and several groups resident per CU (fastest on 1184 tiles x 56 k-tiles);
            // few tiles: sixteen waves split K.
            if (n_tiles32 >= 512)
                MQ_LAUNCH((w4g128_gemv_kernel<8, 1>), dim3(n_tiles32), dim3(512), 0, st, xc, ldx, wt,
                          sT, yc, ldy, tc, N, K, n_pad);
            else
                MQ_LAUNCH((w4g128_gemv_kernel<16, 2>), dim3(n_tiles32), dim3(1024), 0, st, xc, ldx,
                          wt, sT, yc, ldy, tc, N, K, n_pad);
            const int status = launch_status();
            if (status != MQUANT_OK) return status;
        }
        return MQUANT_OK;
    }
    if (T <= 64) return launch_g128<64, 128, 1, 4>(xh, ldx, wp, yh, ldy, T, N, K, st);
    // 96 x 256 when it fills more CUs per round than 128 x 256 (rounds over the CUs x tile
    // rows / measured relative efficiency): 1280 x 3584 makes 196 tiles instead of 140 and
    // runs 12 % faster; with thousands of tiles the taller tile wins by 15 %.
    const double c128 = static_cast<double>(ceil_div(ceil_div(T, 128) * ceil_div(N, 256), kNumCU)) * 128.0;
    const double c96 = static_cast<double>(ceil_div(ceil_div(T, 96) * ceil_div(N, 256), kNumCU)) * 96.0 / 0.9;
    int tile = c96 < c128 ? 1 : 0;
    const int32_t forced = tune_state().g128_tile.load(std::memory_order_relaxed);
    if (forced >= 0) tile = forced;
    if (tile == 1) return launch_g128<96, 256, 1, 8>(xh, ldx, wp, yh, ldy, T, N, K, st);
    return launch_g128<128, 256, 1, 8>(xh, ldx, wp, yh, ldy, T, N, K, st);
}
