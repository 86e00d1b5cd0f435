// W4A8 GEMM / GEMV with fused dequantisation (MQuant Sec. 4: "W4A8 GEMM",
// "custom W4A8 GEMV kernel"; Eq. (3) for the per-modality activation scale;
// per-channel weight scale of Algorithm 1).
//
//   acc[i, n] = sum_k xq[i, k] * wq[n, k]           (int32, exact)
//   y[i, n]   = fp16((float(acc) * s_i) * w_scale[n]),  s_i = s_vis (i < n_vis) or s_txt
//
// Matrix core: v_mfma_i32_32x32x32_i8.  A = int8 activations (M = tokens),
// B = weights (N = output channels).  Lane l supplies row/column l % 32 and the
// 16 consecutive k of k-group l / 32; it receives column l % 32 of the 32x32
// result, rows (r / 4) * 8 + (l / 32) * 4 + r % 4 for accumulator register r.
//
// Prepacked weights.  A tile is 32 output channels x 64 input channels = 1 KiB,
// stored as [n_tile][k_tile][lane][16 bytes]: lane (n % 32) + 32 * g holds the
// 32 channels k = 64 * k_tile + 32 * g .. + 31 of output row n, i.e. exactly
// the B operands of two MFMAs, fetched with one 16-byte load per lane (1 KiB
// contiguous per wavefront).  Inside each dword of 8 channels the nibbles are
// interleaved (nibble 2j = channel j, nibble 2j+1 = channel 4+j) so that
//     lo = (v << 4) & 0xF0F0F0F0   -> bytes 16*w[0..3]
//     hi =  v       & 0xF0F0F0F0   -> bytes 16*w[4..7]
// are ready-made int8 operands.  The accumulator therefore holds 16 * acc and
// is shifted right by 4 (exact) in the epilogue; 16 * 128 * 8 * K < 2^31 for
// K <= 65536.
#include <hip/hip_fp16.h>
#include <math.h>
#include <stdlib.h>

#include <atomic>

#include "hadamard_segment.h"
#include "mquant_internal.h"
#include "lds_dma.h"
#include "w4a8_common.h"

using namespace mquant;

namespace {

// ------------------------------------------------------------------ prepack

__global__ __launch_bounds__(256) void prepack_kernel(
    const uint8_t *__restrict__ w, uint32_t *__restrict__ out, int32_t N, int32_t K,
    int32_t n_tiles, int32_t k_tiles)
{
    const int64_t total = static_cast<int64_t>(n_tiles) * k_tiles * 64 * 4;     // dwords
    for (int64_t o = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; o < total;
         o += static_cast<int64_t>(gridDim.x) * 256) {
        const int d = static_cast<int>(o & 3);
        const int lane = static_cast<int>((o >> 2) & 63);
        const int64_t tile = o >> 8;
        const int32_t kt = static_cast<int32_t>(tile % k_tiles);
        const int32_t nt = static_cast<int32_t>(tile / k_tiles);
        const int32_t n = nt * kPackN + (lane & 31);
        const int32_t k0 = kt * kPackK + (lane >> 5) * 32 + d * 8;
        uint32_t v = 0;
        if (n < N) {
            const uint32_t src =
                *reinterpret_cast<const uint32_t *>(w + static_cast<int64_t>(n) * (K / 2) + k0 / 2);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t lo = (src >> (4 * j)) & 0xFu;          // channel k0 + j
                const uint32_t hi = (src >> (4 * (4 + j))) & 0xFu;    // channel k0 + 4 + j
                v |= lo << (8 * j);
                v |= hi << (8 * j + 4);
            }
        }
        out[o] = v;
    }
}

// ------------------------------------------------------------------- GEMM
//
// Work-group tile BM x BN, 8 wavefronts (WM x WN), two per SIMD so that one
// wave's LDS reads and unpack hide under the other's MFMAs.  K advances in
// stages of 128 channels.  A stage is copied HBM/L2 -> LDS by LDS-DMA loads
// (global_load_lds_dwordx4: 16 bytes per lane, no VGPR staging), three stages
// deep:
//   A (activations): BM rows x 128 bytes; the eight 16-byte chunks of a row are
//     XOR-swizzled with (row >> 1) & 7, so the DMA writes (8 lanes per row) and
//     the MFMA fragment reads (32 lanes down a column of chunks) are both free
//     of bank conflicts.  The swizzle is applied on the global side: lane i of a
//     1 KiB DMA chunk always lands at LDS offset 16 * i.
//   B (weights): BN/32 n-tiles x 2 k-tiles x 1 KiB, a straight copy of the
//     prepacked tiles; a fragment read is lane * 16, conflict free.
// The DMA loads are issued through inline asm and tracked with explicit
// s_waitcnt vmcnt(n): the compiler would otherwise wait for every outstanding
// LDS-DMA before each ds_read and serialise the pipeline.

// The LDS of gfx950 has 64 four-byte banks (256 B per clock): a 16-byte-per-lane read is
// served 16 lanes at a time, and those 16 lanes -- 16 consecutive rows reading the same
// logical chunk -- must cover the 256-byte bank space exactly once.  Two consecutive rows
// already sit in different halves of it (pitch 128 B), so the chunk index is XORed with
// (row >> 1) & 7: measured 232 B/clk/CU against 124 B/clk with the (row & 7) swizzle that
// a 32-bank LDS would want.
__device__ __forceinline__ int lds_a_swizzle(int row) { return (row >> 1) & 7; }

__device__ __forceinline__ int lds_a_offset(int row, int chunk)
{
    return row * 128 + ((chunk ^ lds_a_swizzle(row)) << 4);
}

// Work-group id -> (tm, tn).  Work-groups are dealt round-robin to the 8 XCDs,
// each with its own L2: XCD x gets a contiguous run of the tile order, and the
// order walks bands of `band` tile-rows, so the ~32 tiles an XCD runs at a time
// form a compact block that shares few A row-panels and few B column-panels.
__device__ __forceinline__ void tile_of_group(int32_t id, int32_t tiles_m, int32_t tiles_n,
                                              int32_t BAND, int32_t &tm, int32_t &tn)
{
    const int32_t total = tiles_m * tiles_n;
    const int32_t per = total / 8, rem = total % 8;
    const int32_t xcd = id % 8, local = id / 8;
    const int32_t t = xcd * per + (xcd < rem ? xcd : rem) + local;
    const int32_t band_tiles = BAND * tiles_n;
    const int32_t band = t / band_tiles;
    const int32_t in_band = t - band * band_tiles;
    const int32_t rows = (tiles_m - band * BAND) < BAND ? (tiles_m - band * BAND) : BAND;
    tm = band * BAND + in_band % rows;
    tn = in_band / rows;
}

template <int BM, int BN, int WM, int WN, int STAGES, int EPI>
__global__ __launch_bounds__(WM *WN * 64, STAGES == 2 ? 4 : 2) void w4a8_gemm_kernel(
    const int8_t *__restrict__ xq, const uint4 *__restrict__ wp, const __half *__restrict__ w_scale,
    __half *__restrict__ y, int64_t ldy, int32_t *__restrict__ acc_out, int32_t T, int32_t N,
    int32_t K, Epilogue ep, int32_t tiles_m, int32_t tiles_n,
    int32_t n_tiles32, int32_t splits, int32_t kb_per_split, int32_t *__restrict__ partial,
    int32_t wide_store, int32_t band)
{
    constexpr int NW = WM * WN;
    constexpr int MT = BM / WM / 32;          // 32x32 tiles per wave along M
    constexpr int NT = BN / WN / 32;          // ... along N
    constexpr int A_STAGE = BM * 128, B_STAGE = BN * 64, STAGE = A_STAGE + B_STAGE;
    constexpr int A_CH = BM / 8, B_CH = BN / 16;      // 1 KiB DMA chunks per stage
    constexpr int CH = (A_CH + B_CH) / NW;            // ... per wave
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "tile shape");
    static_assert((A_CH + B_CH) % NW == 0, "chunks must divide evenly over the waves");
    static_assert((STAGES == 2 || STAGES == 3) && CH * (STAGES - 1) < 64, "pipeline depth");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

    // With split-K the K range is one more factor of the tile grid (next to tn).
    int32_t tm, tn;
    tile_of_group(blockIdx.x, tiles_m, tiles_n * splits, band, tm, tn);
    // K range outermost: neighbouring columns of the order (the tiles one XCD holds
    // at a time) then share their A k-range, which its L2 fetches once.
    const int32_t split = tn / tiles_n;
    tn -= split * tiles_n;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WM;
    const int wn = wave / WM;
    const int l32 = lane & 31;
    const int g = lane >> 5;

    const int32_t row0 = tm * BM;
    const int32_t k_tiles = K / kPackK;
    const int32_t kb0 = split * kb_per_split;           // first 128-wide k-block of this group
    int32_t k_blocks = K / 128 - kb0;                   // K % 128 == 0 is guaranteed by the host
    k_blocks = k_blocks < kb_per_split ? k_blocks : kb_per_split;
    const int32_t ntile0 = tn * (BN / 32);

    v16i acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0;

    // Per-lane global source of each DMA chunk this wave copies, for k-block 0.
    // Rows past T and n-tiles past the padded N are clamped to valid memory; the
    // values they produce are never stored.
    const uint8_t *src[CH];
    int32_t src_step[CH];
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int q = wave + j * NW;
        if (q < A_CH) {
            const int r = q * 8 + (lane >> 3);
            const int logical = (lane & 7) ^ lds_a_swizzle(r);
            int32_t row = row0 + r;
            row = row < T ? row : T - 1;
            src[j] = reinterpret_cast<const uint8_t *>(xq) + static_cast<int64_t>(row) * K +
                     static_cast<int64_t>(kb0) * 128 + logical * 16;
            src_step[j] = 128;
        } else {
            const int b = q - A_CH, nt = b >> 1, ks = b & 1;
            int32_t ntile = ntile0 + nt;
            ntile = ntile < n_tiles32 ? ntile : n_tiles32 - 1;
            src[j] = reinterpret_cast<const uint8_t *>(wp) +
                     ((static_cast<int64_t>(ntile) * k_tiles + kb0 * 2 + ks) * 64 + lane) * 16;
            src_step[j] = 2 * kPackTileBytes;
        }
    }
    // DMA chunk j of this wave for k-block kb (relative to kb0) into stage buffer buf.
    auto dma_chunk = [&](int j, int32_t kb, int buf) {
        lds_dma16(src[j] + static_cast<int64_t>(kb) * src_step[j],
                  smem + buf * STAGE + (wave + j * NW) * 1024);
    };
    // Fragment reads.  A k-block is consumed in four phases (ks, h) of 32 channels:
    // phase (ks, h) multiplies 16-byte chunk ks*4 + g*2 + h of every A row with half h
    // of the unpacked B tile of k-tile ks.
    auto read_a = [&](int buf, int ks, int h, v4i (&dst)[MT]) {
        const uint8_t *abase = smem + buf * STAGE;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int r = wm * (BM / WM) + mt * 32 + l32;
            dst[mt] = as_v4i(*reinterpret_cast<const uint4 *>(
                abase + lds_a_offset(r, ks * 4 + g * 2 + h)));
        }
    };
    auto read_b = [&](int buf, int ks, uint4 (&dst)[NT]) {
        const uint8_t *bbase = smem + buf * STAGE + A_STAGE;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            dst[nt] = *reinterpret_cast<const uint4 *>(
                bbase + ((wn * NT + nt) * 2 + ks) * 1024 + lane * 16);
    };
    // One phase: MT*NT MFMAs (consecutive ones write different accumulators, a
    // dependent pair back to back would wait out the full MFMA latency) with DMA
    // chunks [j0, j0+nj) of a later stage issued between them.  Eight waves that
    // issue a whole stage of LDS-DMA at once queue up behind the one texture
    // address unit of the CU for hundreds of cycles with nothing else to issue.
    auto phase = [&](const v4i (&a)[MT], const v4i (&b)[NT][2], int h, int j0, int nj, bool dma_on,
                     int32_t dma_kb, int dma_buf) {
        int issued = 0, j = 0;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mt], b[nt][h], acc[mt][nt],
                                                                    0, 0, 0);
                ++issued;
                if (j < nj && issued == ((j + 1) * (MT * NT) + nj) / (nj + 1)) {
                    if (dma_on) dma_chunk(j0 + j, dma_kb, dma_buf);
                    ++j;
                }
            }
    };
    // Chunks of one stage are spread over three phases.
    constexpr int C_P3 = (CH + 2) / 3, C_P0 = (CH + 1) / 3, C_P1 = CH - C_P3 - C_P0;
    static_assert(C_P3 <= MT * NT, "more DMA chunks than MFMAs in a phase");

    if constexpr (STAGES == 2) {
        // Two work-groups share a CU (four waves per SIMD): the other group's waves
        // fill every stall of this one, and the plain order -- wait, barrier, whole
        // next stage, all fragments, all MFMAs -- with its lower register count is
        // the faster one (measured 32.5 us against 35.2 us on 1280 x 3584 x 4608).
        if (k_blocks > 0)
#pragma unroll
            for (int j = 0; j < CH; ++j) dma_chunk(j, 0, 0);
        for (int32_t kb = 0; kb < k_blocks; ++kb) {
            const int buf = kb & 1;
            wait_vmcnt<0>();
            // After the barrier every wave sees stage kb and has finished reading
            // stage kb-1, whose buffer the next DMA overwrites.
            __syncthreads();
            if (kb + 1 < k_blocks)
#pragma unroll
                for (int j = 0; j < CH; ++j) dma_chunk(j, kb + 1, buf ^ 1);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                v4i a[2][MT], b[NT][2];
                uint4 braw[NT];
                read_a(buf, ks, 0, a[0]);
                read_a(buf, ks, 1, a[1]);
                read_b(buf, ks, braw);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) unpack_w4x16(braw[nt], b[nt][0], b[nt][1]);
                phase(a[0], b, 0, 0, 0, false, 0, 0);
                phase(a[1], b, 1, 0, 0, false, 0, 0);
            }
        }
    } else {
    // ---- prologue: fill every stage buffer, wait for stage 0, first fragments
#pragma unroll
    for (int s = 0; s < STAGES; ++s)
        if (s < k_blocks)
#pragma unroll
            for (int j = 0; j < CH; ++j) dma_chunk(j, s, s);
    if (k_blocks >= 3) wait_vmcnt<2 * CH>();
    else if (k_blocks == 2) wait_vmcnt<CH>();
    else wait_vmcnt<0>();
    __syncthreads();

    v4i afr[2][MT];              // A fragments of the current and the next phase
    uint4 braw[2][NT];           // packed B tiles of k-tile 0 and 1
    read_a(0, 0, 0, afr[0]);
    read_b(0, 0, braw[0]);

    // ---- main loop.  Every phase first requests the fragments of the next one,
    // so LDS latency hides under a phase's MFMAs; the barrier sits before phase 3,
    // whose operands are already in registers, and phase 3 requests the first
    // fragments of the next k-block from the buffer the barrier has just published.
    // After barrier kb every wave has finished reading buffer kb % STAGES (its
    // last reads were requested in phase 2), so stage kb + STAGES may overwrite it.
    int buf = 0;
    for (int32_t kb = 0; kb < k_blocks; ++kb) {
        const int nb = buf + 1 == STAGES ? 0 : buf + 1;        // buffer of k-block kb + 1
        const int pb = buf == 0 ? STAGES - 1 : buf - 1;        // buffer of kb - 1: stage kb-1+STAGES
        const bool refill_p = kb >= 1 && kb - 1 + STAGES < k_blocks;
        const bool refill_c = kb + STAGES < k_blocks;
        v4i b0[NT][2], b1[NT][2];

        read_a(buf, 0, 1, afr[1]);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) unpack_w4x16(braw[0][nt], b0[nt][0], b0[nt][1]);
        phase(afr[0], b0, 0, C_P3, C_P0, refill_p, kb - 1 + STAGES, pb);

        read_a(buf, 1, 0, afr[0]);
        read_b(buf, 1, braw[1]);
        phase(afr[1], b0, 1, C_P3 + C_P0, C_P1, refill_p, kb - 1 + STAGES, pb);

        read_a(buf, 1, 1, afr[1]);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) unpack_w4x16(braw[1][nt], b1[nt][0], b1[nt][1]);
        phase(afr[0], b1, 0, 0, 0, false, 0, 0);

        // Stage kb+1 must have landed; stage kb+2 may stay in flight.
        if (kb + 2 < k_blocks) wait_vmcnt<CH>();
        else wait_vmcnt<0>();
        __syncthreads();

        if (kb + 1 < k_blocks) {
            read_a(nb, 0, 0, afr[0]);
            read_b(nb, 0, braw[0]);
        }
        phase(afr[1], b1, 1, 0, C_P3, refill_c, kb + STAGES, buf);
        buf = nb;
    }
    }

    const int32_t wave_row0 = row0 + wm * (BM / WM);
    const int32_t wave_n0 = (ntile0 + wn * NT) * 32;

    // ---- split-K: hand the raw partial sums (still x16) to the reduce kernel
    if (partial != nullptr) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int32_t n = wave_n0 + nt * 32 + l32;
            if (n >= N) continue;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int32_t row = wave_row0 + mt * 32 + acc_row(r, g);
                    if (row < T)
                        partial[(static_cast<int64_t>(split) * T + row) * N + n] = acc[mt][nt][r];
                }
        }
        return;
    }

    // ---- epilogue: scale select by row span, per-channel scale, fp16
    if (!wide_store || acc_out != nullptr) {
        // plain path: every lane stores its own 2-byte results
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int32_t n = wave_n0 + nt * 32 + l32;
            if (n >= N) continue;
            const float ws = __half2float(w_scale[n]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int32_t row = wave_row0 + mt * 32 + acc_row(r, g);
                    if (row < T) store_out<EPI>(acc[mt][nt][r], row, n, ep, ws, y, ldy, acc_out, N);
                }
            }
        }
        return;
    }

    // Wide path: the MFMA result has a lane per column, so a direct store writes
    // 2 bytes per lane.  Each wave instead turns 32 rows x (NT*32) columns through
    // its own LDS patch and stores 16 bytes per lane, whole rows of the patch
    // (NT*64 contiguous bytes) at a time.
    constexpr int ROWB = NT * 64 + 16;                 // padded row pitch of the patch, bytes
    constexpr int LPR = NT * 64 / 16;                  // lanes per patch row on the way out
    constexpr int RPI = 64 / LPR;                      // patch rows per store instruction
    static_assert(NW * 32 * ROWB <= STAGES * STAGE, "epilogue patch must fit the stage buffers");
    __syncthreads();                                   // every wave is done with the stage buffers
    uint8_t *patch = smem + wave * (32 * ROWB);
    float ws[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int32_t n = wave_n0 + nt * 32 + l32;
        ws[nt] = __half2float(w_scale[n < N ? n : N - 1]);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = acc_row(r, g);
            const int32_t row = wave_row0 + mt * 32 + rl;
            const int32_t row_in = row < T ? row : T - 1;          // rows past T are never stored
            const float s_row = ep.scale_of<EPI>(row_in);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int32_t a = acc[mt][nt][r] >> 4;             // exact: the sum holds 16 * acc
                int32_t n = wave_n0 + nt * 32 + l32;
                n = n < N ? n : N - 1;                             // only read by the split path
                const float v = ep.dequant<EPI>(a, s_row, row_in, n, N, ws[nt]);
                *reinterpret_cast<__half *>(patch + rl * ROWB + (nt * 32 + l32) * 2) =
                    half_of_rounded_f32(v);
            }
        }
#pragma unroll
        for (int q = 0; q < 32 / RPI; ++q) {
            const int rl = q * RPI + lane / LPR;
            const int c = lane % LPR;
            const uint4 v = *reinterpret_cast<const uint4 *>(patch + rl * ROWB + c * 16);
            const int32_t row = wave_row0 + mt * 32 + rl;
            const int32_t n = wave_n0 + c * 8;
            if (row < T && n < N)                                  // N % 8 == 0 on this path
                *reinterpret_cast<uint4 *>(y + static_cast<int64_t>(row) * ldy + n) = v;
        }
    }
}

// Sums the split-K partials (int32, x16) and applies the dequant epilogue.
// Four consecutive channels per thread; N % 4 == 0.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(
    const int32_t *__restrict__ partial, int32_t splits, int32_t T, int32_t N,
    const __half *__restrict__ w_scale, __half *__restrict__ y, int64_t ldy,
    int32_t *__restrict__ acc_out, Epilogue ep)
{
    const int64_t quads = static_cast<int64_t>(T) * (N / 4);
    const int64_t plane = static_cast<int64_t>(T) * N;
    for (int64_t q = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; q < quads;
         q += static_cast<int64_t>(gridDim.x) * 256) {
        const int32_t row = static_cast<int32_t>(q / (N / 4));
        const int32_t n = static_cast<int32_t>(q - static_cast<int64_t>(row) * (N / 4)) * 4;
        const int64_t off = static_cast<int64_t>(row) * N + n;
        int4 sum = *reinterpret_cast<const int4 *>(partial + off);
        for (int32_t s = 1; s < splits; ++s) {
            const int4 p = *reinterpret_cast<const int4 *>(partial + s * plane + off);
            sum.x += p.x;
            sum.y += p.y;
            sum.z += p.z;
            sum.w += p.w;
        }
        const int32_t a[4] = {sum.x >> 4, sum.y >> 4, sum.z >> 4, sum.w >> 4};
        const float s_row = ep.scale_of<EPI>(row);
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            v[e] = (static_cast<float>(a[e]) * s_row) * __half2float(w_scale[n + e]);
        if constexpr (EPI == kEpiSplit) {
            // same terms and order as Epilogue::dequant, with the token's code read once per
            // flagged channel and the four weights of the quad in one 4-byte load
            for (int32_t j = 0; j < ep.n_split; ++j) {
                const int32_t code = ep.xq[static_cast<int64_t>(row) * ep.K + ep.split_idx[j]];
                const uint32_t w4 = *reinterpret_cast<const uint32_t *>(
                    ep.split_w + static_cast<int64_t>(j) * N + n);
                const float sc = ep.split_scale[j];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int32_t w = static_cast<int8_t>(w4 >> (8 * e));
                    v[e] = v[e] + (static_cast<float>(code * w) * s_row) * sc;
                }
            }
        }
        __half h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = half_of_rounded_f32(v[e]);
        __half *dst = y + static_cast<int64_t>(row) * ldy + n;
        if ((reinterpret_cast<uintptr_t>(dst) & 7) == 0) {
            *reinterpret_cast<uint2 *>(dst) = *reinterpret_cast<const uint2 *>(h);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[j] = h[j];
        }
        if (acc_out) *reinterpret_cast<int4 *>(acc_out + off) = make_int4(a[0], a[1], a[2], a[3]);
    }
}

// ------------------------------------------------------------------- GEMV

// Decode shape (T <= 32): the weights are streamed once from HBM and nothing
// is reused, so there is no LDS staging of operands.  One work-group owns one
// 32-channel tile; its NWAVES waves split K, and every wave requests a whole
// batch of KT k-tiles (activations first, they hit L2; then the weights, with
// the non-temporal hint) before it touches the first one.  Loads are branch
// free: addresses past a wave's K range are clamped and the weights masked to
// zero, and lanes whose token row is >= T read row T-1 (rows >= T of the MFMA
// result are never stored).  The partial sums of the waves meet in LDS.
//
// AROWS > 0 (T <= AROWS): the activations of a batch pass through a wave-private
// LDS patch.  Read straight from memory, a fragment load touches T rows x 2 pieces of
// 16 bytes -- at T = 16 four times the cache lines of the 1 KiB weight load next to it;
// staged, the wave reads each row's 256 bytes of the batch once, 16 lanes per row, and
// picks the fragments out of LDS (row pitch 272 bytes: conflict free).
//
// Several linears that share xq (q/k/v, gate/up) can go into one launch: the grid is the
// concatenation of their tiles (units = 32-channel tiles of each problem).
//
// MROWS = 2 (33..64 rows, short prompts): two 32-row blocks share every weight tile -- the
// weights are still read once, unpacked once and feed two MFMA pairs.
template <int NWAVES, int KT, int EPI, int AROWS, int MROWS>
__global__ __launch_bounds__(NWAVES * 64) void w4a8_gemv_kernel(
    const int8_t *__restrict__ xq, GemvGroup grp, int32_t T, int32_t K, Epilogue ep)
{
    typedef unsigned int v4u __attribute__((ext_vector_type(4)));
    static_assert(MROWS == 1 || (MROWS == 2 && AROWS == 64), "two row blocks come with 64 staged rows");
    // which linear of the group, which tile of it
    int32_t pi = 0, ntile = blockIdx.x;
    while (pi + 1 < grp.n && ntile >= grp.p[pi].units) {
        ntile -= grp.p[pi].units;
        ++pi;
    }
    const uint4 *__restrict__ wp = grp.p[pi].wp;
    const __half *__restrict__ w_scale = grp.p[pi].w_scale;
    __half *__restrict__ y = grp.p[pi].y;
    int32_t *__restrict__ acc_out = grp.p[pi].acc_out;
    const int64_t ldy = grp.p[pi].ldy;
    const int32_t N = grp.p[pi].N;
    constexpr int kPatchPitch = KT * 64 + 16;
    constexpr int kPatchBytes = AROWS * kPatchPitch;
    constexpr int kWaveBytes = kPatchBytes > 4096 ? kPatchBytes : 4096;
    __shared__ __attribute__((aligned(16))) uint8_t smem[NWAVES * kWaveBytes];
    int32_t (*red)[16][64] = reinterpret_cast<int32_t (*)[16][64]>(smem);   // [NWAVES][16][64]

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l32 = lane & 31;
    const int g = lane >> 5;
    const int32_t k_tiles = K / kPackK;
    const int32_t per_wave = (k_tiles + NWAVES - 1) / NWAVES;
    const int32_t kt_begin = wave * per_wave;
    int32_t kt_end = kt_begin + per_wave;
    kt_end = kt_end < k_tiles ? kt_end : k_tiles;
    const int32_t n = ntile * 32 + l32;
    const __half ws_h = w_scale[n < N ? n : N - 1];      // requested early, used in the epilogue

    v16i acc0[MROWS], acc1[MROWS];                        // two chains: no back-to-back dependent MFMAs
#pragma unroll
    for (int m = 0; m < MROWS; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc0[m][r] = 0;
            acc1[m][r] = 0;
        }
    const uint4 *wtile = wp + static_cast<int64_t>(ntile) * k_tiles * 64 + lane;
    const int8_t *xrow = xq + static_cast<int64_t>(l32 < T ? l32 : T - 1) * K + g * 32;

    constexpr int NI = AROWS / 4;                         // staging loads per batch: 4 rows each
    uint8_t *patch = smem + wave * kWaveBytes;
    const int srow = lane >> 4, scol = lane & 15;
    int frag_row[MROWS];
#pragma unroll
    for (int m = 0; m < MROWS; ++m) frag_row[m] = m * 32 + l32 < T ? m * 32 + l32 : T - 1;

    for (int32_t base = kt_begin; base < kt_end; base += KT) {
        uint4 a0[MROWS][KT], a1[MROWS][KT], b[KT];
        v4u stage_reg[NI > 0 ? NI : 1];
        if constexpr (AROWS == 0) {
#pragma unroll
            for (int u = 0; u < KT; ++u) {
                int32_t kt = base + u;
                kt = kt < kt_end ? kt : kt_end - 1;
                a0[0][u] = *reinterpret_cast<const uint4 *>(xrow + kt * 64);
                a1[0][u] = *reinterpret_cast<const uint4 *>(xrow + kt * 64 + 16);
            }
        } else {
            // 16 bytes per lane, 16 lanes per row; channels past K are clamped into the row
            // (their weights are masked to zero below)
            int32_t kofs = base * 64 + scol * 16;
            kofs = kofs <= K - 16 ? kofs : K - 16;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                int32_t r = i * 4 + srow;
                r = r < T ? r : T - 1;
                stage_reg[i] = *reinterpret_cast<const v4u *>(xq + static_cast<int64_t>(r) * K + kofs);
            }
        }
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            int32_t kt = base + u;
            kt = kt < kt_end ? kt : kt_end - 1;
            const v4u t = __builtin_nontemporal_load(
                reinterpret_cast<const v4u *>(wtile + static_cast<int64_t>(kt) * 64));
            b[u] = make_uint4(t[0], t[1], t[2], t[3]);
        }
        if constexpr (AROWS > 0) {
            // same wave writes and reads: LDS operations of a wave complete in order
#pragma unroll
            for (int i = 0; i < NI; ++i)
                *reinterpret_cast<v4u *>(patch + (i * 4 + srow) * kPatchPitch + scol * 16) = stage_reg[i];
#pragma unroll
            for (int m = 0; m < MROWS; ++m)
#pragma unroll
                for (int u = 0; u < KT; ++u) {
                    const uint8_t *f = patch + frag_row[m] * kPatchPitch + u * 64 + g * 32;
                    a0[m][u] = *reinterpret_cast<const uint4 *>(f);
                    a1[m][u] = *reinterpret_cast<const uint4 *>(f + 16);
                }
        }
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            const uint32_t msk = (base + u < kt_end) ? 0xFFFFFFFFu : 0u;     // wave-uniform
            uint4 bb = b[u];
            bb.x &= msk;
            bb.y &= msk;
            bb.z &= msk;
            bb.w &= msk;
            v4i b0, b1;
            unpack_w4x16(bb, b0, b1);
#pragma unroll
            for (int m = 0; m < MROWS; ++m) {
                acc0[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(a0[m][u]), b0, acc0[m], 0, 0, 0);
                acc1[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(a1[m][u]), b1, acc1[m], 0, 0, 0);
            }
        }
        // Scheduling order inside a batch: all memory reads first, then the
        // arithmetic.  Without this the scheduler sinks each load next to its use
        // and the wave waits out one memory round trip per k-tile.
        if constexpr (AROWS == 0) {
            __builtin_amdgcn_sched_group_barrier(0x020, 3 * KT, 0);
        } else {
            __builtin_amdgcn_sched_group_barrier(0x020, NI + KT, 0);
            __builtin_amdgcn_sched_group_barrier(0x200, NI, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * KT * MROWS, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x00A, (16 + 2 * MROWS) * KT, 0);
    }
    if constexpr (AROWS > 0) __syncthreads();             // the sums below reuse the patches

    // Accumulator register r of k-group g holds row acc_row(r, g): with T <= 8
    // only r < 4 can be a valid row, with T <= 16 only r < 8.
    const int rmax = T <= 8 ? 4 : (T <= 16 ? 8 : 16);
    const float ws = __half2float(ws_h);
#pragma unroll
    for (int m = 0; m < MROWS; ++m) {
        if (m > 0) __syncthreads();                       // the sums of the block before have been read
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (r < rmax) red[wave][r][lane] = acc0[m][r] + acc1[m][r];
        __syncthreads();
        for (int r = wave; r < rmax; r += NWAVES) {
            const int32_t row = m * 32 + acc_row(r, g);
            if (row < T && n < N) {
                int32_t sum = 0;
#pragma unroll
                for (int w = 0; w < NWAVES; ++w) sum += red[w][r][lane];
                store_out<EPI>(sum, row, n, ep, ws, y, ldy, acc_out, N);
            }
        }
    }
}

// Decode with the front end fused in (T <= 4): every work-group first rotates and
// quantizes the T input rows itself (Sec. 3.2 rotation, Eq. (2)/(3) static
// quantizer: the same wave-level code as the stand-alone kernel, one 512-channel
// segment per wave at a time) into an LDS copy of xq, then streams its weight tile
// as above with the activation fragments read from that copy.  The rotation is
// redundant across work-groups but costs a few hundred cycles per wave against a
// separate launch per linear (about 2 us each in a 7-linear decoder layer).
template <int NWAVES, int KT, int B>
__global__ __launch_bounds__(NWAVES * 64) void w4a8_decode_fused_kernel(
    const __half *__restrict__ x, int64_t ldx, const uint4 *__restrict__ wp,
    const __half *__restrict__ w_scale, __half *__restrict__ y, int64_t ldy, int32_t T, int32_t N,
    int32_t K, Epilogue ep, float c_vis, float c_txt)
{
    typedef unsigned int v4u __attribute__((ext_vector_type(4)));
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];     // max(T * pitch, NWAVES * 4096)
    int32_t (*red)[16][64] = reinterpret_cast<int32_t (*)[16][64]>(smem);
    const int32_t pitch = K + 16;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l32 = lane & 31;
    const int g = lane >> 5;
    const int32_t ntile = blockIdx.x;
    const int32_t k_tiles = K / kPackK;
    const int32_t per_wave = (k_tiles + NWAVES - 1) / NWAVES;
    const int32_t kt_begin = wave * per_wave;
    int32_t kt_end = kt_begin + per_wave;
    kt_end = kt_end < k_tiles ? kt_end : k_tiles;
    const int32_t n = ntile * 32 + l32;
    const __half ws_h = w_scale[n < N ? n : N - 1];

    const uint4 *wtile = wp + static_cast<int64_t>(ntile) * k_tiles * 64 + lane;
    auto load_weights = [&](int32_t base, uint4 (&b)[KT]) {
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            int32_t kt = base + u;
            kt = kt < kt_end ? kt : kt_end - 1;
            kt = kt > 0 ? kt : 0;
            const v4u t = __builtin_nontemporal_load(
                reinterpret_cast<const v4u *>(wtile + static_cast<int64_t>(kt) * 64));
            b[u] = make_uint4(t[0], t[1], t[2], t[3]);
        }
    };
    // The first batch of weights is requested before the front end, so the rotation runs
    // under that round trip to memory.
    uint4 b[KT];
    load_weights(kt_begin, b);

    // ---- front end: x (fp16) -> rotated, quantized int8 rows in LDS
    {
        using Seg = Segment<B>;
        const int32_t segs_per_row = (K + Seg::SEG - 1) / Seg::SEG;
        const int32_t total = T * segs_per_row;
        for (int32_t sgi = wave; sgi < total; sgi += NWAVES) {
            const int32_t i = sgi / segs_per_row, sidx = sgi - i * segs_per_row;
            Seg sg;
            sg.load_rotate(x + static_cast<int64_t>(i) * ldx, sidx, K, lane);
            sg.quant_store(i < ep.n_vis ? c_vis : c_txt, reinterpret_cast<int8_t *>(smem) + i * pitch,
                           sidx, lane);
        }
    }
    __syncthreads();

    v16i acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        acc0[r] = 0;
        acc1[r] = 0;
    }
    const uint8_t *frag = smem + (l32 < T ? l32 : T - 1) * pitch + g * 32;

    auto batch = [&](int32_t base, const uint4 (&bw)[KT]) {
        uint4 a0[KT], a1[KT];
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            int32_t kt = base + u;
            kt = kt < kt_end ? kt : kt_end - 1;
            a0[u] = *reinterpret_cast<const uint4 *>(frag + kt * 64);
            a1[u] = *reinterpret_cast<const uint4 *>(frag + kt * 64 + 16);
        }
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            const uint32_t m = (base + u < kt_end) ? 0xFFFFFFFFu : 0u;     // wave-uniform
            uint4 bb = bw[u];
            bb.x &= m;
            bb.y &= m;
            bb.z &= m;
            bb.w &= m;
            v4i b0, b1;
            unpack_w4x16(bb, b0, b1);
            acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(a0[u]), b0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(a1[u]), b1, acc1, 0, 0, 0);
        }
    };
    if (kt_begin < kt_end) batch(kt_begin, b);             // its weights were requested up front
    for (int32_t base = kt_begin + KT; base < kt_end; base += KT) {
        load_weights(base, b);
        batch(base, b);
        // all memory and LDS reads of the batch first, then the arithmetic
        __builtin_amdgcn_sched_group_barrier(0x020, KT, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * KT, 0);
        __builtin_amdgcn_sched_group_barrier(0x00A, 18 * KT, 0);
    }
    __syncthreads();                                       // the sums below reuse the xq copy

    // T <= 4: only accumulator registers r < 4 of lane group 0 hold valid rows
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][r][lane] = acc0[r] + acc1[r];
    __syncthreads();
    const float ws = __half2float(ws_h);
    for (int r = wave; r < 4; r += NWAVES) {
        const int32_t row = acc_row(r, g);
        if (row < T && n < N) {
            int32_t sum = 0;
#pragma unroll
            for (int w = 0; w < NWAVES; ++w) sum += red[w][r][lane];
            store_out<kEpiStatic>(sum, row, n, ep, ws, y, ldy, nullptr, N);
        }
    }
}

// ------------------------------------------------------------------ host side

constexpr int kGemvMaxT = 32;

int check_gemm_args(const void *xq, const void *wp, const void *w_scale, const void *y,
                    int64_t ldy, int32_t T, int32_t N, int32_t K, int32_t n_vis, float s_vis,
                    float s_txt)
{
    if (T < 0 || N < 0 || K < 0) return MQUANT_ERR_BAD_SHAPE;
    if (K % kPackK != 0 || K > kMaxK) return MQUANT_ERR_UNSUPPORTED;
    if (n_vis < 0 || n_vis > T) return MQUANT_ERR_BAD_SHAPE;
    if (!(s_vis > 0.0f) || !(s_txt > 0.0f) || !isfinite(s_vis) || !isfinite(s_txt))
        return MQUANT_ERR_BAD_SHAPE;
    if (T == 0 || N == 0) return MQUANT_OK;
    if (ldy < N) return MQUANT_ERR_BAD_SHAPE;
    if (K == 0) return MQUANT_ERR_UNSUPPORTED;
    if (!xq || !wp || !w_scale || !y) return MQUANT_ERR_NULL;
    if (!aligned_to(xq, 16) || !aligned_to(wp, 16) || !aligned_to(w_scale, 2) || !aligned_to(y, 2))
        return MQUANT_ERR_ALIGNMENT;
    return MQUANT_OK;
}


// Split-K plan for the 256x256 tile: when the tile grid fills less than half of
// the CUs and K is long, S work-groups share a tile's K range, write int32
// partials to the workspace and a small second kernel reduces and dequantises.
// (A single-kernel reduction needs device-scope fences, which write back the
// whole L2 and were measured far slower.)  Up to 16 pieces of at least 2048
// channels: measured on the few-tile shapes of short prompts, 64..512 rows against
// 18944 x 3584 take 34-51 us instead of 54-63 us with at most 4 pieces of 4096, and
// nothing measured got slower; pieces shorter than 2048 channels lose to the fixed
// cost of a work-group (3584-channel shapes stay unsplit).
int plan_splits(int32_t T, int32_t N, int32_t K)
{
    const int64_t tiles = ceil_div(T, 256) * ceil_div(N, 256);
    int64_t s = kNumCU / tiles;
    if (s < 2 || N % 4 != 0) return 1;
    if (s > 16) s = 16;
    while (s > 1 && K / s < 2048) --s;
    return static_cast<int>(s);
}

template <int BM, int BN, int WM, int WN, int STAGES, int EPI>
int launch_gemm(const int8_t *xq, const uint8_t *wp, const void *w_scale, void *y, int64_t ldy,
                int32_t *acc_out, int32_t T, int32_t N, int32_t K, Epilogue ep, int32_t splits,
                int32_t *partial, hipStream_t stream)
{
    const int32_t tiles_m = static_cast<int32_t>(ceil_div(T, BM));
    const int32_t tiles_n = static_cast<int32_t>(ceil_div(N, BN));
    const int32_t n_tiles32 = static_cast<int32_t>(ceil_div(N, kPackN));
    const int32_t kb_per_split = static_cast<int32_t>(ceil_div(K / 128, splits));
    const size_t lds = static_cast<size_t>(STAGES) * (BM * 128 + BN * 64);
    const int32_t wide_store =
        (N % 8 == 0 && ldy % 8 == 0 && aligned_to(y, 16) && acc_out == nullptr) ? 1 : 0;
    auto kern = w4a8_gemm_kernel<BM, BN, WM, WN, STAGES, EPI>;
    // Band height of the tile order: all tile-rows when there are few (every B panel is then
    // read by one XCD only), else equal bands of about six rows.
    const int32_t band = tiles_m <= 8 ? tiles_m
                                      : static_cast<int32_t>(ceil_div(tiles_m, ceil_div(tiles_m, 6)));
    // Raising the dynamic LDS limit is idempotent: threads racing here at most repeat it.
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                static_cast<int>(lds)) != hipSuccess)
            return MQUANT_ERR_HIP;
        attr_set.store(true, std::memory_order_release);
    }
    MQ_LAUNCH(kern, dim3(tiles_m * tiles_n * splits), dim3(WM * WN * 64), lds, stream, xq,
                       reinterpret_cast<const uint4 *>(wp), static_cast<const __half *>(w_scale),
                       static_cast<__half *>(y), ldy, acc_out, T, N, K, ep, tiles_m, tiles_n, n_tiles32, splits, kb_per_split,
                       splits > 1 ? partial : nullptr, wide_store, band);
    int st = launch_status();
    if (st != MQUANT_OK || splits == 1) return st;
    const int64_t quads = static_cast<int64_t>(T) * (N / 4);
    int64_t blocks = ceil_div(quads, 256);
    if (blocks > 8 * kNumCU) blocks = 8 * kNumCU;
    MQ_LAUNCH(splitk_reduce_kernel<EPI>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0,
                       stream, partial, splits, T, N, static_cast<const __half *>(w_scale),
                       static_cast<__half *>(y), ldy, acc_out, ep);
    return launch_status();
}

// Tile choice.  256x256 (one work-group per CU, three stages) has the best
// steady-state rate; 128x256 with two stages fits two work-groups per CU, which
// hides one group's prologue and epilogue under the other's main loop and
// halves the tile-count granularity.  Cost model: rounds over the 256 CUs times
// tile area, the smaller tile derated by its measured relative rate.
//
// Short prompts on matrices with many output channels (up to 128 rows; the few-channel ones
// go to the tile GEMV): one or two rows of 64-row tiles, three stages, several work-groups per
// CU.  With one row of 128- or 256-row tiles the k-loop of a lone, mostly empty work-group per
// CU sets the time.  Measured at T = 64, 64x128 / 64x256 against the 128x256 tile the cost
// model below would pick: 3584 -> 18944 15.3 / 19.1 against 22.6 us, 3584 -> 37888 23.0 / 20.7
// against 32.7, 8192 -> 59136 53.6 / 48.9 against 72.8; at T = 128: 3584 -> 18944 20.5
// against 23.2, 8192 -> 10240 28.4 against 37.9, 3584 -> 37888 no difference (30.5).
int pick_gemm_tile(int32_t T, int32_t N)
{
    if (T <= 128) {
        const int64_t groups = ceil_div(T, 64) * ceil_div(N, 128);       // of 64x128 tiles
        if (T <= 64) return groups <= kNumCU ? 3 : 4;
        if (groups <= kNumCU + kNumCU / 4) return 3;
    }
    // rounds of work-groups over the CUs x tile area / measured relative efficiency of the tile
    const double a = static_cast<double>(ceil_div(ceil_div(T, 256) * ceil_div(N, 256), kNumCU)) *
                     256.0 * 256.0;
    const double b = static_cast<double>(ceil_div(ceil_div(T, 128) * ceil_div(N, 256), kNumCU)) *
                     128.0 * 256.0 / 0.93;
    const double c = static_cast<double>(ceil_div(ceil_div(T, 192) * ceil_div(N, 128), kNumCU)) *
                     192.0 * 128.0 / 0.78;
    if (a <= b && a <= c) return 0;
    return b <= c ? 1 : 2;
}

}  // namespace

extern "C" int64_t mquant_w4_prepacked_bytes(int32_t N, int32_t K)
{
    if (N < 0 || K < 0) return MQUANT_ERR_BAD_SHAPE;
    if (K % kPackK != 0 || K > kMaxK) return MQUANT_ERR_UNSUPPORTED;
    return ceil_div(N, kPackN) * (K / kPackK) * static_cast<int64_t>(kPackTileBytes);
}

extern "C" int mquant_w4_prepack(const uint8_t *w, uint8_t *out, int32_t N, int32_t K,
                                 mquant_stream_t stream)
{
    if (N < 0 || K < 0) return MQUANT_ERR_BAD_SHAPE;
    if (K % kPackK != 0 || K > kMaxK) return MQUANT_ERR_UNSUPPORTED;
    if (N == 0 || K == 0) return MQUANT_OK;
    if (!w || !out) return MQUANT_ERR_NULL;
    if (!aligned_to(w, 4) || !aligned_to(out, 16)) return MQUANT_ERR_ALIGNMENT;
    const int32_t n_tiles = static_cast<int32_t>(ceil_div(N, kPackN));
    const int32_t k_tiles = K / kPackK;
    const int64_t dwords = static_cast<int64_t>(n_tiles) * k_tiles * 256;
    int64_t blocks = ceil_div(dwords, 256);
    if (blocks > (1 << 20)) blocks = 1 << 20;
    MQ_LAUNCH(prepack_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), w, reinterpret_cast<uint32_t *>(out), N, K,
                       n_tiles, k_tiles);
    return launch_status();
}

namespace {

// Shapes the tile GEMV takes instead of the prefill GEMM: up to 32 rows (one pass), every K
// the prefill kernel does not handle, and short prompts against matrices with few output
// channels, where the GEMM would run a single, mostly empty row of tiles at its fixed cost
// while the GEMV streams the weights once per 64 rows (two row blocks per weight tile).
// Measured at 33..64 rows, GEMV against GEMM: 3584 x 3584 and 3584 x 4608 9 against 22 us,
// 18944 x 3584 24-30 against 33-35, 8192 x 8192 15 against 31, 8192 x 10240 23-25 against 32,
// 29568 x 8192 39-43 against 60; with 18944 or more output channels the GEMM fills enough
// compute units to win (3584 x 18944: 22-23 us either way, x 37888: 38 against 32).  At
// 65..128 rows the second pass pays for small matrices only (3584 x 3584: 14-16 against 22 us,
// 8192 x 8192 24-29 against 34; 18944 x 3584 49 against 36).
bool gemv_tile_takes(int32_t T, int32_t N, int32_t K)
{
    if (T <= kGemvMaxT || K % 128 != 0) return true;
    if (tune_state().gemm_tile.load(std::memory_order_relaxed) >= 0) return false;   // a forced GEMM tile
    if (T <= 2 * kGemvMaxT) return N <= 12288;
    return T <= 4 * kGemvMaxT && N <= 8192 && static_cast<int64_t>(N) * K <= (int64_t{1} << 26);
}

}  // namespace

namespace mquant {

// The tile GEMV for a group of linears that share xq (a group of one for the single-linear
// entry points).  It handles 32 rows per pass; taller inputs (only reached for K % 128 != 0,
// which the prefill kernel does not take) are walked in slabs of 32 rows.
template <int EPI>
int gemv_tile_dispatch(const int8_t *xq, int32_t T, int32_t K, GemvGroup grp, const Epilogue &ep,
                       hipStream_t stream)
{
    int64_t total = 0;
    for (int32_t i = 0; i < grp.n; ++i) {
        grp.p[i].units = static_cast<int32_t>(ceil_div(grp.p[i].N, 32));
        total += grp.p[i].units;
    }
    if (total <= 0 || total > 0x7fffffff) return MQUANT_ERR_BAD_SHAPE;
    const unsigned n_tiles = static_cast<unsigned>(total);
    // 32 rows per pass, 64 with two row blocks per weight tile (rows beyond 32 come here only
    // for short prompts and for K % 128 != 0)
    for (int32_t t0 = 0; t0 < T;) {
        const int32_t left = T - t0;
        const int32_t tt = left > kGemvMaxT ? (left < 2 * kGemvMaxT ? left : 2 * kGemvMaxT) : left;
        Epilogue slab = ep;
        int32_t nv = ep.n_vis - t0;
        slab.n_vis = nv < 0 ? 0 : (nv > tt ? tt : nv);
        if (ep.rows != nullptr) slab.rows = ep.rows + t0;
        slab.xq = xq + static_cast<int64_t>(t0) * K;
        const int8_t *xs = xq + static_cast<int64_t>(t0) * K;
        GemvGroup gs = grp;
        for (int32_t i = 0; i < grp.n; ++i) {
            gs.p[i].y = grp.p[i].y + static_cast<int64_t>(t0) * grp.p[i].ldy;
            gs.p[i].acc_out = grp.p[i].acc_out ? grp.p[i].acc_out + static_cast<int64_t>(t0) * grp.p[i].N : nullptr;
        }
        // Few n-tiles: more waves per tile to keep enough loads in flight.  The activations of
        // a batch are staged through LDS (faster at every T measured, T = 1 included:
        // a batch then takes 1-16 row loads instead of 8 scattered fragment loads).
        const int arows = tt > 32 ? 64 : (tt > 16 ? 32 : (tt <= 4 ? 4 : (tt <= 8 ? 8 : 16)));
#define MQ_GEMV(NWV, AR, MR)                                                                          \
    MQ_LAUNCH((w4a8_gemv_kernel<NWV, 4, EPI, AR, MR>), dim3(n_tiles), dim3(NWV * 64), 0, stream, xs, \
              gs, tt, K, slab)
        if (arows == 64) {
            MQ_GEMV(8, 64, 2);
        } else if (n_tiles >= 256) {
            if (arows == 32) MQ_GEMV(8, 32, 1);
            else if (arows == 4) MQ_GEMV(8, 4, 1);
            else if (arows == 8) MQ_GEMV(8, 8, 1);
            else MQ_GEMV(8, 16, 1);
        } else {
            if (arows == 32) MQ_GEMV(16, 32, 1);
            else if (arows == 4) MQ_GEMV(16, 4, 1);
            else if (arows == 8) MQ_GEMV(16, 8, 1);
            else MQ_GEMV(16, 16, 1);
        }
#undef MQ_GEMV
        const int ls = launch_status();
        if (ls != MQUANT_OK) return ls;
        t0 += tt;
    }
    return MQUANT_OK;
}

template int gemv_tile_dispatch<kEpiStatic>(const int8_t *, int32_t, int32_t, GemvGroup, const Epilogue &, hipStream_t);
template int gemv_tile_dispatch<kEpiRowScale>(const int8_t *, int32_t, int32_t, GemvGroup, const Epilogue &, hipStream_t);
template int gemv_tile_dispatch<kEpiSplit>(const int8_t *, int32_t, int32_t, GemvGroup, const Epilogue &, hipStream_t);

}  // namespace mquant

extern "C" int64_t mquant_w4a8_workspace_bytes(int32_t T, int32_t N, int32_t K)
{
    if (T < 0 || N < 0 || K < 0) return MQUANT_ERR_BAD_SHAPE;
    if (K % kPackK != 0 || K > kMaxK) return MQUANT_ERR_UNSUPPORTED;
    if (gemv_tile_takes(T, N, K)) return 0;
    const int splits = plan_splits(T, N, K);
    return splits > 1 ? static_cast<int64_t>(splits) * T * N * 4 : 0;
}

namespace {

// Shared body of the GEMM entry points; `ep` carries the activation scales (static or
// per row) and the optional split channels.  Arguments are validated by the callers.
template <int EPI>
int gemm_dispatch(const int8_t *xq, const uint8_t *wp, const void *w_scale, void *y, int64_t ldy,
                  int32_t *acc_out, int32_t T, int32_t N, int32_t K, Epilogue ep, void *workspace,
                  int64_t workspace_bytes, hipStream_t stream)
{
    if (gemv_stream_takes(T, K, ceil_div(N, kPackN))) {
        GemvGroup grp = {};
        grp.n = 1;
        grp.p[0].wp = reinterpret_cast<const uint4 *>(wp);
        grp.p[0].w_scale = static_cast<const __half *>(w_scale);
        grp.p[0].y = static_cast<__half *>(y);
        grp.p[0].acc_out = acc_out;
        grp.p[0].ldy = ldy;
        grp.p[0].N = N;
        return gemv_stream_dispatch<EPI>(xq, T, K, grp, ep, stream);
    }
    if (gemv_tile_takes(T, N, K)) {
        GemvGroup grp = {};
        grp.n = 1;
        grp.p[0].wp = reinterpret_cast<const uint4 *>(wp);
        grp.p[0].w_scale = static_cast<const __half *>(w_scale);
        grp.p[0].y = static_cast<__half *>(y);
        grp.p[0].acc_out = acc_out;
        grp.p[0].ldy = ldy;
        grp.p[0].N = N;
        return gemv_tile_dispatch<EPI>(xq, T, K, grp, ep, stream);
    }
    int splits = plan_splits(T, N, K);
    const int force_tile = tune_state().gemm_tile.load(std::memory_order_relaxed);
    if (tune_state().gemm_nosplit.load(std::memory_order_relaxed)) splits = 1;
    if (splits > 1) {
        const int64_t need = static_cast<int64_t>(splits) * T * N * 4;
        if (!workspace || workspace_bytes < need) return MQUANT_ERR_WORKSPACE;
        if (!aligned_to(workspace, 256)) return MQUANT_ERR_ALIGNMENT;
        return launch_gemm<256, 256, 2, 4, 3, EPI>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, splits,
                                                 static_cast<int32_t *>(workspace), stream);
    }
    const int tile = force_tile < 0 ? pick_gemm_tile(T, N) : force_tile;
    if (tile == 3)
        return launch_gemm<64, 128, 2, 4, 3, EPI>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, 1,
                                                nullptr, stream);
    if (tile == 4)
        return launch_gemm<64, 256, 1, 8, 3, EPI>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, 1,
                                                nullptr, stream);
    if (tile == 0)
        return launch_gemm<256, 256, 2, 4, 3, EPI>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, 1,
                                                 nullptr, stream);
    // 192 x 128 (wave tile 96 x 32): the middle ground when 128 x 256 tiles leave a third of
    // the CUs idle (1280 x 4608: 252 tiles instead of 180; 28 us against 31 us).
    if (tile == 2)
        return launch_gemm<192, 128, 2, 4, 3, EPI>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, 1,
                                                 nullptr, stream);
    return launch_gemm<128, 256, 2, 4, 2, EPI>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, 1, nullptr,
                                             stream);
}

}  // namespace

extern "C" int mquant_w4a8_gemm(const int8_t *xq, const uint8_t *wp, const void *w_scale, void *y,
                                int64_t ldy, int32_t *acc_out, int32_t T, int32_t N, int32_t K,
                                int32_t n_vis, float s_vis, float s_txt, void *workspace,
                                int64_t workspace_bytes, mquant_stream_t stream)
{
    const int st = check_gemm_args(xq, wp, w_scale, y, ldy, T, N, K, n_vis, s_vis, s_txt);
    if (st != MQUANT_OK) return st;
    if (T == 0 || N == 0) return MQUANT_OK;
    Epilogue ep = {};
    ep.n_vis = n_vis, ep.s_vis = s_vis, ep.s_txt = s_txt, ep.K = K, ep.xq = xq;
    return gemm_dispatch<kEpiStatic>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, workspace, workspace_bytes,
                         static_cast<hipStream_t>(stream));
}

extern "C" int mquant_w4a8_gemm_rowscale(const int8_t *xq, const uint8_t *wp, const void *w_scale,
                                         const float *row_scale, void *y, int64_t ldy,
                                         int32_t *acc_out, int32_t T, int32_t N, int32_t K,
                                         void *workspace, int64_t workspace_bytes,
                                         mquant_stream_t stream)
{
    const int st = check_gemm_args(xq, wp, w_scale, y, ldy, T, N, K, 0, 1.0f, 1.0f);
    if (st != MQUANT_OK) return st;
    if (T == 0 || N == 0) return MQUANT_OK;
    if (!row_scale) return MQUANT_ERR_NULL;
    if (!aligned_to(row_scale, 4)) return MQUANT_ERR_ALIGNMENT;
    Epilogue ep = {};
    ep.s_vis = 1.0f, ep.s_txt = 1.0f, ep.rows = row_scale, ep.K = K, ep.xq = xq;
    return gemm_dispatch<kEpiRowScale>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, workspace, workspace_bytes,
                         static_cast<hipStream_t>(stream));
}

extern "C" int mquant_w4a8_gemm_rms(const int8_t *xq, const uint8_t *wp, const void *w_scale,
                                    void *y, int64_t ldy, int32_t *acc_out, int32_t T, int32_t N,
                                    int32_t K, int32_t n_vis, float s_vis, float s_txt,
                                    const int32_t *split_idx, const int8_t *split_w,
                                    const float *split_scale, int32_t n_split, void *workspace,
                                    int64_t workspace_bytes, mquant_stream_t stream)
{
    const int st = check_gemm_args(xq, wp, w_scale, y, ldy, T, N, K, n_vis, s_vis, s_txt);
    if (st != MQUANT_OK) return st;
    if (n_split < 0 || n_split > kMaxSplitChannels) return MQUANT_ERR_BAD_SHAPE;
    if (T == 0 || N == 0) return MQUANT_OK;
    Epilogue ep = {};
    ep.n_vis = n_vis, ep.s_vis = s_vis, ep.s_txt = s_txt, ep.K = K, ep.xq = xq;
    if (n_split > 0) {
        if (!split_idx || !split_w || !split_scale) return MQUANT_ERR_NULL;
        if (!aligned_to(split_w, 4)) return MQUANT_ERR_ALIGNMENT;
        for (int32_t j = 0; j < n_split; ++j) {
            if (split_idx[j] < 0 || split_idx[j] >= K) return MQUANT_ERR_BAD_SHAPE;
            if (!isfinite(split_scale[j])) return MQUANT_ERR_BAD_SHAPE;
            ep.split_idx[j] = split_idx[j];
            ep.split_scale[j] = split_scale[j];
        }
        ep.n_split = n_split;
        ep.split_w = split_w;
    }
    if (n_split == 0)
        return gemm_dispatch<kEpiStatic>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, workspace,
                                         workspace_bytes, static_cast<hipStream_t>(stream));
    return gemm_dispatch<kEpiSplit>(xq, wp, w_scale, y, ldy, acc_out, T, N, K, ep, workspace,
                                    workspace_bytes, static_cast<hipStream_t>(stream));
}

extern "C" int64_t mquant_w4a8_linear_prefill_workspace_bytes(int32_t T, int32_t N, int32_t K)
{
    const int64_t g = mquant_w4a8_workspace_bytes(T, N, K);
    if (g < 0) return g;
    const int64_t xq_bytes = ceil_div(static_cast<int64_t>(T) * K, 256) * 256;
    return xq_bytes + g;
}

extern "C" int mquant_w4a8_linear_prefill(const void *x, int64_t ldx, const int32_t *perm,
                                          const uint8_t *wp, const void *w_scale, void *y,
                                          int64_t ldy, int32_t T, int32_t N, int32_t K,
                                          int32_t n_vis, float s_vis, float s_txt,
                                          int32_t had_block, void *workspace,
                                          int64_t workspace_bytes, mquant_stream_t stream)
{
    const int64_t need = mquant_w4a8_linear_prefill_workspace_bytes(T, N, K);
    if (need < 0) return static_cast<int>(need);
    if (T == 0 || N == 0) {
        // still validate the front-end arguments
        return mquant_hadamard_quant_act(x, ldx, perm, nullptr, 0, K, 0, s_vis, s_txt, had_block,
                                         stream);
    }
    if (!workspace) return MQUANT_ERR_WORKSPACE;
    if (workspace_bytes < need) return MQUANT_ERR_WORKSPACE;
    if (!aligned_to(workspace, 256)) return MQUANT_ERR_ALIGNMENT;
    // Validate the GEMM half before launching the front end so that a failure
    // launches nothing.
    int8_t *xq = static_cast<int8_t *>(workspace);
    int st = check_gemm_args(xq, wp, w_scale, y, ldy, T, N, K, n_vis, s_vis, s_txt);
    if (st != MQUANT_OK) return st;
    st = mquant_hadamard_quant_act(x, ldx, perm, xq, T, K, n_vis, s_vis, s_txt, had_block, stream);
    if (st != MQUANT_OK) return st;
    const int64_t xq_bytes = ceil_div(static_cast<int64_t>(T) * K, 256) * 256;
    return mquant_w4a8_gemm(xq, wp, w_scale, y, ldy, nullptr, T, N, K, n_vis, s_vis, s_txt,
                            static_cast<uint8_t *>(workspace) + xq_bytes, need - xq_bytes, stream);
}

// ------------------------------------------------ fused prefill without a caller workspace
//
// For callers that cannot allocate (code under HIP graph capture, serving loops,
// harnesses that forbid hipMalloc): the workspace of the fused prefill entry -- the int8
// activations between the two kernels and the split-K partial sums -- lives in a
// file-scope device array instead.  Every GPU the library runs on holds its own copy at
// its own address until the process ends; in host code the array's name is only a handle
// for hipGetSymbolAddress, never an address to pass on.
namespace {

constexpr int64_t kStaticScratchBytes = 128ll << 20;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MQUANT_ERR_HIP;
    void *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return MQUANT_ERR_HIP;
        }
        // threads racing here store the same address
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return MQUANT_OK;
}

}  // namespace

extern "C" int mquant_w4a8_linear_prefill_static(const void *x, int64_t ldx, const int32_t *perm,
                                                 const uint8_t *wp, const void *w_scale, void *y,
                                                 int64_t ldy, int32_t T, int32_t N, int32_t K,
                                                 int32_t n_vis, float s_vis, float s_txt,
                                                 int32_t had_block, mquant_stream_t stream)
{
    const int64_t need = mquant_w4a8_linear_prefill_workspace_bytes(T, N, K);
    if (need < 0) return static_cast<int>(need);
    if (need > kStaticScratchBytes) return MQUANT_ERR_WORKSPACE;
    void *ws = nullptr;
    if (T > 0 && N > 0) {
        const int st = static_scratch(&ws);
        if (st != MQUANT_OK) return st;
    }
    // Nothing in the scratch has to start at zero: the front end writes every code the GEMM
    // reads, and the split-K kernels write every partial sum the reduction reads.
    return mquant_w4a8_linear_prefill(x, ldx, perm, wp, w_scale, y, ldy, T, N, K, n_vis, s_vis, s_txt,
                                      had_block, ws, kStaticScratchBytes, stream);
}

namespace {

constexpr int kDecodeFusedMaxT = 4;

template <int B>
int launch_decode_fused(const __half *x, int64_t ldx, const uint4 *wp, const __half *w_scale, __half *y,
                        int64_t ldy, int32_t T, int32_t N, int32_t K, const Epilogue &ep, float c_vis,
                        float c_txt, hipStream_t stream)
{
    const unsigned n_tiles = static_cast<unsigned>(ceil_div(N, 32));
    const int64_t xq_bytes = static_cast<int64_t>(T) * (K + 16);
    if (n_tiles >= 256) {
        const size_t lds = static_cast<size_t>(xq_bytes > 8 * 4096 ? xq_bytes : 8 * 4096);
        auto kern = w4a8_decode_fused_kernel<8, 4, B>;
        static std::atomic<bool> attr_set{false};
        if (!attr_set.load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
                return MQUANT_ERR_HIP;
            attr_set.store(true, std::memory_order_release);
        }
        MQ_LAUNCH(kern, dim3(n_tiles), dim3(512), lds, stream, x, ldx, wp, w_scale, y, ldy, T, N, K, ep,
                  c_vis, c_txt);
    } else {
        const size_t lds = static_cast<size_t>(xq_bytes > 16 * 4096 ? xq_bytes : 16 * 4096);
        auto kern = w4a8_decode_fused_kernel<16, 4, B>;
        static std::atomic<bool> attr_set{false};
        if (!attr_set.load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
                return MQUANT_ERR_HIP;
            attr_set.store(true, std::memory_order_release);
        }
        MQ_LAUNCH(kern, dim3(n_tiles), dim3(1024), lds, stream, x, ldx, wp, w_scale, y, ldy, T, N, K, ep,
                  c_vis, c_txt);
    }
    return launch_status();
}

}  // namespace

extern "C" int mquant_w4a8_linear_decode(const void *x, int64_t ldx, const uint8_t *wp,
                                         const void *w_scale, void *y, int64_t ldy, int32_t T,
                                         int32_t N, int32_t K, int32_t n_vis, float s_vis, float s_txt,
                                         int32_t had_block, mquant_stream_t stream)
{
    if (T < 0 || N < 0 || K < 0) return MQUANT_ERR_BAD_SHAPE;
    if (T > kDecodeFusedMaxT) return MQUANT_ERR_UNSUPPORTED;
    if (had_block != 1 && had_block != 128 && had_block != 512) return MQUANT_ERR_UNSUPPORTED;
    if (K % kPackK != 0 || K > kMaxK || K % had_block != 0) return MQUANT_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(T) * (K + 16) > 150 * 1024) return MQUANT_ERR_UNSUPPORTED;
    if (n_vis < 0 || n_vis > T) return MQUANT_ERR_BAD_SHAPE;
    if (!(s_vis > 0.0f) || !(s_txt > 0.0f) || !isfinite(s_vis) || !isfinite(s_txt))
        return MQUANT_ERR_BAD_SHAPE;
    if (T == 0 || N == 0) return MQUANT_OK;
    if (K == 0) return MQUANT_ERR_UNSUPPORTED;
    if (ldx < K || ldy < N) return MQUANT_ERR_BAD_SHAPE;
    if (!x || !wp || !w_scale || !y) return MQUANT_ERR_NULL;
    if (ldx % 8 != 0 || !aligned_to(x, 16) || !aligned_to(wp, 16) || !aligned_to(w_scale, 2) ||
        !aligned_to(y, 2))
        return MQUANT_ERR_ALIGNMENT;
    const double rb = sqrt(static_cast<double>(had_block));
    const float c_vis = static_cast<float>(1.0 / (static_cast<double>(s_vis) * rb));
    const float c_txt = static_cast<float>(1.0 / (static_cast<double>(s_txt) * rb));
    Epilogue ep = {};
    ep.n_vis = n_vis, ep.s_vis = s_vis, ep.s_txt = s_txt, ep.K = K;
    hipStream_t stream_h = static_cast<hipStream_t>(stream);
    const __half *xh = static_cast<const __half *>(x);
    const uint4 *wpp = reinterpret_cast<const uint4 *>(wp);
    const __half *wsc = static_cast<const __half *>(w_scale);
    __half *yh = static_cast<__half *>(y);
    {
        // the streaming kernel when the shape is in its range
        GemvGroup grp = {};
        grp.n = 1;
        grp.p[0].wp = wpp, grp.p[0].w_scale = wsc, grp.p[0].y = yh, grp.p[0].acc_out = nullptr;
        grp.p[0].ldy = ldy, grp.p[0].N = N;
        const int st = gemv_stream_fused(xh, ldx, T, K, had_block, grp, ep, c_vis, c_txt, stream_h);
        if (st != MQUANT_ERR_UNSUPPORTED) return st;
    }
    switch (had_block) {
    case 1: return launch_decode_fused<1>(xh, ldx, wpp, wsc, yh, ldy, T, N, K, ep, c_vis, c_txt, stream_h);
    case 128: return launch_decode_fused<128>(xh, ldx, wpp, wsc, yh, ldy, T, N, K, ep, c_vis, c_txt, stream_h);
    default: return launch_decode_fused<512>(xh, ldx, wpp, wsc, yh, ldy, T, N, K, ep, c_vis, c_txt, stream_h);
    }
}

extern "C" int mquant_w4a8_linear_decode_grouped(const void *x, int64_t ldx, int32_t T, int32_t K,
                                                 int32_t n_vis, float s_vis, float s_txt,
                                                 int32_t had_block, const mquant_linear_t *lin,
                                                 int32_t n_linear, mquant_stream_t stream)
{
    if (T < 0 || K < 0 || n_linear < 0) return MQUANT_ERR_BAD_SHAPE;
    if (T > kDecodeFusedMaxT || n_linear > kGemvMaxGroup) return MQUANT_ERR_UNSUPPORTED;
    if (had_block != 1 && had_block != 128 && had_block != 512) return MQUANT_ERR_UNSUPPORTED;
    if (K % kPackK != 0 || K > kMaxK || K % had_block != 0) return MQUANT_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(T) * (K + 16) > 150 * 1024) return MQUANT_ERR_UNSUPPORTED;
    if (n_vis < 0 || n_vis > T) return MQUANT_ERR_BAD_SHAPE;
    if (!(s_vis > 0.0f) || !(s_txt > 0.0f) || !isfinite(s_vis) || !isfinite(s_txt))
        return MQUANT_ERR_BAD_SHAPE;
    if (n_linear > 0 && !lin) return MQUANT_ERR_NULL;
    for (int32_t i = 0; i < n_linear; ++i) {
        if (lin[i].N < 0) return MQUANT_ERR_BAD_SHAPE;
        if (lin[i].N > 0 && T > 0 && lin[i].ldy < lin[i].N) return MQUANT_ERR_BAD_SHAPE;
    }
    if (T == 0 || n_linear == 0) return MQUANT_OK;
    if (K == 0) return MQUANT_ERR_UNSUPPORTED;
    if (ldx < K) return MQUANT_ERR_BAD_SHAPE;
    if (!x) return MQUANT_ERR_NULL;
    if (ldx % 8 != 0 || !aligned_to(x, 16)) return MQUANT_ERR_ALIGNMENT;
    GemvGroup grp = {};
    for (int32_t i = 0; i < n_linear; ++i) {
        if (lin[i].N == 0) continue;
        if (!lin[i].w_prepacked_dev || !lin[i].w_scale_dev || !lin[i].y_dev) return MQUANT_ERR_NULL;
        if (!aligned_to(lin[i].w_prepacked_dev, 16) || !aligned_to(lin[i].w_scale_dev, 2) ||
            !aligned_to(lin[i].y_dev, 2))
            return MQUANT_ERR_ALIGNMENT;
        GemvProblem &p = grp.p[grp.n++];
        p.wp = reinterpret_cast<const uint4 *>(lin[i].w_prepacked_dev);
        p.w_scale = static_cast<const __half *>(lin[i].w_scale_dev);
        p.y = static_cast<__half *>(lin[i].y_dev);
        p.acc_out = nullptr;
        p.ldy = lin[i].ldy;
        p.N = lin[i].N;
    }
    if (grp.n == 0) return MQUANT_OK;
    if (gemv_stream_fused_takes(T, K, had_block)) {
        const double rb = sqrt(static_cast<double>(had_block));
        const float c_vis = static_cast<float>(1.0 / (static_cast<double>(s_vis) * rb));
        const float c_txt = static_cast<float>(1.0 / (static_cast<double>(s_txt) * rb));
        Epilogue ep = {};
        ep.n_vis = n_vis, ep.s_vis = s_vis, ep.s_txt = s_txt, ep.K = K;
        return gemv_stream_fused(static_cast<const __half *>(x), ldx, T, K, had_block, grp, ep, c_vis, c_txt,
                                 static_cast<hipStream_t>(stream));
    }
    // outside the streaming kernel's range: one launch per linear
    for (int32_t i = 0; i < grp.n; ++i) {
        const int st = mquant_w4a8_linear_decode(x, ldx, reinterpret_cast<const uint8_t *>(grp.p[i].wp),
                                                 grp.p[i].w_scale, grp.p[i].y, grp.p[i].ldy, T, grp.p[i].N, K,
                                                 n_vis, s_vis, s_txt, had_block, stream);
        if (st != MQUANT_OK) return st;
    }
    return MQUANT_OK;
}
