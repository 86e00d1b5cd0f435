// Causal attention on AIFS-ordered tokens and rotary embedding with reordered
// position ids, for gfx950 (MQuant, arXiv 2502.00425: Sec. 3.1, Eq. (5)-(6);
// appendix "Rotary Position Embedding for AIFS").
//
// After the AIFS reorder a token's row index no longer says what it may attend.
// Its original position does: token i attends token j exactly when
// pos[j] <= pos[i] (the unified mask M^u[i,j] = M[pos[i], pos[j]] of the causal
// M; for one visual segment this is the three-region rule of Eq. (6)).  The
// kernel never materialises a [T,T] mask: it compares positions per element on
// the tiles that need it, takes whole tiles unmasked or skips them by the
// min/max of their positions, flash-attention style (online softmax, fp32
// statistics, fp16 MFMA operands).
#include <hip/hip_fp16.h>

#include <climits>
#include <cmath>

#include "lds_dma.h"
#include "mquant_internal.h"

using namespace mquant;

namespace {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

constexpr int kHeadDim = 128;          // the only head size built (28 x 128, 64 x 128 in the paper's models)
constexpr int kBQ = 128;               // queries per work-group (32 per wave)
constexpr int kBK = 64;                // keys per tile
constexpr int kAhead = 4;               // LDS fragment reads in flight ahead of the MFMA that uses them
constexpr int kKTile = kBK * 2 * kHeadDim;   // a key tile in LDS: 64 rows of 256 bytes
constexpr int kVTile = kHeadDim * 2 * kBK;   // a V^T tile in LDS: 128 rows (head channels) of 128 bytes

// Tiles arrive by LDS-DMA (1 KiB per wave instruction, lane i at offset 16 i), so rows cannot
// be padded; instead the 16-byte chunks of a row are XOR-swizzled, on the global side of the
// copy, so that the 16 lanes the LDS serves together (16 consecutive rows, one logical chunk)
// cover the 64 banks exactly once: key rows are 256 bytes (the full bank space), V^T rows 128.
// Chunk c of key row r sits at r * 256 + ((c ^ (r & 15)) << 4), chunk c of V^T row d at
// d * 128 + ((c ^ ((d >> 1) & 7)) << 4).

// Key order inside the V^T rows: the P V product takes its key index from the score registers
// (operand slot i of lane group g is key 16 kk + 8 (i / 4) + 4 g + i % 4), so the transpose
// stores every 16 keys as 0-3, 8-11, 4-7, 12-15 and an operand is one aligned 16-byte chunk.
__device__ __forceinline__ int vt_key_of_slot(int p)
{
    const int x = p & 15;
    return (p & ~15) | (x < 4 ? x : (x < 8 ? x + 4 : (x < 12 ? x - 4 : x)));
}

// The value of the partner lane (lane ^ 32) next to this lane's own: v_permlane32_swap on two
// copies leaves {low half, low half} and {high half, high half}; no LDS traffic, so fragment
// reads that are in flight are not waited for.
__device__ __forceinline__ void halves_of(float x, float &lo, float &hi)
{
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
    lo = __int_as_float(sw[0]);
    hi = __int_as_float(sw[1]);
}

// MFMA 32x32 result register r of lane group g holds row (r/4)*8 + g*4 + r%4.
__device__ __forceinline__ int acc_row(int r, int g) { return (r >> 2) * 8 + g * 4 + (r & 3); }

// ------------------------------------------------------------------- RoPE
//
// x'[2j] = x[2j] cos - x[2j+1] sin, x'[2j+1] = x[2j] sin + x[2j+1] cos with the
// angle pos[i] * theta_j, theta_j = base^(-2j/D): the block-diagonal rotation
// printed in the appendix, with the token's ORIGINAL position as its id.  The
// angle and its sine/cosine are formed in double (a position of 16384 leaves an
// fp32 angle accurate to 1e-3 only); one thread per (token, pair) serves all heads.
struct InvFreq {
    double f[kHeadDim / 2];
};

__global__ __launch_bounds__(256) void rope_kernel(__half *__restrict__ x, int64_t ldx,
                                                   const int32_t *__restrict__ pos, int32_t T,
                                                   int32_t n_heads, InvFreq inv)
{
    constexpr int P = kHeadDim / 2;
    const int64_t total = static_cast<int64_t>(T) * P;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; e < total;
         e += static_cast<int64_t>(gridDim.x) * 256) {
        const int32_t i = static_cast<int32_t>(e / P);
        const int32_t j = static_cast<int32_t>(e - static_cast<int64_t>(i) * P);
        double sn, cs;
        sincos(static_cast<double>(pos[i]) * inv.f[j], &sn, &cs);
        const float c = static_cast<float>(cs), s = static_cast<float>(sn);
        __half2 *row = reinterpret_cast<__half2 *>(x + static_cast<int64_t>(i) * ldx) + j;
        for (int32_t h = 0; h < n_heads; ++h) {
            const float2 v = __half22float2(row[h * P]);
            row[h * P] = __floats2half2_rn(v.x * c - v.y * s, v.x * s + v.y * c);
        }
    }
}

// -------------------------------------------------------- V^T and tile bounds
//
// The P V product wants, per head channel, the eight keys of an MFMA operand in one
// 16-byte chunk, so V goes through a one-off transpose V[T][Hkv*D] -> Vt[Hkv*D][Tp]
// (Tp = T rounded up to the key tile, tail zeroed: a zero probability times an
// uninitialised value could be NaN; keys inside a row in the order of vt_key_of_slot).
// The same launch records min and max position of every key tile.
__global__ __launch_bounds__(256) void vt_kernel(const __half *__restrict__ v, int64_t ldv,
                                                 __half *__restrict__ vt, int32_t T, int32_t Tp,
                                                 int32_t channels, const int32_t *__restrict__ pos,
                                                 int32_t *__restrict__ tile_min,
                                                 int32_t *__restrict__ tile_max)
{
    // 64 tokens x 64 channels per group; 16-byte accesses on both sides (channels is a
    // multiple of 64 here: whole heads of 128).
    __shared__ __attribute__((aligned(16))) __half tile[64][72];
    const int32_t t0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int r8 = threadIdx.x >> 3, c8 = (threadIdx.x & 7) * 8;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int r = half * 32 + r8;
        const int32_t t = t0 + r;
        uint4 val = make_uint4(0u, 0u, 0u, 0u);
        if (t < T) val = *reinterpret_cast<const uint4 *>(v + static_cast<int64_t>(t) * ldv + c0 + c8);
        *reinterpret_cast<uint4 *>(&tile[r][c8]) = val;
    }
    __syncthreads();
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int c = half * 32 + r8;                       // channel row of the transposed tile
        __half out[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = tile[vt_key_of_slot(c8 + i)][c];
        *reinterpret_cast<uint4 *>(vt + static_cast<int64_t>(c0 + c) * Tp + t0 + c8) =
            *reinterpret_cast<const uint4 *>(out);
    }
    if (blockIdx.y == 0 && threadIdx.x < 64) {
        const int32_t t = t0 + threadIdx.x;
        int32_t lo = t < T ? pos[t] : INT_MAX, hi = t < T ? pos[t] : INT_MIN;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            lo = min(lo, __shfl_xor(lo, m, 64));
            hi = max(hi, __shfl_xor(hi, m, 64));
        }
        if (threadIdx.x == 0) {
            tile_min[blockIdx.x] = lo;
            tile_max[blockIdx.x] = hi;
        }
    }
}

// -------------------------------------------------------------- attention
//
// One work-group: 128 queries of one query head, four waves of 32 queries.
// Per key tile (64 keys, shared through LDS):
//   S^T = K Q^T     A = K rows (keys) from LDS, B = Q^T held in registers for the whole
//                   kernel; in the result a LANE is a query, its registers are keys, so
//                   the softmax statistics of a query live in one lane pair
//   P^T             the same registers, as fp16, are the B operand of
//   O^T += V^T P^T  A = V^T rows (head channels) from LDS; the result again has a lane per
//                   query, so the running rescale needs no cross-lane traffic.
// Software pipeline, one tile deep inside a wave: while the exponentials of tile j run on
// the vector ALU, the matrix core computes the scores of tile j+1 (a second score register
// set; the two instruction streams are written interleaved and pinned), so of the three
// parts of a tile -- scores, softmax, P V -- only two are paid in sequence.  Key tiles are
// therefore fetched one step ahead of value tiles.  Tiles travel global -> LDS by LDS-DMA
// (no staging registers), two buffers each for K and V^T, one barrier per tile.
// Tiles whose smallest position exceeds the group's largest query position are skipped
// altogether (no loads); a wave skips the arithmetic of a tile that is masked for all of its
// 32 queries and drops the per-element compare on tiles that are visible to all of them.
__global__ __launch_bounds__(256, 2) void aifs_attention_kernel(
    const __half *__restrict__ q, int64_t ldq, const __half *__restrict__ k, int64_t ldk,
    const __half *__restrict__ vt, int32_t Tp, __half *__restrict__ o, int64_t ldo,
    const int32_t *__restrict__ pos, const int32_t *__restrict__ tile_min,
    const int32_t *__restrict__ tile_max, int32_t T, int32_t group, int32_t n_kv_heads, int32_t n_qblocks,
    int32_t xcds_per_kv, float scale_log2e)
{
    __shared__ __attribute__((aligned(1024))) uint8_t k_lds2[2][kKTile];
    __shared__ __attribute__((aligned(1024))) uint8_t v_lds2[2][kVTile];
    __shared__ int32_t pos_lds2[2][kBK];
    __shared__ int32_t wg_qmax_lds[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    // Work-group ids are dealt round-robin to the 8 XCDs, each with its own L2.  When the
    // key/value heads divide the XCDs evenly (xcds_per_kv > 0), an XCD serves ONE key/value
    // head: its resident work-groups then walk the same key tiles at about the same time and
    // the L2 fetches each tile once for all of them (with heads simply dealt in order every
    // XCD streams all key/value heads and two thirds of the tile requests hit).  Query blocks
    // go from the last to the first: in AIFS order the later blocks of each modality see the
    // most keys, so the long work-groups start first and the short ones fill the end.
    const int32_t n_heads = group * n_kv_heads;
    int32_t head, qblock;
    if (xcds_per_kv > 0) {
        const int32_t xcd = blockIdx.x % 8, n = blockIdx.x / 8;
        const int32_t m = n * xcds_per_kv + xcd % xcds_per_kv;      // item of this key/value head
        if (m >= n_qblocks * group) return;                         // uniform: whole work-group
        head = (xcd / xcds_per_kv) * group + m % group;
        qblock = n_qblocks - 1 - m / group;
    } else {
        head = blockIdx.x % n_heads;
        qblock = n_qblocks - 1 - blockIdx.x / n_heads;
    }
    const int32_t kvh = head / group;
    const int32_t q0 = qblock * kBQ + wave * 32;
    const int32_t n_tiles = Tp / kBK;

    // ---- this lane's query: position and Q^T fragments
    const int32_t qi = q0 + l32;
    const int32_t qrow = qi < T ? qi : T - 1;
    const int32_t my_pos = pos[qrow];
    v8h qf[kHeadDim / 16];
    {
        const __half *qp = q + static_cast<int64_t>(qrow) * ldq + head * kHeadDim + g * 8;
#pragma unroll
        for (int ks = 0; ks < kHeadDim / 16; ++ks)
            qf[ks] = *reinterpret_cast<const v8h *>(qp + ks * 16);
    }
    int32_t qmin = my_pos, qmax = my_pos;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        qmin = min(qmin, __shfl_xor(qmin, m, 64));
        qmax = max(qmax, __shfl_xor(qmax, m, 64));
    }
    if (lane == 0) wg_qmax_lds[wave] = qmax;
    __syncthreads();
    const int32_t wg_qmax = max(max(wg_qmax_lds[0], wg_qmax_lds[1]), max(wg_qmax_lds[2], wg_qmax_lds[3]));

    v16f acc_o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[dt][r] = 0.0f;

    // ---- tile copies: 16 blocks of 1 KiB per tile, four per wave.  A copy instruction takes a
    // wave-uniform base (scalar registers) and a 32-bit offset per lane; block i of a wave lies
    // a fixed stride after block 0, so a lane keeps three offsets in registers and nothing more
    // (full 64-bit addresses per copy, hoisted out of the loop, spilled to scratch memory).
    const uint8_t *kbase = reinterpret_cast<const uint8_t *>(k + kvh * kHeadDim);
    const uint8_t *vbase = reinterpret_cast<const uint8_t *>(vt + static_cast<int64_t>(kvh) * kHeadDim * Tp);
    const uint32_t k_lds_addr = lds_address(&k_lds2[0][0]), v_lds_addr = lds_address(&v_lds2[0][0]);
    const int32_t k_row = wave * 4 + (lane >> 4);          // key row of this lane in block 0 (block i: + 16 i)
    const uint32_t k_chunk = static_cast<uint32_t>(((lane & 15) ^ (k_row & 15)) << 4);
    const int32_t v_d = wave * 8 + (lane >> 3);            // head channel of this lane in block 0 (block i: + 32 i)
    const uint32_t v_lane = static_cast<uint32_t>(v_d) * static_cast<uint32_t>(Tp) * 2u +
                            static_cast<uint32_t>(((lane & 7) ^ ((v_d >> 1) & 7)) << 4);
    const uint32_t k_pitch = static_cast<uint32_t>(ldk) * 2u;
    auto dma_k = [&](int32_t t, int b) {                   // rows past T repeat the last row (masked later)
        const uint8_t *tile = kbase + static_cast<int64_t>(t) * kBK * ldk * 2;
        const int32_t last = T - 1 - t * kBK;              // last valid row of this tile
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int32_t row = k_row + 16 * i;
            row = row < last ? row : last;
            lds_dma16_uniform_base(tile, static_cast<uint32_t>(row) * k_pitch + k_chunk,
                                   k_lds_addr + b * kKTile + (i * 4 + wave) * 1024);
        }
    };
    auto dma_v = [&](int32_t t, int b) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            lds_dma16_uniform_base(vbase + (static_cast<int64_t>(i) * 32 * Tp + static_cast<int64_t>(t) * kBK) * 2, v_lane,
                                   v_lds_addr + b * kVTile + (i * 4 + wave) * 1024);
    };
    auto key_pos = [&](int32_t t) -> int32_t {             // threads 0..63: position of key tid of tile t
        const int32_t key = t * kBK + (tid & 63);
        return key < T ? pos[key] : INT_MAX;
    };
    auto next_tile = [&](int32_t t) {                     // first tile >= t the group needs, or n_tiles
        while (t < n_tiles && tile_min[t] > wg_qmax) ++t;
        return t;
    };
    // LDS fragments: MFMA i of the score product is (ks, kb) = (i / 2, i % 2), of the P V
    // product (kk, dt) = (i / 4, i % 4); consecutive MFMAs write different accumulators.
    const int kswz = l32 & 15, vswz = (l32 >> 1) & 7;
    auto kfrag = [&](const uint8_t *kb_lds, int i) {
        return *reinterpret_cast<const v8h *>(kb_lds + ((i & 1) * 32 + l32) * 256 + ((((i >> 1) * 2 + g) ^ kswz) << 4));
    };
    auto vfrag = [&](const uint8_t *vb_lds, int i) {
        return *reinterpret_cast<const v8h *>(vb_lds + ((i & 3) * 32 + l32) * 128 + ((((i >> 2) * 2 + g) ^ vswz) << 4));
    };
    const v16f zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // scores of one tile on their own (first tile; tiles whose predecessor this wave skips)
    auto scores = [&](const uint8_t *kb_lds, v16f (&s)[2]) {
        v8h fr[kAhead];
#pragma unroll
        for (int i = 0; i < kAhead; ++i) fr[i] = kfrag(kb_lds, i);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2 * (kHeadDim / 16); ++i) {
            s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fr[i % kAhead], qf[i >> 1], i < 2 ? zero16 : s[i & 1], 0, 0, 0);
            if (i + kAhead < 2 * (kHeadDim / 16)) fr[i % kAhead] = kfrag(kb_lds, i + kAhead);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Running statistics in raw-logit units; the exponent is exp2((s - m_ref) * c) as one
    // fused multiply-add per element.  m_ref is the reference maximum the accumulators are
    // scaled to; it follows the true maximum lazily: only when some query's maximum has grown
    // by more than kLazy (a factor 2^kLazy in the probabilities, harmless in fp16 and fp32)
    // are the accumulators rescaled, so most tiles skip the 64 multiplies and the exponential.
    constexpr float kLazy = 8.0f;
    const float lazy_raw = kLazy / scale_log2e;
    float m_ref = -INFINITY, l_run = 0.0f;

    // One step of the pipeline: softmax and P V of tile `cur` (scores in s_cur, values in V
    // buffer par, positions in pos buffer par) while the scores of tile `nxt` (keys in K
    // buffer par ^ 1) go to s_nxt.  On entry a barrier has published those buffers and freed
    // K buffer par (its scores are done) and V buffer par ^ 1 (its P V product is done).
    int32_t cur, nxt;
    int32_t kmin_c, kmax_c, kmin_n, kmax_n;               // bounds of the positions of cur and nxt
    auto step = [&](v16f (&s_cur)[2], v16f (&s_nxt)[2], const int par) {
        const int32_t nn = nxt < n_tiles ? next_tile(nxt + 1) : n_tiles;
        if (nn < n_tiles) dma_k(nn, par);
        if (nxt < n_tiles) dma_v(nxt, par ^ 1);
        int32_t preg = INT_MAX;
        if (tid < kBK && nxt < n_tiles) preg = key_pos(nxt);
        // bounds of nn: requested a whole step before they decide a branch
        const int32_t nn_c = nn < n_tiles ? nn : 0;
        const int32_t kmin_nn = tile_min[nn_c], kmax_nn = tile_max[nn_c];
        const uint8_t *kb_lds = k_lds2[par ^ 1], *vb_lds = v_lds2[par];
        const int32_t *pos_lds = pos_lds2[par];
        const bool need_cur = kmin_c <= qmax;              // else: masked for all 32 queries of the wave
        const bool need_nxt = nxt < n_tiles && kmin_n <= qmax;
        const bool padded = (cur + 1) * kBK > T;           // tile holds keys past the end
        if (need_cur) {
            // ---- mask, online softmax
            if (kmax_c > qmin || padded) {                 // wave-uniform: some (query, key) pair is hidden
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (pos_lds[kb * 32 + acc_row(r, g)] > my_pos) s_cur[kb][r] = -INFINITY;
            }
            float m_new = m_ref;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) m_new = fmaxf(m_new, s_cur[kb][r]);
            {
                float lo, hi;
                halves_of(m_new, lo, hi);                        // the query's other 32 keys
                m_new = fmaxf(lo, hi);
            }
            if (__any(m_new > m_ref + lazy_raw)) {         // also the first visible tile (m_ref = -inf)
                const float m_use = m_new == -INFINITY ? 0.0f : m_new;
                const float alpha = __builtin_amdgcn_exp2f((m_ref - m_use) * scale_log2e);   // exp2(-inf) = 0
                l_run *= alpha;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc_o[dt][r] *= alpha;
                m_ref = m_new;
            }
            const float neg = m_ref == -INFINITY ? 0.0f : -m_ref * scale_log2e;
            float l_add = 0.0f;
            v8h p[4];
            // The two branches below take the offset from different registers (`neg_alone` is
            // a copy the compiler cannot see through): written alike, the compiler merges the
            // exponentials of both and hoists them in front of the branch, out from between
            // the MFMAs of the interleaved one.
            float neg_alone = neg;
            asm volatile("" : "+v"(neg_alone));
            auto exp_pair = [&](int e, float off) {        // elements 2e, 2e+1 of the 32 scores of a lane
                const int kb = e >> 3, r = (e & 7) * 2;
                const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[kb][r], scale_log2e, off));
                const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[kb][r + 1], scale_log2e, off));
                // the denominator sums the probabilities as the P V product sees them (rounded
                // to fp16): one dot-product instruction per pair instead of two additions
                v2h ph;
                ph[0] = static_cast<_Float16>(e0);
                ph[1] = static_cast<_Float16>(e1);
                l_add = __builtin_amdgcn_fdot2(ph, v2h{1, 1}, l_add, false);
                p[kb * 2 + (r >> 3)][r & 7] = ph[0];
                p[kb * 2 + (r >> 3)][(r & 7) + 1] = ph[1];
            };
            v8h fr[kAhead];
            if (need_nxt) {
                // exponentials of this tile interleaved with the score MFMAs of the next one:
                // one MFMA, its fragment read, two exponentials per group, order pinned
#pragma unroll
                for (int i = 0; i < kAhead; ++i) fr[i] = kfrag(kb_lds, i);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    s_nxt[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fr[i % kAhead], qf[i >> 1],
                                                                          i < 2 ? zero16 : s_nxt[i & 1], 0, 0, 0);
                    if (i + kAhead < 16) fr[i % kAhead] = kfrag(kb_lds, i + kAhead);
                    exp_pair(i, neg);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) exp_pair(i, neg_alone);
            }
            // the first V^T fragments travel while the sums are exchanged
#pragma unroll
            for (int i = 0; i < kAhead; ++i) fr[i] = vfrag(vb_lds, i);
            __builtin_amdgcn_sched_barrier(0);
            {
                float lo, hi;
                halves_of(l_add, lo, hi);
                l_add = lo + hi;
            }
            l_run += l_add;
            // ---- O^T += V^T P^T (the four channel blocks alternate; same rotating window)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                acc_o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fr[i % kAhead], p[i >> 2], acc_o[i & 3], 0, 0, 0);
                if (i + kAhead < 16) fr[i % kAhead] = vfrag(vb_lds, i + kAhead);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else if (need_nxt) {
            scores(kb_lds, s_nxt);
        }
        if (tid < kBK) pos_lds2[par ^ 1][tid] = preg;
        wait_vmcnt<0>();                                   // K of nn and V^T of nxt have landed
        __syncthreads();
        cur = nxt;
        nxt = nn;
        kmin_c = kmin_n, kmax_c = kmax_n;
        kmin_n = kmin_nn, kmax_n = kmax_nn;
    };

    // ---- prologue: first tile's keys, values and positions, second tile's keys
    cur = next_tile(0);                                    // exists: every token sees itself
    nxt = cur < n_tiles ? next_tile(cur + 1) : n_tiles;
    if (cur < n_tiles) {
        dma_k(cur, 0);
        dma_v(cur, 0);
        if (nxt < n_tiles) dma_k(nxt, 1);
        if (tid < kBK) pos_lds2[0][tid] = key_pos(cur);
    }
    {
        const int32_t c = cur < n_tiles ? cur : 0, n = nxt < n_tiles ? nxt : 0;
        kmin_c = tile_min[c], kmax_c = tile_max[c];
        kmin_n = tile_min[n], kmax_n = tile_max[n];
    }
    wait_vmcnt<0>();
    __syncthreads();
    v16f s_a[2], s_b[2];
    if (cur < n_tiles && kmin_c <= qmax) scores(k_lds2[0], s_a);
    __syncthreads();                                       // K buffer 0 is free for the third tile
    while (cur < n_tiles) {
        step(s_a, s_b, 0);
        if (cur >= n_tiles) break;
        step(s_b, s_a, 1);
    }

    // ---- normalise and store: lane = query, registers = head channels (4 consecutive per group)
    if (qi < T) {
        const float inv_l = 1.0f / l_run;                  // every token sees at least itself
        __half *orow = o + static_cast<int64_t>(qi) * ldo + head * kHeadDim;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                __half h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = __float2half_rn(acc_o[dt][r4 * 4 + e] * inv_l);
                *reinterpret_cast<uint2 *>(orow + dt * 32 + r4 * 8 + g * 4) = *reinterpret_cast<const uint2 *>(h);
            }
    }
}

int check_heads(int32_t T, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim)
{
    if (T < 0 || n_q_heads < 1 || n_kv_heads < 1) return MQUANT_ERR_BAD_SHAPE;
    if (head_dim != kHeadDim) return MQUANT_ERR_UNSUPPORTED;
    if (n_q_heads % n_kv_heads != 0) return MQUANT_ERR_BAD_SHAPE;
    return MQUANT_OK;
}

int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

}  // namespace

extern "C" int mquant_rope_apply(void *x, int64_t ldx, const int32_t *pos, int32_t T, int32_t n_heads,
                                 int32_t head_dim, double base, mquant_stream_t stream)
{
    if (T < 0 || n_heads < 1) return MQUANT_ERR_BAD_SHAPE;
    if (head_dim != kHeadDim) return MQUANT_ERR_UNSUPPORTED;
    if (!(base > 1.0) || !std::isfinite(base)) return MQUANT_ERR_BAD_SHAPE;
    if (T == 0) return MQUANT_OK;
    if (!x || !pos) return MQUANT_ERR_NULL;
    if (ldx < static_cast<int64_t>(n_heads) * head_dim) return MQUANT_ERR_BAD_SHAPE;
    if (ldx % 2 != 0 || !aligned_to(x, 4) || !aligned_to(pos, 4)) return MQUANT_ERR_ALIGNMENT;
    InvFreq inv;
    for (int j = 0; j < kHeadDim / 2; ++j) inv.f[j] = pow(base, -2.0 * j / kHeadDim);
    int64_t blocks = ceil_div(static_cast<int64_t>(T) * (kHeadDim / 2), 256);
    if (blocks > 65536) blocks = 65536;
    MQ_LAUNCH(rope_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0,
              static_cast<hipStream_t>(stream), static_cast<__half *>(x), ldx, pos, T, n_heads, inv);
    return launch_status();
}

extern "C" int64_t mquant_aifs_attention_workspace_bytes(int32_t T, int32_t n_kv_heads, int32_t head_dim)
{
    if (T < 0 || n_kv_heads < 1) return MQUANT_ERR_BAD_SHAPE;
    if (head_dim != kHeadDim) return MQUANT_ERR_UNSUPPORTED;
    const int64_t Tp = round_up(T, kBK);
    const int64_t vt = round_up(static_cast<int64_t>(n_kv_heads) * head_dim * Tp * 2, 256);
    return vt + round_up(2 * (Tp / kBK) * 4, 256);
}

extern "C" int mquant_aifs_attention(const void *q, int64_t ldq, const void *k, int64_t ldk,
                                     const void *v, int64_t ldv, void *o, int64_t ldo,
                                     const int32_t *pos, int32_t T, int32_t n_q_heads,
                                     int32_t n_kv_heads, int32_t head_dim, void *workspace,
                                     int64_t workspace_bytes, mquant_stream_t stream_)
{
    const int st = check_heads(T, n_q_heads, n_kv_heads, head_dim);
    if (st != MQUANT_OK) return st;
    if (T == 0) return MQUANT_OK;
    if (!q || !k || !v || !o || !pos) return MQUANT_ERR_NULL;
    const int64_t qw = static_cast<int64_t>(n_q_heads) * head_dim, kw = static_cast<int64_t>(n_kv_heads) * head_dim;
    if (ldq < qw || ldo < qw || ldk < kw || ldv < kw) return MQUANT_ERR_BAD_SHAPE;
    if (ldq % 8 != 0 || ldk % 8 != 0 || ldv % 8 != 0 || ldo % 4 != 0 || !aligned_to(q, 16) ||
        !aligned_to(k, 16) || !aligned_to(v, 16) || !aligned_to(o, 8) || !aligned_to(pos, 4))
        return MQUANT_ERR_ALIGNMENT;
    const int64_t need = mquant_aifs_attention_workspace_bytes(T, n_kv_heads, head_dim);
    if (!workspace || workspace_bytes < need) return MQUANT_ERR_WORKSPACE;
    if (!aligned_to(workspace, 256)) return MQUANT_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_);

    const int32_t Tp = static_cast<int32_t>(round_up(T, kBK));
    const int32_t n_tiles = Tp / kBK;
    __half *vt = static_cast<__half *>(workspace);
    int32_t *tile_min = reinterpret_cast<int32_t *>(
        static_cast<uint8_t *>(workspace) + round_up(kw * Tp * 2, 256));
    int32_t *tile_max = tile_min + n_tiles;
    MQ_LAUNCH(vt_kernel, dim3(n_tiles, static_cast<unsigned>(ceil_div(kw, 64))), dim3(256), 0, stream,
              static_cast<const __half *>(v), ldv, vt, T, Tp, static_cast<int32_t>(kw), pos, tile_min,
              tile_max);
    int ls = launch_status();
    if (ls != MQUANT_OK) return ls;
    const float scale_log2e = static_cast<float>(1.4426950408889634 / sqrt(static_cast<double>(head_dim)));
    const int64_t n_qblocks = ceil_div(T, kBQ);
    const int32_t group = n_q_heads / n_kv_heads;
    const int32_t xcds_per_kv = 8 % n_kv_heads == 0 ? 8 / n_kv_heads : 0;
    const int64_t groups = xcds_per_kv > 0 ? 8 * ceil_div(n_qblocks * group, xcds_per_kv) : n_qblocks * n_q_heads;
    if (groups > 0x7fffffff) return MQUANT_ERR_UNSUPPORTED;
    MQ_LAUNCH(aifs_attention_kernel, dim3(static_cast<unsigned>(groups)), dim3(256),
              0, stream, static_cast<const __half *>(q), ldq, static_cast<const __half *>(k), ldk, vt, Tp,
              static_cast<__half *>(o), ldo, pos, tile_min, tile_max, T, group, n_kv_heads,
              static_cast<int32_t>(n_qblocks), xcds_per_kv, scale_log2e);
    return launch_status();
}
