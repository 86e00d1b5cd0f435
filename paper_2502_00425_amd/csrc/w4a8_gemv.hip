// W4A8 GEMV for decode (MQuant Sec. 4: "custom W4A8 GEMV kernel", the decode rows of the
// speed tables): T <= 4 new rows against an [N, K] int4 weight that is streamed from HBM
// exactly once.  Nothing is reused, so the kernel is a read stream with a little arithmetic
// attached, and what decides its speed is how the stream is cut up and kept in flight:
//
//   - A work-group owns 32 / F output channels over all of K (F = 1 or 2) and needs no
//     partner: partial sums meet in LDS, never in memory.  F = 2 (16-channel halves of the
//     prepacked 32-channel tiles, i.e. 256-byte pieces at a stride of 512 bytes) doubles the
//     number of work-groups for matrices with few output tiles (N = 3584 has 112 tiles for
//     256 compute units) and uses the 16x16x64 matrix instruction; F = 1 reads whole 1 KiB
//     tiles and uses the 32x32x32 one.
//   - Every wave keeps DEPTH loads of 1 KiB in flight all the time: the load that refills a
//     register set is issued right after the set has been consumed (a rolling pipeline), so
//     the memory pipe never drains between batches or between the k-range's ends.
//   - The T quantized rows (T * K bytes) are copied to LDS once per work-group while the first
//     loads are in flight; the matrix instruction's token operand is read from there.
//   - Several linears that share their input (q/k/v, gate/up) can go into one launch: the grid
//     is the concatenation of their units.
#include <hip/hip_fp16.h>
#include <math.h>

#include "hadamard_segment.h"
#include "mquant_internal.h"
#include "w4a8_common.h"

using namespace mquant;

namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// HB > 0: the rotate + quantize front end runs inside the kernel (Sec. 3.2 rotation with
// Hadamard block HB, Eq. (2)/(3) static quantizer: the wave-level code of the stand-alone
// kernel).  x is then the fp16 input [T, ldx]; every work-group rotates and quantizes the T
// rows itself, one 512-channel segment per wave at a time (NX = segments per wave), straight
// into the LDS copy that the xq path fills by copying.  The work is redundant across
// work-groups but runs under the latency of the first weight loads, and it saves a launch per
// linear, which at decode costs as much as a small GEMV.
template <int F, int WAVES, int DEPTH, int NX, int EPI, int HB>
__global__ __launch_bounds__(WAVES * 64) void w4a8_gemv_stream_kernel(
    const int8_t *__restrict__ xq, int32_t T, int32_t K, GemvGroup grp, Epilogue ep,
    const __half *__restrict__ x, int64_t ldx, float c_vis, float c_txt)
{
    static_assert(F == 1 || F == 2, "channels per work-group: 32 or 16");
    static_assert(HB == 0 || HB <= 512, "one 512-channel segment per wave and step");
    // 16 bytes that every wave has in cache, for loads past a wave's range
    const uint4 *hot = HB > 0 ? reinterpret_cast<const uint4 *>(x) : reinterpret_cast<const uint4 *>(xq);
    constexpr int CH = 32 / F;                    // output channels of a work-group
    constexpr int STEP = 64 * F;                  // input channels one wave-load covers
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];   // T rows of xq, pitch K + 16
    const int32_t pitch = K + 16;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

    // which linear of the group, which unit of it
    int32_t pi = 0, unit = blockIdx.x;
    while (pi + 1 < grp.n && unit >= grp.p[pi].units) {
        unit -= grp.p[pi].units;
        ++pi;
    }
    const GemvProblem &pr = grp.p[pi];
    const int32_t N = pr.N;
    const int32_t k_tiles = K / kPackK;
    const int32_t loads = k_tiles / F;            // wave-loads of this unit (K % (64 F) == 0)
    const int32_t per_wave = (loads + WAVES - 1) / WAVES;
    const int32_t j0 = wave * per_wave;
    int32_t j1 = j0 + per_wave;
    j1 = j1 < loads ? j1 : loads;
    const int32_t n_mine = j1 > j0 ? j1 - j0 : 0;

    // Lane -> its 16 bytes inside a wave-load, and the first input channel they hold.
    //   F = 1: the whole tile, lane = (channel % 32) + 32 g, channels k = 64 j + 32 g ...
    //   F = 2: half h of two consecutive tiles; lane = c + 16 q, q = 2 * (tile in pair) + g,
    //          channels k = 128 j + 32 q ...
    const int32_t nt = unit / F, h = unit % F;
    int32_t lane_vec, k_lane;
    if constexpr (F == 1) {
        lane_vec = lane;
        k_lane = (lane >> 5) * 32;
    } else {
        const int q = lane >> 4, c = lane & 15;
        lane_vec = (q >> 1) * 64 + (q & 1) * 32 + h * 16 + c;
        k_lane = q * 32;
    }
    const uint4 *wsrc = pr.wp + static_cast<int64_t>(nt) * k_tiles * 64 + lane_vec;
    auto load_w = [&](int32_t j) -> uint4 {
        // Past the wave's range the load stays (the pipeline is branch-free) but reads the first
        // 16 bytes of the input, which every wave has in cache; its value is masked below.
        const uint4 *src = j < j1 ? wsrc + static_cast<int64_t>(j) * (64 * F) : hot;
        const v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src));
        return make_uint4(t[0], t[1], t[2], t[3]);
    };
    uint4 b[DEPTH];
    const int32_t n_ch = nt * 32 + h * CH + (lane & (CH - 1));            // this lane's output channel
    __half ws_h;

    if constexpr (HB > 0) {
        // ---- fused front end: x segments first (they must arrive first), then the weights
        using Seg = Segment<HB>;
        const int32_t spr = (K + Seg::SEG - 1) / Seg::SEG;                  // segments per row
        const int32_t total_seg = T * spr;                                  // <= NX * WAVES
        uint4 raw[NX];
        bool in_range[NX];
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            int32_t sg = wave + i * WAVES;
            sg = sg < total_seg ? sg : total_seg - 1;
            const int32_t r = (sg >= spr ? 1 : 0) + (sg >= 2 * spr ? 1 : 0) + (sg >= 3 * spr ? 1 : 0);
            raw[i] = Seg::load_chunk(x + static_cast<int64_t>(r) * ldx, sg - r * spr, 0, K, lane, in_range[i]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) b[d] = load_w(j0 + d);
        ws_h = pr.w_scale[n_ch < N ? n_ch : N - 1];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int32_t sg = wave + i * WAVES;
            if (sg < total_seg) {                                           // wave-uniform
                const int32_t r = (sg >= spr ? 1 : 0) + (sg >= 2 * spr ? 1 : 0) + (sg >= 3 * spr ? 1 : 0);
                Seg s;
                s.set_chunk(0, raw[i], in_range[i]);
                s.rotate(lane);
                s.quant_store(r < ep.n_vis ? c_vis : c_txt, reinterpret_cast<int8_t *>(smem) + r * pitch,
                              sg - r * spr, lane);
            }
        }
    } else {
    // Loads return in the order they were issued, so the order of issue is the order of
    // arrival: first the T rows of xq (L2 hits; NX 16-byte pieces per thread, branch-free with
    // clamped addresses), then the first DEPTH weight loads (HBM).  The copy of xq into LDS
    // below then waits for the xq pieces only, while the weight loads stay in flight; issued
    // the other way round, every work-group would start with a full memory round trip in
    // which nothing else moves.
    const int32_t vec_per_row = K / 16;
    const int32_t xq_vecs = T * vec_per_row;                              // <= NX * WAVES * 64
    v4u xr[NX];
#pragma unroll
    for (int i = 0; i < NX; ++i) {
        int32_t v = static_cast<int32_t>(threadIdx.x) + i * (WAVES * 64);
        v = v < xq_vecs ? v : xq_vecs - 1;
        xr[i] = *reinterpret_cast<const v4u *>(xq + static_cast<int64_t>(v) * 16);
    }
    __builtin_amdgcn_sched_barrier(0);            // the scheduler must not move weight loads ahead of these
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) b[d] = load_w(j0 + d);
    ws_h = pr.w_scale[n_ch < N ? n_ch : N - 1];
    __builtin_amdgcn_sched_barrier(0);

    // Pieces past the end were clamped to the last one: they store the same bytes to the same
    // place again, which keeps this straight-line code.  Row of a piece without a division
    // (T <= 4).
#pragma unroll
    for (int i = 0; i < NX; ++i) {
        int32_t v = static_cast<int32_t>(threadIdx.x) + i * (WAVES * 64);
        v = v < xq_vecs ? v : xq_vecs - 1;
        const int32_t r = (v >= vec_per_row ? 1 : 0) + (v >= 2 * vec_per_row ? 1 : 0) +
                          (v >= 3 * vec_per_row ? 1 : 0);
        *reinterpret_cast<v4u *>(smem + (v + r) * 16) = xr[i];            // row pitch K + 16
    }
    }
    __syncthreads();

    // token operand of this lane: row (lane % rows of the instruction), clamped to a valid row
    const int m = F == 1 ? (lane & 31) : (lane & 15);
    const uint8_t *arow = smem + (m < T ? m : T - 1) * pitch + k_lane;

    typedef typename std::conditional<F == 1, v16i, v4i>::type acc_t;
    acc_t acc0, acc1;                                   // two chains: no dependent back-to-back pair
#pragma unroll
    for (int r = 0; r < (F == 1 ? 16 : 4); ++r) {
        acc0[r] = 0;
        acc1[r] = 0;
    }

    // Rolling pipeline: step d consumes register set d and at once issues the load that refills
    // it, so DEPTH - 1 or DEPTH loads are in flight at every moment.  The scheduling barrier at
    // the end of a step keeps the compiler from collecting the refills at the end of the
    // unrolled body (which would drain the memory pipe once per DEPTH steps); the token operand
    // of the next step is requested from LDS before the matrix instructions of this one.
    auto read_a = [&](int32_t j, uint4 &a0, uint4 &a1) {
        const int32_t jc = j < j1 ? j : j1 - 1;
        a0 = *reinterpret_cast<const uint4 *>(arow + jc * STEP);
        a1 = *reinterpret_cast<const uint4 *>(arow + jc * STEP + 16);
    };
    uint4 an0 = make_uint4(0, 0, 0, 0), an1 = an0;
    if (n_mine > 0) read_a(j0, an0, an1);
    for (int32_t i = 0; i < n_mine; i += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int32_t j = j0 + i + d;
            const uint4 a0 = an0, a1 = an1;
            read_a(j + 1, an0, an1);
            const uint32_t msk = j < j1 ? 0xFFFFFFFFu : 0u;          // wave-uniform
            uint4 bb = b[d];
            bb.x &= msk;
            bb.y &= msk;
            bb.z &= msk;
            bb.w &= msk;
            b[d] = load_w(j + DEPTH);                                 // refill this register set
            v4i b0, b1;
            unpack_w4x16(bb, b0, b1);
            if constexpr (F == 1) {
                acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(a0), b0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(a1), b1, acc1, 0, 0, 0);
            } else {
                acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_v4i(a0), b0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_v4i(a1), b1, acc1, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __syncthreads();                                   // every wave is done with the xq copy

    // Result rows of the valid tokens (T <= 4) sit in registers 0..3 of the lanes of k-group 0
    // (32x32x32: lanes 0..31; 16x16x64: lanes 0..15), one column per lane.
    int32_t (*red)[4][CH] = reinterpret_cast<int32_t (*)[4][CH]>(smem);      // [WAVES][4][CH]
    if (lane < CH) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][r][lane] = acc0[r] + acc1[r];
    }
    __syncthreads();
    const int t = threadIdx.x;
    // lane c of every wave holds the scale of the unit's channel c
    const float wsf = __shfl(__half2float(ws_h), t % CH, 64);
    if (t < 4 * CH) {
        const int32_t row = t / CH, c = t % CH;
        const int32_t n = nt * 32 + h * CH + c;
        if (row < T && n < N) {
            int32_t sum = 0;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) sum += red[w][row][c];
            store_out<EPI>(sum, row, n, ep, wsf, pr.y, pr.ldy, pr.acc_out, N);
        }
    }
}

// The same stream for up to 16 rows (and for few rows of a very long K): the T rows of xq no
// longer fit LDS as a whole, so they are streamed too.  With every weight load a wave requests
// the 64 F input channels of all rows that go with it (16 rows x 64 F bytes: one or two 16-byte
// loads per lane, 4 lanes per row, fully coalesced), and passes them through a wave-private LDS
// slot on their way into the matrix instruction's token operand (lane = token there).  Two
// slots alternate: the rows of step s + 1 are written while step s is computed.  No barrier is
// involved: a wave's LDS operations complete in order.
template <int F, int WAVES, int DEPTH, int EPI>
__global__ __launch_bounds__(WAVES * 64) void w4a8_gemv_stream_x_kernel(
    const int8_t *__restrict__ xq, int32_t T, int32_t K, GemvGroup grp, Epilogue ep)
{
    static_assert(F == 1 || F == 2, "channels per work-group: 32 or 16");
    constexpr int CH = 32 / F;
    constexpr int STEP = 64 * F;                  // input channels per wave-load
    constexpr int PITCH = STEP + 16;              // row pitch of a slot: conflict-free fragment reads
    constexpr int SLOT = 16 * PITCH;
    constexpr int kSlots = WAVES * 2 * SLOT, kRed = WAVES * 16 * CH * 4;
    __shared__ __attribute__((aligned(16))) uint8_t smem[kSlots > kRed ? kSlots : kRed];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

    int32_t pi = 0, unit = blockIdx.x;
    while (pi + 1 < grp.n && unit >= grp.p[pi].units) {
        unit -= grp.p[pi].units;
        ++pi;
    }
    const GemvProblem &pr = grp.p[pi];
    const int32_t N = pr.N;
    const int32_t k_tiles = K / kPackK;
    const int32_t loads = k_tiles / F;
    const int32_t per_wave = (loads + WAVES - 1) / WAVES;
    const int32_t j0 = wave * per_wave;
    int32_t j1 = j0 + per_wave;
    j1 = j1 < loads ? j1 : loads;
    const int32_t n_mine = j1 > j0 ? j1 - j0 : 0;

    const int32_t nt = unit / F, h = unit % F;
    int32_t lane_vec, k_lane;
    if constexpr (F == 1) {
        lane_vec = lane;
        k_lane = (lane >> 5) * 32;
    } else {
        const int q = lane >> 4, c = lane & 15;
        lane_vec = (q >> 1) * 64 + (q & 1) * 32 + h * 16 + c;
        k_lane = q * 32;
    }
    const uint4 *wsrc = pr.wp + static_cast<int64_t>(nt) * k_tiles * 64 + lane_vec;
    // past the wave's range both loads stay (branch-free pipeline) and read the start of xq
    auto load_w = [&](int32_t j) -> uint4 {
        const uint4 *src = j < j1 ? wsrc + static_cast<int64_t>(j) * (64 * F)
                                  : reinterpret_cast<const uint4 *>(xq);
        const v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src));
        return make_uint4(t[0], t[1], t[2], t[3]);
    };
    // x of a step: lane -> row lane / 4 (clamped to a valid row), piece lane % 4 of 16 F bytes
    const int xr = lane >> 2, xp = lane & 3;
    const int8_t *xsrc = xq + static_cast<int64_t>(xr < T ? xr : T - 1) * K + xp * (16 * F);
    auto load_x = [&](int32_t j, v4u (&dst)[F]) {
        const int8_t *src = j < j1 ? xsrc + static_cast<int64_t>(j) * STEP : xq;
#pragma unroll
        for (int v = 0; v < F; ++v) dst[v] = *reinterpret_cast<const v4u *>(src + v * 16);
    };

    v4u xa[DEPTH][F];
    uint4 b[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        load_x(j0 + d, xa[d]);
        b[d] = load_w(j0 + d);
    }
    const int32_t n_ch = nt * 32 + h * CH + (lane & (CH - 1));
    const __half ws_h = pr.w_scale[n_ch < N ? n_ch : N - 1];
    __builtin_amdgcn_sched_barrier(0);

    uint8_t *slots = smem + wave * (2 * SLOT);
    auto stage_x = [&](int slot, const v4u (&src)[F]) {
#pragma unroll
        for (int v = 0; v < F; ++v)
            *reinterpret_cast<v4u *>(slots + slot * SLOT + xr * PITCH + xp * (16 * F) + v * 16) = src[v];
    };
    const int m = F == 1 ? (lane & 31) : (lane & 15);           // token of this lane in the instruction
    const uint8_t *afrag = slots + (m & 15) * PITCH + k_lane;    // rows 16..31 of the 32-row form repeat
    auto read_a = [&](int slot, uint4 &a0, uint4 &a1) {
        a0 = *reinterpret_cast<const uint4 *>(afrag + slot * SLOT);
        a1 = *reinterpret_cast<const uint4 *>(afrag + slot * SLOT + 16);
    };

    typedef typename std::conditional<F == 1, v16i, v4i>::type acc_t;
    acc_t acc0, acc1;
#pragma unroll
    for (int r = 0; r < (F == 1 ? 16 : 4); ++r) {
        acc0[r] = 0;
        acc1[r] = 0;
    }

    stage_x(0, xa[0]);
    for (int32_t i = 0; i < n_mine; i += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int32_t j = j0 + i + d;
            // DEPTH is even, so the slot of a step is the parity of d
            stage_x((d + 1) & 1, xa[(d + 1) % DEPTH]);            // rows of the next step
            uint4 a0, a1;
            read_a(d & 1, a0, a1);
            const uint32_t msk = j < j1 ? 0xFFFFFFFFu : 0u;       // wave-uniform
            uint4 bb = b[d];
            bb.x &= msk;
            bb.y &= msk;
            bb.z &= msk;
            bb.w &= msk;
            // refill this step's register sets: x before w, the order in which they are needed
            load_x(j + DEPTH, xa[d]);
            b[d] = load_w(j + DEPTH);
            v4i b0, b1;
            unpack_w4x16(bb, b0, b1);
            if constexpr (F == 1) {
                acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(a0), b0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(a1), b1, acc1, 0, 0, 0);
            } else {
                acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_v4i(a0), b0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_v4i(a1), b1, acc1, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __syncthreads();                                   // the sums reuse the slots

    // rows 0..15 of the result: 32x32x32 keeps row (r / 4) * 8 + 4 g + r % 4 in register r < 8 of
    // k-group g; 16x16x64 keeps row 4 q + r in register r of lane group q
    int32_t (*red)[16][CH] = reinterpret_cast<int32_t (*)[16][CH]>(smem);      // [WAVES][16][CH]
    if constexpr (F == 1) {
        const int g = lane >> 5;
#pragma unroll
        for (int r = 0; r < 8; ++r) red[wave][acc_row(r, g)][lane & 31] = acc0[r] + acc1[r];
    } else {
        const int q = lane >> 4;
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][4 * q + r][lane & 15] = acc0[r] + acc1[r];
    }
    __syncthreads();
    const float wsf = __half2float(ws_h);              // this thread's channel below is lane % CH
    for (int32_t idx = threadIdx.x; idx < T * CH; idx += WAVES * 64) {
        const int32_t row = idx / CH, c = idx % CH;
        const int32_t n = nt * 32 + h * CH + c;
        if (n < N) {
            int32_t sum = 0;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) sum += red[w][row][c];
            store_out<EPI>(sum, row, n, ep, wsf, pr.y, pr.ldy, pr.acc_out, N);
        }
    }
}

template <int F, int WAVES, int DEPTH, int EPI>
int launch_stream_x(const int8_t *xq, int32_t T, int32_t K, const GemvGroup &grp, const Epilogue &ep,
                    int32_t total_units, hipStream_t stream)
{
    static_assert(DEPTH % 2 == 0, "slot parity");
    MQ_LAUNCH((w4a8_gemv_stream_x_kernel<F, WAVES, DEPTH, EPI>), dim3(static_cast<unsigned>(total_units)),
              dim3(WAVES * 64), 0, stream, xq, T, K, grp, ep);
    return launch_status();
}

// The T rows of xq pass through registers on their way to LDS: at most NX 16-byte pieces per
// thread, i.e. T * K <= kStreamMaxXq bytes whatever the work-group size.
constexpr int kStreamMaxXq = 80 * 1024;
constexpr int kStreamMaxLds = kStreamMaxXq + 16 * kGemvStreamMaxT;

template <int F, int WAVES, int DEPTH, int NX, int EPI, int HB = 0>
int launch_stream(const int8_t *xq, int32_t T, int32_t K, const GemvGroup &grp, const Epilogue &ep,
                  int32_t total_units, hipStream_t stream, const __half *x = nullptr, int64_t ldx = 0,
                  float c_vis = 0.0f, float c_txt = 0.0f)
{
    size_t lds = static_cast<size_t>(T) * (K + 16);
    const size_t red = static_cast<size_t>(WAVES) * 4 * (32 / F) * 4;
    lds = lds > red ? lds : red;
    auto kern = w4a8_gemv_stream_kernel<F, WAVES, DEPTH, NX, EPI, HB>;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kStreamMaxLds) != hipSuccess)
            return MQUANT_ERR_HIP;
        attr_set.store(true, std::memory_order_release);
    }
    MQ_LAUNCH(kern, dim3(static_cast<unsigned>(total_units)), dim3(WAVES * 64), lds, stream, xq, T, K, grp, ep,
              x, ldx, c_vis, c_txt);
    return launch_status();
}

// NX for the two sizes of xq a variant is compiled for: up to 16 KiB, up to kStreamMaxXq.
template <int F, int WAVES, int DEPTH, int EPI>
int launch_stream_nx(const int8_t *xq, int32_t T, int32_t K, const GemvGroup &grp, const Epilogue &ep,
                     int32_t units, hipStream_t stream)
{
    constexpr int kPer = WAVES * 64 * 16;                  // bytes one piece per thread covers
    constexpr int kSmall = 16 * 1024 / kPer, kLarge = kStreamMaxXq / kPer;
    if (static_cast<int64_t>(T) * K <= 16 * 1024)
        return launch_stream<F, WAVES, DEPTH, kSmall, EPI>(xq, T, K, grp, ep, units, stream);
    return launch_stream<F, WAVES, DEPTH, kLarge, EPI>(xq, T, K, grp, ep, units, stream);
}

}  // namespace

namespace mquant {

// Which shapes the two streaming kernels take (measured against the tile kernel they replace,
// 28 distinct 7B layers, one HIP graph per pass):
//   - up to 4 rows whose T * K bytes fit the LDS copy: every shape (T = 1: 3584 -> 18944 in 8.2 us
//     against 8.9, 18944 -> 3584 in 8.1 against 10.2, 3584 -> 3584 in 3.9 against 4.0);
//   - 5 to 16 rows: matrices with at most 128 output tiles, where 16-channel units double the
//     work-groups (T = 16: 18944 -> 3584 in 11.9 us against 15.5, 3584 -> 3584 in 4.4 against 5.1).
//     With many output tiles the tile kernel, which stages four k-tiles of activations per LDS
//     round trip, stays ahead (3584 -> 18944: 10.9 us against 12.1), and so it does for few rows
//     of a K too long for the LDS copy.
bool gemv_stream_takes(int32_t T, int32_t K, int64_t n_tiles)
{
    if (T < 1 || K % 128 != 0) return false;
    if (T <= kGemvStreamLdsMaxT) return static_cast<int64_t>(T) * K <= kStreamMaxXq;
    return T <= kGemvStreamMaxT && n_tiles <= kNumCU / 2;
}

// Shared by the single-linear entry points (a group of one) and the grouped entry.
template <int EPI>
int gemv_stream_dispatch(const int8_t *xq, int32_t T, int32_t K, GemvGroup grp, const Epilogue &ep,
                         hipStream_t stream)
{
    int64_t tiles = 0;
    for (int32_t i = 0; i < grp.n; ++i) tiles += ceil_div(grp.p[i].N, kPackN);
    // 16-channel units when whole tiles would leave compute units without work (or with a
    // ragged second round): measured on a pure read stream of the same pieces, 224 work-groups
    // of half tiles read the 18944 x 3584 matrix in 6.9 us, 112 of whole tiles in 8.5-9.0 us.
    const bool halves = tiles < 2 * kNumCU;
    const int f = halves ? 2 : 1;
    int64_t total = 0;
    for (int32_t i = 0; i < grp.n; ++i) {
        grp.p[i].units = static_cast<int32_t>(ceil_div(grp.p[i].N, kPackN) * f);
        total += grp.p[i].units;
    }
    if (total <= 0 || total > 0x7fffffff) return MQUANT_ERR_BAD_SHAPE;
    const int32_t units = static_cast<int32_t>(total);
    if (T > kGemvStreamLdsMaxT) {
        // more rows than the LDS copy of xq is compiled for: xq streamed next to the weights
        // (only few-tile matrices come here, see gemv_stream_takes)
        if (halves) return launch_stream_x<2, 8, 4, EPI>(xq, T, K, grp, ep, units, stream);
        return launch_stream_x<1, 4, 4, EPI>(xq, T, K, grp, ep, units, stream);
    }
    if constexpr (EPI == kEpiStatic) {
        // shapes of the work-group for tuning runs (mquant_tune_set); the default is variant 0
        const int32_t variant = tune_state().gemv_variant.load(std::memory_order_relaxed);
        if (variant == 1) {
            if (halves) return launch_stream_nx<2, 8, 4, EPI>(xq, T, K, grp, ep, units, stream);
            return launch_stream_nx<1, 8, 4, EPI>(xq, T, K, grp, ep, units, stream);
        }
        if (variant == 2) {
            if (halves) return launch_stream_nx<2, 8, 8, EPI>(xq, T, K, grp, ep, units, stream);
            return launch_stream_nx<1, 4, 8, EPI>(xq, T, K, grp, ep, units, stream);
        }
        if (variant == 3) {
            if (halves) return launch_stream_nx<2, 4, 16, EPI>(xq, T, K, grp, ep, units, stream);
            return launch_stream_nx<1, 8, 8, EPI>(xq, T, K, grp, ep, units, stream);
        }
    }
    if (halves) return launch_stream_nx<2, 4, 8, EPI>(xq, T, K, grp, ep, units, stream);
    return launch_stream_nx<1, 4, 4, EPI>(xq, T, K, grp, ep, units, stream);
}

// The one-launch decode linear on the streaming kernel (one linear, or several that share
// their input); ERR_UNSUPPORTED when the shape is outside its range (the caller then takes
// another path).
template <int HB>
static int stream_fused_hb(const __half *x, int64_t ldx, int32_t T, int32_t K, GemvGroup grp, const Epilogue &ep,
                           float c_vis, float c_txt, hipStream_t stream)
{
    constexpr int kSegSmall = 2, kSegLarge = 10;                 // segments per wave the kernel is compiled for
    int64_t tiles = 0;
    for (int32_t i = 0; i < grp.n; ++i) tiles += ceil_div(grp.p[i].N, kPackN);
    const bool halves = tiles < 2 * kNumCU;
    int64_t total = 0;
    for (int32_t i = 0; i < grp.n; ++i) {
        grp.p[i].units = static_cast<int32_t>(ceil_div(grp.p[i].N, kPackN) * (halves ? 2 : 1));
        total += grp.p[i].units;
    }
    if (total <= 0 || total > 0x7fffffff) return MQUANT_ERR_BAD_SHAPE;
    const int32_t units = static_cast<int32_t>(total);
    const int64_t segs = static_cast<int64_t>(T) * ceil_div(K, 512);
    if (segs > kSegLarge * 4) return MQUANT_ERR_UNSUPPORTED;
    const bool small = segs <= kSegSmall * 4;
    // Every work-group rotates all segments itself, about half a microsecond per segment and
    // wave, so the few-tile matrices (whose work-groups are alone on their compute unit) take
    // more waves than the plain stream does: measured at T = 1 on the 7B shapes, 3584 -> 3584
    // 3.87 -> 3.65 us with eight waves, 18944 -> 3584 11.1 -> 9.9 us with sixteen; with many
    // output tiles (3584 -> 37888) four waves stay ahead.
    if (halves) {
        if (small) return launch_stream<2, 8, 4, 1, kEpiStatic, HB>(nullptr, T, K, grp, ep, units, stream, x, ldx, c_vis, c_txt);
        return launch_stream<2, 16, 2, 3, kEpiStatic, HB>(nullptr, T, K, grp, ep, units, stream, x, ldx, c_vis, c_txt);
    }
    if (small) return launch_stream<1, 4, 4, kSegSmall, kEpiStatic, HB>(nullptr, T, K, grp, ep, units, stream, x, ldx, c_vis, c_txt);
    return launch_stream<1, 4, 4, kSegLarge, kEpiStatic, HB>(nullptr, T, K, grp, ep, units, stream, x, ldx, c_vis, c_txt);
}

bool gemv_stream_fused_takes(int32_t T, int32_t K, int32_t had_block)
{
    if (T < 1 || T > kGemvStreamLdsMaxT || K % 128 != 0 || static_cast<int64_t>(T) * K > kStreamMaxXq) return false;
    if (static_cast<int64_t>(T) * ceil_div(K, 512) > 40) return false;
    return had_block == 1 || had_block == 128 || had_block == 512;
}

int gemv_stream_fused(const __half *x, int64_t ldx, int32_t T, int32_t K, int32_t had_block, const GemvGroup &grp,
                      const Epilogue &ep, float c_vis, float c_txt, hipStream_t stream)
{
    if (!gemv_stream_fused_takes(T, K, had_block) || grp.n < 1) return MQUANT_ERR_UNSUPPORTED;
    switch (had_block) {
    case 1: return stream_fused_hb<1>(x, ldx, T, K, grp, ep, c_vis, c_txt, stream);
    case 128: return stream_fused_hb<128>(x, ldx, T, K, grp, ep, c_vis, c_txt, stream);
    default: return stream_fused_hb<512>(x, ldx, T, K, grp, ep, c_vis, c_txt, stream);
    }
}

template int gemv_stream_dispatch<kEpiStatic>(const int8_t *, int32_t, int32_t, GemvGroup, const Epilogue &, hipStream_t);
template int gemv_stream_dispatch<kEpiRowScale>(const int8_t *, int32_t, int32_t, GemvGroup, const Epilogue &, hipStream_t);
template int gemv_stream_dispatch<kEpiSplit>(const int8_t *, int32_t, int32_t, GemvGroup, const Epilogue &, hipStream_t);

}  // namespace mquant

extern "C" int mquant_w4a8_gemv_grouped(const int8_t *xq, int32_t T, int32_t K, int32_t n_vis, float s_vis,
                                        float s_txt, const mquant_linear_t *lin, int32_t n_linear,
                                        mquant_stream_t stream)
{
    if (T < 0 || K < 0 || n_linear < 0) return MQUANT_ERR_BAD_SHAPE;
    if (n_linear > kGemvMaxGroup || T > 32) return MQUANT_ERR_UNSUPPORTED;
    if (K % kPackK != 0 || K > kMaxK) return MQUANT_ERR_UNSUPPORTED;
    if (n_vis < 0 || n_vis > T) return MQUANT_ERR_BAD_SHAPE;
    if (!(s_vis > 0.0f) || !(s_txt > 0.0f) || !isfinite(s_vis) || !isfinite(s_txt)) return MQUANT_ERR_BAD_SHAPE;
    if (n_linear > 0 && !lin) return MQUANT_ERR_NULL;
    for (int32_t i = 0; i < n_linear; ++i) {
        if (lin[i].N < 0) return MQUANT_ERR_BAD_SHAPE;
        if (lin[i].N > 0 && T > 0 && lin[i].ldy < lin[i].N) return MQUANT_ERR_BAD_SHAPE;
    }
    if (T == 0 || n_linear == 0) return MQUANT_OK;
    if (K == 0) return MQUANT_ERR_UNSUPPORTED;
    if (!xq) return MQUANT_ERR_NULL;
    if (!aligned_to(xq, 16)) return MQUANT_ERR_ALIGNMENT;
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
    Epilogue ep = {};
    ep.n_vis = n_vis, ep.s_vis = s_vis, ep.s_txt = s_txt, ep.K = K, ep.xq = xq;
    int64_t group_tiles = 0;
    for (int32_t i = 0; i < grp.n; ++i) group_tiles += ceil_div(grp.p[i].N, kPackN);
    // outside the streaming kernels' range: the tile kernel, still one launch for the group
    if (!gemv_stream_takes(T, K, group_tiles))
        return gemv_tile_dispatch<kEpiStatic>(xq, T, K, grp, ep, static_cast<hipStream_t>(stream));
    return gemv_stream_dispatch<kEpiStatic>(xq, T, K, grp, ep, static_cast<hipStream_t>(stream));
}
