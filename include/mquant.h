/*
 * mquant.h -- C ABI of the MI355X (gfx950) W4A8 linear layer with
 * modality-specific static activation scales, the hot path of MQuant
 * (arXiv 2502.00425).
 *
 * The path, in the paper's terms:
 *   E (mixed visual/text tokens)  --AIFS reorder (Sec. 3.1)-->  E^u
 *   E^u --online block-Hadamard rotation (Sec. 3.2, appendix on the
 *         Walsh-Hadamard matrix)--> rotated activations
 *       --static per-tensor int8 quantization, scale s_v for visual rows and
 *         s_t for text rows (Eq. (2), Eq. (3))--> int8 codes
 *       --int4-weight x int8-activation GEMM, int32 accumulation (Sec. 4,
 *         "W4A8 GEMM" / "W4A8 GEMV")--> accumulators
 *       --dequantisation by s_row * s_w[n] (per-channel weight scale of
 *         Algorithm 1)--> fp16 output, rows in AIFS order.
 *
 * Conventions shared by every entry point
 *   - Plain C types only.  "dev" pointers are device (HBM) addresses valid on
 *     the current HIP device, "host" pointers are ordinary host memory.
 *   - The caller owns every buffer, including workspaces; no entry point
 *     allocates or frees device memory.
 *   - Device entry points are asynchronous on `stream` (a hipStream_t passed
 *     as void*; NULL = the default stream) and never synchronise.
 *   - Arguments are validated on the host before anything is launched; a
 *     failed validation launches nothing and returns a negative status.
 *   - Return value: MQUANT_OK (0) or a negative mquant_status_t.  Nothing
 *     throws or aborts across this boundary.
 *   - Zero-sized problems (T == 0, N == 0) are valid no-ops.
 *   - Matrices are row-major.  fp16 means IEEE binary16.  Leading dimensions
 *     are in elements.
 *   - Inputs must be finite; NaN/Inf behaviour is undefined.
 *   - Entry points may be called from several host threads and on several
 *     streams; calls that share an output buffer or a workspace must be
 *     ordered by the caller.
 *   - Environment: MQUANT_DEBUG=1 prints the HIP error text behind an ERR_HIP
 *     status.  Kernel choices (tile shapes, split-K) are made by the library's
 *     cost model; mquant_tune_set() overrides them for tests and tuning runs.
 */
#ifndef MQUANT_H
#define MQUANT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MQUANT_OK = 0,
    MQUANT_ERR_NULL = -1,        /* a required pointer is NULL */
    MQUANT_ERR_BAD_SHAPE = -2,   /* negative size, leading dimension too small, span outside [0,T), n_vis > T ... */
    MQUANT_ERR_UNSUPPORTED = -3, /* legal in the paper's terms but outside what these kernels handle */
    MQUANT_ERR_WORKSPACE = -4,   /* workspace missing or too small */
    MQUANT_ERR_HIP = -5,         /* a HIP runtime call failed (launch error) */
    MQUANT_ERR_ALIGNMENT = -6    /* a pointer or leading dimension is not 16-byte aligned */
} mquant_status_t;

/* One visual segment of the mixed sequence (Sec. 3.1: tokens e^v_m..e^v_n),
 * 0-based, half-open: rows [start, start+len). */
typedef struct {
    int32_t start;
    int32_t len;
} mquant_span_t;

typedef void *mquant_stream_t; /* hipStream_t */

/* Library version (major*10000 + minor*100 + patch). */
int mquant_version(void);

/* Static, NUL-terminated hash of the sources and flags this binary was built from
 * (what the build script computes; "unknown" for a build made without it). */
const char *mquant_build_id(void);

/* Static, NUL-terminated description of a status code. */
const char *mquant_status_string(int status);

/* -------------------------------------------------------------------------
 * AIFS (Attention-Invariant Flexible Switching), Sec. 3.1 and the appendix
 * on rotary position embedding: E^u = (all visual tokens, then all text
 * tokens), each modality in its original order.
 * ---------------------------------------------------------------------- */

/*
 * HOST, synchronous, O(T).  Builds the AIFS index vector.
 *   vis_host[n_spans] : visual segments, sorted by start, disjoint, inside [0,T)
 *   perm_host[T]      : out (may be NULL). Row i of E^u is row perm[i] of E;
 *                       also the position id of row i (the appendix's
 *                       (m..n, 1..m-1, n+1..L)).
 *   inv_perm_host[T]  : out (may be NULL). inv_perm[perm[i]] = i.
 *   n_vis_host        : out (required). Number of visual rows V.
 * Errors: NULL n_vis_host or (n_spans > 0 and NULL vis_host) -> ERR_NULL;
 *         T < 0, n_spans < 0, len < 0, unsorted/overlapping/out-of-range
 *         spans -> ERR_BAD_SHAPE.
 */
int mquant_aifs_build_perm(int32_t T, const mquant_span_t *vis_host, int32_t n_spans,
                           int32_t *perm_host, int32_t *inv_perm_host, int32_t *n_vis_host);

/*
 * DEVICE.  Row gather x_u[i, :] = x[perm[i], :] for fp16 matrices (Sec. 3.1,
 * the reorder that replaces slice/concat of interleaved tokens).
 *   x_dev   : fp16 [T, K], leading dimension ldx  (read)
 *   x_u_dev : fp16 [T, K], leading dimension ldxu (written); must not alias x
 *             (x_u_dev == x_dev is rejected with ERR_BAD_SHAPE; partial overlap is
 *             the caller's responsibility)
 *   perm_dev: int32 [T], every entry in [0, T) (not checked on the device
 *             beyond a clamp: an out-of-range entry reads row 0)
 * Requirements: K % 8 == 0, ldx % 8 == 0, ldxu % 8 == 0, 16-byte aligned
 * base pointers (ERR_ALIGNMENT / ERR_UNSUPPORTED otherwise).
 */
int mquant_aifs_permute(const void *x_dev, int64_t ldx, void *x_u_dev, int64_t ldxu,
                        const int32_t *perm_dev, int32_t T, int32_t K, mquant_stream_t stream);

/*
 * DEVICE.  Unified causal mask M^u[i, j] = M[perm[i], perm[j]] (Eq. (5) ->
 * Eq. (6)); masks are uint8 [T, T], contiguous, non-zero = may attend.
 * mask_u must not alias mask.
 */
int mquant_aifs_remap_mask(const uint8_t *mask_dev, uint8_t *mask_u_dev, const int32_t *perm_dev,
                           int32_t T, mquant_stream_t stream);

/* -------------------------------------------------------------------------
 * Online rotation + modality-specific static quantization (Sec. 3.2; Eq. (2)
 * with z = 0; Eq. (3)).
 * ---------------------------------------------------------------------- */

/*
 * DEVICE.  For every row i of the AIFS-ordered activations and every
 * contiguous block of had_block channels:
 *     u   = x_blk * H_B            (H_B the +-1 Walsh-Hadamard matrix of the
 *                                   Kronecker recursion; fp32 butterflies in
 *                                   stage order h = 1, 2, 4, ..., B/2)
 *     xq  = clamp(round_half_even(u * c_i), -128, 127),
 *     c_i = fp32(1 / (s_i * sqrt(B))),  s_i = s_vis if i < n_vis else s_txt.
 * The orthonormal 1/sqrt(B) of the rotation is folded into c_i.
 *   x_dev    : fp16 [*, K], leading dimension ldx.
 *   perm_dev : NULL -> row i of the output comes from row i of x (x already in
 *              AIFS order); non-NULL int32 [T] -> from row perm[i] (the gather
 *              of mquant_aifs_permute fused in).
 *   xq_dev   : int8 [T, K], contiguous (written).
 *   had_block: power of two in [1, 1024] dividing K; 1 = no rotation.
 *   s_vis, s_txt : finite, > 0.
 * Requirements: K % 8 == 0, ldx % 8 == 0, 16-byte aligned x, 8-byte aligned xq.
 * Errors: ERR_NULL, ERR_BAD_SHAPE (n_vis outside [0,T], ldx < K, scale <= 0),
 *         ERR_UNSUPPORTED (had_block not a supported power of two or not
 *         dividing K, K % 8 != 0), ERR_ALIGNMENT.
 */
int mquant_hadamard_quant_act(const void *x_dev, int64_t ldx, const int32_t *perm_dev,
                              int8_t *xq_dev, int32_t T, int32_t K, int32_t n_vis,
                              float s_vis, float s_txt, int32_t had_block,
                              mquant_stream_t stream);

/*
 * DEVICE.  mquant_hadamard_quant_act at activation bit-width act_bits in 2..8
 * (Eq. (2) with b = act_bits; the W4A4 setting of the accuracy tables is
 * act_bits = 4, codes in [-8, 7]).  The codes still take one int8 each, so the
 * GEMM / GEMV entry points consume them unchanged.  act_bits = 8 is
 * mquant_hadamard_quant_act.  ERR_UNSUPPORTED for act_bits outside 2..8.
 */
int mquant_hadamard_quant_act_bits(const void *x_dev, int64_t ldx, const int32_t *perm_dev,
                                   int8_t *xq_dev, int32_t T, int32_t K, int32_t n_vis,
                                   float s_vis, float s_txt, int32_t had_block, int32_t act_bits,
                                   mquant_stream_t stream);

/*
 * DEVICE.  Calibration statistic of Algorithm 1 (activation scale from
 * calibration samples; Eq. (2): s = max|x| / 127): the maximum |u| over the
 * unnormalised rotation of all T rows, combined into *absmax_dev with max().
 * The caller zeroes *absmax_dev (a float in device memory) beforehand and
 * turns the statistic into a scale with mquant_static_scale_from_absmax.  Same
 * requirements as mquant_hadamard_quant_act.
 */
int mquant_hadamard_absmax(const void *x_dev, int64_t ldx, int32_t T, int32_t K,
                           int32_t had_block, float *absmax_dev, mquant_stream_t stream);

/*
 * HOST, synchronous.  The static scale of Eq. (2), s = max|x_rot| / (2^(b-1) - 1),
 * from the statistic mquant_hadamard_absmax returns: x_rot = u / sqrt(had_block)
 * is the orthonormal rotation, so
 *     *scale_host = fp32( absmax_u / sqrt(had_block) / (2^(act_bits-1) - 1) ),
 * evaluated in double and rounded once.  act_bits = 8 for the W4A8 path.
 * Errors: ERR_NULL (scale_host), ERR_UNSUPPORTED (had_block not a power of two in
 * [1, 1024], act_bits outside 2..8), ERR_BAD_SHAPE (absmax_u negative or not finite).
 * absmax_u == 0 (an all-zero calibration set) yields scale 0, which the quantizer
 * entry points reject: the caller decides what an empty statistic means.
 */
int mquant_static_scale_from_absmax(float absmax_u, int32_t had_block, int32_t act_bits,
                                    float *scale_host);

/*
 * DEVICE.  Per-token dynamic activation quantization, the baseline the speed
 * tables of Sec. 4 compare MSQ against (Sec. 2.2: the scale of Eq. (2) from
 * runtime statistics; appendix on quantization granularity: one scale per
 * token).  Same rotation as mquant_hadamard_quant_act; for every row i
 *   s_i = fp32( max_k |x_rot[i,k]| / 127 ),  xq[i,:] = clamp(rne(x_rot[i,:] / s_i)),
 * an all-zero row gets s_i = 1.  Nothing of a row can be written before the
 * whole row has been read and reduced, which is the cost static scales avoid.
 *   row_scale_dev : fp32 [T] (written), 4-byte aligned
 *   other arguments as in mquant_hadamard_quant_act.
 * Errors: as mquant_hadamard_quant_act; ERR_UNSUPPORTED also when a row does
 *         not fit the registers of one work-group (K > 32768).
 */
int mquant_hadamard_dynquant_act(const void *x_dev, int64_t ldx, const int32_t *perm_dev,
                                 int8_t *xq_dev, float *row_scale_dev, int32_t T, int32_t K,
                                 int32_t had_block, mquant_stream_t stream);

/* -------------------------------------------------------------------------
 * W4A8 GEMM / GEMV (Sec. 4: "W4A8 GEMM", "custom W4A8 GEMV kernel") with the
 * fused dequantisation y = acc * s_row * s_w[n].
 * ---------------------------------------------------------------------- */

/*
 * Size in bytes of the kernel-private weight layout for an [N, K] int4
 * matrix (N padded to a multiple of 32).  Negative status on bad shape.
 */
int64_t mquant_w4_prepacked_bytes(int32_t N, int32_t K);

/*
 * DEVICE, one-off (weights are static).  Reorders the canonical int4 storage
 *   w_canonical_dev : uint8 [N, K/2]; byte n*K/2 + k/2 holds channel k of
 *                     output row n, even k in the low nibble, odd k in the
 *                     high nibble, 4-bit two's complement in [-8, 7]
 * into the tile order the GEMM/GEMV kernels stream
 * (mquant_w4_prepacked_bytes(N, K) bytes, 16-byte aligned).
 * Requirements: K % 64 == 0 (ERR_UNSUPPORTED otherwise), K <= 65536.
 */
int mquant_w4_prepack(const uint8_t *w_canonical_dev, uint8_t *w_prepacked_dev,
                      int32_t N, int32_t K, mquant_stream_t stream);

/* Workspace mquant_w4a8_gemm needs for this shape: 0 except for long-K shapes with few
 * output tiles, which are computed as split-K partial sums (splits * T * N * 4 bytes). */
int64_t mquant_w4a8_workspace_bytes(int32_t T, int32_t N, int32_t K);

/*
 * DEVICE.  acc[i, n] = sum_k xq[i, k] * wq[n, k] in int32 (exact), then
 * y[i, n] = fp16( (float(acc) * s_i) * float(w_scale[n]) ), s_i = s_vis for
 * rows i < n_vis and s_txt otherwise.  Small T (decode) is routed to a
 * weight-streaming GEMV kernel, large T (prefill) to the MFMA GEMM.
 *   xq_dev         : int8 [T, K] contiguous, 16-byte aligned
 *   w_prepacked_dev: output of mquant_w4_prepack for the same (N, K)
 *   w_scale_dev    : fp16 [N]
 *   y_dev          : fp16 [T, N], leading dimension ldy >= N (written)
 *   acc_out_dev    : NULL, or int32 [T, N] contiguous that receives the raw
 *                    accumulators (for verification; costs extra traffic)
 *   workspace_dev  : at least mquant_w4a8_workspace_bytes(T, N, K) bytes,
 *                    256-byte aligned; may be NULL when that size is 0.
 *                    Contents are scratch; concurrent calls must not share it.
 * Errors: ERR_NULL, ERR_BAD_SHAPE, ERR_UNSUPPORTED (K % 64 != 0,
 *         K > 65536), ERR_WORKSPACE, ERR_ALIGNMENT.
 */
int mquant_w4a8_gemm(const int8_t *xq_dev, const uint8_t *w_prepacked_dev,
                     const void *w_scale_dev, void *y_dev, int64_t ldy, int32_t *acc_out_dev,
                     int32_t T, int32_t N, int32_t K, int32_t n_vis, float s_vis, float s_txt,
                     void *workspace_dev, int64_t workspace_bytes, mquant_stream_t stream);

/*
 * DEVICE.  The same GEMM / GEMV with one activation scale per token
 * ("per token scale" of the scheme-comparison table in Sec. 4):
 * y[i, n] = fp16( (float(acc[i, n]) * row_scale[i]) * float(w_scale[n]) ).
 *   row_scale_dev : fp32 [T], e.g. from mquant_hadamard_dynquant_act
 * Other arguments, workspace (mquant_w4a8_workspace_bytes) and errors as in
 * mquant_w4a8_gemm.
 */
int mquant_w4a8_gemm_rowscale(const int8_t *xq_dev, const uint8_t *w_prepacked_dev,
                              const void *w_scale_dev, const float *row_scale_dev, void *y_dev,
                              int64_t ldy, int32_t *acc_out_dev, int32_t T, int32_t N, int32_t K,
                              void *workspace_dev, int64_t workspace_bytes,
                              mquant_stream_t stream);

/*
 * DEVICE.  The GEMM / GEMV for a linear marked by Rotation Magnitude
 * Suppression (Sec. 3.2: split the flagged channels into a separate GEMV, zero
 * their rows in the main weight, add the partial output back; the RMS
 * algorithm of the appendix marks the layers offline).  The main weight
 * w_prepacked_dev holds zeros in the n_split flagged input channels; every
 * flagged channel c_j comes with its own int4 row and scale:
 *   y[i, n] = fp16( (float(acc[i, n]) * s_i) * float(w_scale[n])
 *                   + sum_j (float(xq[i, c_j] * split_w[j, n]) * s_i) * split_scale[j] )
 * in fp32, terms added in the order j = 0, 1, ...
 *   split_idx_host   : HOST int32 [n_split], channel indices in [0, K) (per-layer
 *                      constants; they travel as kernel arguments)
 *   split_w_dev      : DEVICE int8 [n_split, N], int4 values in [-8, 7], one per byte
 *   split_scale_host : HOST fp32 [n_split], finite
 *   n_split          : 0 .. 64; 0 makes the call identical to mquant_w4a8_gemm.
 *                      The epilogue costs O(n_split) per output.
 *   acc_out_dev      : receives the main-path accumulators only
 * Other arguments, workspace and errors as in mquant_w4a8_gemm; ERR_BAD_SHAPE
 * for n_split or an index outside its range or a non-finite scale.
 */
int mquant_w4a8_gemm_rms(const int8_t *xq_dev, const uint8_t *w_prepacked_dev,
                         const void *w_scale_dev, void *y_dev, int64_t ldy, int32_t *acc_out_dev,
                         int32_t T, int32_t N, int32_t K, int32_t n_vis, float s_vis, float s_txt,
                         const int32_t *split_idx_host, const int8_t *split_w_dev,
                         const float *split_scale_host, int32_t n_split,
                         void *workspace_dev, int64_t workspace_bytes, mquant_stream_t stream);

/* One linear of a grouped decode launch: its prepacked weight (mquant_w4_prepack for
 * (N, K)), per-channel scales fp16 [N], and output fp16 [T, N] with leading dimension ldy. */
typedef struct {
    const uint8_t *w_prepacked_dev;
    const void *w_scale_dev;
    void *y_dev;
    int64_t ldy;
    int32_t N;
} mquant_linear_t;

/*
 * DEVICE.  The decode GEMV (Sec. 4, "custom W4A8 GEMV kernel"; the decode rows of the
 * speed tables) for several linears that share their input -- q/k/v, gate/up of a
 * decoder layer -- in ONE launch: for every linear l and row i < T
 *     y_l[i, n] = fp16( (float(sum_k xq[i, k] * wq_l[n, k]) * s_i) * float(w_scale_l[n]) ),
 * exactly what mquant_w4a8_gemm computes for each of them.  At decode a launch streams
 * for a few microseconds, so its fixed cost matters: one launch instead of two or three.
 *   xq_dev   : int8 [T, K] contiguous, 16-byte aligned; T <= 32 (ERR_UNSUPPORTED beyond)
 *   lin_host : HOST array of n_linear (<= 4, ERR_UNSUPPORTED beyond) descriptors; the
 *              outputs must not overlap
 * Errors: as mquant_w4a8_gemm.  T == 0 or n_linear == 0 is a no-op; a linear with
 * N == 0 is skipped.
 */
int mquant_w4a8_gemv_grouped(const int8_t *xq_dev, int32_t T, int32_t K, int32_t n_vis,
                             float s_vis, float s_txt, const mquant_linear_t *lin_host,
                             int32_t n_linear, mquant_stream_t stream);

/* Workspace of the fused prefill entry: the int8 activations plus whatever
 * mquant_w4a8_gemm needs. */
int64_t mquant_w4a8_linear_prefill_workspace_bytes(int32_t T, int32_t N, int32_t K);

/*
 * DEVICE.  The whole path for one linear layer at prefill: x in ORIGINAL
 * token order plus the AIFS index vector -> y in AIFS order.  Equivalent to
 * mquant_hadamard_quant_act(x, perm) into the workspace followed by
 * mquant_w4a8_gemm; the standalone row permute never touches memory.
 * perm_dev may be NULL when x is already in AIFS order.
 */
int mquant_w4a8_linear_prefill(const void *x_dev, int64_t ldx, const int32_t *perm_dev,
                               const uint8_t *w_prepacked_dev, const void *w_scale_dev,
                               void *y_dev, int64_t ldy,
                               int32_t T, int32_t N, int32_t K, int32_t n_vis,
                               float s_vis, float s_txt, int32_t had_block,
                               void *workspace_dev, int64_t workspace_bytes,
                               mquant_stream_t stream);

/*
 * DEVICE.  mquant_w4a8_linear_prefill for callers that cannot allocate device
 * memory or keep a workspace alive: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the
 * same results bit for bit, minus the workspace: the int8 activations and the
 * split-K partial sums go to a 128 MiB device array inside the library
 * (MQUANT_STATIC_SCRATCH_BYTES; one per GPU the library is used on, held until
 * the process ends).  The call allocates and frees nothing.
 * Errors: as mquant_w4a8_linear_prefill; ERR_WORKSPACE when
 * mquant_w4a8_linear_prefill_workspace_bytes(T, N, K) exceeds the array (nothing
 * is launched); ERR_HIP when the array's address cannot be obtained.
 * All calls on one GPU share the array: calls that may overlap on one GPU (two
 * streams, two host threads) race on it and must be ordered by the caller.  Its
 * contents after a call are unspecified.
 */
#define MQUANT_STATIC_SCRATCH_BYTES (128ll << 20)
int mquant_w4a8_linear_prefill_static(const void *x_dev, int64_t ldx, const int32_t *perm_dev,
                                      const uint8_t *w_prepacked_dev, const void *w_scale_dev,
                                      void *y_dev, int64_t ldy,
                                      int32_t T, int32_t N, int32_t K, int32_t n_vis,
                                      float s_vis, float s_txt, int32_t had_block,
                                      mquant_stream_t stream);

/*
 * DEVICE.  The whole path of one linear at decode (T <= 4 new rows) in ONE
 * launch: block-Hadamard rotation and static quantization of x (as
 * mquant_hadamard_quant_act, no gather) inside the weight-streaming GEMV, then
 * the fused dequantisation.  Equivalent to mquant_hadamard_quant_act followed by
 * mquant_w4a8_gemm, bit for bit; saves the separate front-end launch, which at
 * decode costs about as much as a small GEMV.  Every work-group rotates the T rows
 * itself, so the saving holds for T = 1 (7B shapes: 3.7 against 5.7 us for K = N = 3584,
 * even for K = 18944); from T = 2 on the two separate calls are the faster form.
 *   x_dev : fp16 [T, K], leading dimension ldx (multiple of 8), 16-byte aligned
 *   had_block : 1, 128 or 512 (ERR_UNSUPPORTED otherwise, also for T > 4 and for
 *               T * (K + 16) > 150 KiB, the LDS copy of the quantized rows)
 * Other arguments and errors as in mquant_w4a8_gemm; no workspace.
 */
int mquant_w4a8_linear_decode(const void *x_dev, int64_t ldx, const uint8_t *w_prepacked_dev,
                              const void *w_scale_dev, void *y_dev, int64_t ldy, int32_t T, int32_t N,
                              int32_t K, int32_t n_vis, float s_vis, float s_txt, int32_t had_block,
                              mquant_stream_t stream);

/*
 * DEVICE.  mquant_w4a8_linear_decode for several linears that share their input
 * (q/k/v, gate/up of a decoder layer) in ONE launch (Sec. 3.2 rotation, Eq. (2)-(3)
 * quantizer, Sec. 4 GEMV): the T rows of x are rotated and quantized once per
 * work-group, then every linear l gets
 *     y_l[i, n] = fp16( (float(sum_k xq[i, k] * wq_l[n, k]) * s_i) * float(w_scale_l[n]) ),
 * bit for bit what mquant_hadamard_quant_act followed by mquant_w4a8_gemm gives for
 * each of them.  A decoder layer then takes four launches (qkv, o, gate/up, down).
 *   x_dev    : fp16 [T, K], leading dimension ldx (multiple of 8), 16-byte aligned; T <= 4
 *   lin_host : HOST array of n_linear (<= 4, ERR_UNSUPPORTED beyond) descriptors; the
 *              outputs must not overlap
 * Errors: as mquant_w4a8_linear_decode.  T == 0 or n_linear == 0 is a no-op; a linear
 * with N == 0 is skipped.  Shapes beyond the one-launch kernel's range (T * K > 80 KiB)
 * run as one mquant_w4a8_linear_decode launch per linear.
 */
int mquant_w4a8_linear_decode_grouped(const void *x_dev, int64_t ldx, int32_t T, int32_t K,
                                      int32_t n_vis, float s_vis, float s_txt, int32_t had_block,
                                      const mquant_linear_t *lin_host, int32_t n_linear,
                                      mquant_stream_t stream);

/* -------------------------------------------------------------------------
 * Attention on AIFS-ordered tokens (Sec. 3.1, Eq. (5)-(6)) and rotary position
 * embedding with the reordered position ids (appendix "Rotary Position
 * Embedding for AIFS").  fp16 tensors, token-major, heads side by side:
 * q, o [T, n_q_heads * head_dim], k, v [T, n_kv_heads * head_dim]; query head h
 * uses key/value head h / (n_q_heads / n_kv_heads).  head_dim must be 128.
 * ---------------------------------------------------------------------- */

/*
 * DEVICE, in place.  Rotates every head's channel pairs (2j, 2j+1) of token i by
 * the angle pos[i] * base^(-2j/head_dim): the rotary embedding with the token's
 * ORIGINAL position as its id, so that reordered tokens keep their embedding.
 *   x_dev   : fp16 [T, ldx], the first n_heads * head_dim channels of a row are rotated
 *   pos_dev : int32 [T], original position of AIFS row i (the AIFS index vector)
 *   base    : > 1 (10000 in the paper)
 * Errors: ERR_NULL, ERR_BAD_SHAPE, ERR_UNSUPPORTED (head_dim != 128), ERR_ALIGNMENT
 *         (ldx odd, x not 4-byte aligned).
 */
int mquant_rope_apply(void *x_dev, int64_t ldx, const int32_t *pos_dev, int32_t T,
                      int32_t n_heads, int32_t head_dim, double base, mquant_stream_t stream);

/* Workspace of mquant_aifs_attention: the transposed values and two ints per key tile. */
int64_t mquant_aifs_attention_workspace_bytes(int32_t T, int32_t n_kv_heads, int32_t head_dim);

/*
 * DEVICE.  o = softmax(q k^T / sqrt(head_dim) + M^u) v per head, where token i
 * may attend token j exactly when pos[j] <= pos[i]: the unified causal mask
 * M^u[i,j] = M[pos[i], pos[j]] (Eq. (5) -> Eq. (6); for one visual segment the
 * three-region rule printed there), evaluated from the positions per tile; no
 * [T, T] mask is read or written.  fp32 softmax statistics, fp16 MFMA operands.
 *   q_dev, k_dev, v_dev, o_dev : as above, leading dimensions in elements
 *                                (ldq, ldk, ldv multiples of 8, ldo of 4; q, k, v
 *                                16-byte aligned, o 8-byte); o is written
 *   pos_dev       : int32 [T]; any values (ties attend each other)
 *   workspace_dev : mquant_aifs_attention_workspace_bytes(...) bytes, 256-byte
 *                   aligned; scratch, concurrent calls must not share it
 * Errors: ERR_NULL, ERR_BAD_SHAPE (n_q_heads not a multiple of n_kv_heads, a
 *         leading dimension too small), ERR_UNSUPPORTED (head_dim != 128),
 *         ERR_WORKSPACE, ERR_ALIGNMENT.
 */
int mquant_aifs_attention(const void *q_dev, int64_t ldq, const void *k_dev, int64_t ldk,
                          const void *v_dev, int64_t ldv, void *o_dev, int64_t ldo,
                          const int32_t *pos_dev, int32_t T, int32_t n_q_heads, int32_t n_kv_heads,
                          int32_t head_dim, void *workspace_dev, int64_t workspace_bytes,
                          mquant_stream_t stream);

/* -------------------------------------------------------------------------
 * Weight-only W4 linear with group-wise scales (the weight-only setting of
 * Table 13: int4 weight, group size 128, 16-bit activations; group-wise
 * granularity as in the appendix on quantization granularity).  The weight is
 * dequantised to fp16 on its way into the matrix core:
 *   W~[n, k] = fp16(wq[n, k] * s[n, k / 128])        one rounding
 *   y[i, n]  = fp16(sum_k x[i, k] * W~[n, k])        products exact, fp32 sums
 * ---------------------------------------------------------------------- */

/* Bytes of the kernel-private layout (weight tiles, then the scale table) for an
 * [N, K] matrix.  Negative status: ERR_BAD_SHAPE, ERR_UNSUPPORTED (K % 128 != 0). */
int64_t mquant_w4g128_prepacked_bytes(int32_t N, int32_t K);

/*
 * DEVICE, one-off.  Reorders
 *   w_canonical_dev : uint8 [N, K/2], nibble order as for mquant_w4_prepack, 4-byte aligned
 *   scales_dev      : fp16 [N, K/128], scale of output channel n and channel group k/128
 * into out_dev (mquant_w4g128_prepacked_bytes(N, K) bytes, 16-byte aligned).
 * The layout differs from mquant_w4_prepack's: the two are not interchangeable.
 */
int mquant_w4g128_prepack(const uint8_t *w_canonical_dev, const void *scales_dev, uint8_t *out_dev,
                          int32_t N, int32_t K, mquant_stream_t stream);

/*
 * DEVICE.  y = x W~^T as defined above.
 *   x_dev : fp16 [T, ldx], 16-byte aligned, ldx >= K and ldx % 8 == 0 (read only)
 *   w_prepacked_dev : output of mquant_w4g128_prepack for the same (N, K)
 *   y_dev : fp16 [T, ldy] (written: columns 0..N-1 of every row), ldy >= N; 16-byte
 *           stores are used when N % 8 == 0, ldy % 8 == 0 and y_dev is 16-byte aligned
 * Few tokens (decode) are routed to a weight-streaming GEMV kernel, many to the MFMA
 * GEMM.  The summation order is the matrix core's (and, in the GEMV, fixed across the
 * waves that split K) and is not specified; results agree with a double-precision sum
 * to within fp32 accumulation error plus the final fp16 rounding.
 * T == 0 or N == 0 is a no-op.  Errors: ERR_BAD_SHAPE, ERR_UNSUPPORTED (K % 128 != 0 or
 * K == 0), ERR_NULL, ERR_ALIGNMENT, ERR_HIP.
 */
int mquant_w4g128_gemm(const void *x_dev, int64_t ldx, const uint8_t *w_prepacked_dev, void *y_dev,
                       int64_t ldy, int32_t T, int32_t N, int32_t K, mquant_stream_t stream);

/* -------------------------------------------------------------------------
 * Tuning hook (tests and tuning runs; not needed for normal use).
 * ---------------------------------------------------------------------- */

typedef enum {
    MQUANT_TUNE_GEMM_TILE = 0,      /* -1 = cost model; 0 = 256x256, 1 = 128x256, 2 = 192x128,
                                       3 = 64x128, 4 = 64x256 (short prompts) */
    MQUANT_TUNE_GEMM_NOSPLIT = 1,   /* 0 = cost model; 1 = never split K */
    MQUANT_TUNE_G128_TILE = 2,      /* -1 = cost model; 0 = 128x256, 1 = 96x256 (weight-only GEMM) */
    MQUANT_TUNE_GEMV_VARIANT = 3    /* -1 = default; 0..3 = waves per work-group x loads in flight per
                                       wave of the decode GEMV: 4x8|4x4, 8x4|8x4, 8x8|4x8, 4x16|8x8
                                       (16-channel units | 32-channel units) */
} mquant_tune_key_t;

/*
 * HOST.  Overrides one kernel choice of the library for the whole process until
 * it is set back (value -1, or 0 for NOSPLIT).  Results never depend on these
 * choices, only speed; workspace sizes reported before a change may no longer
 * match (NOSPLIT needs none).  Out-of-range keys or values: ERR_BAD_SHAPE and
 * nothing changes.  Thread-safe; calls already running keep the value they read.
 */
int mquant_tune_set(int32_t key, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* MQUANT_H */
