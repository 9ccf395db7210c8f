/*
 * muxq.h -- C ABI of the MI355X (gfx950) MUXQ quantized linear layer.
 *
 * Computes Y = X.W the way the MUXQ paper defines it: abs-max symmetric INT8
 * quantisation (Sec. II-A, Eq. 1-3) applied after the outlier decomposition
 * of Sec. III-C (Eq. 4-7): channels of X holding an element of magnitude
 * above a threshold (6 in the paper) are shrunk by 2^-exp in the main matrix
 * "Body", a compact copy of those shrunk columns forms the small auxiliary
 * matrix "Aux", and Y = Body.W + (2^exp - 1) Aux.W is evaluated with INT8
 * codes and INT32 accumulators, then dequantised to fp16.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or synchronises; every call only enqueues kernels
 *     on `stream` (a hipStream_t passed as void*, NULL = default stream).
 *   - Return value: a muxq_status.  On any status other than MUXQ_OK nothing
 *     has been enqueued and no output has been touched, except MUXQ_ERR_HIP
 *     (a launch failed part-way; outputs are then undefined).
 *   - X is M x K fp16 row-major (K contiguous) with row stride ldx elements:
 *     M tokens by K input channels.  W is K x N fp16 row-major (N contiguous,
 *     the [in, out] orientation of the GPT-2 projection modules of Sec. IV-C).
 *   - Shape rules: M, K, N >= 1; K % 8 == 0; N % 8 == 0; ldx, ldw, ldy
 *     multiples of 8 and >= the row length; fp16 pointers 16-byte aligned;
 *     int8 pointers 16-byte aligned.  r_cap (capacity of the outlier list) is
 *     a multiple of 64 with 0 <= r_cap <= muxq_k_pad(K).  exp in [0, 7].
 *     The worst-case accumulator of Eq. 7, 127^2 (K + (2^exp - 1) r_cap), must fit INT32
 *     (MUXQ_ERR_PARAM otherwise: K up to about 133 thousand).
 *     Size limits (MUXQ_ERR_SHAPE beyond them): M <= 2^24, K <= 2^21,
 *     N <= 2^21, and each packed operand (M x k_pad, N x k_pad codes) below
 *     4 GiB, since the kernels address packed operands with 32-bit offsets.
 *   - INT8 operands of the GEMM (weight codes, Body codes, Aux codes, Aux
 *     weight rows) live in ONE packed layout, chosen so that a wave's
 *     direct-to-LDS load reads 1 KiB of contiguous memory: an R x C matrix of
 *     codes (C % 64 == 0) is cut into blocks of 16 rows x 64 codes; a block is
 *     1 KiB, row-major inside; blocks are ordered row-block-major.  Code
 *     (r, c) sits at byte muxq_packed_index(r, c, C) =
 *     ((r / 16) * (C / 64) + c / 64) * 1024 + (r % 16) * 64 + c % 64, and the
 *     buffer holds muxq_packed_bytes(R, C) = 16 * ceil(R / 16) * C bytes (rows
 *     past R are never written; the GEMM may read them, and what they hold
 *     reaches no output).
 *   - Where the signatures differ from the first plan of this boundary: the stage entry points
 *     muxq_detect_outliers and muxq_build_aux take a caller-provided `scratch` argument (the
 *     library allocates nothing, and the single-read abs-max pass needs room for its row-slab
 *     maxima; the quantiser for its per-channel multipliers), r_cap precedes the outputs so
 *     that inputs come first, and K, N must be multiples of 8 (one 16-byte load or store per
 *     lane), not of 16.
 *   - Non-finite inputs give unspecified codes (never a fault).
 *   - Rounding is round-half-to-even everywhere; codes are clamped to
 *     [-127, 127]; an all-zero quantisation unit gets scale 0 and codes 0.
 */
#ifndef MUXQ_H
#define MUXQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MUXQ_OK = 0,
    MUXQ_ERR_NULL = 1,      /* a required pointer is NULL */
    MUXQ_ERR_SHAPE = 2,     /* a dimension or leading dimension breaks the shape rules */
    MUXQ_ERR_ALIGN = 3,     /* a pointer is not 16-byte aligned */
    MUXQ_ERR_PARAM = 4,     /* exp, r_cap, granularity or threshold out of range */
    MUXQ_ERR_WORKSPACE = 5, /* workspace smaller than muxq_workspace_bytes() */
    MUXQ_ERR_HIP = 6        /* the HIP runtime refused a launch */
} muxq_status;

typedef enum { MUXQ_PER_TENSOR = 0, MUXQ_PER_CHANNEL = 1 } muxq_gran;

/* Activation-side options of muxq_linear_opts.
 * x_gran: MUXQ_X_PER_TENSOR, one scale for the whole Body (the per-tensor
 *     setting), or MUXQ_X_PER_TOKEN, one scale per row of Body (the per-vector
 *     setting of Sec. II-A / Fig. 2(a), the per-vector rows of Table 1):
 *     s_x[m] = max_k |Body[m][k]| / qmax.  Outlier channels are still detected
 *     per channel over all rows, and Aux shares the row's scale.  Needs
 *     r_cap <= 4096 and K <= 131072.
 * ia_bits: activation code width b in [2, 8] (the IA column of Table 1): codes in
 *     [-(2^(b-1) - 1), 2^(b-1) - 1], stored in int8.
 * absmax_ready: see muxq_gelu_absmax.
 * aux_own_scale: the other reading of Eq. 5 (the paper does not say on which scale Aux is
 *     quantised).  Zero, the default: Aux shares Body's scale, its codes are Body's outlier
 *     columns and Eq. 7 is summed on the integer accumulators.  Nonzero: Aux gets the abs-max
 *     scale of its own values, s_aux = max|Aux| / qmax (written to the workspace's x_scale[2],
 *     with qmax / max|Aux| in x_scale[3]; with per-token activations one per row,
 *     s_aux[m] = max_j |Aux[m][j]| / qmax, the fourth array of x_scale, and the factors rho[m]
 *     below the fifth), aux_q = clamp(rne(Aux * (qmax / max|Aux|))), and Eq. 7 becomes
 *       Y = (s_x s_w[n]) acc_body + (2^exp - 1) (s_aux s_w[n]) acc_aux.
 *     The GEMM keeps one set of INT32 accumulators: after the Aux steps it rescales them,
 *     acc <- rne(rho * acc_aux) with rho = (2^exp - 1) s_aux / s_x in binary32, and the Body
 *     steps accumulate on top, so Y = fp16((s_x s_w[n]) * float(acc_body + rne(rho acc_aux)) + b):
 *     within half a unit of s_x s_w[n] (plus binary32 rounding) of the sum above.  Both readings
 *     give the same codes, and the same Y up to that rounding, whenever max|Body| lies on an
 *     outlier channel (s_aux = s_x then). */
typedef enum { MUXQ_X_PER_TENSOR = 0, MUXQ_X_PER_TOKEN = 1 } muxq_x_gran;
typedef struct {
    int32_t x_gran;
    int32_t ia_bits;
    int32_t absmax_ready; /* nonzero: the slab maxima of X already sit in the workspace (written
                             by muxq_gelu_absmax into its absmax_partial region for the same M
                             and K); the pass over X that takes them is skipped.  Ignored where
                             no such pass exists (static list with per-token activations). */
    int32_t aux_own_scale; /* nonzero: Aux on the abs-max scale of its own values (see above) */
    int32_t absmax_slabs; /* with absmax_ready: how many row slabs the producer left (the value
                             muxq_linear_gelu_slabs returned for it); 0 = the count
                             muxq_gelu_absmax writes */
} muxq_act_opts;

/* Where muxq_linear keeps each intermediate inside the caller's workspace
 * (byte offsets from its start; every offset is a multiple of 256). */
typedef struct {
    size_t col_absmax;  /* float  [k_pad]      per-channel max |X|                     */
    size_t col_scale;   /* float  [k_pad]      per-channel quantisation multiplier     */
    size_t col_slot;    /* int32  [k_pad]      position in the outlier list, or -1     */
    size_t col_mask;    /* uint8  [k_pad / 8]  bit i of byte c: channel 8c+i is listed  */
    size_t outlier_idx; /* int32  [max(r_cap,1)] ascending outlier channels, -1 filled */
    size_t n_outliers;  /* int32  [3]          {kept, found, z}: z = zero point of body_q      */
    size_t x_scale;     /* float  [2] {s_x, qmax/amax} (+ {s_aux, qmax/max|Aux|} with aux_own_scale);
                           per token: s_x[M], qmax/amax[M], then int32 z[M], the rows' zero points,
                           then with aux_own_scale s_aux[M] and rho[M] = (2^exp - 1) s_aux[m] / s_x[m] */
    size_t absmax_partial; /* fp16 bits [64][k_pad] per-row-slab channel maxima (scratch)  */
    size_t body_q;      /* int8   packed M x k_pad: codes of Body, zero in the K padding; the
                           channels that are NOT listed hold code + z (z of the call, or of the row) */
    size_t aux_q;       /* int8   packed M x r_cap: codes of Aux, zero past the kept count  */
    size_t w_aux;       /* int8   packed N x r_cap: rows outlier_idx[] of the weight codes  */
    size_t cn;          /* int32  [N]: sum of channel n's weight codes over the unlisted input
                           channels (plus 2^14 when z is one per call: the accumulators then start at
                           z * 2^14); z * cn[n] is taken off the INT32 accumulators in the epilogue */
    size_t total;       /* bytes needed */
    int32_t k_pad;      /* 64 * ceil(K / 64) */
} muxq_ws_layout;

int muxq_version(void);
const char *muxq_status_string(int status);

/* Per-device set-up for the CURRENT HIP device: LDS attributes of the GEMM kernels, the CU
 * count their grids are sized by, the address of the library's static scratch array.
 * Thread-safe and idempotent; queries the device, so it must NOT be called while a stream is
 * being captured into a graph.  Optional otherwise: the first call of an entry point on a
 * device does the same work itself -- call muxq_init() once per device beforehand when that
 * first call would be made under capture.  Returns MUXQ_OK or MUXQ_ERR_HIP. */
int muxq_init(void);

/* K rounded up to the GEMM's K step (64). */
int muxq_k_pad(int K);
/* Size and addressing of the packed layout described above (cols % 64 == 0). */
size_t muxq_packed_bytes(int rows, int cols);
size_t muxq_packed_index(int row, int col, int cols);
/* Bytes of the quantised weight: packed N x muxq_k_pad(K) codes, row n holding
 * output channel n (the transpose of W), zero in the K padding
 * (muxq_packed_bytes(N, muxq_k_pad(K)) bytes), followed, 256-byte aligned, by int32[N]:
 * the sum of each output channel's codes (used by muxq_linear, see "zero point"). */
size_t muxq_wq_bytes(int K, int N);
/* Fills *out; returns MUXQ_OK or a shape/param error. */
int muxq_workspace_layout(int M, int K, int N, int r_cap, muxq_ws_layout *out);
/* = layout.total, or 0 on bad arguments. */
size_t muxq_workspace_bytes(int M, int K, int N, int r_cap);

/* Eq. 2 (offline, once per weight).  W: K x N fp16, row stride ldw.
 * gran = MUXQ_PER_TENSOR: one scale max|W|/127; MUXQ_PER_CHANNEL: one scale
 * per output channel n, max_k|W[k][n]|/127 (the per-vector setting of
 * Fig. 2(a) on the weight side).
 * Out: w_q, muxq_wq_bytes(K, N) bytes, packed N x muxq_k_pad(K);
 *      w_scale, float[1] (per-tensor) or float[N] (per-channel). */
int muxq_quantize_weight(const void *W_fp16, int K, int N, int ldw, int gran,
                         int8_t *w_q, float *w_scale, void *stream);
/* The same with a narrower code width (the W column of Table 2): w_bits in
 * [2, 8], codes in [-(2^(b-1) - 1), 2^(b-1) - 1] stored in int8, scales
 * max|W| / (2^(b-1) - 1).  muxq_quantize_weight is the w_bits = 8 case. */
int muxq_quantize_weight_bits(const void *W_fp16, int K, int N, int ldw, int gran,
                              int w_bits, int8_t *w_q, float *w_scale, void *stream);

/* Combination with per-channel difficulty migration between activations and weights (the
 * SmoothQuant-style scaling Sec. V says the method can be combined with): with positive factors
 * f[k] per input channel, X' = X diag(f)^-1 and W' = diag(f) W have the same product, and the
 * layer then runs on (X', W') like on any other operands -- what is left of a loud channel above
 * the threshold after the migration is still decomposed by Eq. 4-7.  How the factors are chosen
 * (e.g. max|X_k|^a / max|W_k|^(1-a) on calibration data) is the caller's business.
 * factors: DEVICE float[K], all > 0 (not checked; a factor that is zero, negative or not finite
 * gives unspecified codes in its channel).
 * Weight side, offline: muxq_quantize_weight_bits on W'[k][n] = fp16(W[k][n] * f[k]) without
 * materialising W' (factors NULL: plain muxq_quantize_weight_bits).
 * Activation side: X'[m][k] = fp16(X[m][k] / f[k]) (one correctly rounded binary32 division).  In a
 * model this step belongs in the producer of X (SmoothQuant folds it into the preceding
 * normalisation); as a kernel of its own it is an elementwise producer like muxq_gelu_absmax
 * and, like it, can leave the slab maxima of X' for the layer (slabs: see muxq_gelu_absmax; may be
 * NULL).  X_out may be X itself. */
int muxq_quantize_weight_smooth(const void *W_fp16, int K, int N, int ldw, int gran, int w_bits,
                                const float *factors, int8_t *w_q, float *w_scale, void *stream);
int muxq_smooth_absmax(const void *X_fp16, int M, int K, int ldx, const float *factors,
                       void *X_out_fp16, int ldo, void *slabs, void *stream);

/* Sec. III-C outlier criterion.  col_absmax[k] = max_m |X[m][k]| (float[K]);
 * a channel is an outlier channel when col_absmax[k] > threshold (strict).
 * outlier_idx (int32[max(r_cap,1)]) receives the outlier channels in ascending
 * order; if more than r_cap qualify, the r_cap lowest-indexed are kept and the
 * others are treated as normal channels (not an error); unused entries are -1.
 * n_outliers (int32[2]) = {kept, found}.
 * scratch: caller-provided device memory of muxq_detect_scratch_bytes(K)
 *      bytes, 16-byte aligned (row-slab maxima; X is read exactly once and no
 *      atomics or pre-zeroed buffers are involved). */
size_t muxq_detect_scratch_bytes(int K);
int muxq_detect_outliers(const void *X_fp16, int M, int K, int ldx,
                         float threshold, int r_cap, float *col_absmax,
                         int32_t *outlier_idx, int32_t *n_outliers,
                         void *scratch, void *stream);

/* Eq. 4-5 then Eq. 1 on Body.  Takes the outputs of muxq_detect_outliers
 * (the outlier list may also come from elsewhere, e.g. a calibrated static
 * list: ascending, in [0, K), first n_outliers[0] entries used).
 *   Body[m][k] = X[m][k] * 2^-exp on listed channels, X[m][k] elsewhere;
 *   s_x = max|Body| / 127 (derived from col_absmax, no second reduction);
 *   body_q = clamp(rne(Body * (127 / max|Body|)));  aux_q[m][j] = body_q[m][idx[j]]
 *   (Aux equals Body's outlier columns, Eq. 5, and shares Body's scale so
 *   that Eq. 7 can be summed on integers).
 * Out: body_q, packed M x muxq_k_pad(K), columns K..muxq_k_pad(K) zeroed;
 *      aux_q, packed M x r_cap (not touched when r_cap == 0, may then be
 *      NULL), columns past the kept count zeroed;
 *      x_scale float[2] = {s_x, 127/max|Body|}.
 * scratch: caller-provided device memory of 2 * muxq_k_pad(K) * 4 bytes
 *      (per-channel multiplier and list position), 16-byte aligned. */
int muxq_build_aux(const void *X_fp16, int M, int K, int ldx,
                   const float *col_absmax, const int32_t *outlier_idx,
                   const int32_t *n_outliers, int r_cap, int exp,
                   int8_t *body_q, int8_t *aux_q, float *x_scale,
                   void *scratch, void *stream);

/* Zero point.  The matrix pipes draw markedly less power when their operands do not
 * keep changing sign, and on this chip power is what limits the GEMM.  muxq_linear
 * therefore stores the codes of the channels that are not listed as code + z,
 * z = min(c, 127 - c) made even, with c the largest such code of the call (per-tensor
 * activations) or of the row (per-token activations) -- non-negative throughout when c <= 63, the
 * usual case once the outlier channels set the scale -- and its GEMM takes
 * z * (sum of the weight codes those channels meet) off each INT32 accumulator before
 * the dequantisation.  Results are those of Eq. 7, bit for bit; what a reader of the
 * workspace sees differs: body_q holds code + z on the unlisted channels, n_outliers[2]
 * (or the third array of x_scale) holds z, and dbg_acc receives the corrected
 * accumulators.  z = 0 when K > 65536, and in the stage entry points.
 * For the same reason the INT32 accumulators of every GEMM here start at a positive offset
 * (2^18, or z * 2^14 folded into the zero-point term) that the epilogue removes again, in
 * integers: accumulators that hover around zero keep flipping their high bits.  The running
 * sums may pass through the INT32 wrap-around because of it; arithmetic modulo 2^32 keeps the
 * result exact.
 *
 * The whole layer, Eq. 1-7: detect -> Body/Aux -> quantise -> INT8 MFMA GEMM
 * with the Aux product, the (2^exp - 1) recombination and the Eq. 3
 * dequantisation fused into it:
 *   acc[m][n] = sum_k body_q[m][k] w_q[k][n] + (2^exp-1) sum_j aux_q[m][j] w_q[idx[j]][n]
 *   Y[m][n]   = fp16( (s_x * s_w[n]) * float(acc[m][n]) + bias[n] )
 * w_q, w_scale: outputs of muxq_quantize_weight with granularity w_gran.
 * bias_fp16: fp16[N] or NULL.  Y: M x N fp16, row stride ldy.
 * workspace: >= muxq_workspace_bytes(M, K, N, r_cap) bytes, 256-byte aligned
 *      (no defined content needed on entry);
 *      afterwards it holds every intermediate at the muxq_workspace_layout
 *      offsets.  Calls that share a workspace must not overlap in time.  dbg_acc_i32: NULL, or int32 [M][N] that receives acc. */
int muxq_linear(const void *X_fp16, int M, int K, int ldx, const int8_t *w_q,
                const float *w_scale, int w_gran, int N, const void *bias_fp16,
                float threshold, int exp, int r_cap, void *Y_fp16, int ldy,
                void *workspace, size_t workspace_bytes, int32_t *dbg_acc_i32,
                void *stream);

/* muxq_linear with the activation-side options above (opts: HOST pointer, NULL =
 * per-tensor, 8 bits = muxq_linear).  With MUXQ_X_PER_TOKEN the workspace's
 * x_scale holds s_x[M] followed by (2^(b-1) - 1) / max|Body[m]| [M], and
 *   Y[m][n] = fp16( (s_x[m] * s_w[n]) * float(acc[m][n]) + bias[n] ). */
int muxq_linear_opts(const void *X_fp16, int M, int K, int ldx, const int8_t *w_q,
                     const float *w_scale, int w_gran, int N, const void *bias_fp16,
                     float threshold, int exp, int r_cap, void *Y_fp16, int ldy,
                     void *workspace, size_t workspace_bytes, int32_t *dbg_acc_i32,
                     const muxq_act_opts *opts, void *stream);

/* Static (calibrated) outlier channels.  Sec. III-C finds the outlier channels by their
 * magnitude; applied offline to calibration data the same criterion gives a fixed
 * list, and the run-time detection can be dropped: the listed channels are then
 * decomposed (Eq. 4-7) whatever their magnitude in the current X, and no other.
 *
 * muxq_prepare_static (offline, once per weight and list) turns a list into the block the
 * run-time call consumes.  list: DEVICE int32[n_list] (NULL allowed when n_list == 0),
 * strictly ascending channel indices in [0, K); an entry outside that range or not above
 * the previous accepted entry is skipped.  The r_cap lowest accepted entries are listed.
 * static_block: device memory, >= muxq_static_bytes(K, N, r_cap) bytes, 256-byte aligned;
 * it receives, at the muxq_static_layout_of offsets: col_mask (one bit per channel),
 * outlier_idx int32[max(r_cap,1)] (-1 padded), n_outliers int32[2] = {listed, accepted},
 * w_aux = packed N x r_cap rows outlier_idx[] of w_q (the weights of the Aux product). */
typedef struct muxq_static_layout {
    size_t col_mask, outlier_idx, n_outliers, w_aux, total;
    int32_t k_pad;
} muxq_static_layout;
size_t muxq_static_bytes(int K, int N, int r_cap);   /* 0 on bad shapes */
int muxq_static_layout_of(int K, int N, int r_cap, muxq_static_layout *out);
int muxq_prepare_static(const int32_t *list, int n_list, int K, const int8_t *w_q, int N,
                        int r_cap, void *static_block, size_t static_bytes, void *stream);

/* muxq_linear_opts with the channel list of a prepared static block in place of the
 * threshold test (static_block: as written by muxq_prepare_static for the same K, N,
 * r_cap and w_q; read only, may be shared by concurrent calls).  Per-tensor activations:
 * abs-max of X -> scale of Body -> quantise -> GEMM, as muxq_linear without the selection
 * and without the Aux weight gather (the workspace's n_outliers then reads {listed,
 * listed}; the number of accepted entries is in the block).  Per-token activations: ONE pass over X (a row's
 * scale needs only that row once the channels are known) and the GEMM; the workspace's
 * col_absmax, col_scale, col_slot and outlier_idx are then not written. */
int muxq_linear_static(const void *X_fp16, int M, int K, int ldx, const int8_t *w_q,
                       const float *w_scale, int w_gran, int N, const void *bias_fp16,
                       int exp, int r_cap, const void *static_block, void *Y_fp16, int ldy,
                       void *workspace, size_t workspace_bytes, int32_t *dbg_acc_i32,
                       const muxq_act_opts *opts, void *stream);

/* Producer fusion.  Between the two MLP projections of the GPT-2 blocks the method is
 * applied to (Sec. IV-C) sits a GELU; the kernel that applies it can take the per-channel
 * maxima the outlier criterion of Sec. III-C needs while it writes X, and the next
 * muxq_linear then starts at the selection step (one pass over X less).
 *   X[m][k] = fp16( gelu(Y[m][k]) ),  gelu(y) = 0.5 y (1 + tanh(sqrt(2/pi) (y + 0.044715 y^3))),
 * evaluated in binary32 (within one fp16 unit in the last place of the exact value).
 * Y_fp16: M x K, row stride ldy; X_fp16: M x K, row stride ldx, may be Y_fp16 itself (in place,
 * ldx == ldy then).  slabs: the absmax_partial region of the workspace the following
 * muxq_linear_opts / muxq_linear_static call (same M, K; absmax_ready = 1) will be given, i.e.
 * workspace + muxq_workspace_layout(...).absmax_partial; muxq_detect_scratch_bytes(K) bytes,
 * 16-byte aligned.  The maxima are those of the rounded fp16 values written to X. */
int muxq_gelu_absmax(const void *Y_fp16, int M, int K, int ldy, void *X_fp16, int ldx,
                     void *slabs, void *stream);

/* The first projection of the GPT-2 MLP with its activation fused in (Sec. IV-C: c_fc, GELU,
 * c_proj are consecutive, and the method wraps both projections):
 *   H[m][n] = fp16( gelu( fp16( (s_x s_w[n]) acc[m][n] + bias[n] ) ) ),
 * i.e. exactly what muxq_linear_opts followed by muxq_gelu_absmax gives, bit for bit, without the
 * round trip of the 2 M N bytes of Y through memory and without a GELU kernel: the GELU runs in
 * the GEMM's epilogue.  next_slabs (may be NULL): the absmax_partial region of the workspace of
 * the NEXT layer (the one whose input is H: same M, its K = this N), i.e. its workspace +
 * muxq_workspace_layout(M, N, N_next, r_cap_next).absmax_partial; it receives the per-slab column
 * maxima of H, so that the next muxq_linear_opts / muxq_linear_static starts at its selection
 * step with opts.absmax_ready = 1 and opts.absmax_slabs = muxq_linear_gelu_slabs(M, K, N).
 * The GEMM's workgroups take those maxima from the tiles they store (one slab per row of
 * tiles); where the problem is too small for that form of the GEMM, or has more than 64 rows of
 * tiles, one plain pass over H takes them instead (same result, same interface).
 * opts: as muxq_linear_opts (aux_own_scale is not combined with the fused GELU: MUXQ_ERR_PARAM). */
int muxq_linear_gelu_slabs(int M, int K, int N);   /* 0 on bad shapes */
int muxq_linear_gelu(const void *X_fp16, int M, int K, int ldx, const int8_t *w_q,
                     const float *w_scale, int w_gran, int N, const void *bias_fp16,
                     float threshold, int exp, int r_cap, void *H_fp16, int ldh,
                     void *workspace, size_t workspace_bytes, void *next_slabs,
                     const muxq_act_opts *opts, void *stream);

/* The MLP of a GPT-2 block as one call (Sec. IV-C: the method wraps c_fc and c_proj, with the
 * GELU between them):
 *   H = fp16(gelu(muxq_linear(X,  W1) + b1))   M x N1   (muxq_linear_gelu)
 *   Y = muxq_linear(H, W2) + b2                M x N2   (muxq_linear_opts on H, starting at its
 *                                                        selection step: the first layer's GEMM
 *                                                        hands H's channel maxima over)
 * Both layers detect their outlier channels at run time with the same threshold, exp and r_cap
 * and the same opts (x_gran, ia_bits; absmax_ready / absmax_slabs refer to X and the first layer;
 * aux_own_scale must be 0).  Results are bit for bit those of the two calls made one after the
 * other.  H_fp16 (M x N1, row stride ldh) is an output as well as the second layer's input.
 * workspace: muxq_mlp_workspace_bytes(M, K, N1, N2, r_cap) bytes, 256-byte aligned, content
 * undefined on entry; it holds the first layer's workspace (muxq_workspace_layout(M, K, N1, r_cap))
 * at offset 0 and the second layer's (muxq_workspace_layout(M, N1, N2, r_cap)) right behind it, at
 * the first layer's `total` rounded up to 256.  w1_q / w2_q: muxq_quantize_weight of the K x N1 and
 * N1 x N2 weights; bias1 / bias2 may be NULL.  Errors as muxq_linear_opts; nothing is launched when
 * an argument of either layer is refused. */
size_t muxq_mlp_workspace_bytes(int M, int K, int N1, int N2, int r_cap);   /* 0 on bad shapes */
int muxq_mlp(const void *X_fp16, int M, int K, int ldx,
             const int8_t *w1_q, const float *w1_scale, int w1_gran, int N1, const void *bias1_fp16,
             const int8_t *w2_q, const float *w2_scale, int w2_gran, int N2, const void *bias2_fp16,
             float threshold, int exp, int r_cap, void *H_fp16, int ldh, void *Y_fp16, int ldy,
             void *workspace, size_t workspace_bytes, const muxq_act_opts *opts, void *stream);

/* muxq_linear for callers that cannot allocate or be handed a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The intermediates live in a
 * static device array inside the library instead of a caller's workspace: at most
 * muxq_noalloc_max_bytes() (16 MiB) per GPU, held from library load until the process ends.
 * Same arguments and results as muxq_linear minus the workspace and the accumulator export;
 * shapes whose muxq_workspace_bytes(M, K, N, r_cap) exceeds the array are rejected with
 * MUXQ_ERR_WORKSPACE.  Calls no allocating routine.  Every call on a GPU shares that GPU's one
 * array: calls that overlap in time on one GPU (different streams or threads) race.  The first
 * call on a device looks the array's address up (see muxq_init). */
size_t muxq_noalloc_max_bytes(void);
int muxq_linear_noalloc(const void *X_fp16, int M, int K, int ldx, const int8_t *w_q,
                        const float *w_scale, int w_gran, int N, const void *bias_fp16,
                        float threshold, int exp, int r_cap, void *Y_fp16, int ldy, void *stream);

/* The same pipeline with outlier handling switched off (plain Eq. 1-3 with a
 * dynamic per-tensor activation scale): the reference point for MUXQ's
 * overhead.  Workspace as for muxq_linear with r_cap = 0. */
int muxq_linear_naive_int8(const void *X_fp16, int M, int K, int ldx,
                           const int8_t *w_q, const float *w_scale, int w_gran,
                           int N, const void *bias_fp16, void *Y_fp16, int ldy,
                           void *workspace, size_t workspace_bytes,
                           int32_t *dbg_acc_i32, void *stream);

/* The bare GEMM + epilogue of muxq_linear on operands quantised earlier
 * (Eq. 3 / Eq. 7 only).  a_q: packed M x muxq_k_pad(K) codes (K padding zero);
 * w_q: packed weight; aux_q / w_aux / n_outliers may all be NULL (then no Aux
 * product), else aux_q is packed M x r_cap, w_aux packed N x r_cap, both zero
 * past column n_outliers[0], of which ceil(n_outliers[0] / 64) * 64 are used.
 * x_scale: float[>=1], x_scale[0] = s_x. */
int muxq_gemm_i8(const int8_t *a_q, int M, int K, const int8_t *w_q,
                 int N, const int8_t *aux_q, const int8_t *w_aux,
                 const int32_t *n_outliers, int r_cap, int exp,
                 const float *x_scale, const float *w_scale, int w_gran,
                 const void *bias_fp16, void *Y_fp16, int ldy,
                 int32_t *dbg_acc_i32, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MUXQ_H */
