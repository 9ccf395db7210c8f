// Internal launch interface between the C-ABI layer and the gfx950 kernels.
// Every function enqueues on `stream` and returns the hipError_t of the
// launch.  Shapes are validated by the caller (muxq_api.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

namespace muxq {

// Enqueue `kernel` and return the status of THIS launch.  (hipGetLastError() after a
// triple-chevron launch reports the runtime's sticky error word: a failure some earlier,
// unrelated call of the process left there would be taken for a failed launch here.)
// The arguments are converted to the kernel's exact parameter types first.
template <typename... P, size_t... I>
inline hipError_t launch_kernel_impl(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes,
                                     hipStream_t s, std::tuple<P...> &params, std::index_sequence<I...>)
{
    void *ptrs[] = {(void *)&std::get<I>(params)..., nullptr};
    return hipLaunchKernel((const void *)kernel, grid, block, ptrs, lds_bytes, s);
}
template <typename... P, typename... A>
inline hipError_t launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t s,
                                A &&...args)
{
    static_assert(sizeof...(P) == sizeof...(A), "argument count differs from the kernel's parameter list");
    std::tuple<P...> params{static_cast<P>(std::forward<A>(args))...};
    return launch_kernel_impl(kernel, grid, block, lds_bytes, s, params, std::index_sequence_for<P...>{});
}

constexpr int kKStep = 64;  // GEMM K step in bytes/codes; K is padded to it

// Packed layout of every INT8 operand of the GEMM (activation codes, weight
// codes, Aux codes, Aux weight rows): a matrix of R rows x C codes (C % 64 == 0)
// is cut into blocks of 16 rows x 64 codes, each block 1 KiB contiguous
// (row-major inside), blocks ordered row-block-major.  One direct-to-LDS load
// of a wave (64 lanes x 16 B) then reads exactly one contiguous block.
__host__ __device__ inline size_t packed_index(int r, int c, int C)
{
    return ((size_t)(r >> 4) * (size_t)(C >> 6) + (size_t)(c >> 6)) * 1024 + (size_t)((r & 15) * 64 + (c & 63));
}
inline size_t packed_bytes(int R, int C) { return (size_t)((R + 15) / 16 * 16) * (size_t)C; }
// A quantised weight is its packed N x k_pad codes followed (256-byte aligned) by the
// int32 sum of each output channel's codes, which the GEMM epilogue needs to undo the
// zero point that the activation codes of the unlisted channels carry.
inline size_t wq_rowsum_offset(int N, int k_pad) { return (packed_bytes(N, k_pad) + 255) & ~(size_t)255; }
inline size_t wq_total_bytes(int N, int k_pad) { return wq_rowsum_offset(N, k_pad) + (((size_t)N * 4 + 255) & ~(size_t)255); }

// Accumulator offset.  INT32 accumulators that hover around zero change sign all the time,
// and a sign change flips every high bit of a two's-complement word: the matrix pipes draw
// measurably less power (the GEMM is ~2-4 % shorter) when the accumulators stay on one side
// of zero.  With a per-call zero point z the offset is free: the quantiser writes
// cn[n] + kCnBias, the GEMM starts every accumulator at z * kCnBias, and the epilogue's
// acc - z * cn[n] removes exactly that.  2^14 keeps |cn + kCnBias| inside the 24-bit
// multiplier for every K the zero point is used with (K <= 65536: 65536 * 127 + 2^14 < 2^23)
// and is several times the spread of cn (~ 25 sqrt(K) for weight codes of spread 25).
constexpr int32_t kCnBias = 1 << 14;
// Without that route (no zero point: z = 0, no cn, or one z per token) the accumulators start
// at kAccBias and the epilogue subtracts it again: one integer add per output, or none where
// it folds into the correction constant of the channel.
constexpr int32_t kAccBias = 1 << 18;

// ---- device helpers shared by the streaming kernels and the GEMM epilogue -------------------
typedef unsigned short muxq_u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    muxq_u16x2 va = __builtin_bit_cast(muxq_u16x2, a), vb = __builtin_bit_cast(muxq_u16x2, b);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(va, vb));
}

// Running maximum of eight fp16 magnitudes: |fp16| as a 15-bit unsigned integer orders exactly
// like the magnitude.
__device__ __forceinline__ uint4 absmax_step(uint4 mx, uint4 v)
{
    mx.x = pk_max_u16(mx.x, v.x & 0x7fff7fffu);
    mx.y = pk_max_u16(mx.y, v.y & 0x7fff7fffu);
    mx.z = pk_max_u16(mx.z, v.z & 0x7fff7fffu);
    mx.w = pk_max_u16(mx.w, v.w & 0x7fff7fffu);
    return mx;
}

// The activation between the two projections of the GPT-2 MLP (the modules of Sec. IV-C), tanh
// form: gelu(y) = 0.5 y (1 + tanh(sqrt(2/pi) (y + 0.044715 y^3))) = y / (1 + exp(-2 u)),
// evaluated in binary32.  One definition for the stand-alone producer kernel and the GEMM's
// fused epilogue, so that the two give the same fp16 values.
__device__ __forceinline__ float gelu_tanh_f32(float y)
{
    const float u = 0.7978845608028654f * (y + 0.044715f * y * y * y);
    float r = y * __builtin_amdgcn_rcpf(1.0f + __expf(-2.0f * u));
    // The product is a binary32 value in every caller: without this the compiler may fold the
    // multiply and a following conversion to fp16 into one mixed-precision instruction with a
    // single rounding, and the same input would then give different fp16 results in different
    // kernels (seen at near-ties).
    asm("" : "+v"(r));
    return r;
}

struct GemmArgs {
    const int8_t *a_q;      // packed M x k_pad activation codes (Body)
    const int8_t *w_q;      // packed N x k_pad weight codes (row n = output channel n)
    const int8_t *aux_q;    // packed M x r_cap, or nullptr
    const int8_t *w_aux;    // packed N x r_cap, or nullptr
    const int32_t *n_outliers;  // device: [0] = columns of aux_q / w_aux in use, or nullptr
    const float *x_scale;   // device: [0] = s_x, or s_x[M] with x_per_token
    const float *w_scale;   // device: [1] or [N]
    const _Float16 *bias;   // [N] or nullptr
    _Float16 *y;            // [M][ldy]
    int32_t *dbg_acc;       // [M][N] or nullptr
    const int32_t *cn;      // [N] or nullptr: sum of channel n's weight codes over the unlisted
                            // input channels; z * cn[n] is taken off the accumulators
    const int32_t *zero_point;  // device: z, [1], or z[M] with x_per_token (used with cn)
    int32_t cn_bias;        // what the producer of cn added to every entry (0 or kCnBias); the
                            // accumulators then start at z * cn_bias instead of 0 (see kCnBias)
    int M, N, k_pad, r_cap, ldy;
    int exp_shift;          // exp of Eq. 4; the Aux product is weighted by 2^exp - 1
    int w_per_channel;
    int x_per_token;        // one activation scale per row of a_q (per-vector setting)
    int gelu;               // the layer's output goes through the tanh GELU: Y = fp16(gelu(fp16(y)))
    uint16_t *slab_out;     // with gelu, persistent kernels only, or nullptr: workgroups write the
                            // column maxima |Y| of their tile, fp16 bits, to
                            // slab_out[tile_m][n] (row stride slab_ld, zeros for n >= N): the slab
                            // maxima the next layer's selection step folds
    int slab_ld;
    int aux_own_scale;      // Aux was quantised on its own scale: its accumulators are brought onto
                            // Body's scale by rho = (2^exp - 1) s_aux / s_x, rounded to the nearest
                            // integer; one activation scale: s_aux = x_scale[2]; one per token:
                            // rho[m] is the fifth array of x_scale (after s_x, 1/s, z, s_aux)
    long long *wg_ticks;    // measurement aid, or nullptr: workgroup i of a persistent kernel stores
                            // the constant 100 MHz counter at its start in [2 i] and at its end in [2 i + 1]
};

hipError_t launch_fill_u32(uint32_t *p, int n, uint32_t v, hipStream_t s);

// max |v| per column (per_tensor = 0) or over the whole matrix (per_tensor = 1,
// result in out_bits[0]) of a rows x cols fp16 matrix; out_bits must hold
// zeros on entry and receives the binary32 bit patterns of the maxima.
hipError_t launch_col_absmax(const void *x_fp16, int rows, int cols, int ld,
                             int per_tensor, uint32_t *out_bits, hipStream_t s,
                             const float *row_factor = nullptr);
// row_factor (here and in launch_wquant_transpose): row k of the matrix is first replaced by
// fp16(row * row_factor[k]), the weight side of a per-channel difficulty migration.

// Activation path: per-channel abs-max without atomics.  Writes fp16 magnitudes
// partial[slab][k_pad] (slab = a contiguous range of rows) and *n_slabs
// (<= kMaxSlabs); launch_fold_select_scale folds them.
constexpr int kMaxSlabs = 64;
// The number of slabs launch_col_absmax_partial and launch_gelu_absmax_partial write for a
// matrix of `rows` rows (a function of rows and k_pad only).
int absmax_slab_count(int rows, int k_pad);
// x = gelu(y) (tanh form, fp16 in and out, x may be y) and the slab maxima of x in one pass.
// With col_factor the producer is x = fp16(y / col_factor[k]) instead of the GELU (partial may
// then be null: no maxima wanted).
hipError_t launch_gelu_absmax_partial(const void *y_fp16, int rows, int cols, int ld_in, void *x_fp16,
                                      int ld_out, int k_pad, uint16_t *partial, hipStream_t s,
                                      const float *col_factor = nullptr);
hipError_t launch_col_absmax_partial(const void *x_fp16, int rows, int cols, int ld, int k_pad,
                                    uint16_t *partial, int *n_slabs, hipStream_t s);

// qmax below is the largest code magnitude, 2^(bits-1) - 1 (127 for the INT8 of
// Eq. 1-2), passed as a float.

// Fold of the slab maxima, outlier selection and (do_scale) scale derivation in
// one launch of one workgroup; col_scale / x_scale may be null without do_scale
// (col_slot and col_mask too, when the caller does not need them).  col_mask holds
// one byte per 8 channels, bit i = channel 8 c + i is a listed outlier channel.
hipError_t launch_fold_select_scale(const uint16_t *partial, int n_slabs, int K, int k_pad,
                                    float threshold, int r_cap, int exp, float qmax, int do_scale,
                                    float *col_absmax, int32_t *idx, int32_t *n_outliers,
                                    int32_t *col_slot, uint8_t *col_mask, float *col_scale,
                                    float *x_scale, hipStream_t s,
                                    const uint8_t *static_mask = nullptr,
                                    int32_t *zero_point = nullptr, float *aux_scale_out = nullptr);
// aux_scale_out (with do_scale): receives {s_aux, qmax / max|Aux|}, the abs-max scale of Aux's
// own values (the listed channels after the shift), for the own-scale reading of Eq. 5.
// static_mask (one bit per channel) replaces the threshold test by a list fixed offline.
// launch_static_list prepares such a list: col_mask, the padded index list, n_outliers =
// {listed, accepted}, and (r_cap > 0) the packed N x r_cap Aux weight rows.
hipError_t launch_static_list(const int32_t *list, int n_list, int K, int k_pad, int r_cap,
                              uint8_t *col_mask, int32_t *idx, int32_t *n_outliers, const int8_t *w_q,
                              int N, int8_t *w_aux, hipStream_t s);

// Outlier selection and/or scale derivation (one workgroup).
//   do_select: build idx / n_outliers / col_slot from col_absmax > threshold;
//   otherwise col_slot is rebuilt from the given idx / n_outliers.
//   do_scale: derive x_scale and col_scale (needs col_slot, col_scale != null).
hipError_t launch_select_scale(const float *col_absmax, int K, int k_pad, float threshold,
                               int r_cap, int exp, float qmax, int do_select, int do_scale,
                               int32_t *idx, int32_t *n_outliers, int32_t *col_slot,
                               float *col_scale, float *x_scale, hipStream_t s);

// Body/Aux quantisation with one activation scale; when w_aux != null the same
// launch also gathers the Aux weight rows w_aux[n][j] = w_q[n][idx[j]] (zero past
// n_outliers[0]).
hipError_t launch_quantize_body(const void *x_fp16, int M, int K, int ldx, int k_pad, float qmax,
                                const float *col_scale, const int32_t *col_slot,
                                const int32_t *n_outliers, int r_cap, int8_t *body_q,
                                int8_t *aux_q, const int8_t *w_q, int N, const int32_t *idx,
                                int8_t *w_aux, hipStream_t s, const int8_t *w_aux_given = nullptr,
                                const int32_t *zero_point = nullptr,
                                const int32_t *w_row_sum = nullptr, int32_t *cn = nullptr,
                                int32_t cn_bias = 0, const float *aux_scale = nullptr, int exp = 0);
// aux_scale (device {s_aux, qmax / max|Aux|}, with exp): Aux codes on that scale instead of Body's.
// zero_point (device scalar z from launch_fold_select_scale): unlisted channels are stored as
// code + z.  cn (with w_row_sum, and w_aux_given when w_aux is not gathered here) receives
// w_row_sum[n] - sum_j w_aux[n][j]; the GEMM takes z * cn[n] off its accumulators.

// The same with one activation scale per row (token): x_scale receives s_x[M]
// followed by qmax / max|Body[m]| [M].  Needs col_mask
// (launch_fold_select_scale without do_scale).
hipError_t launch_quantize_rows_token(const void *x_fp16, int M, int K, int ldx, int k_pad, float qmax,
                                      int exp, const uint8_t *col_mask, const int32_t *n_outliers,
                                      int r_cap, int8_t *body_q, int8_t *aux_q, float *x_scale,
                                      const int8_t *w_q, int N, const int32_t *idx, int8_t *w_aux,
                                      hipStream_t s, const int8_t *w_aux_given = nullptr,
                                      const int32_t *w_row_sum = nullptr, int32_t *cn = nullptr,
                                      int aux_own = 0);
// aux_own: Aux codes on the abs-max scale of each row's own Aux values; x_scale then also receives
// s_aux[M] (fourth array, after the row's zero points) and the GEMM's per-token factors
// rho[M] = (2^exp - 1) s_aux[m] / s_x[m] (fifth).

// Weight side: w_scale holds abs-max values (binary32) on entry to
// quantize_transpose; finalize turns them into scales amax / qmax.
hipError_t launch_wquant_transpose(const void *w_fp16, int K, int N, int ldw,
                                   int k_pad, const float *amax,
                                   int per_channel, float qmax, int8_t *w_q, int32_t *row_sum,
                                   hipStream_t s, const float *row_factor = nullptr);
hipError_t launch_wscale_finalize(float *w_scale, int n, float qmax, hipStream_t s);

hipError_t launch_gemm(const GemmArgs &a, hipStream_t s);
// Rows per output tile of the persistent form launch_gemm picks for this problem (256 or 128),
// or 0 when it picks the register-staged form (which does not write slab_out).
int gemm_persistent_tile_rows(int M, int N, int k_pad);

// Per-device set-up of the GEMM kernels for the CURRENT device: the LDS attribute of the
// persistent kernels and the CU count their grid is sized by.  Thread-safe, idempotent, and
// NOT capturable into a graph (it queries the device and sets function attributes).
// launch_gemm calls it itself when the current device has not been prepared yet.
hipError_t gemm_prepare_device();

}  // namespace muxq
