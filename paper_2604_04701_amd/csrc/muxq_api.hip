// C ABI of the MUXQ library (declared in include/muxq.h): argument checks and
// kernel sequencing only.  Nothing here allocates, frees or synchronises.
#include "../../include/muxq.h"
#include "../../include/muxq_measure.h"
#include "muxq_kernels.h"

#include <math.h>

#include <atomic>
#include <mutex>

// Scratch of muxq_linear_noalloc: the intermediates of one muxq_linear call (what a caller's
// workspace holds otherwise), in a static device array, so that the entry point needs no
// allocation and no workspace argument.  Each GPU the library runs on holds its own copy, at its
// own address, until the process ends.  In host code the name below is only a stand-in for the
// symbol, never a device address: the per-device address comes from hipGetSymbolAddress
// (noalloc_scratch_ptr) and only that pointer is handed to kernels.
constexpr size_t kNoallocBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kNoallocBytes];

namespace {

constexpr int kVersion = 100;

inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }
inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
inline int kpad(int K) { return (K + muxq::kKStep - 1) / muxq::kKStep * muxq::kKStep; }

int check_dims(int M, int K, int N)
{
    if (M < 1 || K < 1 || N < 1) return MUXQ_ERR_SHAPE;
    if (K % 8 != 0 || N % 8 != 0) return MUXQ_ERR_SHAPE;
    if (K > (1 << 21) || N > (1 << 21) || M > (1 << 24)) return MUXQ_ERR_SHAPE;   // grid limits
    // the kernels address packed operands with 32-bit byte offsets
    if (muxq::packed_bytes(M, kpad(K)) >= (1ull << 32) || muxq::packed_bytes(N, kpad(K)) >= (1ull << 32))
        return MUXQ_ERR_SHAPE;
    return MUXQ_OK;
}

int check_rcap(int K, int r_cap)
{
    if (r_cap < 0 || r_cap % 64 != 0 || r_cap > kpad(K)) return MUXQ_ERR_PARAM;
    return MUXQ_OK;
}

// Launch the GEMM, bracketed by the caller's two events if there are any (muxq_linear_timed).
hipError_t gemm_with_events(const muxq::GemmArgs &g, hipStream_t s, hipEvent_t e0 = nullptr,
                            hipEvent_t e1 = nullptr)
{
    hipError_t err;
    if (e0 && (err = hipEventRecord(e0, s)) != hipSuccess) return err;
    if ((err = muxq::launch_gemm(g, s)) != hipSuccess) return err;
    if (e1 && (err = hipEventRecord(e1, s)) != hipSuccess) return err;
    return hipSuccess;
}

#define MUXQ_TRY(expr)                          \
    do {                                        \
        if ((expr) != hipSuccess) return MUXQ_ERR_HIP; \
    } while (0)

// Accumulator bound of Eq. 7: |acc| <= 127^2 (K + (2^exp - 1) r_cap) must fit int32.
bool acc_fits(int K, int r_cap, int exp)
{
    double bound = 127.0 * 127.0 * ((double)K + (double)((1 << exp) - 1) * r_cap);
    return bound < 2147483647.0;
}

inline float qmax_of(int bits) { return (float)((1 << (bits - 1)) - 1); }

// Address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

hipError_t noalloc_scratch_ptr(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_acquire);
        if (p == nullptr) {
            if ((e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return e;
            if (p == nullptr) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return hipSuccess;
}

int linear_impl(const void *X, int M, int K, int ldx, const int8_t *w_q, const float *w_scale,
                int w_gran, int N, const void *bias, float threshold, int exp, int r_cap,
                void *Y, int ldy, void *workspace, size_t workspace_bytes, int32_t *dbg_acc,
                void *stream, int x_gran = MUXQ_X_PER_TENSOR, int ia_bits = 8,
                const void *static_block = nullptr, bool absmax_ready = false,
                hipEvent_t gemm_start = nullptr, hipEvent_t gemm_stop = nullptr,
                int64_t *wg_ticks = nullptr, bool aux_own = false, int absmax_slabs = 0,
                bool gelu = false, void *next_slabs = nullptr, bool validate_only = false)
{
    if ((x_gran != MUXQ_X_PER_TENSOR && x_gran != MUXQ_X_PER_TOKEN) || ia_bits < 2 || ia_bits > 8)
        return MUXQ_ERR_PARAM;
    // the per-token quantiser keeps list positions in 16 bits and stages a row's Aux codes
    // in LDS (4 * r_cap bytes per workgroup)
    if (x_gran == MUXQ_X_PER_TOKEN && (r_cap > 4096 || K > (1 << 17))) return MUXQ_ERR_PARAM;
    // Aux on its own scale is not combined with the fused GELU
    if (aux_own && gelu) return MUXQ_ERR_PARAM;
    if (r_cap == 0) aux_own = false;
    if (absmax_slabs < 0 || absmax_slabs > muxq::kMaxSlabs) return MUXQ_ERR_PARAM;
    if (next_slabs && !aligned(next_slabs, 16)) return MUXQ_ERR_ALIGN;
    const float qmax = qmax_of(ia_bits);
    if (!X || !w_q || !w_scale || !Y || !workspace) return MUXQ_ERR_NULL;
    int st = check_dims(M, K, N);
    if (st) return st;
    if (ldx < K || ldx % 8 || ldy < N || ldy % 8) return MUXQ_ERR_SHAPE;
    if ((st = check_rcap(K, r_cap))) return st;
    if (exp < 0 || exp > 7 || (w_gran != MUXQ_PER_TENSOR && w_gran != MUXQ_PER_CHANNEL) ||
        threshold != threshold || !acc_fits(K, r_cap, exp))
        return MUXQ_ERR_PARAM;
    if (!aligned(X, 16) || !aligned(w_q, 16) || !aligned(Y, 16) || !aligned(workspace, 256) ||
        !aligned(w_scale, 4) || (bias && !aligned(bias, 2)) || (dbg_acc && !aligned(dbg_acc, 16)))
        return MUXQ_ERR_ALIGN;
    muxq_ws_layout L;
    if ((st = muxq_workspace_layout(M, K, N, r_cap, &L))) return st;
    if (workspace_bytes < L.total) return MUXQ_ERR_WORKSPACE;
    if (validate_only) return MUXQ_OK;       // (the static block's layout cannot fail after check_rcap)

    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    float *col_absmax = (float *)(ws + L.col_absmax);
    float *col_scale = (float *)(ws + L.col_scale);
    int32_t *col_slot = (int32_t *)(ws + L.col_slot);
    int32_t *idx = (int32_t *)(ws + L.outlier_idx);
    int32_t *n_out = (int32_t *)(ws + L.n_outliers);
    float *x_scale = (float *)(ws + L.x_scale);
    int8_t *body_q = (int8_t *)(ws + L.body_q);
    int8_t *aux_q = (int8_t *)(ws + L.aux_q);
    int8_t *w_aux = (int8_t *)(ws + L.w_aux);
    uint16_t *partial = (uint16_t *)(ws + L.absmax_partial);
    const int k_pad = L.k_pad;

    // four launches: slab maxima -> fold + select (+ scales) -> quantise (+ Aux weight
    // gather in the same launch) -> GEMM.  With a static block the channel list and the Aux
    // weight rows are given: no gather, and in the per-token setting no pass for the
    // channel maxima either (two launches).
    int n_slabs = 0;
    const bool per_token = x_gran == MUXQ_X_PER_TOKEN;
    const uint8_t *static_mask = nullptr;
    const uint8_t *col_mask = (const uint8_t *)(ws + L.col_mask);
    if (static_block != nullptr) {
        muxq_static_layout SL;
        if ((st = muxq_static_layout_of(K, N, r_cap, &SL))) return st;
        const char *sb = (const char *)static_block;
        static_mask = (const uint8_t *)(sb + SL.col_mask);
        w_aux = (int8_t *)(sb + SL.w_aux);                   // read only from here on
        if (per_token) {
            col_mask = static_mask;
            n_out = (int32_t *)(sb + SL.n_outliers);         // read only
        }
    }
    const bool gather = static_block == nullptr && r_cap > 0;
    // the unlisted channels carry a zero point (see muxq.h): one per call, or one per token
    int32_t *zero_point = per_token ? (int32_t *)x_scale + 2 * (size_t)M : (int32_t *)(ws + L.n_outliers) + 2;
    int32_t *cn = (int32_t *)(ws + L.cn);
    const int32_t *w_row_sum = (const int32_t *)(w_q + muxq::wq_rowsum_offset(N, k_pad));
    if (!(per_token && static_block != nullptr)) {
        if (absmax_ready)     // a producer of X has left the slab maxima in the workspace
            n_slabs = absmax_slabs > 0 ? absmax_slabs : muxq::absmax_slab_count(M, k_pad);
        else
            MUXQ_TRY(muxq::launch_col_absmax_partial(X, M, K, ldx, k_pad, partial, &n_slabs, s));
        MUXQ_TRY(muxq::launch_fold_select_scale(partial, n_slabs, K, k_pad, threshold, r_cap, exp, qmax,
                                                per_token ? 0 : 1, col_absmax, idx, n_out, col_slot,
                                                (uint8_t *)(ws + L.col_mask), col_scale, x_scale, s,
                                                static_mask, per_token ? nullptr : zero_point,
                                                aux_own && !per_token ? x_scale + 2 : nullptr));
    }
    if (per_token)
        MUXQ_TRY(muxq::launch_quantize_rows_token(X, M, K, ldx, k_pad, qmax, exp, col_mask, n_out, r_cap,
                                                  body_q, aux_q, x_scale, w_q, N, idx,
                                                  gather ? w_aux : nullptr, s,
                                                  gather ? nullptr : (r_cap ? w_aux : nullptr),
                                                  w_row_sum, cn, aux_own ? 1 : 0));
    else
        MUXQ_TRY(muxq::launch_quantize_body(X, M, K, ldx, k_pad, qmax, col_scale, col_slot, n_out,
                                            r_cap, body_q, aux_q, w_q, N, idx,
                                            gather ? w_aux : nullptr, s,
                                            gather ? nullptr : (r_cap ? w_aux : nullptr), zero_point,
                                            w_row_sum, cn, muxq::kCnBias, aux_own ? x_scale + 2 : nullptr,
                                            exp));

    muxq::GemmArgs g{};
    g.a_q = body_q;
    g.w_q = w_q;
    g.aux_q = r_cap ? aux_q : nullptr;
    g.w_aux = r_cap ? w_aux : nullptr;
    g.n_outliers = r_cap ? n_out : nullptr;
    g.x_scale = x_scale;
    g.w_scale = w_scale;
    g.bias = (const _Float16 *)bias;
    g.y = (_Float16 *)Y;
    g.dbg_acc = dbg_acc;
    g.cn = cn;
    g.zero_point = zero_point;
    g.cn_bias = per_token ? 0 : muxq::kCnBias;
    g.M = M; g.N = N; g.k_pad = k_pad; g.r_cap = r_cap; g.ldy = ldy;
    g.exp_shift = exp;
    g.w_per_channel = w_gran == MUXQ_PER_CHANNEL;
    g.x_per_token = per_token;
    g.aux_own_scale = aux_own;
    g.wg_ticks = (long long *)wg_ticks;
    g.gelu = gelu;
    // the column maxima of the output, for the next layer: from the GEMM's own tiles when it
    // runs as a persistent kernel with at most kMaxSlabs rows of tiles, else by a pass over Y
    const int k_pad_next = kpad(N);
    const int tile_rows = muxq::gemm_persistent_tile_rows(M, N, k_pad);
    const bool slabs_from_gemm = gelu && next_slabs != nullptr && tile_rows > 0 &&
                                 (M + tile_rows - 1) / tile_rows <= muxq::kMaxSlabs;
    if (slabs_from_gemm) {
        g.slab_out = (uint16_t *)next_slabs;
        g.slab_ld = k_pad_next;
    }
    MUXQ_TRY(gemm_with_events(g, s, gemm_start, gemm_stop));
    if (gelu && next_slabs != nullptr && !slabs_from_gemm) {
        int n_next = 0;
        MUXQ_TRY(muxq::launch_col_absmax_partial(Y, M, N, ldy, k_pad_next, (uint16_t *)next_slabs, &n_next, s));
    }
    return MUXQ_OK;
}

}  // namespace

extern "C" {

int muxq_version(void) { return kVersion; }

const char *muxq_status_string(int status)
{
    switch (status) {
    case MUXQ_OK: return "ok";
    case MUXQ_ERR_NULL: return "a required pointer is NULL";
    case MUXQ_ERR_SHAPE: return "dimension or leading dimension breaks the shape rules";
    case MUXQ_ERR_ALIGN: return "pointer not sufficiently aligned";
    case MUXQ_ERR_PARAM: return "parameter out of range";
    case MUXQ_ERR_WORKSPACE: return "workspace too small";
    case MUXQ_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
    }
}

int muxq_init(void)
{
    MUXQ_TRY(muxq::gemm_prepare_device());
    void *p = nullptr;
    MUXQ_TRY(noalloc_scratch_ptr(&p));
    return MUXQ_OK;
}

size_t muxq_noalloc_max_bytes(void) { return kNoallocBytes; }

int muxq_linear_noalloc(const void *X, int M, int K, int ldx, const int8_t *w_q, const float *w_scale,
                        int w_gran, int N, const void *bias, float threshold, int exp, int r_cap, void *Y,
                        int ldy, void *stream)
{
    // sizes first: a shape that does not fit the static array is refused before anything else
    // happens (bad shapes get their own status from the layout call)
    muxq_ws_layout L;
    const int st = muxq_workspace_layout(M, K, N, r_cap, &L);
    if (st) return st;
    if (L.total > kNoallocBytes) return MUXQ_ERR_WORKSPACE;
    void *ws = nullptr;
    MUXQ_TRY(noalloc_scratch_ptr(&ws));
    // Nothing in the array has to start at zero: every kernel of the call writes what the next
    // one reads (the same contract as a caller's workspace, which needs no defined content).
    return linear_impl(X, M, K, ldx, w_q, w_scale, w_gran, N, bias, threshold, exp, r_cap, Y, ldy, ws,
                       kNoallocBytes, nullptr, stream);
}

int muxq_linear_timed(const void *X, int M, int K, int ldx, const int8_t *w_q, const float *w_scale,
                      int w_gran, int N, const void *bias, float threshold, int exp, int r_cap, void *Y,
                      int ldy, void *workspace, size_t workspace_bytes, const muxq_act_opts *opts,
                      void *gemm_start, void *gemm_stop, int64_t *wg_ticks, void *stream)
{
    if (!gemm_start || !gemm_stop) return MUXQ_ERR_NULL;
    if (wg_ticks && !aligned(wg_ticks, 8)) return MUXQ_ERR_ALIGN;
    const int x_gran = opts ? opts->x_gran : MUXQ_X_PER_TENSOR;
    const int ia_bits = opts ? opts->ia_bits : 8;
    return linear_impl(X, M, K, ldx, w_q, w_scale, w_gran, N, bias, threshold, exp, r_cap, Y, ldy,
                       workspace, workspace_bytes, nullptr, stream, x_gran, ia_bits, nullptr,
                       opts && opts->absmax_ready, (hipEvent_t)gemm_start, (hipEvent_t)gemm_stop, wg_ticks,
                       opts && opts->aux_own_scale, opts ? opts->absmax_slabs : 0);
}

int muxq_k_pad(int K) { return K < 1 ? 0 : kpad(K); }

size_t muxq_wq_bytes(int K, int N)
{
    if (K < 1 || N < 1) return 0;
    return muxq::wq_total_bytes(N, kpad(K));
}

size_t muxq_packed_bytes(int rows, int cols)
{
    if (rows < 1 || cols < 0 || cols % 64) return 0;
    return muxq::packed_bytes(rows, cols);
}

size_t muxq_packed_index(int row, int col, int cols)
{
    return muxq::packed_index(row, col, cols);
}

int muxq_workspace_layout(int M, int K, int N, int r_cap, muxq_ws_layout *out)
{
    if (!out) return MUXQ_ERR_NULL;
    int st = check_dims(M, K, N);
    if (st) return st;
    if ((st = check_rcap(K, r_cap))) return st;
    const size_t kp = (size_t)kpad(K);
    size_t off = 0;
    out->k_pad = (int32_t)kp;
    out->col_absmax = off;  off += up256(kp * 4);
    out->col_scale = off;   off += up256(kp * 4);
    out->col_slot = off;    off += up256(kp * 4);
    out->col_mask = off;    off += up256(kp / 8);
    out->outlier_idx = off; off += up256((size_t)(r_cap > 0 ? r_cap : 1) * 4);
    out->n_outliers = off;  off += 256;
    out->x_scale = off;     off += up256((size_t)(M > 1 ? M : 1) * 5 * 4);
    out->absmax_partial = off; off += up256((size_t)muxq::kMaxSlabs * kp * 2);
    out->body_q = off;      off += up256(muxq::packed_bytes(M, (int)kp));
    out->aux_q = off;       off += up256(muxq::packed_bytes(M, r_cap));
    out->w_aux = off;       off += up256(muxq::packed_bytes(N, r_cap));
    out->cn = off;          off += up256((size_t)N * 4);
    out->total = off;
    return MUXQ_OK;
}

int muxq_static_layout_of(int K, int N, int r_cap, muxq_static_layout *out)
{
    if (!out) return MUXQ_ERR_NULL;
    int st = check_dims(1, K, N);
    if (st) return st;
    if ((st = check_rcap(K, r_cap))) return st;
    const size_t kp = (size_t)kpad(K);
    size_t off = 0;
    out->k_pad = (int32_t)kp;
    out->col_mask = off;    off += up256(kp / 8);
    out->outlier_idx = off; off += up256((size_t)(r_cap > 0 ? r_cap : 1) * 4);
    out->n_outliers = off;  off += 256;
    out->w_aux = off;       off += up256(muxq::packed_bytes(N, r_cap));
    out->total = off;
    return MUXQ_OK;
}

size_t muxq_static_bytes(int K, int N, int r_cap)
{
    muxq_static_layout L;
    return muxq_static_layout_of(K, N, r_cap, &L) == MUXQ_OK ? L.total : 0;
}

int muxq_prepare_static(const int32_t *list, int n_list, int K, const int8_t *w_q, int N, int r_cap,
                        void *static_block, size_t static_bytes, void *stream)
{
    if (!w_q || !static_block || (n_list > 0 && !list)) return MUXQ_ERR_NULL;
    if (n_list < 0) return MUXQ_ERR_PARAM;
    muxq_static_layout L;
    int st = muxq_static_layout_of(K, N, r_cap, &L);
    if (st) return st;
    if (!aligned(w_q, 16) || !aligned(static_block, 256) || (list && !aligned(list, 4))) return MUXQ_ERR_ALIGN;
    if (static_bytes < L.total) return MUXQ_ERR_WORKSPACE;
    char *sb = (char *)static_block;
    MUXQ_TRY(muxq::launch_static_list(list, n_list, K, L.k_pad, r_cap, (uint8_t *)(sb + L.col_mask),
                                      (int32_t *)(sb + L.outlier_idx), (int32_t *)(sb + L.n_outliers),
                                      w_q, N, (int8_t *)(sb + L.w_aux), (hipStream_t)stream));
    return MUXQ_OK;
}

int muxq_linear_static(const void *X, int M, int K, int ldx, const int8_t *w_q, const float *w_scale,
                       int w_gran, int N, const void *bias, int exp, int r_cap,
                       const void *static_block, void *Y, int ldy, void *workspace,
                       size_t workspace_bytes, int32_t *dbg_acc, const muxq_act_opts *opts,
                       void *stream)
{
    if (!static_block) return MUXQ_ERR_NULL;
    if (!aligned(static_block, 256)) return MUXQ_ERR_ALIGN;
    const int x_gran = opts ? opts->x_gran : MUXQ_X_PER_TENSOR;
    const int ia_bits = opts ? opts->ia_bits : 8;
    return linear_impl(X, M, K, ldx, w_q, w_scale, w_gran, N, bias, 0.0f, exp, r_cap, Y, ldy, workspace,
                       workspace_bytes, dbg_acc, stream, x_gran, ia_bits, static_block,
                       opts && opts->absmax_ready, nullptr, nullptr, nullptr,
                       opts && opts->aux_own_scale, opts ? opts->absmax_slabs : 0);
}

size_t muxq_workspace_bytes(int M, int K, int N, int r_cap)
{
    muxq_ws_layout L;
    return muxq_workspace_layout(M, K, N, r_cap, &L) == MUXQ_OK ? L.total : 0;
}

int muxq_quantize_weight(const void *W, int K, int N, int ldw, int gran, int8_t *w_q,
                         float *w_scale, void *stream)
{
    return muxq_quantize_weight_bits(W, K, N, ldw, gran, 8, w_q, w_scale, stream);
}

int muxq_quantize_weight_bits(const void *W, int K, int N, int ldw, int gran, int w_bits,
                              int8_t *w_q, float *w_scale, void *stream)
{
    return muxq_quantize_weight_smooth(W, K, N, ldw, gran, w_bits, nullptr, w_q, w_scale, stream);
}

int muxq_quantize_weight_smooth(const void *W, int K, int N, int ldw, int gran, int w_bits,
                                const float *factors, int8_t *w_q, float *w_scale, void *stream)
{
    if (!W || !w_q || !w_scale) return MUXQ_ERR_NULL;
    if (factors && !aligned(factors, 4)) return MUXQ_ERR_ALIGN;
    if (w_bits < 2 || w_bits > 8) return MUXQ_ERR_PARAM;
    const float qmax = qmax_of(w_bits);
    int st = check_dims(1, K, N);
    if (st) return st;
    if (ldw < N || ldw % 8) return MUXQ_ERR_SHAPE;
    if (gran != MUXQ_PER_TENSOR && gran != MUXQ_PER_CHANNEL) return MUXQ_ERR_PARAM;
    if (!aligned(W, 16) || !aligned(w_q, 16) || !aligned(w_scale, 4)) return MUXQ_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    const int per_channel = gran == MUXQ_PER_CHANNEL;
    const int n_scales = per_channel ? N : 1;
    // w_scale first holds the abs-max values (as binary32), then the scales.
    MUXQ_TRY(muxq::launch_fill_u32((uint32_t *)w_scale, n_scales, 0u, s));
    MUXQ_TRY(muxq::launch_col_absmax(W, K, N, ldw, !per_channel, (uint32_t *)w_scale, s, factors));
    int32_t *row_sum = (int32_t *)(w_q + muxq::wq_rowsum_offset(N, kpad(K)));
    MUXQ_TRY(muxq::launch_fill_u32((uint32_t *)row_sum, N, 0u, s));
    MUXQ_TRY(muxq::launch_wquant_transpose(W, K, N, ldw, kpad(K), w_scale, per_channel, qmax, w_q,
                                           row_sum, s, factors));
    MUXQ_TRY(muxq::launch_wscale_finalize(w_scale, n_scales, qmax, s));
    return MUXQ_OK;
}

size_t muxq_detect_scratch_bytes(int K)
{
    return K < 1 ? 0 : (size_t)muxq::kMaxSlabs * (size_t)kpad(K) * 2;
}

int muxq_detect_outliers(const void *X, int M, int K, int ldx, float threshold, int r_cap,
                         float *col_absmax, int32_t *outlier_idx, int32_t *n_outliers,
                         void *scratch, void *stream)
{
    if (!X || !col_absmax || !outlier_idx || !n_outliers || !scratch) return MUXQ_ERR_NULL;
    int st = check_dims(M, K, 8);
    if (st) return st;
    if (ldx < K || ldx % 8) return MUXQ_ERR_SHAPE;
    if ((st = check_rcap(K, r_cap))) return st;
    if (threshold != threshold) return MUXQ_ERR_PARAM;
    if (!aligned(X, 16) || !aligned(col_absmax, 4) || !aligned(outlier_idx, 4) ||
        !aligned(n_outliers, 4) || !aligned(scratch, 16))
        return MUXQ_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    int n_slabs = 0;
    MUXQ_TRY(muxq::launch_col_absmax_partial(X, M, K, ldx, kpad(K), (uint16_t *)scratch, &n_slabs, s));
    MUXQ_TRY(muxq::launch_fold_select_scale((const uint16_t *)scratch, n_slabs, K, kpad(K), threshold,
                                            r_cap, 0, 127.0f, 0, col_absmax, outlier_idx, n_outliers, nullptr,
                                            nullptr, nullptr, nullptr, s));
    return MUXQ_OK;
}

int muxq_build_aux(const void *X, int M, int K, int ldx, const float *col_absmax,
                   const int32_t *outlier_idx, const int32_t *n_outliers, int r_cap, int exp,
                   int8_t *body_q, int8_t *aux_q, float *x_scale, void *scratch, void *stream)
{
    if (!X || !col_absmax || !outlier_idx || !n_outliers || !body_q || !x_scale || !scratch ||
        (r_cap > 0 && !aux_q))
        return MUXQ_ERR_NULL;
    int st = check_dims(M, K, 8);
    if (st) return st;
    const int k_pad = kpad(K);
    if (ldx < K || ldx % 8) return MUXQ_ERR_SHAPE;
    if ((st = check_rcap(K, r_cap))) return st;
    if (exp < 0 || exp > 7) return MUXQ_ERR_PARAM;
    if (!aligned(X, 16) || !aligned(body_q, 16) || !aligned(scratch, 16) ||
        (aux_q && !aligned(aux_q, 16)) || !aligned(x_scale, 4))
        return MUXQ_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    float *col_scale = (float *)scratch;
    int32_t *col_slot = (int32_t *)scratch + k_pad;
    MUXQ_TRY(muxq::launch_select_scale(col_absmax, K, k_pad, 0.f, r_cap, exp, 127.0f, 0, 1,
                                       const_cast<int32_t *>(outlier_idx),
                                       const_cast<int32_t *>(n_outliers), col_slot, col_scale,
                                       x_scale, s));
    MUXQ_TRY(muxq::launch_quantize_body(X, M, K, ldx, k_pad, 127.0f, col_scale, col_slot, n_outliers,
                                        r_cap, body_q, aux_q, nullptr, 0, nullptr, nullptr, s));
    return MUXQ_OK;
}

int muxq_linear(const void *X, int M, int K, int ldx, const int8_t *w_q, const float *w_scale,
                int w_gran, int N, const void *bias, float threshold, int exp, int r_cap, void *Y,
                int ldy, void *workspace, size_t workspace_bytes, int32_t *dbg_acc, void *stream)
{
    return linear_impl(X, M, K, ldx, w_q, w_scale, w_gran, N, bias, threshold, exp, r_cap, Y, ldy,
                       workspace, workspace_bytes, dbg_acc, stream);
}

int muxq_linear_opts(const void *X, int M, int K, int ldx, const int8_t *w_q, const float *w_scale,
                     int w_gran, int N, const void *bias, float threshold, int exp, int r_cap,
                     void *Y, int ldy, void *workspace, size_t workspace_bytes, int32_t *dbg_acc,
                     const muxq_act_opts *opts, void *stream)
{
    const int x_gran = opts ? opts->x_gran : MUXQ_X_PER_TENSOR;
    const int ia_bits = opts ? opts->ia_bits : 8;
    return linear_impl(X, M, K, ldx, w_q, w_scale, w_gran, N, bias, threshold, exp, r_cap, Y, ldy,
                       workspace, workspace_bytes, dbg_acc, stream, x_gran, ia_bits, nullptr,
                       opts && opts->absmax_ready, nullptr, nullptr, nullptr,
                       opts && opts->aux_own_scale, opts ? opts->absmax_slabs : 0);
}

int muxq_linear_gelu_slabs(int M, int K, int N)
{
    if (check_dims(M, K, N)) return 0;
    const int tile_rows = muxq::gemm_persistent_tile_rows(M, N, kpad(K));
    if (tile_rows > 0 && (M + tile_rows - 1) / tile_rows <= muxq::kMaxSlabs) return (M + tile_rows - 1) / tile_rows;
    return muxq::absmax_slab_count(M, kpad(N));
}

int muxq_linear_gelu(const void *X, int M, int K, int ldx, const int8_t *w_q, const float *w_scale,
                     int w_gran, int N, const void *bias, float threshold, int exp, int r_cap, void *H,
                     int ldh, void *workspace, size_t workspace_bytes, void *next_slabs,
                     const muxq_act_opts *opts, void *stream)
{
    const int x_gran = opts ? opts->x_gran : MUXQ_X_PER_TENSOR;
    const int ia_bits = opts ? opts->ia_bits : 8;
    return linear_impl(X, M, K, ldx, w_q, w_scale, w_gran, N, bias, threshold, exp, r_cap, H, ldh,
                       workspace, workspace_bytes, nullptr, stream, x_gran, ia_bits, nullptr,
                       opts && opts->absmax_ready, nullptr, nullptr, nullptr,
                       opts && opts->aux_own_scale, opts ? opts->absmax_slabs : 0, true, next_slabs);
}

size_t muxq_mlp_workspace_bytes(int M, int K, int N1, int N2, int r_cap)
{
    muxq_ws_layout L1, L2;
    if (muxq_workspace_layout(M, K, N1, r_cap, &L1) || muxq_workspace_layout(M, N1, N2, r_cap, &L2)) return 0;
    return up256(L1.total) + L2.total;
}

int muxq_mlp(const void *X, int M, int K, int ldx, const int8_t *w1_q, const float *w1_scale, int w1_gran,
             int N1, const void *bias1, const int8_t *w2_q, const float *w2_scale, int w2_gran, int N2,
             const void *bias2, float threshold, int exp, int r_cap, void *H, int ldh, void *Y, int ldy,
             void *workspace, size_t workspace_bytes, const muxq_act_opts *opts, void *stream)
{
    if (!workspace) return MUXQ_ERR_NULL;
    if (!aligned(workspace, 256)) return MUXQ_ERR_ALIGN;
    const int x_gran = opts ? opts->x_gran : MUXQ_X_PER_TENSOR;
    const int ia_bits = opts ? opts->ia_bits : 8;
    if (opts && opts->aux_own_scale) return MUXQ_ERR_PARAM;
    muxq_ws_layout L1, L2;
    int st;
    if ((st = muxq_workspace_layout(M, K, N1, r_cap, &L1))) return st;
    if ((st = muxq_workspace_layout(M, N1, N2, r_cap, &L2))) return st;
    const size_t off2 = up256(L1.total);
    if (workspace_bytes < off2 + L2.total) return MUXQ_ERR_WORKSPACE;
    char *ws1 = (char *)workspace, *ws2 = ws1 + off2;
    void *slabs2 = ws2 + L2.absmax_partial;
    const int n_slabs = muxq_linear_gelu_slabs(M, K, N1);
    // both layers' arguments are checked before the first kernel is launched
    for (int pass = 0; pass < 2; ++pass) {
        const bool dry = pass == 0;
        st = linear_impl(X, M, K, ldx, w1_q, w1_scale, w1_gran, N1, bias1, threshold, exp, r_cap, H, ldh, ws1,
                         L1.total, nullptr, stream, x_gran, ia_bits, nullptr, opts && opts->absmax_ready,
                         nullptr, nullptr, nullptr, false, opts ? opts->absmax_slabs : 0, true, slabs2, dry);
        if (st) return st;
        st = linear_impl(H, M, N1, ldh, w2_q, w2_scale, w2_gran, N2, bias2, threshold, exp, r_cap, Y, ldy, ws2,
                         L2.total, nullptr, stream, x_gran, ia_bits, nullptr, true, nullptr, nullptr, nullptr,
                         false, n_slabs, false, nullptr, dry);
        if (st) return st;
    }
    return MUXQ_OK;
}

int muxq_gelu_absmax(const void *Y, int M, int K, int ldy, void *X, int ldx, void *slabs, void *stream)
{
    if (!Y || !X || !slabs) return MUXQ_ERR_NULL;
    if (M < 1 || K < 1 || K % 8 != 0 || K > (1 << 21) || M > (1 << 24)) return MUXQ_ERR_SHAPE;
    if (ldy < K || ldy % 8 || ldx < K || ldx % 8) return MUXQ_ERR_SHAPE;
    if (!aligned(Y, 16) || !aligned(X, 16) || !aligned(slabs, 16)) return MUXQ_ERR_ALIGN;
    MUXQ_TRY(muxq::launch_gelu_absmax_partial(Y, M, K, ldy, X, ldx, kpad(K), (uint16_t *)slabs,
                                              (hipStream_t)stream));
    return MUXQ_OK;
}

int muxq_smooth_absmax(const void *X, int M, int K, int ldx, const float *factors, void *X_out, int ldo,
                       void *slabs, void *stream)
{
    if (!X || !X_out || !factors) return MUXQ_ERR_NULL;
    if (M < 1 || K < 1 || K % 8 != 0 || K > (1 << 21) || M > (1 << 24)) return MUXQ_ERR_SHAPE;
    if (ldx < K || ldx % 8 || ldo < K || ldo % 8) return MUXQ_ERR_SHAPE;
    if (!aligned(X, 16) || !aligned(X_out, 16) || !aligned(factors, 4) || (slabs && !aligned(slabs, 16)))
        return MUXQ_ERR_ALIGN;
    MUXQ_TRY(muxq::launch_gelu_absmax_partial(X, M, K, ldx, X_out, ldo, kpad(K), (uint16_t *)slabs,
                                              (hipStream_t)stream, factors));
    return MUXQ_OK;
}

int muxq_linear_naive_int8(const void *X, int M, int K, int ldx, const int8_t *w_q,
                           const float *w_scale, int w_gran, int N, const void *bias, void *Y,
                           int ldy, void *workspace, size_t workspace_bytes, int32_t *dbg_acc,
                           void *stream)
{
    return linear_impl(X, M, K, ldx, w_q, w_scale, w_gran, N, bias, INFINITY, 0, 0, Y, ldy,
                       workspace, workspace_bytes, dbg_acc, stream);
}

int muxq_gemm_i8(const int8_t *a_q, int M, int K, const int8_t *w_q, int N,
                 const int8_t *aux_q, const int8_t *w_aux, const int32_t *n_outliers, int r_cap,
                 int exp, const float *x_scale, const float *w_scale, int w_gran,
                 const void *bias, void *Y, int ldy, int32_t *dbg_acc, void *stream)
{
    if (!a_q || !w_q || !x_scale || !w_scale || !Y) return MUXQ_ERR_NULL;
    int st = check_dims(M, K, N);
    if (st) return st;
    const int k_pad = kpad(K);
    if (ldy < N || ldy % 8) return MUXQ_ERR_SHAPE;
    const bool with_aux = aux_q || w_aux || n_outliers;
    if (with_aux && (!aux_q || !w_aux || !n_outliers)) return MUXQ_ERR_NULL;
    if (!with_aux) r_cap = 0;
    if ((st = check_rcap(K, r_cap))) return st;
    if (exp < 0 || exp > 7 || (w_gran != MUXQ_PER_TENSOR && w_gran != MUXQ_PER_CHANNEL) ||
        !acc_fits(K, r_cap, exp))
        return MUXQ_ERR_PARAM;
    if (!aligned(a_q, 16) || !aligned(w_q, 16) || !aligned(Y, 16) ||
        (with_aux && (!aligned(aux_q, 16) || !aligned(w_aux, 16))) ||
        (dbg_acc && !aligned(dbg_acc, 16)))
        return MUXQ_ERR_ALIGN;
    muxq::GemmArgs g{};
    g.a_q = a_q;
    g.w_q = w_q;
    g.aux_q = r_cap ? aux_q : nullptr;
    g.w_aux = r_cap ? w_aux : nullptr;
    g.n_outliers = r_cap ? n_outliers : nullptr;
    g.x_scale = x_scale;
    g.w_scale = w_scale;
    g.bias = (const _Float16 *)bias;
    g.y = (_Float16 *)Y;
    g.dbg_acc = dbg_acc;
    g.M = M; g.N = N; g.k_pad = k_pad; g.r_cap = r_cap; g.ldy = ldy;
    g.exp_shift = exp;
    g.w_per_channel = w_gran == MUXQ_PER_CHANNEL;
    g.x_per_token = 0;
    MUXQ_TRY(gemm_with_events(g, (hipStream_t)stream));
    return MUXQ_OK;
}

}  // extern "C"
