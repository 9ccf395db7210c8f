// INT8 x INT8 -> INT32 MFMA GEMM of the MUXQ linear layer for gfx950, with the
// Aux product, the (2^exp - 1) recombination (Eq. 7) and the dequantising
// epilogue (Eq. 3) fused in.
//
// Orientation.  Both operands are stored K-contiguous: activations a_q[m][k]
// and the packed weight w_q[n][k].  The MFMA computes D = A.B with A = a
// 32(n) x 32(k) block of the weight and B = a 32(k) x 32(m) block of the
// activations, i.e. the tile of Y transposed.  In the 32x32 accumulator layout
// each lane then owns ONE token m and runs of 4 consecutive output channels
// n, which are contiguous in row-major Y: the epilogue stores 8-byte fp16x4
// packets without any shuffle.
//
// K loop.  The Aux product is simply a few extra K tiles placed FIRST: the
// accumulators after the Aux tiles hold acc_aux; they are multiplied once by
// c = 2^exp - 1 and the Body tiles are then accumulated on top, which gives
// acc_body + c * acc_aux in exact integer arithmetic with one set of
// accumulators.  The number of Aux tiles is read from device memory
// (n_outliers[0]) so no host synchronisation is needed.
//
// Tiling.  Workgroup tile TN x TM (output channels x tokens), K step BK = 64
// codes, WN x WM waves, each wave FN x FM fragments of 32 x 32.  Global ->
// registers -> LDS staging with two LDS buffers and one barrier per K step;
// the next tile's global loads are issued before the MFMAs of the current
// tile.  LDS rows are BK bytes with the 16-byte chunks XOR-swizzled by the
// row number so that the ds_read_b128 fragment loads (32 rows x same chunk)
// and the ds_write_b128 stores are bank-conflict free without padding.
//
// Workgroup -> tile map.  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2.  Tiles are grouped in super-tiles of sup_m x sup_n tiles
// (<= 32, one per CU of an XCD); workgroup i belongs to XCD i % 8 and the
// workgroups an XCD runs concurrently form one compact super-tile, so its L2
// holds (sup_m + sup_n) operand panels for sup_m * sup_n tiles.
#include "muxq_kernels.h"

namespace muxq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

struct TileMap {
    int tiles_m, tiles_n, sup_m, sup_n, super_n, n_super;
};

template <int BK>
__device__ __forceinline__ int swizzle(int row, int chunk)
{
    if constexpr (BK == 64)
        return chunk ^ ((row >> 1) & 3);
    else
        return chunk ^ (row & 7);
}

template <int TN, int TM, int BK, int WN, int WM>
__global__ __launch_bounds__(WN *WM * 64) void k_gemm_i8(const GemmArgs a, const TileMap tm)
{
    constexpr int NT = WN * WM * 64;
    constexpr int CH = BK / 16;              // 16-byte chunks per LDS row
    constexpr int FN = TN / WN / 32, FM = TM / WM / 32;
    constexpr int ROWS_PER_PASS = NT / CH;
    constexpr int W_LD = TN / ROWS_PER_PASS, X_LD = TM / ROWS_PER_PASS;
    constexpr int BUF_BYTES = (TN + TM) * BK;
    static_assert(TN % ROWS_PER_PASS == 0 && TM % ROWS_PER_PASS == 0, "tile/threads mismatch");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // ---- workgroup -> tile --------------------------------------------------
    const int S = tm.sup_m * tm.sup_n;
    const int wg = blockIdx.x;
    const int xcd = wg & 7, j = wg >> 3;
    const int w_in = j % S, st = (j / S) * 8 + xcd;
    if (st >= tm.n_super) return;
    const int tile_m = (st / tm.super_n) * tm.sup_m + w_in / tm.sup_n;
    const int tile_n = (st % tm.super_n) * tm.sup_n + w_in % tm.sup_n;
    if (tile_m >= tm.tiles_m || tile_n >= tm.tiles_n) return;
    const int m0 = tile_m * TM, n0 = tile_n * TN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_n = (wave % WN) * (TN / WN), wave_m = (wave / WN) * (TM / WM);

    // ---- K-tile schedule: Aux tiles first, then Body tiles -------------------
    int used = 0;
    if (a.n_outliers != nullptr && a.r_cap > 0) used = max(0, min(a.n_outliers[0], a.r_cap));
    used = __builtin_amdgcn_readfirstlane(used);
    const int t_aux = (used + BK - 1) / BK;
    const int t_all = t_aux + a.k_pad / BK;

    // ---- global -> LDS staging roles -----------------------------------------
    const int ld_chunk = tid % CH, ld_row = tid / CH;
    int w_row[W_LD], x_row[X_LD];     // clamped global rows
    int w_lds[W_LD], x_lds[X_LD];     // byte offsets inside one LDS buffer
#pragma unroll
    for (int i = 0; i < W_LD; ++i) {
        int r = ld_row + i * ROWS_PER_PASS;
        w_row[i] = min(n0 + r, a.N - 1);
        w_lds[i] = r * BK + swizzle<BK>(r, ld_chunk) * 16;
    }
#pragma unroll
    for (int i = 0; i < X_LD; ++i) {
        int r = ld_row + i * ROWS_PER_PASS;
        x_row[i] = min(m0 + r, a.M - 1);
        x_lds[i] = TN * BK + r * BK + swizzle<BK>(r, ld_chunk) * 16;
    }
    v4i stage_w[W_LD], stage_x[X_LD];

    // Issue the global loads of K tile t into the staging registers.
#define MUXQ_LOAD_TILE(t_)                                                                   \
    do {                                                                                     \
        const int tt_ = (t_);                                                                \
        const bool aux_ = tt_ < t_aux;                                                       \
        const int8_t *wp_ = aux_ ? a.w_aux : a.w_q;                                          \
        const int8_t *xp_ = aux_ ? a.aux_q : a.a_q;                                          \
        const int ldw_ = aux_ ? a.r_cap : a.ldw, ldx_ = aux_ ? a.r_cap : a.lda;              \
        const int k0_ = (aux_ ? tt_ : tt_ - t_aux) * BK + ld_chunk * 16;                     \
        _Pragma("unroll") for (int i = 0; i < W_LD; ++i)                                     \
            stage_w[i] = *(const v4i *)(wp_ + (size_t)w_row[i] * ldw_ + k0_);                \
        _Pragma("unroll") for (int i = 0; i < X_LD; ++i)                                     \
            stage_x[i] = *(const v4i *)(xp_ + (size_t)x_row[i] * ldx_ + k0_);                \
    } while (0)
    // Write the staging registers into LDS buffer buf_.
#define MUXQ_STORE_TILE(buf_)                                                                \
    do {                                                                                     \
        unsigned char *sb_ = lds + (buf_) * BUF_BYTES;                                       \
        _Pragma("unroll") for (int i = 0; i < W_LD; ++i) *(v4i *)(sb_ + w_lds[i]) = stage_w[i]; \
        _Pragma("unroll") for (int i = 0; i < X_LD; ++i) *(v4i *)(sb_ + x_lds[i]) = stage_x[i]; \
    } while (0)

    // ---- fragment read offsets -------------------------------------------------
    const int fr = lane & 31, fh = lane >> 5;   // row inside a 32-row fragment, K half
    v16i acc[FN][FM];
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[fn][fm][v] = 0;

    // One K tile: prefetch the following tile, run the MFMAs of this one out of
    // LDS buffer (t & 1), park the prefetched tile in the other buffer.
#define MUXQ_K_TILE(t_)                                                                      \
    do {                                                                                     \
        MUXQ_LOAD_TILE(min((t_) + 1, t_all - 1)); /* the last tile re-reads itself, unused */ \
        const unsigned char *base = lds + ((t_) & 1) * BUF_BYTES;                            \
        _Pragma("unroll") for (int kk = 0; kk < BK / 32; ++kk) {                             \
            v4i wf[FN], xf[FM];                                                              \
            _Pragma("unroll") for (int fn = 0; fn < FN; ++fn) {                              \
                int r = wave_n + fn * 32 + fr;                                               \
                wf[fn] = *(const v4i *)(base + r * BK + swizzle<BK>(r, kk * 2 + fh) * 16);   \
            }                                                                                \
            _Pragma("unroll") for (int fm = 0; fm < FM; ++fm) {                              \
                int r = wave_m + fm * 32 + fr;                                               \
                xf[fm] = *(const v4i *)(base + TN * BK + r * BK +                            \
                                        swizzle<BK>(r, kk * 2 + fh) * 16);                   \
            }                                                                                \
            _Pragma("unroll") for (int fn = 0; fn < FN; ++fn)                                \
                _Pragma("unroll") for (int fm = 0; fm < FM; ++fm)                            \
                    acc[fn][fm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[fn], xf[fm],      \
                                                                        acc[fn][fm], 0, 0, 0); \
        }                                                                                    \
        MUXQ_STORE_TILE(((t_) + 1) & 1);                                                     \
        __syncthreads();                                                                     \
    } while (0)

    MUXQ_LOAD_TILE(0);
    MUXQ_STORE_TILE(0);
    __syncthreads();

    if (t_aux > 0) {
        for (int t = 0; t < t_aux; ++t) MUXQ_K_TILE(t);
        // acc now holds acc_aux; Eq. 7 weights it by c = 2^exp - 1.
        const int c = a.c_mult;
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) {
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[fn][fm][v] *= c;
                __builtin_amdgcn_sched_barrier(0);   // one fragment at a time: short live ranges
            }
    }
    for (int t = t_aux; t < t_all; ++t) MUXQ_K_TILE(t);
#undef MUXQ_K_TILE
#undef MUXQ_LOAD_TILE
#undef MUXQ_STORE_TILE

    // ---- epilogue: Eq. 3 dequantisation, fp16 store ----------------------------
    const float sx = a.x_scale[0];
    const float sw0 = a.w_scale[0];
#pragma unroll
    for (int fn = 0; fn < FN; ++fn) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n = n0 + wave_n + fn * 32 + 8 * g + 4 * fh;
            if (n >= a.N) continue;          // N % 8 == 0: a run of 4 is in or out as a whole
            float sc[4], bs[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sc[i] = sx * (a.w_per_channel ? a.w_scale[n + i] : sw0);
                bs[i] = a.bias ? (float)a.bias[n + i] : 0.f;
            }
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) {
                const int m = m0 + wave_m + fm * 32 + fr;
                if (m >= a.M) continue;
                f16x4 out;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float y = sc[i] * (float)acc[fn][fm][4 * g + i];
                    if (a.bias) y = y + bs[i];
                    out[i] = (_Float16)y;
                }
                *(f16x4 *)(a.y + (size_t)m * a.ldy + n) = out;
                if (a.dbg_acc) {
                    v4i raw = {acc[fn][fm][4 * g], acc[fn][fm][4 * g + 1], acc[fn][fm][4 * g + 2],
                               acc[fn][fm][4 * g + 3]};
                    *(v4i *)(a.dbg_acc + (size_t)m * a.N + n) = raw;
                }
                __builtin_amdgcn_sched_barrier(0);   // keep the accumulator reads short-lived
            }
        }
    }
}

template <int TN, int TM, int BK, int WN, int WM>
hipError_t launch_cfg(const GemmArgs &a, hipStream_t s)
{
    TileMap tm;
    tm.tiles_m = (a.M + TM - 1) / TM;
    tm.tiles_n = (a.N + TN - 1) / TN;
    tm.sup_m = min(4, tm.tiles_m);
    tm.sup_n = min(32 / tm.sup_m, tm.tiles_n);
    const int super_m = (tm.tiles_m + tm.sup_m - 1) / tm.sup_m;
    tm.super_n = (tm.tiles_n + tm.sup_n - 1) / tm.sup_n;
    tm.n_super = super_m * tm.super_n;
    const int S = tm.sup_m * tm.sup_n;
    const int grid = ((tm.n_super + 7) / 8) * 8 * S;
    constexpr int lds_bytes = 2 * (TN + TM) * BK;
    auto kern = k_gemm_i8<TN, TM, BK, WN, WM>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WN * WM * 64), lds_bytes, s, a, tm);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmArgs &a, hipStream_t s)
{
    // Largest tile that still gives every CU work; small problems take small tiles.
    const long t256 = (long)((a.M + 255) / 256) * ((a.N + 255) / 256);
    const long t128 = (long)((a.M + 127) / 128) * ((a.N + 127) / 128);
    if (t256 >= 192) return launch_cfg<256, 256, 64, 2, 4>(a, s);
    if (t128 >= 128) return launch_cfg<128, 128, 64, 2, 2>(a, s);
    return launch_cfg<64, 64, 64, 2, 2>(a, s);
}

}  // namespace muxq
