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
// Power.  Under INT8 MFMA load the chip is power-limited, and what the matrix pipes
// draw depends on how much their operands toggle.  Two things keep that down without
// changing any result: the activation codes of the unlisted channels come with a
// zero point (non-negative; the epilogue takes z * cn[n] off the accumulators), and
// the accumulators start at a positive offset instead of 0, so that they do not keep
// changing sign (see kCnBias / kAccBias; the Aux weighting lets the offset pass
// through, the epilogue removes it).  The weights are the first MFMA operand and the
// narrow activation codes the second: the other way round draws more.
//
// Three kernels share that scheme:
//   k_gemm_i8_persist8  256 x 256 tile, 8 waves (2 per SIMD), K step 64, one
//                   persistent workgroup per CU.  Operand tiles go global -> LDS
//                   directly (buffer_load_dwordx4 ... lds, no staging registers)
//                   into a ring of LDS stages, two K steps ahead; fragments are
//                   double-buffered in registers so ds_read_b128 of the next K
//                   sub-step overlaps the MFMAs of the current one; one
//                   workgroup barrier per K step, placed between the two
//                   sub-steps so that it never waits on data.
//   k_gemm_i8_persist4  the same kernel body with a 128 x 128 tile and 4 waves,
//                   two workgroups per CU, for problems with too few 256 x 256
//                   tiles to fill 256 CUs but a long K loop.
//   k_gemm_i8_small register-staged tiles of 128 x 128 or 64 x 64 for short K
//                   loops and small problems.
//
// LDS rows are 64 bytes (one K step); the four 16-byte chunks of a row are
// XOR-swizzled with row bits so that a ds_read_b128 of 32 rows x one chunk is
// spread over all banks without padding (a direct-to-LDS load needs the LDS
// image of a wave to be contiguous, so padding is not an option; the swizzle
// is applied on the global-address side instead).
//
// Workgroup -> tile map.  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2.  Tiles are grouped in super-tiles of sup_m x sup_n tiles
// (<= 32, one per CU of an XCD); workgroup i belongs to XCD i % 8 and the
// workgroups an XCD runs concurrently form one compact super-tile, so its L2
// holds (sup_m + sup_n) operand panels for sup_m * sup_n tiles.
#include "muxq_kernels.h"

#include <atomic>
#include <mutex>

namespace muxq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;   // K step (bytes of one LDS row)

struct TileMap {
    int tiles_m, tiles_n, sup_m, sup_n, super_n, n_super;
};

// 16-byte chunk position of logical chunk `chunk` in LDS row `row`.
template <int SWZ>
__device__ __forceinline__ int swizzle(int row, int chunk)
{
    if constexpr (SWZ == 0)
        return chunk ^ ((row >> 1) & 3);
    else if constexpr (SWZ == 1)
        return chunk ^ ((row >> 2) & 3);
    else if constexpr (SWZ == 2)
        return chunk ^ (row & 3);
    else
        return chunk;
}

__device__ __forceinline__ bool tile_of_workgroup(const TileMap &tm, int &tile_m, int &tile_n)
{
    const int S = tm.sup_m * tm.sup_n;
    const int wg = blockIdx.x;
    const int xcd = wg & 7, j = wg >> 3;
    const int w_in = j % S, st = (j / S) * 8 + xcd;
    if (st >= tm.n_super) return false;
    tile_m = (st / tm.super_n) * tm.sup_m + w_in / tm.sup_n;
    tile_n = (st % tm.super_n) * tm.sup_n + w_in % tm.sup_n;
    return tile_m < tm.tiles_m && tile_n < tm.tiles_n;
}

// acc <- c * acc with c = 2^e - 1, as (acc << e) - acc (two full-rate VALU ops).  The
// accumulators start at an offset B (see kCnBias) that is to come through unscaled:
// c * (acc - B) + B = c * acc - fix with fix = (c - 1) * B.
template <int FN, int FM>
__device__ __forceinline__ void scale_acc(v16i (&acc)[FN][FM], int e, int fix)
{
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
        {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[fn][fm][v] = (int)(((unsigned)acc[fn][fm][v] << e) - (unsigned)acc[fn][fm][v] - (unsigned)fix);
            // one fragment at a time: keeps the number of temporaries small when the
            // accumulators live in the accumulation registers
            __builtin_amdgcn_sched_barrier(0);
        }
}

// The same step when Aux was quantised on a scale of its own (s_aux, the other reading of
// Eq. 5): the Aux accumulators are brought onto Body's scale, acc <- rne(rho * acc) with
// rho = (2^e - 1) s_aux / s_x <= 2^e - 1, and the Body steps then accumulate on top as before.
// Against the sum of Eq. 7 taken after dequantisation this rounds the Aux term to a whole
// unit of s_x s_w[n]: at most half such a unit of error per output.
template <int FN, int FM>
__device__ __forceinline__ void scale_acc_rho(v16i (&acc)[FN][FM], float rho, int bias)
{
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
        {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[fn][fm][v] = (int)__builtin_rintf(rho * (float)(acc[fn][fm][v] - bias)) + bias;
            __builtin_amdgcn_sched_barrier(0);
        }
}

// The same with one activation scale per token: a lane's accumulators of fragment column fm
// belong to one token, whose factor rho[fm] the row quantiser left behind the token scales.
template <int FN, int FM>
__device__ __forceinline__ void scale_acc_rho_tok(v16i (&acc)[FN][FM], const float (&rho)[FM], int bias)
{
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
        {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[fn][fm][v] = (int)__builtin_rintf(rho[fm] * (float)(acc[fn][fm][v] - bias)) + bias;
            __builtin_amdgcn_sched_barrier(0);
        }
}

// Where the per-token factors rho[m] = (2^e - 1) s_aux[m] / s_x[m] of such a launch are:
// the fifth array of x_scale (after s_x[M], qmax / max|Body[m]|, z[m], s_aux[M]).
__device__ __forceinline__ const float *aux_rho_tok(const GemmArgs &a) { return a.x_scale + 4 * (size_t)a.M; }

// (2^e - 1) s_aux / s_x of a launch whose Aux codes have their own scale, else 0.
__device__ __forceinline__ float aux_rho(const GemmArgs &a)
{
    if (!a.aux_own_scale || a.x_per_token) return 0.f;
    const float sx = a.x_scale[0], sa = a.x_scale[2];
    return sx > 0.f ? ((float)((1 << a.exp_shift) - 1) * sa) / sx : 0.f;
}

// Eq. 3: Y = fp16((s_x * s_w[n]) * float(acc) + bias[n]).  Lane layout of the
// 32x32 accumulator: token m = lane % 32, output channels
// n = 8 * (v / 4) + 4 * (lane / 32) + v % 4 for register v of 16, so a lane holds
// runs of 4 channels of ONE token: stored directly, a wave instruction would
// touch 32 rows of Y with 16 bytes each.  Instead each wave transposes its
// fp16 results through a private LDS patch, 32 tokens at a time, and writes
// whole rows of its sub-tile (FN * 64 contiguous bytes per token, 16 B per lane).
// `patch` is this wave's LDS area of 32 * (FN * 64 + 16) bytes; the row padding
// of 16 B spreads the 8-byte writes of the 32 tokens over the banks.
template <int FN, int FM>
__device__ __forceinline__ void epilogue(const GemmArgs &a, const v16i (&acc)[FN][FM], int m_base,
                                         int n_base, int lane, unsigned char *patch, int sub_bias)
{
    constexpr int ROW_BYTES = FN * 64 + 16;
    constexpr int LANES_PER_ROW = FN * 4;              // 16-byte pieces per row
    constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
    const int fr = lane & 31, fh = lane >> 5;
    const bool has_bias = a.bias != nullptr;

#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
        // this lane's token: its own activation scale in the per-token setting
        const int m_tok = a.x_per_token ? min(m_base + fm * 32 + fr, a.M - 1) : 0;
        const float sx = a.x_scale[m_tok];
        // ... and its zero point: z * cn[n] comes off the accumulators (|cn| < 2^23)
        const int negz = a.cn != nullptr ? -a.zero_point[m_tok] : 0;
        // registers -> LDS patch [token][channel]
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int nl = fn * 32 + 8 * g + 4 * fh;
                const int n = n_base + nl;
                const int ns = n < a.N ? n : 0;      // N % 8 == 0: a run of 4 is in or out as a whole
                float sc[4], bs[4] = {0.f, 0.f, 0.f, 0.f};
                // what comes off the accumulator: z * cn[n] and the explicit part of its start value
                int zc[4] = {-sub_bias, -sub_bias, -sub_bias, -sub_bias};
                if (a.cn != nullptr) {
                    const int4 c4 = *(const int4 *)(a.cn + ns);
                    zc[0] += __mul24(c4.x, negz); zc[1] += __mul24(c4.y, negz);
                    zc[2] += __mul24(c4.z, negz); zc[3] += __mul24(c4.w, negz);
                }
                if (a.w_per_channel) {
                    const float4 w4 = *(const float4 *)(a.w_scale + ns);
                    sc[0] = sx * w4.x; sc[1] = sx * w4.y; sc[2] = sx * w4.z; sc[3] = sx * w4.w;
                } else {
                    const float s = sx * a.w_scale[0];
                    sc[0] = sc[1] = sc[2] = sc[3] = s;
                }
                if (has_bias) {
                    const f16x4 b4 = *(const f16x4 *)(a.bias + ns);
                    bs[0] = (float)b4[0]; bs[1] = (float)b4[1]; bs[2] = (float)b4[2]; bs[3] = (float)b4[3];
                }
                f16x4 out;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float y = sc[i] * (float)(acc[fn][fm][4 * g + i] + zc[i]);
                    if (has_bias) y = y + bs[i];
                    out[i] = (_Float16)y;
                    // fused activation: on the fp16 value the layer would have stored
                    if (a.gelu) out[i] = (_Float16)gelu_tanh_f32((float)out[i]);
                }
                *(f16x4 *)(patch + fr * ROW_BYTES + nl * 2) = out;
            }
        // LDS patch -> Y, whole rows
#pragma unroll
        for (int p = 0; p < 32 / ROWS_PER_PASS; ++p) {
            const int row = p * ROWS_PER_PASS + lane / LANES_PER_ROW;
            const int piece = lane % LANES_PER_ROW;
            const v4i v = *(const v4i *)(patch + row * ROW_BYTES + piece * 16);
            const int m = m_base + fm * 32 + row, n = n_base + piece * 8;
            // streaming store: Y is written once and never re-read here, keep it out of
            // the way of the operand panels in L2
            if (m < a.M && n < a.N)
                __builtin_nontemporal_store(v, (v4i *)(a.y + (size_t)m * a.ldy + n));
        }
    }

    if (a.dbg_acc != nullptr) {        // raw accumulators, debugging aid: plain per-lane stores
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n_base + fn * 32 + 8 * g + 4 * fh;
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) {
                    const int m = m_base + fm * 32 + fr;
                    if (n >= a.N || m >= a.M) continue;
                    v4i raw = {acc[fn][fm][4 * g], acc[fn][fm][4 * g + 1], acc[fn][fm][4 * g + 2],
                               acc[fn][fm][4 * g + 3]};
                    if (a.cn != nullptr)
                        raw -= *(const v4i *)(a.cn + n) * a.zero_point[a.x_per_token ? m : 0];
                    raw -= sub_bias;
                    *(v4i *)(a.dbg_acc + (size_t)m * a.N + n) = raw;
                }
            }
    }
}

// Epilogue of the persistent kernel, with a smaller patch: the wave's LDS patch
// holds 32 tokens x 64 channels (two fragments), so a tile's epilogue runs
// FM x FN/2 rounds of { 8 ds_write_b64, 4 ds_read_b128, 4 stores of 8 rows x 128 B }.
// Exactly FM * (FN / 2) * 4 store instructions are issued for a full tile.
// The vector-memory counter completes in issue order, so a vector load issued
// here would have to wait for every operand load still in flight; three forms:
//   EPI_PLAIN   per-tensor weight scale, no bias: the only scale is the launch
//               constant `s_tensor`; no loads at all.
//   EPI_STAGED  per-channel weight scales, a bias and/or per-token activation
//               scales: the wave's constants were fetched straight into `chan`
//               (LDS) by direct-to-LDS loads issued with the tile's first K step
//               (raw values: FN * 32 weight scales, then FN * 32 fp16 bias values,
//               then FM * 32 token scales); again no loads here.
//   EPI_LOADS   the wave loads its constants itself (one batch) and also exports
//               the raw accumulators when asked: the debugging path, which
//               drains the memory queue once per tile.
enum { EPI_PLAIN = 0, EPI_STAGED = 1, EPI_LOADS = 2 };
constexpr int kChanFloats = 128 + 64 + 64 + 128 + 64 + 64;   // per-wave LDS for the tile's constants

// ZC (compile time, PLAIN form only; the other forms test a.cn): the accumulators carry a
// zero-point term z * cn[n] (cn per channel, int32, staged behind the other constants; z
// per launch, or per token, staged as well), which is taken off first -- in integers
// (one 24-bit multiply-add), so the result is the accumulator of Eq. 7 exactly.
// SUB (compile time): the accumulators started at an offset that no zero-point term removes
// (see kAccBias); `sub_bias` comes off.  false: the caller knows it is zero.
// WCH, TOK, BIAS (compile time, STAGED form; -1 = decided at run time from `a`): per-channel
// weight scales, per-token activation scales, a bias.  The common combinations are compiled
// separately: a run-time flag costs a select or an add of zero per output, and this epilogue
// is bound by its vector ALU work (seven operations per output in the general form, four in
// the plain one).
// GELU (compile time): the result goes through the tanh GELU, applied to the fp16 value the
// layer would have stored, and `mx` (FN / 2 entries) collects, per lane, the running maxima of
// the |fp16| values the lane stores (its 8 channels of each half, over its rows).
template <int FN, int FM, int ROW_BYTES, int MODE, bool ZC = false, bool SUB = true, int WCH = -1,
          int TOK = -1, int BIAS = -1, bool GELU = false>
__device__ __forceinline__ void epilogue_patch(const GemmArgs &a, const v16i (&acc)[FN][FM],
                                               int m_base, int n_base, int lane,
                                               unsigned char *patch, float *chan, float sx,
                                               float sw0, float s_tensor, int z_launch, int sub_bias,
                                               uint4 *mx = nullptr)
{
    if (!SUB) sub_bias = 0;
    const bool w_chan = WCH < 0 ? a.w_per_channel != 0 : WCH != 0;
    const bool x_tok = TOK < 0 ? a.x_per_token != 0 : TOK != 0;
    const bool has_bias = BIAS < 0 ? a.bias != nullptr : BIAS != 0;
    static_assert((FN == 4 || FN == 2) && FM == 2, "the constants' layout holds up to 128 channels and 64 tokens per wave");
    constexpr bool PLAIN = MODE == EPI_PLAIN;
    const int fr = lane & 31, fh = lane >> 5;
    _Float16 *const chan_bias = (_Float16 *)(chan + 128);
    float *const chan_tok = chan + 128 + 64;
    int *const chan_zc = (int *)(chan + 256);      // cn of the wave's 128 channels
    int *const chan_ztok = (int *)(chan + 384);    // z of the wave's 64 tokens (per-token setting)
    const bool has_zc = PLAIN ? ZC : a.cn != nullptr;
    if (MODE == EPI_LOADS) {                   // same raw layout as the staged form
        const int n = n_base + 2 * lane;
        float2 sw = make_float2(0.f, 0.f);
        _Float16 b0 = (_Float16)0.f, b1 = (_Float16)0.f;
        if (n < a.N) {                         // N % 8 == 0: a pair is in or out as a whole
            if (a.w_per_channel) sw = *(const float2 *)(a.w_scale + n);
            if (a.bias != nullptr) { b0 = a.bias[n]; b1 = a.bias[n + 1]; }
        }
        float sxm = 0.f;
        if (a.x_per_token && m_base + lane < a.M) sxm = a.x_scale[m_base + lane];
        *(float2 *)(chan + 2 * lane) = sw;
        chan_bias[2 * lane] = b0;
        chan_bias[2 * lane + 1] = b1;
        chan_tok[lane] = sxm;
        int z0 = 0, z1 = 0, zt = 0;
        if (a.cn != nullptr && n < a.N) { z0 = a.cn[n]; z1 = a.cn[n + 1]; }
        if (a.cn != nullptr && a.x_per_token && m_base + lane < a.M) zt = a.zero_point[m_base + lane];
        chan_zc[2 * lane] = z0;
        chan_zc[2 * lane + 1] = z1;
        chan_ztok[lane] = zt;
    }

#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
        int negz = 0;                              // this lane's token
        if (has_zc) negz = -((!PLAIN && x_tok) ? chan_ztok[fm * 32 + fr] : z_launch);
#pragma unroll
        for (int h = 0; h < FN / 2; ++h) {
#pragma unroll
            for (int f2 = 0; f2 < 2; ++f2) {
                // the four corrections of this fragment in one batch of LDS reads: read one
                // by one inside the pinned loop below, each would expose its latency
                v4i zq[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
                if (has_zc) {
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        zq[g] = *(const v4i *)(chan_zc + h * 64 + f2 * 32 + 8 * g + 4 * fh);
                }
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int fn = 2 * h + f2;
                    const int nl = f2 * 32 + 8 * g + 4 * fh;          // channel inside the pair
                    float4 sc = make_float4(s_tensor, s_tensor, s_tensor, s_tensor);
                    float4 bs = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (!PLAIN) {
                        // Eq. 3: one binary32 product of the two scales, whichever granularity
                        float4 w = make_float4(sw0, sw0, sw0, sw0);
                        if (w_chan) w = *(const float4 *)(chan + h * 64 + nl);
                        const float sxx = x_tok ? chan_tok[fm * 32 + fr] : sx;
                        sc = make_float4(sxx * w.x, sxx * w.y, sxx * w.z, sxx * w.w);
                        if (has_bias) {
                            const f16x4 b4 = *(const f16x4 *)(chan_bias + h * 64 + nl);
                            bs = make_float4((float)b4[0], (float)b4[1], (float)b4[2], (float)b4[3]);
                        }
                    }
                    const float scv[4] = {sc.x, sc.y, sc.z, sc.w}, bsv[4] = {bs.x, bs.y, bs.z, bs.w};
                    const v4i z4 = zq[g];
                    f16x4 out;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float y = scv[i] * (float)(__mul24(z4[i], negz) + (acc[fn][fm][4 * g + i] - sub_bias));
                        if (!PLAIN && BIAS != 0) y = y + bsv[i];   // + 0 without a bias: changes no finite value
                        out[i] = (_Float16)y;
                        if (GELU) out[i] = (_Float16)gelu_tanh_f32((float)out[i]);
                    }
                    *(f16x4 *)(patch + fr * ROW_BYTES + nl * 2) = out;
                    __builtin_amdgcn_sched_barrier(0);   // bounds the live temporaries (see scale_acc)
                }
            }
            // patch -> Y: 8 lanes cover the 128 bytes of one token, 8 tokens per instruction
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int row = p * 8 + (lane >> 3), piece = lane & 7;
                const v4i v = *(const v4i *)(patch + row * ROW_BYTES + piece * 16);
                const int m = m_base + fm * 32 + row, n = n_base + h * 64 + piece * 8;
                if (m < a.M && n < a.N) {
                    __builtin_nontemporal_store(v, (v4i *)(a.y + (size_t)m * a.ldy + n));
                    if (GELU) mx[h] = absmax_step(mx[h], __builtin_bit_cast(uint4, v));
                }
            }
        }
    }

    if (MODE == EPI_LOADS && a.dbg_acc != nullptr) {   // raw accumulators, debugging aid: plain per-lane stores
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n_base + fn * 32 + 8 * g + 4 * fh;
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) {
                    const int m = m_base + fm * 32 + fr;
                    if (n >= a.N || m >= a.M) continue;
                    v4i raw = {acc[fn][fm][4 * g], acc[fn][fm][4 * g + 1], acc[fn][fm][4 * g + 2],
                               acc[fn][fm][4 * g + 3]};
                    if (a.cn != nullptr)
                        raw -= *(const v4i *)(a.cn + n) * a.zero_point[a.x_per_token ? m : 0];
                    raw -= sub_bias;
                    *(v4i *)(a.dbg_acc + (size_t)m * a.N + n) = raw;
                }
            }
    }
}

__device__ __forceinline__ int aux_tiles(const GemmArgs &a)
{
    int used = 0;
    if (a.n_outliers != nullptr && a.r_cap > 0) used = max(0, min(a.n_outliers[0], a.r_cap));
    used = __builtin_amdgcn_readfirstlane(used);
    return (used + BK - 1) / BK;
}

// s_waitcnt that only constrains vmcnt (gfx9 encoding: vmcnt[3:0] | expcnt[6:4]
// | lgkmcnt[11:8] | vmcnt[5:4] << 14).
constexpr int waitcnt_vm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }
// ... and additionally waits for every LDS access of this wave (lgkmcnt = 0).
constexpr int waitcnt_vm_lds(int n) { return (n & 15) | (7 << 4) | (0 << 8) | ((n >> 4) << 14); }
constexpr int waitcnt_lds_only() { return waitcnt_vm_lds(63); }

// --------------------------------------------------------------------------
// Persistent form of the 256 x 256 kernel: one workgroup per CU walks a list of
// tiles, and the K steps of all its tiles form ONE continuous stream through
// the LDS ring.  The operand loads of the next tile's first K steps are issued
// during the last K steps of the current tile, so there is no load latency at
// tile boundaries, and the stores of a tile's epilogue drain while the next
// tile is already being computed.  The epilogue's LDS patches lie behind the
// ring, so the ring keeps filling during an epilogue.
//
// The four DMA instructions of a K step are spread over the first eight MFMAs
// (one per two MFMAs) instead of being issued back to back: a burst of 32 DMA
// instructions per CU backs up the texture-address unit, and a wave blocked on
// issuing a load cannot issue its MFMAs either.
//
// Ragged edges clamp the 16-row BLOCK index of an operand load (never the row),
// so every lane offset is a launch constant: rows of the last block beyond M or
// N are read from the padded packed buffer and only feed outputs that are never
// stored.
// --------------------------------------------------------------------------
struct PersistTile {
    int v;            // virtual workgroup index of the tile, >= total when exhausted
    int tile_m, tile_n;
};

__device__ __forceinline__ bool tile_of_virtual(const TileMap &tm, int v, int &tile_m, int &tile_n)
{
    const int S = tm.sup_m * tm.sup_n;
    const int xcd = v & 7, j = v >> 3;
    const int w_in = j % S, st = (j / S) * 8 + xcd;
    if (st >= tm.n_super) return false;
    tile_m = (st / tm.super_n) * tm.sup_m + w_in / tm.sup_n;
    tile_n = (st % tm.super_n) * tm.sup_n + w_in % tm.sup_n;
    return tile_m < tm.tiles_m && tile_n < tm.tiles_n;
}

// First valid tile at or after virtual index v, stepping by the grid size.
__device__ __forceinline__ PersistTile next_tile(const TileMap &tm, int v, int total, int stride)
{
    PersistTile p;
    p.tile_m = p.tile_n = 0;
    while (v < total && !tile_of_virtual(tm, v, p.tile_m, p.tile_n)) v += stride;
    p.v = v;
    return p;
}

// The tile is 2 x NWAVES/2 waves of FN x FM fragments of 32 x 32.  Built as
// NWAVES = 8, FN = 4, FM = 2 (256 x 256, two waves per SIMD, each 128 (n) x 64 (m))
// and NWAVES = 4, FN = 2, FM = 2 (128 x 128, for problems with few tiles).
// OWN (compile time): the launch's Aux codes have a scale of their own (GemmArgs::aux_own_scale),
// 1 with one activation scale per launch, 2 with one per token; forms of their own so that the
// usual kernel's register allocation does not carry the floating-point rescale of the
// accumulators (nor the per-launch form the per-token factors: 109 spilled registers in one kernel).
// GELU (compile time): the fused-activation form (GemmArgs::gelu): every epilogue applies the
// GELU and, with slab_out, the workgroup leaves the column maxima of its tile of Y.
template <int STAGES, int NWAVES, int FN, int FM, int OWN = 0, bool GELU = false>
__device__ __forceinline__ void gemm_persist_body(const GemmArgs &a, const TileMap &tm,
                                                  const int total_virtual)
{
    constexpr int WN = 2, WM = NWAVES / WN, TN = WN * FN * 32, TM = WM * FM * 32, SWZ = 1;
    constexpr int NMFMA = FN * FM;           // MFMAs per wave per K sub-step
    constexpr int NFRAG = FN + FM;           // fragment reads per wave per K sub-step
    constexpr int STAGE_BYTES = (TN + TM) * BK;
    constexpr int RING_BYTES = STAGES * STAGE_BYTES;
    constexpr int DEPTH = STAGES - 1;        // K steps in flight ahead of the one being computed
    constexpr int LH = TN / 16 / NWAVES;     // DMA instructions per wave per K step and operand
    static_assert(TN == TM && TN % (16 * NWAVES) == 0, "the waves share the blocks of both operands evenly");
    constexpr int LOADS = 2 * LH;
    constexpr int DMA_EVERY = NMFMA / LOADS; // one DMA instruction per this many MFMAs
    constexpr int PATCH_ROW = 2 * 64 + 16;   // epilogue patch: 32 tokens x 64 channels fp16 (+ pad)
    constexpr int PATCH_BYTES = 32 * PATCH_ROW;
    // global stores per wave per full tile (with the fused GELU one more: the column maxima)
    constexpr int STORES = FM * (FN / 2) * 4 + (GELU ? 1 : 0);
    static_assert(NMFMA % LOADS == 0 && NFRAG <= NMFMA, "schedule does not fit");
    static_assert((DEPTH - 1) * LOADS + STORES + 8 < 64, "vmcnt has 6 bits");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    typedef __attribute__((address_space(3))) void *lptr_t;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_n = (wave % WN) * (FN * 32), wave_m = (wave / WN) * (FM * 32);
    unsigned char *const patch = lds + RING_BYTES + wave * PATCH_BYTES;
    float *const chan = (float *)(lds + RING_BYTES + NWAVES * PATCH_BYTES) + wave * kChanFloats;

    const int t_aux = aux_tiles(a);
    const int k_tiles = a.k_pad / BK;
    const int stride = (int)gridDim.x;

    PersistTile cur_tile = next_tile(tm, (int)blockIdx.x, total_virtual, stride);
    if (cur_tile.v >= total_virtual) return;
    if (a.wg_ticks != nullptr) {             // measurement aid: when this workgroup started
        if (tid == 0) a.wg_ticks[2 * blockIdx.x] = wall_clock64();
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // keeps the store out of the loop's load accounting
    }
    // launch constants of the epilogue, fetched before any operand load is in flight
    const float sx = a.x_scale[0];
    const float sw0 = a.w_scale[0];
    const float s_tensor = sx * sw0;
    const bool plain = !a.w_per_channel && !a.x_per_token && a.bias == nullptr && a.dbg_acc == nullptr;
    const bool has_zc = a.cn != nullptr;
    const int z_launch = has_zc && !a.x_per_token ? a.zero_point[0] : 0;
    // where the accumulators start (see kCnBias), and what the Aux weighting has to take off
    const int fold_bias = z_launch * a.cn_bias;            // comes off with z * cn[n]
    const int sub_bias = fold_bias != 0 ? 0 : kAccBias;    // comes off by itself (see kAccBias)
    const int acc_bias = fold_bias + sub_bias, acc_fix = ((1 << a.exp_shift) - 2) * acc_bias;
    const float rho = OWN == 1 ? aux_rho(a) : 0.f;
    const bool staged = !plain && a.dbg_acc == nullptr;
    const bool consts = staged || (plain && has_zc);     // the tile's constants come by DMA
    constexpr int CONST_LOADS = 8;           // weight scales (2), bias, token scales, cn (2), token z, token rho: always all eight

    // ---- DMA side -------------------------------------------------------------
    // One buffer_load ... lds instruction moves one 1 KiB block of the packed layout
    // (16 rows x 64 B) into 1 KiB of contiguous LDS: lane l lands at byte 16 l, i.e.
    // row l / 4, physical chunk l % 4, and fetches the logical chunk the swizzle maps
    // there.  The address is resource base + per-lane offset (a launch constant) +
    // a scalar offset (row block and K step), so a load costs one scalar add.
    // The stream of K steps runs DEPTH steps ahead of the compute loop, through the
    // phases { Aux steps, Body steps } of one tile after the other.
    const unsigned lane_off = (unsigned)((lane >> 2) * 64 + swizzle<SWZ>(lane >> 2, lane & 3) * 16);
    const unsigned body_rowblock = (unsigned)k_tiles * 1024u;          // bytes per 16 packed rows
    const unsigned aux_rowblock = (unsigned)(a.r_cap / BK) * 1024u;
    const int nblk_n = (a.N + 15) >> 4, nblk_m = (a.M + 15) >> 4;
    constexpr int RSRC_FLAGS = 0x00020000;   // raw buffer of dwords, offset checked against the size
    // resources of the phase the stream is in (rebuilt at each phase change, which is rare)
    __amdgpu_buffer_rsrc_t r_w, r_x;

    PersistTile dma_tile = cur_tile;
    bool d_aux;                 // phase of the stream
    int d_left;                 // K steps left in the phase
    unsigned d_w[LH], d_x[LH];  // scalar byte offsets of the next step's blocks
#define MUXQ_DMA_PHASE(aux_)                                                                    \
    do {                                                                                        \
        const bool ax_ = (aux_);                                                                \
        const unsigned rb_ = ax_ ? aux_rowblock : body_rowblock;                                \
        _Pragma("unroll") for (int i_ = 0; i_ < LH; ++i_) {                                     \
            d_w[i_] = rb_ * (unsigned)min(dma_tile.tile_n * (TN / 16) + i_ * NWAVES + wave, nblk_n - 1); \
            d_x[i_] = rb_ * (unsigned)min(dma_tile.tile_m * (TM / 16) + i_ * NWAVES + wave, nblk_m - 1); \
        }                                                                                       \
        r_w = __builtin_amdgcn_make_buffer_rsrc((void *)(ax_ ? a.w_aux : a.w_q), 0,             \
                                                (int)((unsigned)nblk_n * rb_), RSRC_FLAGS);     \
        r_x = __builtin_amdgcn_make_buffer_rsrc((void *)(ax_ ? a.aux_q : a.a_q), 0,             \
                                                (int)((unsigned)nblk_m * rb_), RSRC_FLAGS);     \
        d_aux = ax_;                                                                            \
        d_left = ax_ ? t_aux : k_tiles;                                                         \
    } while (0)
    // Rare path, once per phase: Aux -> Body of the same tile, Body -> next tile.
    // After the last step of the last tile the stream keeps re-reading that step
    // into stages nobody reads, so the number of loads in flight stays uniform.
#define MUXQ_DMA_NEXT_PHASE                                                                     \
    do {                                                                                        \
        if (d_aux) {                                                                            \
            MUXQ_DMA_PHASE(false);                                                              \
        } else {                                                                                \
            const PersistTile nx_ = next_tile(tm, dma_tile.v + stride, total_virtual, stride);  \
            if (nx_.v < total_virtual) {                                                        \
                dma_tile = nx_;                                                                 \
                MUXQ_DMA_PHASE(t_aux > 0);                                                      \
            } else {                                                                            \
                _Pragma("unroll") for (int i_ = 0; i_ < LH; ++i_) { d_w[i_] -= 1024u; d_x[i_] -= 1024u; } \
                d_left = 1;                                                                     \
            }                                                                                   \
        }                                                                                       \
    } while (0)
    MUXQ_DMA_PHASE(t_aux > 0);
    int st_dma = 0;                            // byte offset of the stage the next DMA fills
    // DMA instruction j of a step: j even -> weight block j / 2, j odd -> activation block j / 2
#define MUXQ_DMA(j_)                                                                            \
    do {                                                                                        \
        if ((j_) % 2 == 0)                                                                      \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r_w,                      \
                (lptr_t)(lds + st_dma + (((j_) / 2) * NWAVES + wave) * 1024), 16, lane_off, d_w[(j_) / 2], 0, 0); \
        else                                                                                    \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r_x,                      \
                (lptr_t)(lds + st_dma + TN * BK + (((j_) / 2) * NWAVES + wave) * 1024), 16, lane_off, d_x[(j_) / 2], 0, 0); \
    } while (0)
#define MUXQ_DMA_STEP_DONE                                                                      \
    do {                                                                                        \
        _Pragma("unroll") for (int i_ = 0; i_ < LH; ++i_) { d_w[i_] += 1024u; d_x[i_] += 1024u; } \
        --d_left;                                                                               \
        st_dma = st_dma + STAGE_BYTES == RING_BYTES ? 0 : st_dma + STAGE_BYTES;                 \
    } while (0)

    // ---- fragment read addresses (byte offsets inside a stage) --------------------
    const int fr = lane & 31, fh = lane >> 5;
    int w_rd[2], x_rd[2];                      // [kk]
    {
        const int rw = wave_n + fr, rx = wave_m + fr;   // + 32 * f keeps the swizzle bits
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            w_rd[kk] = rw * BK + swizzle<SWZ>(rw, kk * 2 + fh) * 16;
            x_rd[kk] = TN * BK + rx * BK + swizzle<SWZ>(rx, kk * 2 + fh) * 16;
        }
    }
    // fragment read q of a K sub-step: q < FN -> weight fragment q, else activation fragment q - FN
#define MUXQ_RD(wf_, xf_, stage_base_, kk_, q_)                                                 \
    do {                                                                                        \
        if ((q_) < FN) wf_[(q_)] = *(const v4i *)((stage_base_) + w_rd[kk_] + (q_) * 32 * BK);  \
        else xf_[(q_) - FN] = *(const v4i *)((stage_base_) + x_rd[kk_] + ((q_) - FN) * 32 * BK); \
    } while (0)
#define MUXQ_MFMA(q_, wf_, xf_)                                                                 \
    acc[(q_) / FM][(q_) % FM] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf_[(q_) / FM], xf_[(q_) % FM], acc[(q_) / FM][(q_) % FM], 0, 0, 0)
#define MUXQ_PIN __builtin_amdgcn_sched_barrier(0)

    // ---- prologue: DEPTH K steps in flight, step 0 landed, its first fragments read ----
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
#pragma unroll
        for (int j = 0; j < LOADS; ++j) MUXQ_DMA(j);
        MUXQ_DMA_STEP_DONE;
        if (d_left == 0) MUXQ_DMA_NEXT_PHASE;
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm((DEPTH - 1) * LOADS));
    __builtin_amdgcn_s_barrier();
    v4i wfA[FN], xfA[FM], wfB[FN], xfB[FM];
#pragma unroll
    for (int q = 0; q < NFRAG; ++q) MUXQ_RD(wfA, xfA, lds, 0, q);
    __builtin_amdgcn_s_waitcnt(waitcnt_lds_only());

    int st_cur = 0;                // byte offset of the stage being computed
    bool stores_pending = false;   // the previous tile's stores may still be in the vmcnt queue

    // One K step.  First half: MFMAs on the fragments of K sub-step 0; in their shadow
    // the fragment reads of sub-step 1 and this step's DMA instructions, spread evenly
    // (a burst of loads backs up the address unit, and a wave blocked on issuing a load
    // cannot issue its MFMAs either).  The stage the DMA refills was last read in the
    // first half of the previous step, i.e. before the barrier every wave has passed
    // since.  Then the next K step must have landed (this wave's part: everything but
    // the newest DEPTH - 1 steps of DMA, which complete in issue order; everybody's
    // part: the barrier), and the fragment reads of this stage must be complete before
    // another wave may refill it after the barrier.  Second half: sub-step 1, and the
    // first fragments of the next step.
    // Wave priority: the second half of a step runs at a higher priority than the first
    // (which carries the DMA instructions).  Of the two waves of a SIMD the one further
    // along then wins the issue arbitration: 6 % fewer cycles per tile, 2 % less time
    // (the chip is power-limited: most of a cycle gain comes back as a lower clock).
    // Only in the 8-wave form: with two 4-wave workgroups per CU it costs 3-4 %.
    // The first step of a tile (FIRST_ = 1) is written out on its own: only there can
    // the previous tile's stores still sit in the queue, and only there are the tile's
    // epilogue constants fetched (straight into the wave's `chan`: they queue behind the
    // step's operand loads and land K steps before use), so the steady-state step keeps
    // a single wait and no branches.
#define MUXQ_KSTEP(FIRST_)                                                                      \
    do {                                                                                        \
        const unsigned char *const cur_ = lds + st_cur;                                         \
        if (NWAVES == 8) __builtin_amdgcn_s_setprio(0);                                         \
        MUXQ_PIN;                                                                               \
        _Pragma("unroll") for (int q = 0; q < NMFMA; ++q) {                                     \
            MUXQ_MFMA(q, wfA, xfA);                                                             \
            if (q < NFRAG) MUXQ_RD(wfB, xfB, cur_, 1, q);                                       \
            if (q % DMA_EVERY == 0) MUXQ_DMA(q / DMA_EVERY);                                    \
            if (q == NMFMA - 1) MUXQ_DMA_STEP_DONE;                                             \
            MUXQ_PIN;                                                                           \
        }                                                                                       \
        if (FIRST_) {                                                                           \
            if (consts) {                                                                       \
                MUXQ_CONST_LOADS;                                                               \
                if (stores_pending)                                                             \
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds((DEPTH - 1) * LOADS + STORES + CONST_LOADS)); \
                else                                                                            \
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds((DEPTH - 1) * LOADS + CONST_LOADS)); \
            } else if (stores_pending) {                                                        \
                __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds((DEPTH - 1) * LOADS + STORES));       \
            } else {                                                                            \
                __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds((DEPTH - 1) * LOADS));                \
            }                                                                                   \
            stores_pending = false;                                                             \
        } else {                                                                                \
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds((DEPTH - 1) * LOADS));                    \
        }                                                                                       \
        __builtin_amdgcn_s_barrier();                                                           \
        if (NWAVES == 8) __builtin_amdgcn_s_setprio(1);                                         \
        MUXQ_PIN;                                                                               \
        const int st_next_ = st_cur + STAGE_BYTES == RING_BYTES ? 0 : st_cur + STAGE_BYTES;     \
        const unsigned char *const nxt_ = lds + st_next_;                                       \
        _Pragma("unroll") for (int q = 0; q < NMFMA; ++q) {                                     \
            MUXQ_MFMA(q, wfB, xfB);                                                             \
            if (q < NFRAG) MUXQ_RD(wfA, xfA, nxt_, 0, q);                                       \
            if (q == NMFMA - 2 && d_left == 0) MUXQ_DMA_NEXT_PHASE;                             \
            if (q == NMFMA - 1) st_cur = st_next_;                                              \
            MUXQ_PIN;                                                                           \
        }                                                                                       \
        __builtin_amdgcn_s_waitcnt(waitcnt_lds_only());                                         \
    } while (0)
    // The constants' resources are built on the spot (a feature that is off gets a
    // zero-sized resource, whose loads return zeros without touching memory).  Whole
    // offsets go into the per-lane operand: that is the part the buffer range check
    // covers, so channels past N and tokens past M read zeros.
#define MUXQ_CONST_LOADS                                                                        \
    do {                                                                                        \
        const __amdgpu_buffer_rsrc_t r_ws_ = __builtin_amdgcn_make_buffer_rsrc(                 \
            (void *)a.w_scale, 0, a.w_per_channel ? a.N * 4 : 0, RSRC_FLAGS);                   \
        const __amdgpu_buffer_rsrc_t r_bias_ = __builtin_amdgcn_make_buffer_rsrc(               \
            a.bias != nullptr ? (void *)a.bias : (void *)a.w_scale, 0,                          \
            a.bias != nullptr ? a.N * 2 : 0, RSRC_FLAGS);                                       \
        const __amdgpu_buffer_rsrc_t r_xs_ = __builtin_amdgcn_make_buffer_rsrc(                 \
            (void *)a.x_scale, 0, a.x_per_token ? a.M * 4 : 0, RSRC_FLAGS);                     \
        const __amdgpu_buffer_rsrc_t r_zc_ = __builtin_amdgcn_make_buffer_rsrc(                 \
            has_zc ? (void *)a.cn : (void *)a.w_scale, 0, has_zc ? a.N * 4 : 0, RSRC_FLAGS);    \
        const bool ztok_ = has_zc && a.x_per_token;                                             \
        const __amdgpu_buffer_rsrc_t r_zt_ = __builtin_amdgcn_make_buffer_rsrc(                 \
            ztok_ ? (void *)a.zero_point : (void *)a.w_scale, 0, ztok_ ? a.M * 4 : 0, RSRC_FLAGS); \
        const int n_w_ = cur_tile.tile_n * TN + wave_n, m_w_ = cur_tile.tile_m * TM + wave_m;   \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_ws_, (lptr_t)chan, 4, (n_w_ + lane) * 4, 0, 0, 0); \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_ws_, (lptr_t)(chan + 64), 4, (n_w_ + 64 + lane) * 4, 0, 0, 0); \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_bias_, (lptr_t)(chan + 128), 4, (n_w_ + 2 * lane) * 2, 0, 0, 0); \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_xs_, (lptr_t)(chan + 192), 4, (m_w_ + lane) * 4, 0, 0, 0); \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_zc_, (lptr_t)(chan + 256), 4, (n_w_ + lane) * 4, 0, 0, 0); \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_zc_, (lptr_t)(chan + 320), 4, (n_w_ + 64 + lane) * 4, 0, 0, 0); \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_zt_, (lptr_t)(chan + 384), 4, (m_w_ + lane) * 4, 0, 0, 0); \
        const bool rtok_ = OWN == 2;                                                            \
        const __amdgpu_buffer_rsrc_t r_rho_ = __builtin_amdgcn_make_buffer_rsrc(                \
            rtok_ ? (void *)aux_rho_tok(a) : (void *)a.w_scale, 0, rtok_ ? a.M * 4 : 0, RSRC_FLAGS); \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_rho_, (lptr_t)(chan + 448), 4, (m_w_ + lane) * 4, 0, 0, 0); \
    } while (0)

#define MUXQ_EPI_STAGED(SUB_, WCH_, TOK_, BIAS_)                                                  \
    epilogue_patch<FN, FM, PATCH_ROW, EPI_STAGED, false, SUB_, WCH_, TOK_, BIAS_>(                  \
        a, acc, m_base, n_base, lane, patch, chan, sx, sw0, s_tensor, z_launch, sub_bias)
#define MUXQ_EPI_GELU(MODE_, ZC_, SUB_, WCH_, TOK_, BIAS_)                                        \
    epilogue_patch<FN, FM, PATCH_ROW, MODE_, ZC_, SUB_, WCH_, TOK_, BIAS_, true>(                   \
        a, acc, m_base, n_base, lane, patch, chan, sx, sw0, s_tensor, z_launch, sub_bias, mxh)
    // fused-GELU form: per-wave then per-workgroup column maxima of the tile, behind the
    // waves' epilogue constants in LDS: [WM][TN] fp16 magnitudes
    unsigned short *const wg_colmax =
        (unsigned short *)(lds + RING_BYTES + NWAVES * PATCH_BYTES + NWAVES * kChanFloats * 4);

    const int t_all = t_aux + k_tiles;
    while (cur_tile.v < total_virtual) {
        v16i acc[FN][FM];
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int fm = 0; fm < FM; ++fm)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[fn][fm][v] = acc_bias;

        // The Aux steps, then (after weighting the Aux accumulators by c = 2^exp - 1)
        // the Body steps.
        MUXQ_KSTEP(1);
#pragma unroll 1
        for (int t = 1; t < t_all; ++t) {
            if (t == t_aux) {                                    // acc_aux -> c * acc_aux
                if constexpr (OWN == 2) {
                    // one factor per token: staged with the tile's constants (issued with the
                    // first K step, so everything older has to land first), or fetched here by
                    // the form that loads its constants itself
                    float rho_t[FM];
                    const float *rho_g = aux_rho_tok(a);
                    if (!consts) {
#pragma unroll
                        for (int fm = 0; fm < FM; ++fm)
                            rho_t[fm] = rho_g[min(cur_tile.tile_m * TM + wave_m + fm * 32 + (lane & 31), a.M - 1)];
                    }
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds(0));
                    asm volatile("" ::: "memory");       // the reads below stay behind the wait
                    if (consts) {
#pragma unroll
                        for (int fm = 0; fm < FM; ++fm) rho_t[fm] = chan[448 + fm * 32 + (lane & 31)];
                    }
                    scale_acc_rho_tok<FN, FM>(acc, rho_t, acc_bias);
                } else if constexpr (OWN == 1) scale_acc_rho<FN, FM>(acc, rho, acc_bias);
                else scale_acc<FN, FM>(acc, a.exp_shift, acc_fix);
            }
            MUXQ_KSTEP(0);
        }

        // ---- epilogue of this tile; the ring keeps its loads in flight meanwhile ----
        const int m_base = cur_tile.tile_m * TM + wave_m, n_base = cur_tile.tile_n * TN + wave_n;
        const bool full = cur_tile.tile_m * TM + TM <= a.M && cur_tile.tile_n * TN + TN <= a.N;
        // a one-step tile has not yet waited past its constants' loads
        if (consts && t_all == 1) __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        if constexpr (GELU) {
            uint4 mxh[FN / 2];
#pragma unroll
            for (int h = 0; h < FN / 2; ++h) mxh[h] = make_uint4(0, 0, 0, 0);
            if (plain && has_zc && sub_bias == 0) MUXQ_EPI_GELU(EPI_PLAIN, true, false, -1, -1, -1);
            else if (plain && has_zc) MUXQ_EPI_GELU(EPI_PLAIN, true, true, -1, -1, -1);
            else if (plain) MUXQ_EPI_GELU(EPI_PLAIN, false, true, -1, -1, -1);
            else if (staged && !a.x_per_token && !a.w_per_channel && sub_bias == 0)
                MUXQ_EPI_GELU(EPI_STAGED, false, false, 0, 0, 1);      // the usual c_fc: a bias, one scale each
            else if (staged) MUXQ_EPI_GELU(EPI_STAGED, false, true, -1, -1, -1);
            else MUXQ_EPI_GELU(EPI_LOADS, false, true, -1, -1, -1);
            if (a.slab_out != nullptr) {
                // A lane holds the maxima of its 8 channels of each half over the rows it stored;
                // the 8 lane groups of a wave hold different rows: fold them through the wave's
                // patch (a wave's LDS operations execute in order), then the WM waves that share
                // the channels through wg_colmax, and every wave stores TN / NWAVES channels.
#pragma unroll
                for (int h = 0; h < FN / 2; ++h) {
                    // (lanes exchange data through LDS here: the fences keep the compiler from
                    // moving one lane's accesses across the other lanes' -- to a single lane
                    // the addresses it reads and the one it writes look unrelated)
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    *(uint4 *)(patch + lane * 16) = mxh[h];
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    if (lane < 8) {
                        uint4 m = make_uint4(0, 0, 0, 0);
#pragma unroll
                        for (int g = 0; g < 8; ++g) m = absmax_step(m, *(const uint4 *)(patch + (g * 8 + lane) * 16));
                        *(uint4 *)(wg_colmax + (wave / WN) * TN + wave_n + h * 64 + lane * 8) = m;
                    }
                }
                __builtin_amdgcn_s_waitcnt(waitcnt_lds_only());
                __builtin_amdgcn_s_barrier();
                constexpr int CH_PER_WAVE = TN / NWAVES;          // 32 channels, lanes 0..3
                const int c0 = wave * CH_PER_WAVE + lane * 8;
                const int n = cur_tile.tile_n * TN + c0;
                // (in a full tile every wave issues this store: the wait counts rely on it)
                if (lane < CH_PER_WAVE / 8 && n < a.slab_ld) {
                    uint4 m = make_uint4(0, 0, 0, 0);
#pragma unroll
                    for (int wm = 0; wm < WM; ++wm) m = absmax_step(m, *(const uint4 *)(wg_colmax + wm * TN + c0));
                    *(uint4 *)(a.slab_out + (size_t)cur_tile.tile_m * a.slab_ld + n) = m;
                }
            }
        } else
        if (plain && has_zc && sub_bias == 0) {
            epilogue_patch<FN, FM, PATCH_ROW, EPI_PLAIN, true, false>(a, acc, m_base, n_base, lane, patch, chan, sx, sw0, s_tensor, z_launch, 0);
        } else if (plain && has_zc) {
            epilogue_patch<FN, FM, PATCH_ROW, EPI_PLAIN, true>(a, acc, m_base, n_base, lane, patch, chan, sx, sw0, s_tensor, z_launch, sub_bias);
        } else if (plain) {
            epilogue_patch<FN, FM, PATCH_ROW, EPI_PLAIN>(a, acc, m_base, n_base, lane, patch, chan, sx, sw0, s_tensor, z_launch, sub_bias);
        } else if (staged && !a.x_per_token && sub_bias == 0) {
            // one activation scale, the accumulators' offset folded away: per-channel weight
            // scales with or without a bias, or a bias alone
            if (!a.w_per_channel) MUXQ_EPI_STAGED(false, 0, 0, 1);
            else if (a.bias != nullptr) MUXQ_EPI_STAGED(false, 1, 0, 1);
            else MUXQ_EPI_STAGED(false, 1, 0, 0);
        } else if (staged && !a.x_per_token) {
            // the same with the offset taken off here (no zero point: the naive pipeline)
            if (!a.w_per_channel) MUXQ_EPI_STAGED(true, 0, 0, 1);
            else if (a.bias != nullptr) MUXQ_EPI_STAGED(true, 1, 0, 1);
            else MUXQ_EPI_STAGED(true, 1, 0, 0);
        } else if (staged && a.w_per_channel && a.x_per_token) {
            // the per-vector setting
            if (a.bias != nullptr) MUXQ_EPI_STAGED(true, 1, 1, 1);
            else MUXQ_EPI_STAGED(true, 1, 1, 0);
        } else if (staged) {
            epilogue_patch<FN, FM, PATCH_ROW, EPI_STAGED>(a, acc, m_base, n_base, lane, patch, chan, sx, sw0, s_tensor, z_launch, sub_bias);
        } else {
            epilogue_patch<FN, FM, PATCH_ROW, EPI_LOADS>(a, acc, m_base, n_base, lane, patch, chan, sx, sw0, s_tensor, z_launch, sub_bias);
        }
        if ((plain || staged) && full && (!GELU || a.slab_out != nullptr)) {
            stores_pending = true;           // exactly STORES stores and no loads were issued
        } else {
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // unknown number of vector-memory operations: drain
        }
        cur_tile = next_tile(tm, cur_tile.v + stride, total_virtual, stride);
    }
    // Drain the unused tail loads before the workgroup's LDS is released.
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lds(0));
    if (a.wg_ticks != nullptr && tid == 0) a.wg_ticks[2 * blockIdx.x + 1] = wall_clock64();
#undef MUXQ_KSTEP
#undef MUXQ_CONST_LOADS
#undef MUXQ_DMA_PHASE
#undef MUXQ_DMA_NEXT_PHASE
#undef MUXQ_DMA
#undef MUXQ_DMA_STEP_DONE
#undef MUXQ_RD
#undef MUXQ_MFMA
#undef MUXQ_PIN
#undef MUXQ_EPI_STAGED
#undef MUXQ_EPI_GELU
}

template <int STAGES, int OWN = 0, bool GELU = false>
__global__ __launch_bounds__(512) void k_gemm_i8_persist8(const GemmArgs a, const TileMap tm,
                                                          const int total_virtual)
{
    gemm_persist_body<STAGES, 8, 4, 2, OWN, GELU>(a, tm, total_virtual);
}

// 128 x 128 tiles, 4 waves of 64 x 64, a deeper ring: for problems with too few
// 256 x 256 tiles to fill the chip, where the load latency of a short K loop
// is what has to be hidden.
template <int STAGES, int OWN = 0, bool GELU = false>
__global__ __launch_bounds__(256) void k_gemm_i8_persist4(const GemmArgs a, const TileMap tm,
                                                          const int total_virtual)
{
    gemm_persist_body<STAGES, 4, 2, 2, OWN, GELU>(a, tm, total_virtual);
}

// --------------------------------------------------------------------------
// Small tiles (TN x TM in {128 x 128, 64 x 64}), 4 waves, register staging.
// --------------------------------------------------------------------------
template <int TN, int TM>
__global__ __launch_bounds__(256) void k_gemm_i8_small(const GemmArgs a, const TileMap tm)
{
    constexpr int WN = 2, WM = 2, NT = 256, CH = BK / 16, SWZ = 1;
    constexpr int FN = TN / WN / 32, FM = TM / WM / 32;
    constexpr int ROWS_PER_PASS = NT / CH;
    constexpr int W_LD = TN / ROWS_PER_PASS, X_LD = TM / ROWS_PER_PASS;
    constexpr int BUF_BYTES = (TN + TM) * BK;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF_BYTES];

    int tile_m, tile_n;
    if (!tile_of_workgroup(tm, tile_m, tile_n)) return;
    const int m0 = tile_m * TM, n0 = tile_n * TN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_n = (wave % WN) * (TN / WN), wave_m = (wave / WN) * (TM / WM);
    const int t_aux = aux_tiles(a);
    const int t_all = t_aux + a.k_pad / BK;
    // where the accumulators start (see kCnBias), and what the Aux weighting has to take off
    const int fold_bias = (a.cn != nullptr && !a.x_per_token) ? a.zero_point[0] * a.cn_bias : 0;
    const int sub_bias = fold_bias != 0 ? 0 : kAccBias;    // comes off by itself (see kAccBias)
    const int acc_bias = fold_bias + sub_bias, acc_fix = ((1 << a.exp_shift) - 2) * acc_bias;
    const float rho = aux_rho(a);

    const int ld_chunk = tid % CH, ld_row = tid / CH;
    int w_row[W_LD], x_row[X_LD], w_lds[W_LD], x_lds[X_LD];
#pragma unroll
    for (int i = 0; i < W_LD; ++i) {
        int r = ld_row + i * ROWS_PER_PASS;
        w_row[i] = min(n0 + r, a.N - 1);
        w_lds[i] = r * BK + swizzle<SWZ>(r, ld_chunk) * 16;
    }
#pragma unroll
    for (int i = 0; i < X_LD; ++i) {
        int r = ld_row + i * ROWS_PER_PASS;
        x_row[i] = min(m0 + r, a.M - 1);
        x_lds[i] = TN * BK + r * BK + swizzle<SWZ>(r, ld_chunk) * 16;
    }
    v4i stage_w[W_LD], stage_x[X_LD];
#define MUXQ_LOAD_TILE(t_)                                                                   \
    do {                                                                                     \
        const int tt_ = (t_);                                                                \
        const bool aux_ = tt_ < t_aux;                                                       \
        const int8_t *wp_ = aux_ ? a.w_aux : a.w_q;                                          \
        const int8_t *xp_ = aux_ ? a.aux_q : a.a_q;                                          \
        const size_t rb_ = (size_t)((aux_ ? a.r_cap : a.k_pad) / BK) * 1024; /* 16 packed rows */ \
        const size_t k0_ = (size_t)(aux_ ? tt_ : tt_ - t_aux) * 1024 + ld_chunk * 16;        \
        _Pragma("unroll") for (int i = 0; i < W_LD; ++i)                                     \
            stage_w[i] = *(const v4i *)(wp_ + (size_t)(w_row[i] >> 4) * rb_ +                \
                                        (w_row[i] & 15) * 64 + k0_);                         \
        _Pragma("unroll") for (int i = 0; i < X_LD; ++i)                                     \
            stage_x[i] = *(const v4i *)(xp_ + (size_t)(x_row[i] >> 4) * rb_ +                \
                                        (x_row[i] & 15) * 64 + k0_);                         \
    } while (0)
#define MUXQ_STORE_TILE(buf_)                                                                \
    do {                                                                                     \
        unsigned char *sb_ = lds + (buf_) * BUF_BYTES;                                       \
        _Pragma("unroll") for (int i = 0; i < W_LD; ++i) *(v4i *)(sb_ + w_lds[i]) = stage_w[i]; \
        _Pragma("unroll") for (int i = 0; i < X_LD; ++i) *(v4i *)(sb_ + x_lds[i]) = stage_x[i]; \
    } while (0)

    const int fr = lane & 31, fh = lane >> 5;
    v16i acc[FN][FM];
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[fn][fm][v] = acc_bias;

    MUXQ_LOAD_TILE(0);
    MUXQ_STORE_TILE(0);
    __syncthreads();
    for (int t = 0; t < t_all; ++t) {
        if (t == t_aux && t_aux > 0) {
            if (a.aux_own_scale && a.x_per_token) {
                float rho_t[FM];
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
                    rho_t[fm] = aux_rho_tok(a)[min(m0 + wave_m + fm * 32 + (lane & 31), a.M - 1)];
                scale_acc_rho_tok<FN, FM>(acc, rho_t, acc_bias);
            } else if (a.aux_own_scale) scale_acc_rho<FN, FM>(acc, rho, acc_bias);
            else scale_acc<FN, FM>(acc, a.exp_shift, acc_fix);
        }
        MUXQ_LOAD_TILE(min(t + 1, t_all - 1));   // the last tile re-reads itself, unused
        __builtin_amdgcn_sched_barrier(0);       // keep the prefetch ahead of the MFMAs
        const unsigned char *base = lds + (t & 1) * BUF_BYTES;
#pragma unroll
        for (int kk = 0; kk < BK / 32; ++kk) {
            v4i wf[FN], xf[FM];
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
                int r = wave_n + fn * 32 + fr;
                wf[fn] = *(const v4i *)(base + r * BK + swizzle<SWZ>(r, kk * 2 + fh) * 16);
            }
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) {
                int r = wave_m + fm * 32 + fr;
                xf[fm] = *(const v4i *)(base + TN * BK + r * BK + swizzle<SWZ>(r, kk * 2 + fh) * 16);
            }
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
                    acc[fn][fm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[fn], xf[fm],
                                                                        acc[fn][fm], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        MUXQ_STORE_TILE((t + 1) & 1);
        __syncthreads();
    }
#undef MUXQ_LOAD_TILE
#undef MUXQ_STORE_TILE
    // (the loop ends on a barrier: every wave is done with the operand tiles)
    static_assert(4 * 32 * (FN * 64 + 16) <= 2 * BUF_BYTES, "epilogue patch does not fit");
    epilogue<FN, FM>(a, acc, m0 + wave_m, n0 + wave_n, lane, lds + wave * (32 * (FN * 64 + 16)), sub_bias);
}

// --------------------------------------------------------------------------
// The same tiles for problems with no more tiles than CUs.  Those are bound by memory round
// trips, not by bytes or MFMAs (a kernel starts with cold caches, and a load that something
// waits for costs 0.5-2 us): the operand loads of CS K steps are issued together and wait in
// registers while the previous CS steps are computed out of LDS, so the loop waits once per CS
// steps instead of once per step.  It costs registers and LDS (two workgroups per CU), which
// is why problems with several workgroups per CU keep the kernel above.
// --------------------------------------------------------------------------
template <int TN, int TM, int CS>
__global__ __launch_bounds__(256) void k_gemm_i8_small_deep(const GemmArgs a, const TileMap tm)
{
    constexpr int WN = 2, WM = 2, NT = 256, CH = BK / 16, SWZ = 1;
    constexpr int FN = TN / WN / 32, FM = TM / WM / 32;
    constexpr int ROWS_PER_PASS = NT / CH;
    constexpr int W_LD = TN / ROWS_PER_PASS, X_LD = TM / ROWS_PER_PASS;
    constexpr int STEP_BYTES = (TN + TM) * BK;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];     // CS * STEP_BYTES

    int tile_m, tile_n;
    if (!tile_of_workgroup(tm, tile_m, tile_n)) return;
    const int m0 = tile_m * TM, n0 = tile_n * TN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_n = (wave % WN) * (TN / WN), wave_m = (wave / WN) * (TM / WM);
    const int t_aux = aux_tiles(a);
    const int t_all = t_aux + a.k_pad / BK;
    const int n_chunks = (t_all + CS - 1) / CS;
    // where the accumulators start (see kCnBias), and what the Aux weighting has to take off
    const int fold_bias = (a.cn != nullptr && !a.x_per_token) ? a.zero_point[0] * a.cn_bias : 0;
    const int sub_bias = fold_bias != 0 ? 0 : kAccBias;    // comes off by itself (see kAccBias)
    const int acc_bias = fold_bias + sub_bias, acc_fix = ((1 << a.exp_shift) - 2) * acc_bias;
    const float rho = aux_rho(a);

    const int ld_chunk = tid % CH, ld_row = tid / CH;
    int w_row[W_LD], x_row[X_LD], w_lds[W_LD], x_lds[X_LD];
#pragma unroll
    for (int i = 0; i < W_LD; ++i) {
        int r = ld_row + i * ROWS_PER_PASS;
        w_row[i] = min(n0 + r, a.N - 1);
        w_lds[i] = r * BK + swizzle<SWZ>(r, ld_chunk) * 16;
    }
#pragma unroll
    for (int i = 0; i < X_LD; ++i) {
        int r = ld_row + i * ROWS_PER_PASS;
        x_row[i] = min(m0 + r, a.M - 1);
        x_lds[i] = TN * BK + r * BK + swizzle<SWZ>(r, ld_chunk) * 16;
    }
    v4i stage_w[CS][W_LD], stage_x[CS][X_LD];
    // the K steps [c * CS, c * CS + CS) of the tile (Aux steps first; past the end the last
    // step is read again, unused) -> registers
    auto load_chunk = [&](int c) {
#pragma unroll
        for (int sl = 0; sl < CS; ++sl) {
            const int tt = min(c * CS + sl, t_all - 1);
            const bool aux = tt < t_aux;
            const int8_t *wp = aux ? a.w_aux : a.w_q;
            const int8_t *xp = aux ? a.aux_q : a.a_q;
            const size_t rb = (size_t)((aux ? a.r_cap : a.k_pad) / BK) * 1024;   // 16 packed rows
            const size_t k0 = (size_t)(aux ? tt : tt - t_aux) * 1024 + ld_chunk * 16;
#pragma unroll
            for (int i = 0; i < W_LD; ++i)
                stage_w[sl][i] = *(const v4i *)(wp + (size_t)(w_row[i] >> 4) * rb + (w_row[i] & 15) * 64 + k0);
#pragma unroll
            for (int i = 0; i < X_LD; ++i)
                stage_x[sl][i] = *(const v4i *)(xp + (size_t)(x_row[i] >> 4) * rb + (x_row[i] & 15) * 64 + k0);
        }
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int sl = 0; sl < CS; ++sl) {
            unsigned char *sb = lds + sl * STEP_BYTES;
#pragma unroll
            for (int i = 0; i < W_LD; ++i) *(v4i *)(sb + w_lds[i]) = stage_w[sl][i];
#pragma unroll
            for (int i = 0; i < X_LD; ++i) *(v4i *)(sb + x_lds[i]) = stage_x[sl][i];
        }
    };

    const int fr = lane & 31, fh = lane >> 5;
    v16i acc[FN][FM];
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[fn][fm][v] = acc_bias;

    load_chunk(0);
    store_chunk();
    __syncthreads();
    for (int c = 0; c < n_chunks; ++c) {
        const bool more = c + 1 < n_chunks;
        if (more) load_chunk(c + 1);
        __builtin_amdgcn_sched_barrier(0);       // keep the prefetch ahead of the MFMAs
#pragma unroll
        for (int sl = 0; sl < CS; ++sl) {
            const int t = c * CS + sl;
            if (t >= t_all) break;
            if (t == t_aux && t_aux > 0) {
                if (a.aux_own_scale && a.x_per_token) {
                    float rho_t[FM];
#pragma unroll
                    for (int fm = 0; fm < FM; ++fm)
                        rho_t[fm] = aux_rho_tok(a)[min(m0 + wave_m + fm * 32 + (lane & 31), a.M - 1)];
                    scale_acc_rho_tok<FN, FM>(acc, rho_t, acc_bias);
                } else if (a.aux_own_scale) scale_acc_rho<FN, FM>(acc, rho, acc_bias);
                else scale_acc<FN, FM>(acc, a.exp_shift, acc_fix);
            }
            const unsigned char *base = lds + sl * STEP_BYTES;
#pragma unroll
            for (int kk = 0; kk < BK / 32; ++kk) {
                v4i wf[FN], xf[FM];
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) {
                    int r = wave_n + fn * 32 + fr;
                    wf[fn] = *(const v4i *)(base + r * BK + swizzle<SWZ>(r, kk * 2 + fh) * 16);
                }
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) {
                    int r = wave_m + fm * 32 + fr;
                    xf[fm] = *(const v4i *)(base + TN * BK + r * BK + swizzle<SWZ>(r, kk * 2 + fh) * 16);
                }
#pragma unroll
                for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                    for (int fm = 0; fm < FM; ++fm)
                        acc[fn][fm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[fn], xf[fm],
                                                                            acc[fn][fm], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();                         // every wave is done with the tiles in LDS
        if (more) {
            store_chunk();
            __syncthreads();
        }
    }
    // (the loop ends on a barrier: every wave is done with the operand tiles)
    static_assert(4 * 32 * (FN * 64 + 16) <= CS * STEP_BYTES, "epilogue patch does not fit");
    epilogue<FN, FM>(a, acc, m0 + wave_m, n0 + wave_n, lane, lds + wave * (32 * (FN * 64 + 16)), sub_bias);
}

TileMap make_tile_map(const GemmArgs &a, int TN, int TM, int &grid)
{
    TileMap tm;
    tm.tiles_m = (a.M + TM - 1) / TM;
    tm.tiles_n = (a.N + TN - 1) / TN;
    tm.sup_m = min(4, tm.tiles_m);
    tm.sup_n = min(32 / tm.sup_m, tm.tiles_n);
    const int super_m = (tm.tiles_m + tm.sup_m - 1) / tm.sup_m;
    tm.super_n = (tm.tiles_n + tm.sup_n - 1) / tm.sup_n;
    tm.n_super = super_m * tm.super_n;
    grid = ((tm.n_super + 7) / 8) * 8 * tm.sup_m * tm.sup_n;
    return tm;
}

// LDS bytes of a persistent kernel: the operand ring, the waves' epilogue patches and constants.
template <int STAGES, int NWAVES>
constexpr int persist_lds_bytes()
{
    constexpr int TILE = NWAVES == 8 ? 256 : 128;
    return STAGES * 2 * TILE * BK + NWAVES * (32 * (2 * 64 + 16) + kChanFloats * 4) +
           (NWAVES / 2) * TILE * 2;          // + the fused-GELU form's column maxima [WM][TN] fp16
}

// K steps whose loads a workgroup of k_gemm_i8_small_deep issues together (64 staging registers,
// 64 KiB of LDS).
constexpr int kDeepSteps = 8;

// What the launcher needs to know about a device, found once per device (gemm_prepare_device).
constexpr int kMaxDevices = 64;
std::atomic<int> g_device_cus[kMaxDevices];      // 0 = not prepared yet
std::mutex g_prepare_mutex;

hipError_t prepare_current_device(int dev)
{
    std::lock_guard<std::mutex> lock(g_prepare_mutex);
    if (g_device_cus[dev].load(std::memory_order_acquire) != 0) return hipSuccess;
    hipError_t e = hipFuncSetAttribute((const void *)k_gemm_i8_persist8<3>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, persist_lds_bytes<3, 8>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)k_gemm_i8_persist4<3>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, persist_lds_bytes<3, 4>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)k_gemm_i8_persist8<3, 1>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, persist_lds_bytes<3, 8>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)k_gemm_i8_persist4<3, 1>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, persist_lds_bytes<3, 4>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)k_gemm_i8_persist8<3, 2>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, persist_lds_bytes<3, 8>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)k_gemm_i8_persist4<3, 2>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, persist_lds_bytes<3, 4>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)k_gemm_i8_persist8<3, 0, true>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, persist_lds_bytes<3, 8>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)k_gemm_i8_persist4<3, 0, true>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, persist_lds_bytes<3, 4>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)k_gemm_i8_small_deep<64, 64, kDeepSteps>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, kDeepSteps * 128 * BK);
    if (e != hipSuccess) return e;
    int cus = 0;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    int n_cu = cus > 0 ? cus / 8 * 8 : 8;   // a multiple of the 8 XCDs keeps workgroup i on XCD i % 8
    if (n_cu < 8) n_cu = 8;
    g_device_cus[dev].store(n_cu, std::memory_order_release);
    return hipSuccess;
}

// CU count (rounded down to a multiple of 8) of the current device, preparing it on first use.
hipError_t current_device_cus(int &n_cu)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    n_cu = g_device_cus[dev].load(std::memory_order_acquire);
    if (n_cu != 0) return hipSuccess;
    if ((e = prepare_current_device(dev)) != hipSuccess) return e;
    n_cu = g_device_cus[dev].load(std::memory_order_acquire);
    return hipSuccess;
}

template <int STAGES, int NWAVES>
hipError_t launch_persist(const GemmArgs &a, hipStream_t s)
{
    static_assert(STAGES == 3, "gemm_prepare_device sets the LDS attribute of the 3-stage forms");
    static_assert(NWAVES == 8 || NWAVES == 4, "built forms");
    constexpr int TILE = NWAVES == 8 ? 256 : 128;
    int total;
    const TileMap tm = make_tile_map(a, TILE, TILE, total);
    constexpr int lds_bytes = persist_lds_bytes<STAGES, NWAVES>();
    constexpr int wgs_per_cu = 160 * 1024 / lds_bytes;     // by LDS; registers allow at least as many
    static_assert(wgs_per_cu >= 1, "ring too deep");
    void (*kern)(const GemmArgs, const TileMap, const int);
    if constexpr (NWAVES == 8)
        kern = a.gelu ? k_gemm_i8_persist8<STAGES, 0, true>
               : !a.aux_own_scale ? k_gemm_i8_persist8<STAGES>
               : a.x_per_token ? k_gemm_i8_persist8<STAGES, 2> : k_gemm_i8_persist8<STAGES, 1>;
    else
        kern = a.gelu ? k_gemm_i8_persist4<STAGES, 0, true>
               : !a.aux_own_scale ? k_gemm_i8_persist4<STAGES>
               : a.x_per_token ? k_gemm_i8_persist4<STAGES, 2> : k_gemm_i8_persist4<STAGES, 1>;
    int n_cu = 0;
    const hipError_t e = current_device_cus(n_cu);
    if (e != hipSuccess) return e;
    const int grid = total < n_cu * wgs_per_cu ? total : n_cu * wgs_per_cu;
    return launch_kernel(kern, dim3(grid), dim3(NWAVES * 64), lds_bytes, s, a, tm, total);
}

template <int TN, int TM>
hipError_t launch_small(const GemmArgs &a, hipStream_t s)
{
    int grid;
    const TileMap tm = make_tile_map(a, TN, TM, grid);
    if constexpr (TN == 64) {
        int n_cu = 0;                             // (prepares the device on first use: LDS attribute)
        const hipError_t e = current_device_cus(n_cu);
        if (e != hipSuccess) return e;
        if ((long)tm.tiles_m * tm.tiles_n <= n_cu)
            return launch_kernel(k_gemm_i8_small_deep<64, 64, kDeepSteps>, dim3(grid), dim3(256),
                                 kDeepSteps * 128 * BK, s, a, tm);
    }
    return launch_kernel(k_gemm_i8_small<TN, TM>, dim3(grid), dim3(256), 0, s, a, tm);
}

}  // namespace

hipError_t gemm_prepare_device()
{
    int n_cu = 0;
    return current_device_cus(n_cu);
}

// 0: register-staged 64 x 64, 1: register-staged 128 x 128, 2: persistent 128 x 128,
// 3: persistent 256 x 256.
static int gemm_form(int M, int N, int k_pad)
{
    // Which form runs a shape fastest was measured over a grid of 168 GPT-2-scale shapes
    // (M 128..16384, K 768..4096, N 768..5120, each form forced in turn); this rule loses
    // 1 % to the best form on average and at most about 15 %.  The 256 x 256 form wins as
    // soon as its tiles give more than half of the CUs work; below that the 128 x 128
    // DMA-ring form wins when the K loop is long enough for its ring to matter, and plain
    // register-staged workgroups, several per CU, when it is short.
    const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256);
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (t256 >= 144) return 3;
    if (k_pad >= 2048) return 2;
    if (k_pad < 1024) return t128 <= 320 ? 0 : 1;
    if (t128 < 128) return 0;
    return t128 <= 384 ? 2 : 1;
}

int gemm_persistent_tile_rows(int M, int N, int k_pad)
{
    const int f = gemm_form(M, N, k_pad);
    return f == 3 ? 256 : f == 2 ? 128 : 0;
}

hipError_t launch_gemm(const GemmArgs &a, hipStream_t s)
{
    switch (gemm_form(a.M, a.N, a.k_pad)) {
    case 3: return launch_persist<3, 8>(a, s);
    case 2: return launch_persist<3, 4>(a, s);
    case 1: return launch_small<128, 128>(a, s);
    default: return launch_small<64, 64>(a, s);
    }
}

}  // namespace muxq
