// Streaming (HBM-bound) kernels of the MUXQ linear layer for gfx950:
// per-channel abs-max, outlier selection + scale derivation, Body/Aux
// quantisation, Aux weight-row gather, and the offline weight quantiser.
//
// Layout idea shared by the two passes over X: a workgroup is 4 waves; each
// wave reads whole 1 KiB row segments (64 lanes x 16 B = 512 fp16 channels),
// so every thread owns 8 fixed channels and keeps their state in registers
// while it walks down the rows.  X is read exactly once per pass.
#include "muxq_kernels.h"

namespace muxq {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t half_mag_to_f32_bits(uint32_t h)
{
    float f = (float)__builtin_bit_cast(_Float16, (unsigned short)h);
    return __float_as_uint(f);
}

__global__ void k_fill_u32(uint32_t *p, int n, uint32_t v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Sec. III-C criterion, first half: column maxima of |X|.
// fp16( fp32(h) * f ) on eight packed fp16 values: the smoothed weight row W'[k][:] = W[k][:] f[k]
// of the difficulty migration (rounded to fp16, the format a layer receives its operands in).
__device__ __forceinline__ uint4 scale8_fp16(uint4 raw, float f)
{
    const f16x8 h = __builtin_bit_cast(f16x8, raw);
    f16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float v = (float)h[i] * f;
        asm("" : "+v"(v));            // one binary32 rounding, then one to fp16 (see gelu_tanh_f32)
        o[i] = (_Float16)v;
    }
    return __builtin_bit_cast(uint4, o);
}

// row_factor (may be null): row r of x is multiplied by row_factor[r] first (see scale8_fp16).
template <bool kPerTensor>
__global__ __launch_bounds__(256) void k_col_absmax(const uint16_t *__restrict__ x, int rows,
                                                    int cols, int ld, int rows_per_block,
                                                    uint32_t *__restrict__ out_bits,
                                                    const float *__restrict__ row_factor)
{
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int col0 = (blockIdx.x * 64 + tx) * 8;
    const bool active = col0 < cols;
    const int r0 = blockIdx.y * rows_per_block;
    const int r1 = min(rows, r0 + rows_per_block);
    uint4 mx = make_uint4(0, 0, 0, 0);
    if (active) {
        const uint16_t *p = x + col0;
        int row = r0 + ty;
        if (row_factor != nullptr) {
            for (; row < r1; row += 4)
                mx = absmax_step(mx, scale8_fp16(*(const uint4 *)(p + (size_t)row * ld), row_factor[row]));
        }
        for (; row + 12 < r1; row += 16) {
            uint4 v0 = *(const uint4 *)(p + (size_t)row * ld);
            uint4 v1 = *(const uint4 *)(p + (size_t)(row + 4) * ld);
            uint4 v2 = *(const uint4 *)(p + (size_t)(row + 8) * ld);
            uint4 v3 = *(const uint4 *)(p + (size_t)(row + 12) * ld);
            mx = absmax_step(absmax_step(absmax_step(absmax_step(mx, v0), v1), v2), v3);
        }
        for (; row < r1; row += 4)
            mx = absmax_step(mx, *(const uint4 *)(p + (size_t)row * ld));
    }
    __shared__ uint4 red[256];
    red[threadIdx.x] = mx;
    __syncthreads();
    if (ty != 0) return;
    for (int j = 1; j < 4; ++j) {
        uint4 o = red[tx + 64 * j];
        mx.x = pk_max_u16(mx.x, o.x);
        mx.y = pk_max_u16(mx.y, o.y);
        mx.z = pk_max_u16(mx.z, o.z);
        mx.w = pk_max_u16(mx.w, o.w);
    }
    const uint32_t w[4] = {mx.x, mx.y, mx.z, mx.w};
    if (kPerTensor) {
        uint32_t m = 0;
        for (int i = 0; i < 4; ++i) m = max(m, max(w[i] & 0xffffu, w[i] >> 16));
        for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
        if (tx == 0 && m) atomicMax(out_bits, half_mag_to_f32_bits(m));
    } else if (active) {
        for (int i = 0; i < 4; ++i) {
            uint32_t lo = w[i] & 0xffffu, hi = w[i] >> 16;
            if (lo) atomicMax(out_bits + col0 + 2 * i, half_mag_to_f32_bits(lo));
            if (hi) atomicMax(out_bits + col0 + 2 * i + 1, half_mag_to_f32_bits(hi));
        }
    }
}

// Same reduction for the activation path, without atomics or a zeroed output:
// workgroup (bx, by) writes the maxima of its row slab as fp16 magnitudes to
// partial[by][k]; k_select_scale folds the slabs.  8 waves per workgroup, each
// thread keeps 8 channels and has four 16-byte loads in flight.
__global__ __launch_bounds__(512) void k_col_absmax_partial(const uint16_t *__restrict__ x, int rows,
                                                            int cols, int ld, int k_pad,
                                                            int rows_per_block,
                                                            uint16_t *__restrict__ partial)
{
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int col0 = (blockIdx.x * 64 + tx) * 8;
    const bool active = col0 < cols;
    const int r0 = blockIdx.y * rows_per_block;
    const int r1 = min(rows, r0 + rows_per_block);
    uint4 mx = make_uint4(0, 0, 0, 0);
    if (active) {
        const uint16_t *p = x + col0;
        int row = r0 + ty;
        for (; row + 24 < r1; row += 32) {
            uint4 v0 = *(const uint4 *)(p + (size_t)row * ld);
            uint4 v1 = *(const uint4 *)(p + (size_t)(row + 8) * ld);
            uint4 v2 = *(const uint4 *)(p + (size_t)(row + 16) * ld);
            uint4 v3 = *(const uint4 *)(p + (size_t)(row + 24) * ld);
            mx = absmax_step(absmax_step(absmax_step(absmax_step(mx, v0), v1), v2), v3);
        }
        for (; row < r1; row += 8)
            mx = absmax_step(mx, *(const uint4 *)(p + (size_t)row * ld));
    }
    __shared__ uint4 red[512];
    red[threadIdx.x] = mx;
    __syncthreads();
    if (ty != 0 || col0 >= k_pad) return;
    for (int j = 1; j < 8; ++j) {
        uint4 o = red[tx + 64 * j];
        mx.x = pk_max_u16(mx.x, o.x);
        mx.y = pk_max_u16(mx.y, o.y);
        mx.z = pk_max_u16(mx.z, o.z);
        mx.w = pk_max_u16(mx.w, o.w);
    }
    *(uint4 *)(partial + (size_t)blockIdx.y * k_pad + col0) = mx;   // zeros in the K padding
}

// Producer fusion: the slab maxima above, taken by the kernel that produces X instead of by a
// pass of their own.  The producer here is the activation between the two projections of the
// GPT-2 MLP (the modules of Sec. IV-C): x = gelu(y), tanh form,
//   gelu(y) = 0.5 y (1 + tanh(sqrt(2/pi) (y + 0.044715 y^3))) = y / (1 + exp(-2 u)),
// evaluated in binary32 and rounded once to fp16; the maxima are those of the rounded
// values, so the selection step sees exactly what a separate pass over x_out would give.
// Same grid and slab layout as k_col_absmax_partial; x_out may be y itself.
// SMOOTH: the producer is the activation side of the difficulty migration instead,
// x = fp16(y / f[k]) with positive per-channel factors (one correctly rounded binary32 division).
template <bool SMOOTH>
__global__ __launch_bounds__(512) void k_gelu_absmax_partial(const uint16_t *y, int rows,
                                                             int cols, int ld_in, uint16_t *x_out,
                                                             int ld_out, int k_pad, int rows_per_block,
                                                             uint16_t *__restrict__ partial,
                                                             const float *__restrict__ col_factor)
{
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int col0 = (blockIdx.x * 64 + tx) * 8;
    const bool active = col0 < cols;
    const int r0 = blockIdx.y * rows_per_block;
    const int r1 = min(rows, r0 + rows_per_block);
    uint4 mx = make_uint4(0, 0, 0, 0);
    if (active) {
        float fk[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) fk[i] = SMOOTH ? col_factor[col0 + i] : 1.0f;
        auto one = [&](int row, uint4 raw) {
            const f16x8 h = __builtin_bit_cast(f16x8, raw);
            f16x8 g;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (SMOOTH) {
                    float v = (float)h[i] / fk[i];
                    asm("" : "+v"(v));
                    g[i] = (_Float16)v;
                } else {
                    g[i] = (_Float16)gelu_tanh_f32((float)h[i]);
                }
            }
            const uint4 out = __builtin_bit_cast(uint4, g);
            *(uint4 *)(x_out + (size_t)row * ld_out + col0) = out;
            mx = absmax_step(mx, out);
        };
        const uint16_t *p = y + col0;
        int row = r0 + ty;
        for (; row + 24 < r1; row += 32) {
            uint4 v0 = *(const uint4 *)(p + (size_t)row * ld_in);
            uint4 v1 = *(const uint4 *)(p + (size_t)(row + 8) * ld_in);
            uint4 v2 = *(const uint4 *)(p + (size_t)(row + 16) * ld_in);
            uint4 v3 = *(const uint4 *)(p + (size_t)(row + 24) * ld_in);
            one(row, v0);
            one(row + 8, v1);
            one(row + 16, v2);
            one(row + 24, v3);
        }
        for (; row < r1; row += 8) one(row, *(const uint4 *)(p + (size_t)row * ld_in));
    }
    __shared__ uint4 red[512];
    red[threadIdx.x] = mx;
    __syncthreads();
    if (ty != 0 || col0 >= k_pad || partial == nullptr) return;
    for (int j = 1; j < 8; ++j) {
        uint4 o = red[tx + 64 * j];
        mx.x = pk_max_u16(mx.x, o.x);
        mx.y = pk_max_u16(mx.y, o.y);
        mx.z = pk_max_u16(mx.z, o.z);
        mx.w = pk_max_u16(mx.w, o.w);
    }
    *(uint4 *)(partial + (size_t)blockIdx.y * k_pad + col0) = mx;   // zeros in the K padding
}

// Sec. III-C criterion, second half (ascending outlier list with the capacity
// rule), and the scale of Eq. 1 taken on Body = X with listed channels shrunk
// by 2^-exp (Eq. 4): max|Body| = max_k col_absmax[k] * mult[k].
__global__ __launch_bounds__(1024) void k_select_scale(
    const float *__restrict__ col_absmax, int K, int k_pad, float threshold, int r_cap, int exp,
    float qmax, int do_select, int do_scale, int32_t *__restrict__ idx, int32_t *__restrict__ n_outliers,
    int32_t *__restrict__ col_slot, float *__restrict__ col_scale, float *__restrict__ x_scale)
{
    __shared__ int s_wave_tot[16];
    __shared__ uint32_t s_amax_bits;
    __shared__ float s_inv;
    const int tid = threadIdx.x;
    const int per = (K + 1023) / 1024;
    const int kb = min(K, tid * per), ke = min(K, kb + per);
    if (tid == 0) s_amax_bits = 0;

    if (do_select) {
        int cnt = 0;
        for (int k = kb; k < ke; ++k) cnt += col_absmax[k] > threshold;
        // exclusive prefix over the 1024 threads: wave scan, then the 16 wave totals
        int incl = cnt;
        const int lane = tid & 63, wv = tid >> 6;
        for (int off = 1; off < 64; off <<= 1) {
            int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (lane == 63) s_wave_tot[wv] = incl;
        __syncthreads();
        int wave_base = 0, total = 0;
        for (int w = 0; w < 16; ++w) {
            const int tw = s_wave_tot[w];
            if (w < wv) wave_base += tw;
            total += tw;
        }
        int rank = wave_base + incl - cnt;
        for (int k = kb; k < ke; ++k) {
            int slot = -1;
            if (col_absmax[k] > threshold) {
                if (rank < r_cap) {
                    slot = rank;
                    idx[rank] = k;
                }
                ++rank;
            }
            if (col_slot) col_slot[k] = slot;
        }
        const int used = min(total, r_cap);
        if (tid == 0) {
            n_outliers[0] = used;
            n_outliers[1] = total;
        }
        for (int j = used + tid; j < max(r_cap, 1); j += 1024) idx[j] = -1;
        if (col_slot)
            for (int k = K + tid; k < k_pad; k += 1024) col_slot[k] = -1;
    } else {
        for (int k = tid; k < k_pad; k += 1024) col_slot[k] = -1;
        __syncthreads();
        const int used = max(0, min(n_outliers[0], r_cap));
        for (int j = tid; j < used; j += 1024) {
            int k = idx[j];
            if (k >= 0 && k < K) col_slot[k] = j;
        }
    }
    __syncthreads();
    if (!do_scale) return;

    const float shrink = __uint_as_float((uint32_t)(127 - exp) << 23);  // 2^-exp
    float amax = 0.f;
    for (int k = kb; k < ke; ++k) {
        float v = col_absmax[k] * (col_slot[k] >= 0 ? shrink : 1.0f);
        amax = fmaxf(amax, v);
    }
    // one LDS atomic per wave: 64 lanes on one address are served one after the other
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    if ((tid & 63) == 0) atomicMax(&s_amax_bits, __float_as_uint(amax));
    __syncthreads();
    if (tid == 0) {
        float a = __uint_as_float(s_amax_bits);
        float s = 0.f, inv = 0.f;
        if (a > 0.f) {
            s = a / qmax;       // correctly rounded fp32 divisions (Eq. 1)
            inv = qmax / a;
        }
        x_scale[0] = s;
        x_scale[1] = inv;
        s_inv = inv;
    }
    __syncthreads();
    const float inv = s_inv;
    for (int k = tid; k < k_pad; k += 1024)
        col_scale[k] = k < K ? inv * (col_slot[k] >= 0 ? shrink : 1.0f) : 0.f;
}

// Workgroup barrier for data exchanged through LDS only: waits for this wave's LDS
// operations but not for its global stores.  (__syncthreads() also waits until every
// earlier global store of the wave has been acknowledged, 1-3 us each time in the
// one-workgroup selection kernels, whose stores nobody reads before the kernel ends.)
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0), vmcnt and expcnt unconstrained
    __builtin_amdgcn_s_barrier();
}

// Selection and scales for one workgroup of NT threads, shared by the kernels
// below.  A thread owns 8 consecutive channels per round (rounds of 8 * NT
// channels); `load8(k0, v)` supplies their abs-max values (zero in the K padding).
// Writes col_absmax (when the loader folded it), the ascending outlier list with
// the capacity rule (Sec. III-C), n_outliers = {kept, found}, col_slot, and with
// do_scale the scale of Eq. 1 taken on Body (Eq. 4: listed channels shrunk by
// 2^-exp): x_scale = {s_x, qmax / max|Body|} and the per-channel multipliers
// (qmax = 2^(bits-1) - 1, 127 for the INT8 of Eq. 1).
template <int NT, bool STATIC, class Load8>
__device__ __forceinline__ void select_scale_block(Load8 load8, bool write_absmax, int K, int k_pad,
                                                   float threshold, int r_cap, int exp, float qmax,
                                                   int do_scale,
                                                   float *col_absmax, int32_t *idx,
                                                   int32_t *n_outliers, int32_t *col_slot,
                                                   uint8_t *col_mask, float *col_scale,
                                                   float *x_scale,
                                                   const uint8_t *static_mask = nullptr,
                                                   int32_t *zero_point = nullptr,
                                                   float *aux_scale_out = nullptr)
{
    constexpr int NW = NT / 64, ROUND = NT * 8;
    __shared__ int s_wave_tot[NW];
    __shared__ uint32_t s_amax_bits, s_nmax_bits, s_lmax_bits;
    __shared__ float s_inv;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) { s_amax_bits = 0; s_nmax_bits = 0; s_lmax_bits = 0; }
    const float shrink = __uint_as_float((uint32_t)(127 - exp) << 23);  // 2^-exp
    float lmax = 0.f;                               // max |Aux|: listed channels, after the shift
    const bool vec_ok = (((uintptr_t)col_absmax | (uintptr_t)col_slot | (uintptr_t)col_scale) & 15) == 0;
    float amax = 0.f;
    float nmax = 0.f;                               // abs-max over the channels that are not listed
    int base = 0;                                   // outlier channels found in earlier rounds
    bool shrunk0[8];                                // round 0: which of this thread's channels are listed
    for (int c0 = 0; c0 < k_pad; c0 += ROUND) {
        const int k0 = c0 + tid * 8;
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
        if (k0 < k_pad) {
            load8(k0, v);
            // (K is a multiple of 8: a thread's 8 channels are inside K or outside as a whole;
            // a lane-strided scalar store touches 32 lines per instruction, a vector store 8)
            if (write_absmax && k0 < K) {
                if (vec_ok) {
                    *(float4 *)(col_absmax + k0) = make_float4(v[0], v[1], v[2], v[3]);
                    *(float4 *)(col_absmax + k0 + 4) = make_float4(v[4], v[5], v[6], v[7]);
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) col_absmax[k0 + i] = v[i];
                }
            }
        }
        // candidate channels: over the threshold (Sec. III-C), or, with a list fixed
        // offline, the channels of that list whatever their magnitude now
        uint32_t cand = 0;
        if (STATIC && k0 < K) cand = static_mask[k0 >> 3];
        // ascending ranks: exclusive prefix of the per-thread counts over the workgroup
        int cnt = 0;
        if (STATIC) {
            cnt = __builtin_popcount(cand);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) cnt += (k0 + i < K && v[i] > threshold) ? 1 : 0;
        }
        int incl = cnt;
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        lds_barrier();                             // s_wave_tot of the previous round is consumed
        if (lane == 63) s_wave_tot[wv] = incl;
        lds_barrier();
        int wave_base = 0, total = 0;
        for (int w = 0; w < NW; ++w) {
            const int tw = s_wave_tot[w];
            if (w < wv) wave_base += tw;
            total += tw;
        }
        int rank = base + wave_base + incl - cnt;
        uint32_t listed = 0;                         // bit i: channel k0 + i is a listed outlier channel
        int slots[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int slot = -1;
            if (STATIC ? ((cand >> i) & 1u) != 0 : (k0 + i < K && v[i] > threshold)) {
                if (rank < r_cap) {
                    slot = rank;
                    idx[rank] = k0 + i;
                }
                ++rank;
            }
            slots[i] = slot;
            if (c0 == 0) shrunk0[i] = slot >= 0;
            listed |= (slot >= 0 ? 1u : 0u) << i;
            amax = fmaxf(amax, v[i] * (slot >= 0 ? shrink : 1.0f));
            nmax = fmaxf(nmax, slot >= 0 ? 0.f : v[i]);
            lmax = fmaxf(lmax, slot >= 0 ? v[i] * shrink : 0.f);
        }
        if (col_slot != nullptr && k0 < k_pad) {
            if (vec_ok) {
                *(int4 *)(col_slot + k0) = make_int4(slots[0], slots[1], slots[2], slots[3]);
                *(int4 *)(col_slot + k0 + 4) = make_int4(slots[4], slots[5], slots[6], slots[7]);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) col_slot[k0 + i] = slots[i];
            }
        }
        if (col_mask != nullptr && k0 < k_pad) col_mask[k0 >> 3] = (uint8_t)listed;
        base += total;
    }
    const int used = min(base, r_cap);
    if (tid == 0) {
        n_outliers[0] = used;
        n_outliers[1] = base;
    }
    for (int j = used + tid; j < max(r_cap, 1); j += NT) idx[j] = -1;
    if (!do_scale) return;

    // one LDS atomic per wave: 64 lanes on one address are served one after the other
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    for (int off = 32; off > 0; off >>= 1) nmax = fmaxf(nmax, __shfl_xor(nmax, off));
    if (aux_scale_out != nullptr)
        for (int off = 32; off > 0; off >>= 1) lmax = fmaxf(lmax, __shfl_xor(lmax, off));
    if (lane == 0) {
        atomicMax(&s_amax_bits, __float_as_uint(amax));
        atomicMax(&s_nmax_bits, __float_as_uint(nmax));
        if (aux_scale_out != nullptr) atomicMax(&s_lmax_bits, __float_as_uint(lmax));
    }
    lds_barrier();
    if (tid == 0) {
        const float a = __uint_as_float(s_amax_bits);
        float s = 0.f, inv = 0.f;
        if (a > 0.f) {
            s = a / qmax;       // correctly rounded fp32 divisions (Eq. 1)
            inv = qmax / a;
        }
        x_scale[0] = s;
        x_scale[1] = inv;
        s_inv = inv;
        if (aux_scale_out != nullptr) {
            // Aux on the abs-max scale of its own values (the other reading of Eq. 5)
            const float al = __uint_as_float(s_lmax_bits);
            aux_scale_out[0] = al > 0.f ? al / qmax : 0.f;
            aux_scale_out[1] = al > 0.f ? qmax / al : 0.f;
        }
        if (zero_point != nullptr) {
            // Zero point z of the unlisted channels' codes.  Their codes lie in [-c, c] with
            // c the code of their largest magnitude (the quantiser is monotone); stored as
            // code + z with z = min(c, 127 - c) made even they stay inside int8 and, when
            // c <= 63, are all non-negative.  (Even: z rides on the constant whose addition
            // does the rounding, and ties go to the even SUM.)  The GEMM epilogue takes z * (sum of the weights they meet)
            // off the INT32 accumulator again, so results do not change; what changes is the
            // sign toggling in the matrix pipes, and with it the power they draw.
            const float t = fminf(__builtin_rintf(__uint_as_float(s_nmax_bits) * inv), qmax);
            const int c = (int)t;
            // (the epilogue multiplies z by a sum of up to K weight codes in 24 bits)
            zero_point[0] = K <= 65536 ? min(c + (c & 1), (127 - c) & ~1) : 0;
        }
    }
    lds_barrier();
    const float inv = s_inv;
    if (tid * 8 < k_pad) {                          // round 0 from registers
        const int k0 = tid * 8;
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = k0 + i < K ? inv * (shrunk0[i] ? shrink : 1.0f) : 0.f;
        *(float4 *)(col_scale + k0) = make_float4(o[0], o[1], o[2], o[3]);
        *(float4 *)(col_scale + k0 + 4) = make_float4(o[4], o[5], o[6], o[7]);
    }
    // later rounds: each thread re-reads the col_slot entries it wrote itself
    for (int c0 = ROUND; c0 < k_pad; c0 += ROUND) {
        const int k0 = c0 + tid * 8;
        if (k0 >= k_pad) continue;
        const int4 a = *(const int4 *)(col_slot + k0), b = *(const int4 *)(col_slot + k0 + 4);
        const int sl[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = k0 + i < K ? inv * (sl[i] >= 0 ? shrink : 1.0f) : 0.f;
        *(float4 *)(col_scale + k0) = make_float4(o[0], o[1], o[2], o[3]);
        *(float4 *)(col_scale + k0 + 4) = make_float4(o[4], o[5], o[6], o[7]);
    }
}

__device__ __forceinline__ void widen8(uint4 mx, float (&v)[8])
{
    const uint32_t w[4] = {mx.x, mx.y, mx.z, mx.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = (float)__builtin_bit_cast(_Float16, (unsigned short)(w[i] & 0xffffu));
        v[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(w[i] >> 16));
    }
}

// Second launch of muxq_linear and muxq_detect_outliers: fold the slabs (col_absmax[k] = max over
// slabs, widened to binary32) and select, in one workgroup.  STATIC: the candidates are
// the channels of `static_mask` (a list fixed offline) instead of those over the threshold.
template <bool STATIC>
__global__ __launch_bounds__(1024) void k_fold_select_scale(
    const uint16_t *__restrict__ partial, int n_slabs, int K, int k_pad, float threshold, int r_cap,
    int exp, float qmax, int do_scale, float *__restrict__ col_absmax, int32_t *__restrict__ idx,
    int32_t *__restrict__ n_outliers, int32_t *__restrict__ col_slot, uint8_t *__restrict__ col_mask,
    float *__restrict__ col_scale, float *__restrict__ x_scale, const uint8_t *__restrict__ static_mask,
    int32_t *__restrict__ zero_point, float *__restrict__ aux_scale_out)
{
    // Few channels and many slabs (K <= 2048 at M in the thousands) leave most threads idle while
    // the others wait for one batch of loads after the other: thread t then takes channel group
    // t % G and the slabs t / G, t / G + P, ..., so that a group's slabs are fetched by P threads
    // at once, and the P partial maxima meet in LDS (64 slabs of 1024 channels: 4.2 us -> 1.8 us
    // inside the kernel).  With more channels the fold is bound by what one CU can fetch
    // (~100 GB/s), and with few slabs there is one batch anyway: both are faster as they were.
    // (Indices past the last slab are clamped, not branched around: re-reading a slab changes no
    // maximum, a branch per load would serialise the loads.)
    __shared__ uint4 s_part[1024];
    const int G = k_pad / 8;
    if (G <= 256 && n_slabs > 16) {
        const int P = 1024 / G;
        const int t = threadIdx.x, g = t % G, p = t / G;
        if (p < P) {
            uint4 mx = make_uint4(0, 0, 0, 0);
            const uint16_t *src = partial + (size_t)g * 8;
            const int last = n_slabs - 1;
            for (int sl = p; sl < n_slabs; sl += 8 * P) {
                uint4 q[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) q[j] = *(const uint4 *)(src + (size_t)min(sl + j * P, last) * k_pad);
#pragma unroll
                for (int j = 0; j < 8; ++j) mx = absmax_step(mx, q[j]);
            }
            s_part[t] = mx;
        }
        __syncthreads();
        auto load8 = [&](int k0, float (&v)[8]) {
            uint4 m = s_part[k0 >> 3];
            for (int q = 1; q < P; ++q) m = absmax_step(m, s_part[q * G + (k0 >> 3)]);
            widen8(m, v);
        };
        select_scale_block<1024, STATIC>(load8, true, K, k_pad, threshold, r_cap, exp, qmax, do_scale,
                                         col_absmax, idx, n_outliers, col_slot, col_mask, col_scale, x_scale,
                                         static_mask, zero_point, aux_scale_out);
        return;
    }
    auto load8 = [&](int k0, float (&v)[8]) {
        uint4 mx = make_uint4(0, 0, 0, 0);
        int sl = 0;
        for (; sl + 7 < n_slabs; sl += 8) {      // eight independent loads in flight
            uint4 q[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = *(const uint4 *)(partial + (size_t)(sl + j) * k_pad + k0);
#pragma unroll
            for (int j = 0; j < 8; ++j) mx = absmax_step(mx, q[j]);
        }
        for (; sl < n_slabs; ++sl)
            mx = absmax_step(mx, *(const uint4 *)(partial + (size_t)sl * k_pad + k0));
        widen8(mx, v);
    };
    select_scale_block<1024, STATIC>(load8, true, K, k_pad, threshold, r_cap, exp, qmax, do_scale,
                                     col_absmax, idx, n_outliers, col_slot, col_mask, col_scale, x_scale,
                                     static_mask, zero_point, aux_scale_out);
}

// Eq. 1 code of x * scale, left in the low byte of the returned word: the product is
// rounded to binary32, clamped to [-qmax, qmax] (v_med3_f32), and adding 1.5 * 2^23 then
// rounds it to the nearest integer, ties to even, in the adder itself and leaves that
// integer, two's complement, in the low mantissa bits.  Rounding after the clamp equals
// clamping after rounding because the bounds are integers.  Four VALU ops per element
// with the fp16 -> fp32 conversion; the streaming quantisers are not far from ALU-bound.
__device__ __forceinline__ uint32_t quant_word(float x, float scale, float qmax,
                                               float magic = 12582912.0f)
{
    const float t = __builtin_amdgcn_fmed3f(x * scale, -qmax, qmax);
    return __float_as_uint(t + magic);      // magic = 1.5 * 2^23 (+ a zero point: code + z)
}

// The low bytes of four such words as one dword (a in byte 0).
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    const uint32_t lo = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);   // {a.byte0, b.byte0, 0, 0}
    const uint32_t hi = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
    return lo | (hi << 16);
}

// Role of the extra workgroups of the two quantiser launches (workgroup `wg` of `n_wgs`,
// 256 threads): 16 lanes per output channel n (a wave takes four channels, a workgroup
// sixteen, strided over N).  Gathers the Aux weight rows (Eq. 7: only rows outlier_idx[]
// of W meet Aux; w_aux_given when they were gathered offline) and writes what the
// epilogue's zero-point correction multiplies by z:
//   cn[n] = sum over the unlisted channels k of w_q[n][k]
//         = w_row_sum[n] - sum_j w_aux[n][j]   (+ cn_bias, see kCnBias).
__device__ __forceinline__ void gather_aux_weights_and_cn(
    int wg, int n_wgs, const int8_t *__restrict__ w_q, int N, int k_pad, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ n_outliers, int r_cap, int8_t *__restrict__ w_aux,
    const int8_t *__restrict__ w_aux_given, const int32_t *__restrict__ w_row_sum,
    int32_t *__restrict__ cn, int32_t cn_bias)
{
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int used = r_cap > 0 ? max(0, min(n_outliers[0], r_cap)) : 0;
    const int sub = tx & 15;
    for (long n0 = (long)wg * 16 + ty * 4; n0 < N; n0 += (long)n_wgs * 16) {
        const long n = n0 + (tx >> 4);
        const bool live = n < N;
        // issued ahead of the gather, so that its latency is not added to the chain's
        const int row_sum = (cn != nullptr && live) ? w_row_sum[n] : 0;
        int sum = 0;
        if (live) {
            for (int j = sub; j < r_cap; j += 16) {
                int8_t v = 0;
                if (w_aux != nullptr) {
                    if (j < used) {
                        const int k = idx[j];
                        if (k >= 0 && k < k_pad) v = w_q[packed_index((int)n, k, k_pad)];
                    }
                    w_aux[packed_index((int)n, j, r_cap)] = v;
                } else if (w_aux_given != nullptr && j < used) {
                    v = w_aux_given[packed_index((int)n, j, r_cap)];
                }
                sum += (int)v;
            }
        }
        if (cn != nullptr) {
            for (int off = 8; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
            if (sub == 0 && live) cn[n] = row_sum - sum + cn_bias;     // bias: see kCnBias
        }
    }
}

// Eq. 4-5 and Eq. 1 in one pass over X: each code is
// clamp(rne(X[m][k] * col_scale[k])) with col_scale[k] = (127/max|Body|) * 2^-exp
// on outlier channels (an exact power-of-two factor, so the single fp32
// rounding equals rounding Body * (127/max|Body|)).  Threads that own an
// outlier channel also drop its code into the compact Aux matrix.
__global__ __launch_bounds__(256) void k_quantize_body(
    const uint16_t *__restrict__ x, int M, int K, int ldx, int k_pad, int rows_per_block, float qmax,
    const float *__restrict__ col_scale, const int32_t *__restrict__ col_slot,
    const int32_t *__restrict__ n_outliers, int r_cap, int8_t *__restrict__ body_q,
    int8_t *__restrict__ aux_q, int quant_blocks_y, const int8_t *__restrict__ w_q, int N,
    const int32_t *__restrict__ idx, int8_t *__restrict__ w_aux,
    const int8_t *__restrict__ w_aux_given, const int32_t *__restrict__ zero_point,
    const int32_t *__restrict__ w_row_sum, int32_t *__restrict__ cn, int32_t cn_bias,
    const float *__restrict__ aux_scale, int exp)
{
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    if ((int)blockIdx.y >= quant_blocks_y) {
        // Extra workgroups of the same launch: Aux weight rows and cn.  They come last in
        // dispatch order; dispatched first they slow the streaming part.
        const int wg = ((int)blockIdx.y - quant_blocks_y) * (int)gridDim.x + (int)blockIdx.x;
        const int n_wgs = ((int)gridDim.y - quant_blocks_y) * (int)gridDim.x;   // grid.y is capped
        gather_aux_weights_and_cn(wg, n_wgs, w_q, N, k_pad, idx, n_outliers, r_cap, w_aux, w_aux_given,
                                  w_row_sum, cn, cn_bias);
        return;
    }
    const int col0 = (blockIdx.x * 64 + tx) * 8;
    const int r0 = blockIdx.y * rows_per_block;
    const int r1 = min(M, r0 + rows_per_block);

    if (r_cap > 0 && blockIdx.x == 0) {   // zero the unused tail of the Aux rows
        const int used = max(0, min(n_outliers[0], r_cap));
        for (int row = r0 + ty; row < r1; row += 4)
            for (int j = used + tx; j < r_cap; j += 64) aux_q[packed_index(row, j, r_cap)] = 0;
    }
    if (col0 >= k_pad) return;
    if (col0 >= K) {                      // K padding of Body
        for (int row = r0 + ty; row < r1; row += 4)
            *(uint2 *)(body_q + packed_index(row, col0, k_pad)) = make_uint2(0, 0);
        return;
    }
    float sc[8];
    int slot[8];
    {
        float4 a = *(const float4 *)(col_scale + col0), b = *(const float4 *)(col_scale + col0 + 4);
        int4 c = *(const int4 *)(col_slot + col0), d = *(const int4 *)(col_slot + col0 + 4);
        sc[0] = a.x; sc[1] = a.y; sc[2] = a.z; sc[3] = a.w;
        sc[4] = b.x; sc[5] = b.y; sc[6] = b.z; sc[7] = b.w;
        slot[0] = c.x; slot[1] = c.y; slot[2] = c.z; slot[3] = c.w;
        slot[4] = d.x; slot[5] = d.y; slot[6] = d.z; slot[7] = d.w;
    }
    bool has_aux = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) has_aux |= slot[i] >= 0;
    has_aux = has_aux && r_cap > 0;
    // unlisted channels are stored as code + z (see the selection kernel): z rides on the
    // rounding constant, so it costs nothing here
    const float z = zero_point != nullptr ? (float)zero_point[0] : 0.f;
    float magic[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) magic[i] = 12582912.0f + (slot[i] < 0 ? z : 0.f);
    // Aux on a scale of its own (aux_scale = {s_aux, qmax / max|Aux|}): its codes are no longer
    // Body's; the multiplier is (qmax / max|Aux|) 2^-exp, exact like col_scale's
    const bool aux_own = aux_scale != nullptr && has_aux;
    const float aux_mul = aux_own ? aux_scale[1] * __uint_as_float((uint32_t)(127 - exp) << 23) : 0.f;

    const uint16_t *p = x + col0;
    auto do_row = [&](int row, uint4 raw) {
        f16x8 h = __builtin_bit_cast(f16x8, raw);
        uint32_t q[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = quant_word((float)h[i], sc[i], qmax, magic[i]);
        uint2 packed;
        packed.x = pack_low_bytes(q[0], q[1], q[2], q[3]);
        packed.y = pack_low_bytes(q[4], q[5], q[6], q[7]);
        *(uint2 *)(body_q + packed_index(row, col0, k_pad)) = packed;
        if (has_aux) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (slot[i] >= 0) {
                    const uint32_t code = aux_own ? quant_word((float)h[i], aux_mul, qmax) : q[i];
                    aux_q[packed_index(row, slot[i], r_cap)] = (int8_t)(code & 0xffu);
                }
        }
    };
    int row = r0 + ty;
    for (; row + 12 < r1; row += 16) {
        uint4 v0 = *(const uint4 *)(p + (size_t)row * ldx);
        uint4 v1 = *(const uint4 *)(p + (size_t)(row + 4) * ldx);
        uint4 v2 = *(const uint4 *)(p + (size_t)(row + 8) * ldx);
        uint4 v3 = *(const uint4 *)(p + (size_t)(row + 12) * ldx);
        do_row(row, v0);
        do_row(row + 4, v1);
        do_row(row + 8, v2);
        do_row(row + 12, v3);
    }
    for (; row < r1; row += 4) do_row(row, *(const uint4 *)(p + (size_t)row * ldx));
}

// ---- per-token form of the Body/Aux quantisation --------------------------------------
// One activation scale per row of Body (the per-vector setting of Sec. II-A, Fig. 2(a)),
// s_x[m] = max_k |Body[m][k]| / qmax.  A wave owns whole rows.  Which channels are listed
// outlier channels (Eq. 4: shrunk by 2^-exp) comes as one bit per channel from col_mask
// (one byte per 16-byte chunk of 8 channels, written by the selection kernel or taken from
// a static block); a listed channel's position in the ascending list is the number of
// listed channels below it.
// x_scale: [0, M) receives s_x[m], [M, 2M) qmax / max|Body[m]|, [2M, 3M) the row's zero
// point as int32.  Every workgroup also takes a share of the Aux weight gather (the one
// k_quantize_body's extra workgroups do); workgroups past `quant_wgs` do only that.

// Once per workgroup (256 threads, all of them call): the chunk masks into mask_lds, the
// list position of each chunk's first listed channel into pos_lds, and (idx_lds != nullptr)
// the ascending list itself.  Returns the number of listed channels.  Ends with a barrier.
__device__ __forceinline__ int token_mask_prologue(const uint8_t *__restrict__ col_mask, int K,
                                                   int n_chunks_all, int r_cap, uint8_t *mask_lds,
                                                   uint16_t *pos_lds, int32_t *idx_lds)
{
    __shared__ int s_wave_tot[4];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int base = 0;
    for (int c0 = 0; c0 < n_chunks_all; c0 += 256) {
        const int c = c0 + (int)threadIdx.x;
        const uint32_t m = (c < n_chunks_all && c * 8 < K) ? (uint32_t)col_mask[c] : 0u;
        const int cnt = __builtin_popcount(m);
        int incl = cnt;
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        __syncthreads();                                     // s_wave_tot of the last round is consumed
        if (lane == 63) s_wave_tot[wv] = incl;
        __syncthreads();
        int wave_base = 0, total = 0;
        for (int w = 0; w < 4; ++w) {
            if (w < wv) wave_base += s_wave_tot[w];
            total += s_wave_tot[w];
        }
        if (c < n_chunks_all) {
            int slot = base + wave_base + incl - cnt;
            mask_lds[c] = (uint8_t)m;
            pos_lds[c] = (uint16_t)slot;
            if (idx_lds != nullptr)
                for (uint32_t mm = m; mm != 0 && slot < r_cap; mm &= mm - 1, ++slot)
                    idx_lds[slot] = c * 8 + __builtin_ctz(mm);
        }
        base += total;
    }
    __syncthreads();
    return min(base, r_cap);
}

// The row's scale, inverse and zero point from max|Body| (amax) and the largest magnitude
// on an unlisted channel (nmax); lane 0 stores them.  Returns the rounding constant of the
// unlisted channels, 1.5 * 2^23 + z.
__device__ __forceinline__ float token_row_scale(float amax, float nmax, float qmax, bool with_z, int row,
                                                 int M, float *__restrict__ x_scale, float &inv)
{
    float sx = 0.f;
    inv = 0.f;
    if (amax > 0.f) {
        sx = amax / qmax;     // correctly rounded fp32 divisions (Eq. 1)
        inv = qmax / amax;
    }
    // the row's zero point (see the selection kernel), from c, the largest code among the
    // row's unlisted channels
    int z = 0;
    if (with_z) {
        const int c = (int)fminf(__builtin_rintf(nmax * inv), qmax);
        z = min(c + (c & 1), (127 - c) & ~1);      // even: see the selection kernel
    }
    if ((threadIdx.x & 63) == 0) {
        x_scale[row] = sx;
        x_scale[M + row] = inv;
        ((int32_t *)x_scale)[2 * (size_t)M + row] = z;
    }
    return 12582912.0f + (float)z;
}

// Aux on a scale of its own, one per token (the other reading of Eq. 5 in the per-vector
// setting): s_aux[m] = max_j |Aux[m][j]| / qmax goes to the fourth array of x_scale, the factor
// rho[m] = (2^exp - 1) s_aux[m] / s_x[m] that brings the Aux accumulators onto Body's grid in
// the GEMM to the fifth; returns qmax / max_j |Aux[m][j]|.  aux_amax: the row's largest
// |Aux| value (listed channels after the shift), the same in every lane.
__device__ __forceinline__ float token_aux_scale(float aux_amax, float amax, float qmax, int exp, int row,
                                                 int M, float *__restrict__ x_scale)
{
    float sa = 0.f, ia = 0.f;
    if (aux_amax > 0.f) {
        sa = aux_amax / qmax;
        ia = qmax / aux_amax;
    }
    const float sx = amax > 0.f ? amax / qmax : 0.f;          // what token_row_scale wrote
    const float rho = sx > 0.f ? ((float)((1 << exp) - 1) * sa) / sx : 0.f;
    if ((threadIdx.x & 63) == 0) {
        x_scale[3 * (size_t)M + row] = sa;
        x_scale[4 * (size_t)M + row] = rho;
    }
    return ia;
}

// Rows that fit in LDS (four per workgroup).  Per row a wave
//   1. copies the row into LDS (lane l takes the chunks l, l + 64, ...; the first row is on
//      its way while the workgroup prepares the masks, every later one while the wave works
//      on the row before it);
//   2. takes the listed channels out of that copy: lane j keeps x[row][idx[j]] aside and
//      zeroes it in the copy, so that steps 3 and 5 need no per-channel case;
//   3. max over the copy (fp16 magnitudes compared as integers, two per instruction) = the
//      largest unlisted magnitude; max|Body| = max(that, 2^-exp * largest listed one), exact;
//   4. scale and zero point; lane j quantises its listed channel from the Body value (Eq. 4:
//      exact product with 2^-exp, then the one rounded product of Eq. 1, no zero point) into
//      the row's Aux codes (Eq. 5);
//   5. quantises chunk by chunk as code + z; the few lanes whose chunk holds a listed channel
//      put the Aux code into the packed word before the store;
//   6. writes the row's Aux codes with one coalesced store.
// Lanes exchange data through the wave's own LDS regions without barriers: a wave's LDS
// instructions execute in order.
// Dynamic LDS: k_pad/8 mask bytes, k_pad/8 uint16 positions, r_cap int32 list entries; per
// wave r_cap Aux bytes, r_cap fp16 listed values and k_pad fp16 of row.
__global__ __launch_bounds__(256) void k_quantize_rows_token(
    const uint16_t *__restrict__ x, int M, int K, int ldx, int k_pad, int rows_per_wave, float qmax,
    int exp, const uint8_t *__restrict__ col_mask, const int32_t *__restrict__ n_outliers, int r_cap,
    int8_t *__restrict__ body_q, int8_t *__restrict__ aux_q, float *__restrict__ x_scale,
    int quant_wgs, const int8_t *__restrict__ w_q, int N, const int32_t *__restrict__ idx,
    int8_t *__restrict__ w_aux, const int8_t *__restrict__ w_aux_given,
    const int32_t *__restrict__ w_row_sum, int32_t *__restrict__ cn, int aux_own)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if ((int)blockIdx.x >= quant_wgs) {      // workgroups with no rows: their share of the gather only
        if (w_aux != nullptr || cn != nullptr)
            gather_aux_weights_and_cn((int)blockIdx.x, (int)gridDim.x, w_q, N, k_pad, idx, n_outliers, r_cap,
                                      w_aux, w_aux_given, w_row_sum, cn, 0);
        return;
    }
    extern __shared__ __attribute__((aligned(16))) unsigned char tok_lds[];
    const int n_chunks_all = k_pad / 8, n_chunks = K / 8;       // 16-byte chunks per row: padded, real
    uint8_t *const mask_lds = tok_lds;                                               // [n_chunks_all]
    uint16_t *const pos_lds = (uint16_t *)(tok_lds + ((n_chunks_all + 15) & ~15));   // [n_chunks_all]
    int32_t *const idx_lds = (int32_t *)(pos_lds + ((n_chunks_all + 7) & ~7));       // [r_cap]
    int8_t *const per_wave = (int8_t *)(idx_lds + r_cap);
    int8_t *const aux_row = per_wave + wv * r_cap;                                   // [r_cap]
    uint16_t *const listed_x = (uint16_t *)(per_wave + 4 * r_cap) + wv * r_cap;      // [r_cap]
    uint4 *const row_lds = (uint4 *)(per_wave + 12 * r_cap) + (size_t)wv * n_chunks_all;
    uint16_t *const row_half = (uint16_t *)row_lds;

    const int wave_global = blockIdx.x * 4 + wv;
    const int r0 = wave_global * rows_per_wave, r1 = min(M, r0 + rows_per_wave);
    // A row travels memory -> registers -> LDS in two steps, so that the loads of the next row
    // are in flight while the wave works on the current one: the first kPrefetch chunks of a
    // lane (rows of up to 64 * 8 * kPrefetch channels entirely) wait in registers, the rest of
    // a longer row is copied at the second step.
    constexpr int kPrefetch = 8;
    uint4 pf[kPrefetch];
    const bool full = n_chunks >= 64 * kPrefetch;             // no per-chunk bound checks then
    auto row_issue = [&](int row) {
        const uint16_t *src = x + (size_t)row * ldx;
        if (full) {
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u) pf[u] = *(const uint4 *)(src + (size_t)(64 * u + lane) * 8);
        } else {
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u)
                pf[u] = 64 * u + lane < n_chunks ? *(const uint4 *)(src + (size_t)(64 * u + lane) * 8)
                                                 : make_uint4(0, 0, 0, 0);
        }
    };
    auto row_commit = [&](int row) {
        if (full) {
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u) row_lds[64 * u + lane] = pf[u];
        } else {
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u)
                if (64 * u + lane < n_chunks) row_lds[64 * u + lane] = pf[u];
        }
        const uint16_t *src = x + (size_t)row * ldx;
        for (int c = 64 * kPrefetch + lane; c < n_chunks; c += 64)
            row_lds[c] = *(const uint4 *)(src + (size_t)c * 8);
    };
    if (r0 < r1) {
        row_issue(r0);
        row_commit(r0);
    }

    for (int j = lane * 4; j < r_cap; j += 256) *(uint32_t *)(aux_row + j) = 0u;
    const int used = token_mask_prologue(col_mask, K, n_chunks_all, r_cap, mask_lds, pos_lds, idx_lds);
    const float shrink = __uint_as_float((uint32_t)(127 - exp) << 23);  // 2^-exp
    const bool with_z = cn != nullptr && K <= 65536;

    for (int row = r0; row < r1; ++row) {
        if (row + 1 < r1) row_issue(row + 1);
        // ---- listed channels out of the copy ----
        float lmax = 0.f;
        for (int j = lane; j < used; j += 64) {
            const int k = idx_lds[j];
            const uint16_t hb = row_half[k];
            row_half[k] = 0;
            listed_x[j] = hb;
            lmax = fmaxf(lmax, (float)__builtin_bit_cast(_Float16, (unsigned short)(hb & 0x7fffu)));
        }
        __builtin_amdgcn_wave_barrier();
        // ---- the row's abs-max ----
        uint32_t m2 = 0;
#pragma unroll 4
        for (int c = lane; c < n_chunks; c += 64) {
            const uint4 raw = row_lds[c];
            m2 = pk_max_u16(pk_max_u16(m2, raw.x & 0x7fff7fffu),
                            pk_max_u16(pk_max_u16(raw.y & 0x7fff7fffu, raw.z & 0x7fff7fffu),
                                       raw.w & 0x7fff7fffu));
        }
        const uint32_t top = max(m2 & 0xffffu, m2 >> 16);        // magnitudes order like integers
        float nmax = fmaxf(0.f, (float)__builtin_bit_cast(_Float16, (unsigned short)top));
        float amax = fmaxf(nmax, lmax * shrink);
        for (int off = 32; off > 0; off >>= 1) {
            amax = fmaxf(amax, __shfl_xor(amax, off));
            nmax = fmaxf(nmax, __shfl_xor(nmax, off));
        }
        float inv;
        const float magic_z = token_row_scale(amax, nmax, qmax, with_z, row, M, x_scale, inv);
        float inv_aux = inv;                         // Aux shares the row's scale, or has its own
        if (aux_own) {
            for (int off = 32; off > 0; off >>= 1) lmax = fmaxf(lmax, __shfl_xor(lmax, off));
            inv_aux = token_aux_scale(lmax * shrink, amax, qmax, exp, row, M, x_scale);
        }
        // ---- Aux codes ----
        for (int j = lane; j < used; j += 64) {
            const float b = (float)__builtin_bit_cast(_Float16, listed_x[j]) * shrink;
            aux_row[j] = (int8_t)(quant_word(b, inv_aux, qmax) & 0xffu);
        }
        __builtin_amdgcn_wave_barrier();
        // ---- Body codes ----
#pragma unroll 2
        for (int c = lane; c < n_chunks; c += 64) {
            const uint4 raw = row_lds[c];
            const uint32_t mask = mask_lds[c];
            const f16x8 h = __builtin_bit_cast(f16x8, raw);
            uint32_t q[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) q[i] = quant_word((float)h[i], inv, qmax, magic_z);
            uint2 packed;
            packed.x = pack_low_bytes(q[0], q[1], q[2], q[3]);
            packed.y = pack_low_bytes(q[4], q[5], q[6], q[7]);
            if (mask != 0 && r_cap > 0) {
                int slot = pos_lds[c];
                for (uint32_t mm = mask; mm != 0; mm &= mm - 1, ++slot) {
                    const int i = __builtin_ctz(mm);
                    const int sl = min(slot, r_cap - 1);
                    // Body's code of a listed channel: the Aux code, unless Aux has its own scale
                    const uint32_t code =
                        aux_own ? quant_word((float)__builtin_bit_cast(_Float16, listed_x[sl]) * shrink, inv, qmax) & 0xffu
                                : (uint32_t)(uint8_t)aux_row[sl];
                    const uint32_t sh = (uint32_t)(i & 3) * 8u;
                    if (i < 4)
                        packed.x = (packed.x & ~(0xffu << sh)) | (code << sh);
                    else
                        packed.y = (packed.y & ~(0xffu << sh)) | (code << sh);
                }
            }
            *(uint2 *)(body_q + packed_index(row, c * 8, k_pad)) = packed;
        }
        for (int c = n_chunks + lane; c < n_chunks_all; c += 64)          // K padding of Body
            *(uint2 *)(body_q + packed_index(row, c * 8, k_pad)) = make_uint2(0, 0);
        for (int j = lane * 4; j < r_cap; j += 256)
            *(uint32_t *)(aux_q + packed_index(row, j, r_cap)) = *(const uint32_t *)(aux_row + j);
        if (row + 1 < r1) row_commit(row + 1);
    }
    // every workgroup of the launch takes a share of the Aux weight gather: here its memory
    // latency hides behind the other waves' rows (workgroups that did nothing else would wait
    // for the LDS of a finished one and run after the streaming part)
    if (w_aux != nullptr || cn != nullptr)
        gather_aux_weights_and_cn((int)blockIdx.x, (int)gridDim.x, w_q, N, k_pad, idx, n_outliers, r_cap,
                                  w_aux, w_aux_given, w_row_sum, cn, 0);
}

// Rows too long for LDS: the same result with each row read twice from memory (abs-max,
// then codes) and the listed channels told apart by the chunk masks in both passes.
// Dynamic LDS: k_pad/8 mask bytes, k_pad/8 uint16 positions, 4 x r_cap Aux bytes.
__global__ __launch_bounds__(256) void k_quantize_rows_token_long(
    const uint16_t *__restrict__ x, int M, int K, int ldx, int k_pad, int rows_per_wave, float qmax,
    int exp, const uint8_t *__restrict__ col_mask, const int32_t *__restrict__ n_outliers, int r_cap,
    int8_t *__restrict__ body_q, int8_t *__restrict__ aux_q, float *__restrict__ x_scale,
    int quant_wgs, const int8_t *__restrict__ w_q, int N, const int32_t *__restrict__ idx,
    int8_t *__restrict__ w_aux, const int8_t *__restrict__ w_aux_given,
    const int32_t *__restrict__ w_row_sum, int32_t *__restrict__ cn, int aux_own)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if ((int)blockIdx.x >= quant_wgs) {      // workgroups with no rows: their share of the gather only
        if (w_aux != nullptr || cn != nullptr)
            gather_aux_weights_and_cn((int)blockIdx.x, (int)gridDim.x, w_q, N, k_pad, idx, n_outliers, r_cap,
                                      w_aux, w_aux_given, w_row_sum, cn, 0);
        return;
    }
    extern __shared__ __attribute__((aligned(16))) unsigned char tok_lds[];
    const int n_chunks_all = k_pad / 8;
    uint8_t *const mask_lds = tok_lds;
    uint16_t *const pos_lds = (uint16_t *)(tok_lds + ((n_chunks_all + 15) & ~15));
    int8_t *const aux_row = (int8_t *)(pos_lds + ((n_chunks_all + 7) & ~7)) + wv * r_cap;

    for (int j = lane * 4; j < r_cap; j += 256) *(uint32_t *)(aux_row + j) = 0u;
    token_mask_prologue(col_mask, K, n_chunks_all, r_cap, mask_lds, pos_lds, nullptr);
    const float shrink = __uint_as_float((uint32_t)(127 - exp) << 23);  // 2^-exp
    const bool with_z = cn != nullptr && K <= 65536;

    // max |Body| over a chunk's 8 channels (exact: |x| and |x| 2^-exp are binary32 values);
    // nmax: the same over its unlisted channels only.  The few lanes whose chunk holds a
    // listed channel first take those magnitudes out one by one.
    auto chunk_amax = [&](uint4 raw, uint32_t mask, float &nmax, float &lmax_row) -> float {
        uint32_t w[4] = {raw.x & 0x7fff7fffu, raw.y & 0x7fff7fffu, raw.z & 0x7fff7fffu,
                         raw.w & 0x7fff7fffu};
        float lmax = 0.f;                                        // largest |x| on listed channels
        for (uint32_t mm = mask; mm != 0; mm &= mm - 1) {
            const int i = __builtin_ctz(mm), d = i >> 1;
            const uint32_t sh = (uint32_t)(i & 1) * 16u;
            const uint32_t word = d == 0 ? w[0] : d == 1 ? w[1] : d == 2 ? w[2] : w[3];
            const float v = (float)__builtin_bit_cast(_Float16, (unsigned short)((word >> sh) & 0xffffu));
            lmax = fmaxf(lmax, v);
            const uint32_t keep = ~(0xffffu << sh);
            w[0] = d == 0 ? w[0] & keep : w[0];
            w[1] = d == 1 ? w[1] & keep : w[1];
            w[2] = d == 2 ? w[2] & keep : w[2];
            w[3] = d == 3 ? w[3] & keep : w[3];
        }
        const uint32_t m = pk_max_u16(pk_max_u16(w[0], w[1]), pk_max_u16(w[2], w[3]));
        const uint32_t top = max(m & 0xffffu, m >> 16);          // magnitudes order like integers
        const float a = (float)__builtin_bit_cast(_Float16, (unsigned short)top);
        nmax = fmaxf(nmax, a);
        lmax_row = fmaxf(lmax_row, lmax);
        return fmaxf(a, lmax * shrink);
    };
    auto load_chunk = [&](int row, int c) -> uint4 {            // zeros in the K padding
        return c * 8 < K ? *(const uint4 *)(x + (size_t)row * ldx + c * 8) : make_uint4(0, 0, 0, 0);
    };

    const int wave_global = blockIdx.x * 4 + wv;
    const int r0 = wave_global * rows_per_wave, r1 = min(M, r0 + rows_per_wave);
    for (int row = r0; row < r1; ++row) {
        // ---- pass 1: the row's abs-max ----
        float amax = 0.f, nmax = 0.f, lmax_row = 0.f;
        for (int c0 = lane; c0 < n_chunks_all; c0 += 256) {     // four chunks in flight per lane
            uint4 raw[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                raw[u] = c0 + 64 * u < n_chunks_all ? load_chunk(row, c0 + 64 * u) : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + 64 * u;
                if (c < n_chunks_all) amax = fmaxf(amax, chunk_amax(raw[u], mask_lds[c], nmax, lmax_row));
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            amax = fmaxf(amax, __shfl_xor(amax, off));
            nmax = fmaxf(nmax, __shfl_xor(nmax, off));
        }
        float inv;
        const float magic_z = token_row_scale(amax, nmax, qmax, with_z, row, M, x_scale, inv);
        float inv_aux = inv;                         // Aux shares the row's scale, or has its own
        if (aux_own) {
            for (int off = 32; off > 0; off >>= 1) lmax_row = fmaxf(lmax_row, __shfl_xor(lmax_row, off));
            inv_aux = token_aux_scale(lmax_row * shrink, amax, qmax, exp, row, M, x_scale);
        }
        // ---- pass 2: codes, chunk by chunk ----
        // Every channel is quantised as an unlisted one (code + z); the few lanes whose chunk
        // holds a listed channel then redo those codes from the Body value (Eq. 4: exact
        // product with 2^-exp, then the one rounded product of Eq. 1, no zero point), put them
        // into the packed word and drop them into the row's Aux codes.
#pragma unroll 2
        for (int c = lane; c < n_chunks_all; c += 64) {
            const uint4 raw = load_chunk(row, c);
            const uint32_t mask = mask_lds[c];
            const f16x8 h = __builtin_bit_cast(f16x8, raw);
            const float magic = c * 8 >= K ? 12582912.0f : magic_z;     // K padding: plain zeros
            uint32_t q[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) q[i] = quant_word((float)h[i], inv, qmax, magic);
            uint2 packed;
            packed.x = pack_low_bytes(q[0], q[1], q[2], q[3]);
            packed.y = pack_low_bytes(q[4], q[5], q[6], q[7]);
            if (mask != 0 && r_cap > 0) {
                int slot = pos_lds[c];
                for (uint32_t mm = mask; mm != 0 && slot < r_cap; mm &= mm - 1, ++slot) {
                    const int i = __builtin_ctz(mm), d = i >> 1;
                    const uint32_t word = d == 0 ? raw.x : d == 1 ? raw.y : d == 2 ? raw.z : raw.w;
                    const float x_i = (float)__builtin_bit_cast(
                        _Float16, (unsigned short)((word >> ((uint32_t)(i & 1) * 16u)) & 0xffffu));
                    const uint32_t code = quant_word(x_i * shrink, inv, qmax) & 0xffu;
                    const uint32_t sh = (uint32_t)(i & 3) * 8u;
                    if (i < 4)
                        packed.x = (packed.x & ~(0xffu << sh)) | (code << sh);
                    else
                        packed.y = (packed.y & ~(0xffu << sh)) | (code << sh);
                    aux_row[slot] = (int8_t)(aux_own ? quant_word(x_i * shrink, inv_aux, qmax) & 0xffu : code);
                }
            }
            *(uint2 *)(body_q + packed_index(row, c * 8, k_pad)) = packed;
        }
        for (int j = lane * 4; j < r_cap; j += 256)
            *(uint32_t *)(aux_q + packed_index(row, j, r_cap)) = *(const uint32_t *)(aux_row + j);
    }
    // every workgroup of the launch takes a share of the Aux weight gather: here its memory
    // latency hides behind the other waves' rows (workgroups that did nothing else would wait
    // for the LDS of a finished one and run after the streaming part)
    if (w_aux != nullptr || cn != nullptr)
        gather_aux_weights_and_cn((int)blockIdx.x, (int)gridDim.x, w_q, N, k_pad, idx, n_outliers, r_cap,
                                  w_aux, w_aux_given, w_row_sum, cn, 0);
}

// A channel list fixed offline (Sec. III-C criterion applied to calibration data), made
// ready for the run-time kernels: entries that are not inside [0, K) or not above the
// previous accepted entry are skipped; the r_cap lowest accepted entries are listed, the
// count of all accepted entries is reported beside the number listed.
__global__ __launch_bounds__(256) void k_static_list(const int32_t *__restrict__ list, int n_list, int K,
                                                     int k_pad, int r_cap, uint8_t *__restrict__ col_mask,
                                                     int32_t *__restrict__ idx, int32_t *__restrict__ n_outliers)
{
    for (int c = threadIdx.x; c < k_pad / 8; c += 256) col_mask[c] = 0;
    for (int j = threadIdx.x; j < max(r_cap, 1); j += 256) idx[j] = -1;
    __syncthreads();
    if (threadIdx.x != 0) return;
    int kept = 0, prev = -1;
    for (int j = 0; j < n_list; ++j) {
        const int k = list[j];
        if (k <= prev || k >= K) continue;
        if (kept < r_cap) {
            idx[kept] = k;
            col_mask[k >> 3] |= (uint8_t)(1u << (k & 7));
        }
        ++kept;
        prev = k;
    }
    n_outliers[0] = min(kept, r_cap);
    n_outliers[1] = kept;
}

// Eq. 7: the rows outlier_idx[] of the quantised weight, as the packed N x r_cap operand of
// the Aux product (4 output channels per workgroup, strided over N).
__global__ __launch_bounds__(256) void k_gather_aux_weights(const int8_t *__restrict__ w_q, int N, int k_pad,
                                                            const int32_t *__restrict__ idx,
                                                            const int32_t *__restrict__ n_outliers,
                                                            int r_cap, int8_t *__restrict__ w_aux)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int used = max(0, min(n_outliers[0], r_cap));
    for (long n = (long)blockIdx.x * 4 + wv; n < N; n += (long)gridDim.x * 4)
        for (int j = lane; j < r_cap; j += 64) {
            int8_t v = 0;
            if (j < used) {
                const int k = idx[j];
                if (k >= 0 && k < k_pad) v = w_q[packed_index((int)n, k, k_pad)];
            }
            w_aux[packed_index((int)n, j, r_cap)] = v;
        }
}

// Eq. 2 codes, written transposed into the packed layout: W is K x N (N
// contiguous); the GEMM wants each output channel's K codes contiguous, so a
// 64 x 64 tile goes through LDS.
__global__ __launch_bounds__(256) void k_wquant_transpose(const uint16_t *__restrict__ w, int K,
                                                          int N, int ldw, int k_pad,
                                                          const float *__restrict__ amax,
                                                          int per_channel, float qmax,
                                                          int8_t *__restrict__ w_q,
                                                          int32_t *__restrict__ row_sum,
                                                          const float *__restrict__ row_factor)
{
    __shared__ __attribute__((aligned(16))) int8_t tile[64][68];  // [n][k]
    const int k0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    const int nc = threadIdx.x & 7, kr = threadIdx.x >> 3;
    const int n = n0 + nc * 8;
    float inv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float a = 0.f;
        if (n + i < N) a = per_channel ? amax[n + i] : amax[0];
        inv[i] = a > 0.f ? qmax / a : 0.f;
    }
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int kl = kr + 32 * pass, k = k0 + kl;
        int q[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (k < K && n < N) {
            uint4 raw = *(const uint4 *)(w + (size_t)k * ldw + n);
            if (row_factor != nullptr) raw = scale8_fp16(raw, row_factor[k]);     // W' = fp16(W f[k])
            f16x8 h = __builtin_bit_cast(f16x8, raw);
#pragma unroll
            for (int i = 0; i < 8; ++i) q[i] = (int)(int8_t)(quant_word((float)h[i], inv[i], qmax) & 0xffu);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) tile[nc * 8 + i][kl] = (int8_t)q[i];
    }
    __syncthreads();
    const int nl = threadIdx.x >> 2, chunk = threadIdx.x & 3;
    if (n0 + nl < N) {
        const uint32_t *src = (const uint32_t *)&tile[nl][chunk * 16];
        uint4 v = make_uint4(src[0], src[1], src[2], src[3]);
        *(uint4 *)(w_q + packed_index(n0 + nl, k0 + chunk * 16, k_pad)) = v;
    }
    // row_sum[n] += the sum of this tile's codes of output channel n (pre-zeroed by the
    // caller): the constant of the activation zero-point correction in the GEMM epilogue
    int part = 0;
    {
        const int8_t *src = &tile[nl][chunk * 16];
#pragma unroll
        for (int i = 0; i < 16; ++i) part += (int)src[i];
    }
    part += __shfl_xor(part, 1);
    part += __shfl_xor(part, 2);
    if (chunk == 0 && n0 + nl < N && part != 0) atomicAdd(row_sum + n0 + nl, part);
}

__global__ void k_wscale_finalize(float *w_scale, int n, float qmax)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        float a = w_scale[i];
        w_scale[i] = a > 0.f ? a / qmax : 0.f;
    }
}

int rows_per_block_for(int rows, int col_blocks, bool streaming_store = false)
{
    // aim at ~8 workgroups per CU (256 CUs), at least 16 rows per wave pass; twice as many when
    // the matrix is larger than the 256 MB memory-side cache holds (16384 x 5120, cold: the
    // quantiser takes 53.8 us instead of 58.8 us; smaller matrices do not care)
    const bool from_hbm = streaming_store &&
                          2.0 * (double)rows * 512.0 * (double)col_blocks >= 128.0 * 1024.0 * 1024.0;
    int want_blocks_y = max(1, (from_hbm ? 4096 : 2048) / max(1, col_blocks));
    int rpb = (rows + want_blocks_y - 1) / want_blocks_y;
    rpb = max(rpb, 32);
    return (rpb + 3) & ~3;
}

}  // namespace

hipError_t launch_fill_u32(uint32_t *p, int n, uint32_t v, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    return launch_kernel(k_fill_u32, dim3((n + 255) / 256), dim3(256), 0, s, p, n, v);
}

hipError_t launch_col_absmax(const void *x_fp16, int rows, int cols, int ld, int per_tensor,
                             uint32_t *out_bits, hipStream_t s, const float *row_factor)
{
    const int gx = (cols / 8 + 63) / 64;
    const int rpb = rows_per_block_for(rows, gx);
    dim3 grid(gx, (rows + rpb - 1) / rpb);
    if (per_tensor)
        return launch_kernel(k_col_absmax<true>, grid, dim3(256), 0, s, (const uint16_t *)x_fp16,
                           rows, cols, ld, rpb, out_bits, row_factor);
    return launch_kernel(k_col_absmax<false>, grid, dim3(256), 0, s, (const uint16_t *)x_fp16,
                         rows, cols, ld, rpb, out_bits, row_factor);
}

// Grid of the slab-maxima kernels: gx column blocks of 512 channels, gy row slabs.
static void absmax_grid(int rows, int k_pad, int &gx, int &gy, int &rpb)
{
    gx = (k_pad / 8 + 63) / 64;
    // Enough workgroups to fill the chip, at most kMaxSlabs slabs, at least 16 rows each.  How many
    // depends on where X comes from (measured on the MI355X, 256 CUs).  Out of the 256 MB
    // memory-side cache a pass is bound by what is in flight, and 320 workgroups beat 256
    // (8192 x 4096: 11.7 us against 17.4 us).  From HBM, i.e. when X is larger than that cache
    // holds, it is bound by the slowest CU, and a grid of at most one workgroup per CU beats one
    // that leaves a quarter of the CUs with two (2 GiB of X: 6.2 TB/s against 5.3 TB/s;
    // 16384 x 5120, cold: 38.9 us against 44.1 us for the pass and the fold).
    const bool from_hbm = 2.0 * (double)rows * (double)k_pad >= 128.0 * 1024.0 * 1024.0;
    gy = max(1, min(kMaxSlabs, from_hbm ? 256 / gx : (320 + gx - 1) / gx));
    gy = max(1, min(gy, (rows + 15) / 16));
    rpb = (rows + gy - 1) / gy;
    rpb = (rpb + 7) & ~7;
    gy = (rows + rpb - 1) / rpb;
}

hipError_t launch_col_absmax_partial(const void *x_fp16, int rows, int cols, int ld, int k_pad,
                                    uint16_t *partial, int *n_slabs, hipStream_t s)
{
    int gx, gy, rpb;
    absmax_grid(rows, k_pad, gx, gy, rpb);
    *n_slabs = gy;
    return launch_kernel(k_col_absmax_partial, dim3(gx, gy), dim3(512), 0, s,
                       (const uint16_t *)x_fp16, rows, cols, ld, k_pad, rpb, partial);
}

int absmax_slab_count(int rows, int k_pad)
{
    int gx, gy, rpb;
    absmax_grid(rows, k_pad, gx, gy, rpb);
    return gy;
}

hipError_t launch_gelu_absmax_partial(const void *y_fp16, int rows, int cols, int ld_in, void *x_fp16,
                                      int ld_out, int k_pad, uint16_t *partial, hipStream_t s,
                                      const float *col_factor)
{
    int gx, gy, rpb;
    absmax_grid(rows, k_pad, gx, gy, rpb);
    if (col_factor != nullptr)
        return launch_kernel(k_gelu_absmax_partial<true>, dim3(gx, gy), dim3(512), 0, s, (const uint16_t *)y_fp16,
                             rows, cols, ld_in, (uint16_t *)x_fp16, ld_out, k_pad, rpb, partial, col_factor);
    return launch_kernel(k_gelu_absmax_partial<false>, dim3(gx, gy), dim3(512), 0, s, (const uint16_t *)y_fp16,
                         rows, cols, ld_in, (uint16_t *)x_fp16, ld_out, k_pad, rpb, partial, col_factor);
}

hipError_t launch_fold_select_scale(const uint16_t *partial, int n_slabs, int K, int k_pad,
                                    float threshold, int r_cap, int exp, float qmax, int do_scale,
                                    float *col_absmax, int32_t *idx, int32_t *n_outliers,
                                    int32_t *col_slot, uint8_t *col_mask, float *col_scale,
                                    float *x_scale, hipStream_t s, const uint8_t *static_mask,
                                    int32_t *zero_point, float *aux_scale_out)
{
    if (static_mask != nullptr)
        return launch_kernel(k_fold_select_scale<true>, dim3(1), dim3(1024), 0, s, partial, n_slabs, K, k_pad,
                           threshold, r_cap, exp, qmax, do_scale, col_absmax, idx, n_outliers, col_slot,
                           col_mask, col_scale, x_scale, static_mask, zero_point, aux_scale_out);
    return launch_kernel(k_fold_select_scale<false>, dim3(1), dim3(1024), 0, s, partial, n_slabs, K, k_pad,
                         threshold, r_cap, exp, qmax, do_scale, col_absmax, idx, n_outliers, col_slot,
                         col_mask, col_scale, x_scale, static_mask, zero_point, aux_scale_out);
}

hipError_t launch_select_scale(const float *col_absmax, int K, int k_pad, float threshold,
                               int r_cap, int exp, float qmax, int do_select, int do_scale, int32_t *idx,
                               int32_t *n_outliers, int32_t *col_slot, float *col_scale,
                               float *x_scale, hipStream_t s)
{
    return launch_kernel(k_select_scale, dim3(1), dim3(1024), 0, s, col_absmax, K, k_pad, threshold,
                       r_cap, exp, qmax, do_select, do_scale, idx, n_outliers, col_slot, col_scale,
                       x_scale);
}

hipError_t launch_static_list(const int32_t *list, int n_list, int K, int k_pad, int r_cap,
                              uint8_t *col_mask, int32_t *idx, int32_t *n_outliers, const int8_t *w_q,
                              int N, int8_t *w_aux, hipStream_t s)
{
    const hipError_t e = launch_kernel(k_static_list, dim3(1), dim3(256), 0, s, list, n_list, K, k_pad,
                                       r_cap, col_mask, idx, n_outliers);
    if (e != hipSuccess || r_cap == 0) return e;
    const int wgs = min((N + 3) / 4, 1 << 16);
    return launch_kernel(k_gather_aux_weights, dim3(wgs), dim3(256), 0, s, w_q, N, k_pad, idx, n_outliers,
                         r_cap, w_aux);
}

hipError_t launch_quantize_body(const void *x_fp16, int M, int K, int ldx, int k_pad, float qmax,
                                const float *col_scale, const int32_t *col_slot,
                                const int32_t *n_outliers, int r_cap, int8_t *body_q,
                                int8_t *aux_q, const int8_t *w_q, int N, const int32_t *idx,
                                int8_t *w_aux, hipStream_t s, const int8_t *w_aux_given,
                                const int32_t *zero_point, const int32_t *w_row_sum, int32_t *cn,
                                int32_t cn_bias, const float *aux_scale, int exp)
{
    const int gx = (k_pad / 8 + 63) / 64;
    const int rpb = rows_per_block_for(M, gx, true);
    const int gy = (M + rpb - 1) / rpb;
    // extra workgroups gather the Aux weight rows and write the zero-point correction
    // (16 output channels per workgroup)
    if (r_cap == 0) w_aux = nullptr;
    const int gather_wgs = (w_aux != nullptr || cn != nullptr) ? (N + 15) / 16 : 0;
    const int gy_extra = min((gather_wgs + gx - 1) / gx, 65535 - gy);   // grid.y limit; the gather strides
    return launch_kernel(k_quantize_body, dim3(gx, gy + gy_extra), dim3(256), 0, s,
                       (const uint16_t *)x_fp16, M, K, ldx, k_pad, rpb, qmax, col_scale, col_slot,
                       n_outliers, r_cap, body_q, aux_q, gy, w_q, N, idx, w_aux, w_aux_given, zero_point,
                       w_row_sum, cn, cn_bias, aux_scale, exp);
}

hipError_t launch_quantize_rows_token(const void *x_fp16, int M, int K, int ldx, int k_pad, float qmax,
                                      int exp, const uint8_t *col_mask, const int32_t *n_outliers,
                                      int r_cap, int8_t *body_q, int8_t *aux_q, float *x_scale,
                                      const int8_t *w_q, int N, const int32_t *idx, int8_t *w_aux,
                                      hipStream_t s, const int8_t *w_aux_given,
                                      const int32_t *w_row_sum, int32_t *cn, int aux_own)
{
    // about four waves per SIMD over the chip (measured best), at most 16 rows per wave
    int rpw = (M + 4095) / 4096;
    rpw = max(1, min(rpw, 16));
    const int quant_wgs = (M + 4 * rpw - 1) / (4 * rpw);
    if (r_cap == 0) w_aux = nullptr;
    // 16 output channels per workgroup and step of the gather; workgroups without rows are
    // added when the ones with rows are fewer than that
    const int gather_wgs = (w_aux != nullptr || cn != nullptr) ? (N + 15) / 16 : 0;
    const dim3 grid(max(quant_wgs, gather_wgs)), block(256);
    const uint16_t *x = (const uint16_t *)x_fp16;
    const int n_chunks = k_pad / 8;
    const size_t masks = (size_t)((n_chunks + 15) & ~15) + (size_t)((n_chunks + 7) & ~7) * 2;
    const size_t small = masks + 4 * (size_t)r_cap;
    const size_t with_rows = masks + 16 * (size_t)r_cap + 4 * (size_t)n_chunks * 16;
    if (with_rows <= 64 * 1024)     // rows of up to ~8000 channels; four workgroups per CU up to ~4600
        return launch_kernel(k_quantize_rows_token, grid, block, with_rows, s, x, M, K, ldx, k_pad, rpw,
                           qmax, exp, col_mask, n_outliers, r_cap, body_q, aux_q, x_scale, quant_wgs,
                           w_q, N, idx, w_aux, w_aux_given, w_row_sum, cn, aux_own);
    return launch_kernel(k_quantize_rows_token_long, grid, block, small, s, x, M, K, ldx, k_pad, rpw,
                         qmax, exp, col_mask, n_outliers, r_cap, body_q, aux_q, x_scale, quant_wgs,
                         w_q, N, idx, w_aux, w_aux_given, w_row_sum, cn, aux_own);
}

hipError_t launch_wquant_transpose(const void *w_fp16, int K, int N, int ldw, int k_pad,
                                   const float *amax, int per_channel, float qmax, int8_t *w_q,
                                   int32_t *row_sum, hipStream_t s, const float *row_factor)
{
    dim3 grid(k_pad / 64, (N + 63) / 64);
    return launch_kernel(k_wquant_transpose, grid, dim3(256), 0, s, (const uint16_t *)w_fp16, K, N,
                       ldw, k_pad, amax, per_channel, qmax, w_q, row_sum, row_factor);
}

hipError_t launch_wscale_finalize(float *w_scale, int n, float qmax, hipStream_t s)
{
    return launch_kernel(k_wscale_finalize, dim3((n + 255) / 256), dim3(256), 0, s, w_scale, n, qmax);
}

}  // namespace muxq
