// Measurement aid: the rate at which this chip issues v_mfma_i32_32x32x32_i8
// when nothing else competes -- operands in registers, no LDS, no memory --
// on operand codes the caller supplies.  The INT8 matrix pipes of an MI355X
// are power-limited: the same instruction stream runs near the published
// 5.0 POP/s on all-zero operands and well below it on codes that toggle, so
// the ceiling for a given workload has to be measured with that workload's
// codes.  The benchmark reports it next to the GEMM's own rate.
#include "../../include/muxq_measure.h"
#include "muxq_kernels.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Each wave runs `iters` rounds of 8 independent MFMAs (4 weight-side x 2
// activation-side fragments, the wave tile of the GEMM kernel).  Fragments are
// 16 bytes per lane, taken from the sample buffers at lane-dependent offsets.
__global__ __launch_bounds__(256) void k_mfma_probe(const int8_t *__restrict__ a_codes,
                                                    const int8_t *__restrict__ b_codes,
                                                    unsigned n_chunks, int iters,
                                                    long long *__restrict__ clocks, int *sink)
{
    v4i a[4], b[2];
    const unsigned t = blockIdx.x * 256u + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = *(const v4i *)(a_codes + (size_t)((t * 7u + i * 131u) % n_chunks) * 16);
#pragma unroll
    for (int i = 0; i < 2; ++i) b[i] = *(const v4i *)(b_codes + (size_t)((t * 13u + i * 257u + 5u) % n_chunks) * 16);
    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    int s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    if (s == 0x12345678) sink[0] = s;                 // keeps the accumulators alive
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clocks[0] = c1 - c0;                          // shader clocks
        clocks[1] = w1 - w0;                          // ticks of the constant 100 MHz counter
    }
}

}  // namespace

extern "C" int muxq_probe_mfma_rate(const int8_t *a_codes, const int8_t *b_codes, size_t n_bytes,
                                    int iters, int n_workgroups, int64_t *clocks_out, void *stream)
{
    if (!a_codes || !b_codes || !clocks_out) return MUXQ_ERR_NULL;
    if (n_bytes < 16 || iters < 1 || n_workgroups < 1 || n_bytes / 16 > 0xffffffffull)
        return MUXQ_ERR_PARAM;
    if (((uintptr_t)a_codes | (uintptr_t)b_codes) % 16 || (uintptr_t)clocks_out % 8) return MUXQ_ERR_ALIGN;
    // clocks_out[2] doubles as the sink word of the (never taken) keep-alive store
    const hipError_t e = muxq::launch_kernel(k_mfma_probe, dim3(n_workgroups), dim3(256), 0,
                                             (hipStream_t)stream, a_codes, b_codes,
                                             (unsigned)(n_bytes / 16), iters, (long long *)clocks_out,
                                             (int *)(clocks_out + 2));
    return e == hipSuccess ? MUXQ_OK : MUXQ_ERR_HIP;
}
