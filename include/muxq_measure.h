/*
 * muxq_measure.h -- measurement aids of the MUXQ library (same shared object, same
 * conventions as muxq.h).  Nothing here is part of the layer: a benchmark uses these to time
 * the dominant kernel inside the whole call and to find what the matrix pipes of the box at
 * hand can sustain.  Product code includes muxq.h only.
 */
#ifndef MUXQ_MEASURE_H
#define MUXQ_MEASURE_H

#include "muxq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* muxq_linear_opts with two caller-owned hipEvent_t handles (passed as void*, both non-NULL):
 * `gemm_start` is recorded on `stream` immediately before, `gemm_stop` immediately after, the
 * GEMM kernel of the call, so that the dominant kernel can be timed inside the pipeline on
 * the stream it runs on.  wg_ticks: NULL, or device int64[2048]: when the GEMM runs as one of
 * the persistent kernels (at most 1024 workgroups, workgroup i on XCD i % 8), workgroup i
 * stores the constant 100 MHz counter at its start in [2 i] and at its end in [2 i + 1]
 * (entries of workgroups that do not exist are left alone), which shows how evenly the XCDs
 * finish.  No state is kept between calls. */
int muxq_linear_timed(const void *X_fp16, int M, int K, int ldx, const int8_t *w_q,
                      const float *w_scale, int w_gran, int N, const void *bias_fp16,
                      float threshold, int exp, int r_cap, void *Y_fp16, int ldy,
                      void *workspace, size_t workspace_bytes, const muxq_act_opts *opts,
                      void *gemm_start, void *gemm_stop, int64_t *wg_ticks, void *stream);

/* The issue rate of the INT8 MFMA instruction the GEMM uses (v_mfma_i32_32x32x32_i8) with
 * operands held in registers and nothing else running, on operand codes sampled from
 * a_codes / b_codes (device pointers, 16-byte aligned, n_bytes >= 16 each).  The matrix pipes
 * of this chip are power-limited, so the ceiling depends on the codes; a benchmark passes the
 * packed weight and Body codes of its workload.  Enqueues one kernel of n_workgroups x 4
 * waves, each running `iters` rounds of 8 MFMAs: n_workgroups * 4 * iters * 8 * 65536
 * operations in all (time it with events).  clocks_out: device int64[3]; [0] receives the
 * shader clocks and [1] the ticks of the constant 100 MHz counter spent by one wave, [2] is
 * scratch. */
int muxq_probe_mfma_rate(const int8_t *a_codes, const int8_t *b_codes, size_t n_bytes,
                         int iters, int n_workgroups, int64_t *clocks_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MUXQ_MEASURE_H */
