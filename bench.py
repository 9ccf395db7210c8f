#!/usr/bin/env python3
"""Benchmark of the MUXQ quantized linear layer on one MI355X.

One "step" = one muxq_linear call: the whole hot path (per-channel abs-max and
outlier detection, scale derivation, Body/Aux quantisation, Aux weight gather,
INT8 MFMA GEMM with fused Aux product and dequantising epilogue) over one batch
of synthetic outlier-bearing activations that is already resident in HBM.
Weights are quantised once, outside the timed region (offline step of Eq. 2).

Prints ONE JSON line: effective INT8 TOPS of muxq_linear (2*M*N*K / time; Aux
and padding work is not credited), the roofline of the dominant kernel (the
GEMM, timed inside the pipeline with HIP events on the launch stream), the
overhead over plain INT8, and the CPU oracle timed on this machine's host cores.
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0     # MI355X dense INT8, published
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps first; the chip needs some 20 ms of load to settle its clocks")
    ap.add_argument("--config", type=int, default=5, help="workload configuration 1..5")
    ap.add_argument("--case", type=int, default=0, help="which linear of the configuration")
    ap.add_argument("--cpu-rows", type=int, default=8192,
                    help="rows of X the CPU oracle baseline processes (0 = skip)")
    ap.add_argument("--no-detail", action="store_true")
    return ap.parse_args()


class Hip:
    """The few HIP runtime calls the bench needs for raw events."""

    def __init__(self):
        self.lib = C.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.lib.hipEventSynchronize.argtypes = [C.c_void_p]
        self.lib.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.lib.hipEventDestroy.argtypes = [C.c_void_p]

    def event(self):
        e = C.c_void_p()
        assert self.lib.hipEventCreate(C.byref(e)) == 0
        return e

    def elapsed_ms(self, a, b):
        assert self.lib.hipEventSynchronize(b) == 0
        ms = C.c_float()
        assert self.lib.hipEventElapsedTime(C.byref(ms), a, b) == 0
        return ms.value


def timed(fn, steps, torch):
    """Wall time per call over `steps` calls, device idle on both sides."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 "
              "(no collectives or sharding are built)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2604_04701_amd import binding as B
    from paper_2604_04701_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()                                   # fail loudly if the HIP library is missing
    case = synth.config_cases(args.config)[args.case]
    M, K, N, r_cap, e = case.M, case.K, case.N, case.r_cap, case.exp
    X, W, _ = synth.make_case(case)
    dev = "cuda"
    Xd, Wd = torch.from_numpy(X).to(dev), torch.from_numpy(W).to(dev)
    w_q, w_scale = B.muxq_quantize_weight(Wd, case.w_gran)
    del Wd
    ws = B.alloc_workspace(M, K, N, r_cap)
    ws0 = B.alloc_workspace(M, K, N, 0)
    Y = torch.empty((M, N), dtype=torch.float16, device=dev)
    lay = B.workspace_layout(M, K, N, r_cap)

    def step():
        B.muxq_linear(Xd, w_q, w_scale, N, case.w_gran, threshold=case.threshold, exp=e,
                      r_cap=r_cap, out=Y, workspace=ws)

    def step_naive():
        B.muxq_linear_naive_int8(Xd, w_q, w_scale, N, case.w_gran, out=Y, workspace=ws0)

    for _ in range(args.warmup):
        step()
    t_step = timed(step, args.steps, torch)
    useful_ops = 2.0 * M * N * K
    value = useful_ops / t_step / 1e12

    # ---- dominant kernel (GEMM) timed inside the pipeline, HIP events on the launch stream
    hip = Hip()
    evs = [(hip.event(), hip.event()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    for a, b in evs:
        B.muxq_set_profile_events(a, b)
        step()
    torch.cuda.synchronize()
    gemm_ms = sorted(hip.elapsed_ms(a, b) for a, b in evs)
    t_gemm = sum(gemm_ms) / len(gemm_ms) / 1e3
    n_used = int(B.ws_view(ws, lay, "n_outliers", M, N, r_cap)[0].item())
    # HBM-side bytes per GEMM launch from the committed counter runs (FETCH_SIZE / WRITE_SIZE,
    # calibrated against a plain copy); only quoted for the workload they were taken on.
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "gemm_config5_hbm_traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        if tj.get("workload") == case.name:
            traffic = tj["traffic_bytes"]
    t256, t128 = -(-M // 256) * -(-N // 256), -(-M // 128) * -(-N // 128)
    kernel = ("k_gemm_i8_persist8" if t256 >= 144 else
              "k_gemm_i8_persist4" if lay.k_pad >= 2048 or (lay.k_pad >= 1024 and 128 <= t128 <= 384)
              else "k_gemm_i8_small")
    roof = {"bound": "mfma", "kernel": kernel, "achieved": useful_ops / t_gemm / 1e12,
            "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
            "frac": useful_ops / t_gemm / 1e12 / INT8_MFMA_PEAK_TOPS, "traffic": traffic,
            "traffic_unit": "bytes per launch between the L2s and the fabric (Infinity Cache + HBM), FETCH_SIZE + WRITE_SIZE",
            "algorithmic_bytes": float(M) * K + float(N) * K + 2.0 * M * N,
            "avg_launch_ms": t_gemm * 1e3, "min_launch_ms": gemm_ms[0],
            "ops_per_launch": useful_ops}

    # ---- what the MFMA pipes alone sustain on this machine (power-limited: depends on the codes)
    ceiling = None
    if not args.no_detail:
        body_codes = ws[lay.body_q:lay.body_q + M * lay.k_pad].view(torch.int8)
        zeros = torch.zeros(1 << 20, dtype=torch.int8, device=dev)
        B.muxq_probe_mfma_rate(w_q, body_codes, iters=2000)                      # warm-up
        z_tops, z_ghz = B.muxq_probe_mfma_rate(zeros, zeros, iters=8000)
        B.muxq_probe_mfma_rate(w_q, body_codes, iters=8000)
        c_tops, c_ghz = B.muxq_probe_mfma_rate(w_q, body_codes, iters=8000)
        ceiling = {"unit": "TOP/s", "all_zero_operands": z_tops, "all_zero_shader_ghz": z_ghz,
                   "workload_codes": c_tops, "workload_codes_shader_ghz": c_ghz,
                   "gemm_frac_of_workload_ceiling": roof["achieved"] / c_tops,
                   "note": "register-only v_mfma_i32_32x32x32_i8 loop (muxq_probe_mfma_rate) on this "
                           "workload's packed weight and Body codes; the chip lowers its clock under "
                           "MFMA load on toggling data"}

    detail = {}
    if not args.no_detail:
        for _ in range(2):
            step_naive()
        t_naive = timed(step_naive, args.steps, torch)
        # operands of the stand-alone GEMM legs: the stage entry points' codes (no zero point on
        # them; the whole call's Body codes in the workspace carry one and need its correction)
        col_absmax, idx, n_o = B.muxq_detect_outliers(Xd, case.threshold, r_cap)
        body_q, aux_q, x_scale = B.muxq_build_aux(Xd, col_absmax, idx, n_o, r_cap, e)
        w_aux = B.ws_packed(ws, lay, "w_aux", M, N, r_cap)
        n_out = B.ws_view(ws, lay, "n_outliers", M, N, r_cap)

        def bare_gemm():
            B.muxq_gemm_i8(body_q, M, K, w_q, N, x_scale, w_scale, case.w_gran, out=Y)

        def aux_gemm():
            B.muxq_gemm_i8(body_q, M, K, w_q, N, x_scale, w_scale, case.w_gran, aux_q=aux_q,
                           w_aux=w_aux, n_outliers=n_out, r_cap=r_cap, exp=e, out=Y)

        for _ in range(2):
            bare_gemm()
        t_bare = timed(bare_gemm, args.steps, torch)
        t_auxg = timed(aux_gemm, args.steps, torch)
        # the per-vector setting (one activation scale per token, one weight scale per channel)
        Wd2 = torch.from_numpy(W).to(dev)
        w_q_c, w_scale_c = B.muxq_quantize_weight(Wd2, "channel")
        del Wd2

        def step_vector():
            B.muxq_linear(Xd, w_q_c, w_scale_c, N, "channel", threshold=case.threshold, exp=e,
                          r_cap=r_cap, out=Y, workspace=ws, x_gran="token")

        for _ in range(3):
            step_vector()
        t_vector = timed(step_vector, args.steps, torch)
        # static (calibrated) channel list, per-vector setting: one pass over X and the GEMM
        static_ms = None
        try:
            idx_now = B.ws_view(ws, lay, "outlier_idx", M, N, r_cap)[:n_used].clone()
            block = B.muxq_prepare_static(idx_now, K, w_q_c, N, r_cap)

            def step_static():
                B.muxq_linear_static(Xd, w_q_c, w_scale_c, N, block, "channel", exp=e, r_cap=r_cap, out=Y,
                                     workspace=ws, x_gran="token")

            for _ in range(3):
                step_static()
            static_ms = timed(step_static, args.steps, torch) * 1e3
        except Exception as ex:
            print(f"bench.py: static-list leg not timed ({type(ex).__name__}: {ex})", file=sys.stderr)
        # producer fusion: the GELU that produces a layer's input leaves the slab maxima for the
        # layer, whose own pass over its input then falls away.  Both calls run on gelu(X).
        fused_ms = unfused_ms = gelu_ms = torch_gelu_ms = None
        try:
            Xg = torch.empty_like(Xd)

            def step_on_gelu_output(ready):
                B.muxq_linear(Xg, w_q, w_scale, N, case.w_gran, threshold=case.threshold, exp=e,
                              r_cap=r_cap, out=Y, workspace=ws, absmax_ready=ready)

            B.muxq_gelu_absmax(Xd, ws, lay, out=Xg)          # Xg and its slab maxima in ws
            for _ in range(3):
                step_on_gelu_output(True)
            def chain(ready):                                # GELU, then the layer on its output
                B.muxq_gelu_absmax(Xd, ws, lay, out=Xg)
                step_on_gelu_output(ready)

            fused_ms = timed(lambda: chain(True), args.steps, torch) * 1e3
            unfused_ms = timed(lambda: chain(False), args.steps, torch) * 1e3
            gelu_ms = timed(lambda: B.muxq_gelu_absmax(Xd, ws, lay, out=Xg), args.steps, torch) * 1e3
            torch_gelu_ms = timed(lambda: torch.nn.functional.gelu(Xd, approximate="tanh"), args.steps, torch) * 1e3
            del Xg
            step()                                           # the workspace again holds X's intermediates
        except Exception as ex:
            print(f"bench.py: producer-fusion leg not timed ({type(ex).__name__}: {ex})", file=sys.stderr)
        # the same call recorded once into a HIP graph and replayed (the call is capturable:
        # four kernel launches, no allocation, memset or host synchronisation); reported
        # because on this stack a replay has so far been slower than the eager launches
        graph_ms = None
        try:
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                step()
            for _ in range(3):
                gr.replay()
            graph_ms = timed(gr.replay, args.steps, torch) * 1e3
            del gr
        except Exception as ex:
            print(f"bench.py: graph replay not timed ({type(ex).__name__}: {ex})", file=sys.stderr)
        # context only: the vendor library's plain INT8 GEMM (INT32 output, no Aux product, no
        # dequantisation) on the same Body and weight codes, through torch._int_mm
        vendor_ms = None
        try:
            a_codes = B.unpack(body_q, M, lay.k_pad)[:, :K].contiguous()
            b_codes = B.unpack(w_q, N, lay.k_pad)[:, :K].contiguous().t()       # [K, N], K-contiguous
            for _ in range(5):
                torch._int_mm(a_codes, b_codes)
            vendor_ms = timed(lambda: torch._int_mm(a_codes, b_codes), max(10, args.steps // 2), torch) * 1e3
            del a_codes, b_codes
        except Exception as ex:                       # shapes the library does not take, older torch
            vendor_ms = None
            print(f"bench.py: vendor INT8 GEMM not timed ({type(ex).__name__})", file=sys.stderr)
        t_detect = timed(lambda: B.muxq_detect_outliers(Xd, case.threshold, r_cap), args.steps, torch)
        t_build = timed(lambda: B.muxq_build_aux(Xd, col_absmax, idx, n_o, r_cap, e), args.steps, torch)
        # the same two entry points with cold caches: a 768 MiB fill between iterations evicts
        # the L2s and the 256 MB memory-side cache; one pair of events per iteration
        flush = torch.empty(768 << 20, dtype=torch.uint8, device=dev)

        def timed_cold(fn, n=12):
            ts = []
            for i in range(n):
                flush.fill_(i)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                fn()
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            ts.sort()
            return ts[len(ts) // 2] / 1e3

        t_detect_cold = timed_cold(lambda: B.muxq_detect_outliers(Xd, case.threshold, r_cap))
        t_build_cold = timed_cold(lambda: B.muxq_build_aux(Xd, col_absmax, idx, n_o, r_cap, e))
        del flush
        s1_bytes = 2.0 * M * K + 4.0 * K
        s3_bytes = 3.0 * M * K + 1.0 * M * r_cap
        detail = {
            "outlier_channels_found": n_used,
            "ms_muxq_linear": t_step * 1e3, "ms_naive_int8_linear": t_naive * 1e3,
            "ms_bare_gemm": t_bare * 1e3, "ms_gemm_with_aux": t_auxg * 1e3,
            "ms_muxq_linear_per_token_x_per_channel_w": t_vector * 1e3,
            "overhead_vs_naive_pipeline": t_step / t_naive - 1.0,
            "overhead_vs_bare_gemm": t_step / t_bare - 1.0,
            "bare_gemm_tops": useful_ops / t_bare / 1e12,
            "bare_gemm_frac_of_int8_peak": useful_ops / t_bare / 1e12 / INT8_MFMA_PEAK_TOPS,
            "detect_outliers_ms": t_detect * 1e3, "detect_GBs": s1_bytes / t_detect / 1e9,
            "detect_frac_of_hbm": s1_bytes / t_detect / 1e9 / HBM_PEAK_GBS,
            "build_aux_ms": t_build * 1e3, "build_aux_GBs": s3_bytes / t_build / 1e9,
            "build_aux_frac_of_hbm": s3_bytes / t_build / 1e9 / HBM_PEAK_GBS,
            "ms_vendor_int8_gemm_int32_out": vendor_ms, "ms_muxq_linear_graph_replay": graph_ms,
            "ms_muxq_linear_static_list_per_token_x_per_channel_w": static_ms,
            "ms_gelu_then_muxq_linear": unfused_ms,
            "ms_gelu_then_muxq_linear_absmax_from_producer": fused_ms,
            "ms_gelu_with_absmax": gelu_ms, "ms_torch_gelu_tanh": torch_gelu_ms,
            "detect_outliers_cold_ms": t_detect_cold * 1e3, "detect_cold_GBs": s1_bytes / t_detect_cold / 1e9,
            "build_aux_cold_ms": t_build_cold * 1e3, "build_aux_cold_GBs": s3_bytes / t_build_cold / 1e9,
            "note": "detect/build timings are whole entry points (2-3 small launches each), warm caches",
        }

    cpu = None
    if args.cpu_rows > 0:
        from oracle import muxq_oracle as orc
        rows = min(args.cpu_rows, M)
        Xs = np.ascontiguousarray(X[:rows])
        wpack = orc.quantize_weight(W, case.w_gran)          # offline step, not timed
        t0 = time.perf_counter()
        o = orc.linear(Xs, wpack=wpack, threshold=case.threshold, e=e, r_cap=r_cap)
        t_cpu = time.perf_counter() - t0
        cpu = {"value": 2.0 * rows * N * K / t_cpu / 1e12, "unit": "TOP/s", "cores": orc.n_threads(),
               "kind": "oracle", "seconds": t_cpu,
               "sample": f"first {rows} of {M} rows of X through the whole activation-side path "
                         f"(detect, Body/Aux, quantise, INT32 products, dequantise); weights pre-quantised"}
        # the sample doubles as a parity spot check of the GPU result (scales differ: sample vs full X,
        # so only shapes/finite-ness are asserted here; parity proper lives in tests/)
        assert np.isfinite(o["y32"]).all()

    out = {
        "metric": "muxq_linear effective INT8 TOPS + % MFMA peak; overhead vs plain INT8 GEMM",
        "value": value, "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config {args.config}: {case.name}, X {M}x{K} fp16 with {case.r} "
                               f"outlier channels, W {K}x{N}, per-{case.w_gran} INT8, exp={e}, "
                               f"threshold={case.threshold}, r_cap={r_cap}",
                   "M": M, "K": K, "N": N},
        "frac_of_int8_mfma_peak": value / INT8_MFMA_PEAK_TOPS,
        "roofline": roof, "cpu_baseline": cpu, "mfma_ceiling": ceiling, "detail": detail,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
