#!/usr/bin/env python3
"""Benchmark of the MUXQ quantized linear layer on one MI355X.

One "step" = one muxq_linear call: the whole hot path (per-channel abs-max and
outlier detection, scale derivation, Body/Aux quantisation, Aux weight gather,
INT8 MFMA GEMM with fused Aux product and dequantising epilogue) over one batch
of synthetic outlier-bearing activations that is already resident in HBM.
Weights are quantised once, outside the timed region (offline step of Eq. 2).

Timing protocol.  An idle chip needs tens of milliseconds of load before its
clocks reach their working state, so the run first repeats the step until at
least 50 ms of GPU time have passed (`settle_ms`), then does the --warmup steps,
then times exactly --steps steps between two device synchronisations
(`ms_per_step`).  The figure of the first --steps steps on the idle chip is
kept as `ms_per_step_cold_start`.  The three legs of the overhead figures
(muxq_linear, the naive INT8 pipeline, the bare GEMM) are timed interleaved,
A B C A B C ..., with one pair of events per call, and compared by their
medians, so that all three see the same clock state.

Prints ONE JSON line: effective INT8 TOPS of muxq_linear (2*M*N*K / time; Aux
and padding work is not credited), the roofline of the dominant kernel (the
GEMM, timed inside the pipeline with HIP events on the launch stream), the
overhead over plain INT8, the CPU oracle timed on this machine's host cores, and the
comparison of the GPU result with that oracle run (exit status 1 if it fails).
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
Y_REL_TOL = 1e-2                 # max |Y_gpu - Y_oracle| <= 1e-2 * max |Y_fp32|


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50, help="untimed steps right before the timed ones")
    ap.add_argument("--settle-ms", type=float, default=50.0,
                    help="GPU time of untimed steps before the warm-up, for the clocks to settle")
    ap.add_argument("--config", type=int, default=5, help="workload configuration 1..5")
    ap.add_argument("--case", type=int, default=0, help="which linear of the configuration")
    ap.add_argument("--cpu-rows", type=int, default=8192,
                    help="rows of Y the CPU oracle baseline computes and the GPU result is checked on (0 = skip)")
    ap.add_argument("--no-detail", action="store_true")
    ap.add_argument("--cold-streaming", type=int, default=0, metavar="N",
                    help="run ONLY N rounds of {768 MiB fill, muxq_detect_outliers, 768 MiB fill, "
                         "muxq_build_aux} (plus N warm rounds without the fills) and print their timings: "
                         "the command a kernel trace of the two streaming passes on cold caches is taken with")
    ap.add_argument("--cold-flush", choices=["read", "write"], default="read")
    ap.add_argument("--cold-rows", type=int, default=0, metavar="M",
                    help="with --cold-streaming: M rows of activations of the configuration's recipe instead "
                         "of its own M (e.g. 262144 rows of 4096 channels = 2 GiB, eight times the "
                         "memory-side cache: every pass then streams from HBM whatever ran before)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this size (a dispatch of known traffic, "
                         "for scaling the FETCH_SIZE / WRITE_SIZE counters of a profiler run)")
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


def median(v):
    v = sorted(v)
    n = len(v)
    return v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def interleaved(legs, rounds, torch, batch=1):
    """legs: {name: fn}.  Runs the legs round-robin `rounds` times, one pair of events per leg and
    round on the launch stream (around `batch` back-to-back calls of the leg), nothing else in
    between; returns {name: median seconds per call}."""
    names = list(legs)
    evs = {n: [] for n in names}
    for n in names:                       # one untimed pass: lazy loading, caches
        legs[n]()
    torch.cuda.synchronize()
    for _ in range(rounds):
        for n in names:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _i in range(batch):
                legs[n]()
            b.record()
            evs[n].append((a, b))
    torch.cuda.synchronize()
    return {n: median([a.elapsed_time(b) for a, b in evs[n]]) / 1e3 / batch for n in names}


def cold_streaming(args, case, Xd, B, torch):
    """The two streaming passes over X (S1: channel maxima and outlier list; S3: Body / Aux
    quantisation) with the caches emptied before every call, then warm.  Prints one JSON line."""
    M, K = Xd.shape
    r_cap, e = case.r_cap, case.exp
    # Emptying the caches: READING 768 MiB of other data replaces what the L2s and the 256 MB
    # memory-side cache hold with clean lines.  (Writing that much instead leaves them full of
    # dirty lines, and the pass under test then also pays for their write-back: it measures
    # about half the rate.  --cold-flush write shows that figure.)
    flush = torch.zeros(768 << 18, dtype=torch.int32, device=Xd.device)
    col_absmax, idx, n_o = B.muxq_detect_outliers(Xd, case.threshold, r_cap)
    B.muxq_build_aux(Xd, col_absmax, idx, n_o, r_cap, e)

    def once(fn, cold, i):
        if cold and args.cold_flush == "write":
            flush.fill_(i & 255)
        elif cold:
            flush.sum()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b)

    res = {}
    for cold in (True, False):
        td, tb = [], []
        for i in range(args.cold_streaming):
            td.append(once(lambda: B.muxq_detect_outliers(Xd, case.threshold, r_cap), cold, 2 * i))
            tb.append(once(lambda: B.muxq_build_aux(Xd, col_absmax, idx, n_o, r_cap, e), cold, 2 * i + 1))
        tag = "cold" if cold else "warm"
        res[f"detect_outliers_{tag}_ms"], res[f"build_aux_{tag}_ms"] = median(td), median(tb)
    s1, s3 = 2.0 * M * K + 4.0 * K, 3.0 * M * K + 1.0 * M * r_cap
    res.update(workload=case.name, M=M, K=K, s1_algorithmic_bytes=s1, s3_algorithmic_bytes=s3,
               detect_cold_GBs=s1 / res["detect_outliers_cold_ms"] / 1e6,
               build_aux_cold_GBs=s3 / res["build_aux_cold_ms"] / 1e6,
               flush=args.cold_flush,
               note="whole entry points (2 launches each) timed with events; per-kernel durations come "
                    "from a kernel trace of this command: the first N dispatches of each kernel are cold")
    print(json.dumps(res))


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
    B.muxq_init()
    case = synth.config_cases(args.config)[args.case]
    if args.cold_streaming > 0 and args.cold_rows > 0:
        # the same recipe on more rows, generated on the device (2 GiB from the host generator
        # would take minutes): N(0,1) with the case's outlier channels and gains
        import dataclasses
        case = dataclasses.replace(case, M=args.cold_rows, name=f"{case.name}_rows{args.cold_rows}")
        g = torch.Generator(device="cuda").manual_seed(case.seed)
        Xd = torch.randn((case.M, case.K), generator=g, device="cuda", dtype=torch.float16)
        rng = np.random.default_rng(case.seed)
        ch = np.sort(rng.choice(case.K, size=min(case.r, case.K), replace=False))
        lo, hi = case.gain
        gains = rng.uniform(lo, hi, size=len(ch)) if lo != hi else np.full(len(ch), lo)
        Xd[:, torch.from_numpy(ch).cuda()] *= torch.from_numpy(gains.astype(np.float16)).cuda()
        cold_streaming(args, case, Xd, B, torch)
        return
    M, K, N, r_cap, e = case.M, case.K, case.N, case.r_cap, case.exp
    X, W, _ = synth.make_case(case)
    dev = "cuda"
    Xd, Wd = torch.from_numpy(X).to(dev), torch.from_numpy(W).to(dev)
    w_q, w_scale = B.muxq_quantize_weight(Wd, case.w_gran)
    del Wd
    if args.cold_streaming > 0:
        cold_streaming(args, case, Xd, B, torch)
        return
    ws = B.alloc_workspace(M, K, N, r_cap)
    ws0 = B.alloc_workspace(M, K, N, 0)
    Y = torch.empty((M, N), dtype=torch.float16, device=dev)
    Y2 = torch.empty((M, N), dtype=torch.float16, device=dev)     # output of the comparison legs
    lay = B.workspace_layout(M, K, N, r_cap)

    def step():
        B.muxq_linear(Xd, w_q, w_scale, N, case.w_gran, threshold=case.threshold, exp=e,
                      r_cap=r_cap, out=Y, workspace=ws)

    def step_naive():
        B.muxq_linear_naive_int8(Xd, w_q, w_scale, N, case.w_gran, out=Y2, workspace=ws0)

    # The dominant kernel is timed inside the pipeline with pairs of HIP events recorded on the
    # launch stream around the GEMM kernel (muxq_linear_timed = muxq_linear plus the two event
    # records), over --steps calls that follow the timed region back to back, with nothing but
    # a synchronisation in between.  (The timed region itself runs plain muxq_linear: two host
    # event records per call are a visible share of a 25 us call on the small configurations.)
    hip = Hip()
    evs = [(hip.event(), hip.event()) for _ in range(args.steps)]
    wg_ticks = torch.zeros(2048, dtype=torch.int64, device=dev)
    Y_result = torch.empty_like(Y)

    def gemm_event_steps():
        for a, b in evs:
            B.muxq_linear_timed(Xd, w_q, w_scale, N, a, b, case.w_gran, threshold=case.threshold,
                                exp=e, r_cap=r_cap, out=Y, workspace=ws)
        torch.cuda.synchronize()
        return sorted(hip.elapsed_ms(a, b) for a, b in evs)

    torch.cuda.synchronize()
    # ---- the figure an idle chip gives (first calls after start-up), kept for reference
    step()
    t_cold_start = timed(step, args.steps, torch)
    gemm_ms_cold = gemm_event_steps()
    # ---- settle: repeat the step until enough GPU time has passed
    settle_calls, t_settle = 0, 0.0
    chunk = max(1, int(0.010 / max(t_cold_start, 1e-6)))
    while t_settle < args.settle_ms * 1e-3:
        t_settle += timed(step, chunk, torch) * chunk
        settle_calls += chunk
    # ---- warm-up, then exactly --steps timed steps, then the same number with the GEMM's events
    for _ in range(args.warmup):
        step()
    t_step = timed(step, args.steps, torch)
    gemm_ms = gemm_event_steps()
    Y_result.copy_(Y)                          # what the parity check below compares
    useful_ops = 2.0 * M * N * K
    value = useful_ops / t_step / 1e12
    t_gemm = sum(gemm_ms) / len(gemm_ms) / 1e3
    # one more call that also exports when each workgroup of the GEMM started and ended
    a, b = evs[0]
    B.muxq_linear_timed(Xd, w_q, w_scale, N, a, b, case.w_gran, threshold=case.threshold, exp=e,
                        r_cap=r_cap, out=Y, workspace=ws, wg_ticks=wg_ticks)
    torch.cuda.synchronize()
    n_used = int(B.ws_view(ws, lay, "n_outliers", M, N, r_cap)[0].item())
    t256, t128 = -(-M // 256) * -(-N // 256), -(-M // 128) * -(-N // 128)
    kernel = ("k_gemm_i8_persist8" if t256 >= 144 else
              "k_gemm_i8_persist4" if lay.k_pad >= 2048 or (lay.k_pad >= 1024 and 128 <= t128 <= 384)
              else "k_gemm_i8_small")
    # how evenly the 8 XCDs finish (last call; workgroup i runs on XCD i % 8; ticks of 10 ns)
    xcd = None
    tk = wg_ticks.cpu().numpy().reshape(-1, 2)
    live = tk[:, 1] > 0
    if kernel != "k_gemm_i8_small" and live.any():
        t0 = tk[live, 0].min()
        on = lambda x: live & (np.arange(len(tk)) % 8 == x)
        xs = [x for x in range(8) if on(x).any()]
        ends = [float((tk[on(x), 1] - t0).max()) / 100.0 for x in xs]
        starts = [float((tk[on(x), 0] - t0).max()) / 100.0 for x in xs]
        xcd = {"end_us_after_first_start": ends, "last_start_us": starts,
               "spread_frac": (max(ends) - min(ends)) / max(ends), "kernel_us_by_ticks": max(ends)}
    # HBM-side bytes per GEMM launch come from profiler runs of this same command (FETCH_SIZE /
    # WRITE_SIZE counters scaled by a plain copy); quoted with their source, only for the
    # workload they were taken on, and never measured inside this run.
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "gemm_config5_hbm_traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        if tj.get("workload") == case.name:
            traffic, traffic_src = tj["traffic_bytes"], "profiles/gemm_config5_hbm_traffic.txt (rocprofv3 --pmc runs; not measured in this run)"
    roof = {"bound": "mfma", "kernel": kernel, "achieved": useful_ops / t_gemm / 1e12,
            "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
            "frac": useful_ops / t_gemm / 1e12 / INT8_MFMA_PEAK_TOPS, "traffic": traffic,
            "traffic_source": traffic_src,
            "traffic_unit": "bytes per launch between the L2s and the fabric (Infinity Cache + HBM), FETCH_SIZE + WRITE_SIZE",
            "algorithmic_bytes": float(M) * K + float(N) * K + 2.0 * M * N,
            "avg_launch_ms": t_gemm * 1e3, "min_launch_ms": gemm_ms[0], "max_launch_ms": gemm_ms[-1],
            "avg_launch_ms_cold_start": sum(gemm_ms_cold) / len(gemm_ms_cold),
            "ops_per_launch": useful_ops, "xcd_finish": xcd}

    if args.calibration_copy_mib > 0:
        n = args.calibration_copy_mib << 20
        src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

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
        # operands of the stand-alone GEMM legs.  (1) the codes of the stage entry points (plain
        # codes, correct Y); (2) the very bytes the GEMM inside muxq_linear reads: the workspace's
        # Body codes, whose unlisted channels carry the call's zero point -- muxq_gemm_i8 has no
        # correction for it, so that leg's Y is not the layer's output and goes to a spare buffer;
        # it is the like-for-like reference of overhead (B): same kernel, same operand bytes.
        col_absmax, idx, n_o = B.muxq_detect_outliers(Xd, case.threshold, r_cap)
        body_q, aux_q, x_scale = B.muxq_build_aux(Xd, col_absmax, idx, n_o, r_cap, e)
        w_aux = B.ws_packed(ws, lay, "w_aux", M, N, r_cap)
        n_out = B.ws_view(ws, lay, "n_outliers", M, N, r_cap)
        step()
        ws_body = B.ws_packed(ws, lay, "body_q", M, N, r_cap)
        ws_xscale = B.ws_view(ws, lay, "x_scale", M, N, r_cap)

        def bare_gemm():
            B.muxq_gemm_i8(ws_body, M, K, w_q, N, ws_xscale, w_scale, case.w_gran, out=Y2)

        def bare_gemm_plain():
            B.muxq_gemm_i8(body_q, M, K, w_q, N, x_scale, w_scale, case.w_gran, out=Y2)

        def aux_gemm():
            B.muxq_gemm_i8(body_q, M, K, w_q, N, x_scale, w_scale, case.w_gran, aux_q=aux_q,
                           w_aux=w_aux, n_outliers=n_out, r_cap=r_cap, exp=e, out=Y2)

        rounds = max(10, args.steps)
        # calls of well under 0.1 ms are bound by the host's launches: a pair of events per call
        # would then time the host's gaps, so such legs are timed in batches of 8 calls
        batch = 8 if t_step < 1e-4 else 1
        t3 = interleaved({"muxq": step, "naive": step_naive, "bare": bare_gemm,
                          "bare_plain": bare_gemm_plain, "aux": aux_gemm}, rounds, torch, batch)
        # the per-vector setting (one activation scale per token, one weight scale per channel)
        Wd2 = torch.from_numpy(W).to(dev)
        w_q_c, w_scale_c = B.muxq_quantize_weight(Wd2, "channel")
        del Wd2

        def step_vector():
            B.muxq_linear(Xd, w_q_c, w_scale_c, N, "channel", threshold=case.threshold, exp=e,
                          r_cap=r_cap, out=Y2, workspace=ws, x_gran="token")

        for _ in range(3):
            step_vector()
        t_vector = timed(step_vector, args.steps, torch)
        # static (calibrated) channel list, per-vector setting: one pass over X and the GEMM
        static_ms = None
        try:
            idx_now = B.ws_view(ws, lay, "outlier_idx", M, N, r_cap)[:n_used].clone()
            block = B.muxq_prepare_static(idx_now, K, w_q_c, N, r_cap)

            def step_static():
                B.muxq_linear_static(Xd, w_q_c, w_scale_c, N, block, "channel", exp=e, r_cap=r_cap, out=Y2,
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
                              r_cap=r_cap, out=Y2, workspace=ws, absmax_ready=ready)

            def chain(ready):                                # GELU, then the layer on its output
                B.muxq_gelu_absmax(Xd, ws, lay, out=Xg)
                step_on_gelu_output(ready)

            tg = interleaved({"fused": lambda: chain(True), "unfused": lambda: chain(False),
                              "gelu": lambda: B.muxq_gelu_absmax(Xd, ws, lay, out=Xg),
                              "torch_gelu": lambda: torch.nn.functional.gelu(Xd, approximate="tanh")},
                             max(10, args.steps // 2), torch)
            fused_ms, unfused_ms = tg["fused"] * 1e3, tg["unfused"] * 1e3
            gelu_ms, torch_gelu_ms = tg["gelu"] * 1e3, tg["torch_gelu"] * 1e3
            del Xg
        except Exception as ex:
            print(f"bench.py: producer-fusion leg not timed ({type(ex).__name__}: {ex})", file=sys.stderr)
        # the MLP pair of a GPT-2 block (Sec. IV-C): this workload as c_fc, the GELU, then c_proj
        # (N -> K).  unfused: layer, GELU kernel (hands the maxima over), layer; fused: the GELU
        # in the first GEMM's epilogue, the maxima from its tiles; plain: nothing handed over.
        mlp = None
        if N == 4 * K:
            try:
                W2 = synth.make_w(N, K, np.random.default_rng(case.seed + 77))
                w_q2, w_scale2 = B.muxq_quantize_weight(torch.from_numpy(W2).to(dev), case.w_gran)
                del W2
                b1 = torch.zeros(N, dtype=torch.float16, device=dev)
                ws2 = B.alloc_workspace(M, N, K, r_cap)
                lay2 = B.workspace_layout(M, N, K, r_cap)
                Hb = torch.empty((M, N), dtype=torch.float16, device=dev)
                Yo = torch.empty((M, K), dtype=torch.float16, device=dev)
                kw = dict(threshold=case.threshold, exp=e, r_cap=r_cap)
                n_sl = B.lib().muxq_linear_gelu_slabs(M, K, N)

                def mlp_plain():
                    B.muxq_linear(Xd, w_q, w_scale, N, case.w_gran, bias=b1, out=Hb, workspace=ws, **kw)
                    torch.nn.functional.gelu(Hb, approximate="tanh")
                    B.muxq_linear(Hb, w_q2, w_scale2, K, case.w_gran, out=Yo, workspace=ws2, **kw)

                def mlp_unfused():
                    B.muxq_linear(Xd, w_q, w_scale, N, case.w_gran, bias=b1, out=Hb, workspace=ws, **kw)
                    B.muxq_gelu_absmax(Hb, ws2, lay2, out=Hb)
                    B.muxq_linear(Hb, w_q2, w_scale2, K, case.w_gran, out=Yo, workspace=ws2,
                                  absmax_ready=True, **kw)

                def mlp_fused():
                    B.muxq_linear_gelu(Xd, w_q, w_scale, N, case.w_gran, bias=b1, out=Hb, workspace=ws,
                                       next_workspace=ws2, next_layout=lay2, **kw)
                    B.muxq_linear(Hb, w_q2, w_scale2, K, case.w_gran, out=Yo, workspace=ws2,
                                  absmax_ready=True, absmax_slabs=n_sl, **kw)

                _, _, ws_mlp = B.muxq_mlp(Xd, w_q, w_scale, N, w_q2, w_scale2, K, case.w_gran, bias1=b1,
                                          out_h=Hb, out=Yo, **kw)

                def mlp_one_call():
                    B.muxq_mlp(Xd, w_q, w_scale, N, w_q2, w_scale2, K, case.w_gran, bias1=b1, out_h=Hb,
                               out=Yo, workspace=ws_mlp, **kw)

                tm = interleaved({"plain": mlp_plain, "unfused": mlp_unfused, "fused": mlp_fused,
                                  "one_call": mlp_one_call}, max(10, args.steps // 2), torch, batch)
                mlp = {"shape": f"{M} x {K} -> {N} -> {K}", "slabs_from_gemm": n_sl,
                       "ms_two_layers_and_torch_gelu": tm["plain"] * 1e3,
                       "ms_two_layers_and_gelu_kernel_handing_maxima_over": tm["unfused"] * 1e3,
                       "ms_gelu_fused_into_first_gemm": tm["fused"] * 1e3,
                       "ms_muxq_mlp_one_call": tm["one_call"] * 1e3,
                       "fused_vs_plain": tm["fused"] / tm["plain"]}
                del w_q2, ws2, Hb, Yo, ws_mlp
                step()
            except Exception as ex:
                print(f"bench.py: MLP leg not timed ({type(ex).__name__}: {ex})", file=sys.stderr)
        # the same call recorded once into a HIP graph and replayed (the call is capturable:
        # four kernel launches, no allocation, memset or host synchronisation); reported
        # because on this stack a replay has so far been slower than the eager launches
        graph_ms = None
        try:
            step()
            torch.cuda.synchronize()
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
        # The same GEMM kernel on all-zero operand codes: nothing toggles in the matrix pipes, the
        # chip keeps its clock, and what is left is what the kernel's structure allows (operand
        # feed, LDS, barriers, epilogue, stores).  The gap to the workload's codes is the power limit.
        zero_ms = None
        try:
            zb, zw = torch.zeros_like(body_q), torch.zeros_like(w_q)

            def gemm_zero():
                B.muxq_gemm_i8(zb, M, K, zw, N, x_scale, w_scale, case.w_gran, out=Y2)
            n_z = max(20, args.steps)
            for _ in range(n_z):                       # lets the clock come up
                gemm_zero()
            zero_ms = interleaved({"zero": gemm_zero}, n_z, torch, batch)["zero"] * 1e3
            del zb, zw
            for _ in range(10):                        # back to the workload's clock state
                step()
        except Exception as ex:
            print(f"bench.py: zero-code GEMM not timed ({type(ex).__name__}: {ex})", file=sys.stderr)
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
            return median(ts) / 1e3

        t_detect_cold = timed_cold(lambda: B.muxq_detect_outliers(Xd, case.threshold, r_cap))
        t_build_cold = timed_cold(lambda: B.muxq_build_aux(Xd, col_absmax, idx, n_o, r_cap, e))
        del flush
        step()                                           # the workspace again holds X's intermediates
        s1_bytes = 2.0 * M * K + 4.0 * K
        s3_bytes = 3.0 * M * K + 1.0 * M * r_cap
        detail = {
            "outlier_channels_found": n_used,
            "interleaved_rounds": rounds, "interleaved_batch": batch,
            "ms_muxq_linear": t3["muxq"] * 1e3, "ms_naive_int8_linear": t3["naive"] * 1e3,
            "ms_bare_gemm": t3["bare"] * 1e3, "ms_bare_gemm_plain_codes": t3["bare_plain"] * 1e3,
            "ms_gemm_with_aux": t3["aux"] * 1e3,
            "ms_bare_gemm_all_zero_codes": zero_ms,
            "bare_gemm_all_zero_codes_frac_of_int8_peak":
                (useful_ops / (zero_ms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS) if zero_ms else None,
            "ms_muxq_linear_per_token_x_per_channel_w": t_vector * 1e3,
            "overhead_vs_naive_pipeline": t3["muxq"] / t3["naive"] - 1.0,
            "overhead_vs_bare_gemm": t3["muxq"] / t3["bare"] - 1.0,
            "overhead_vs_bare_gemm_plain_codes": t3["muxq"] / t3["bare_plain"] - 1.0,
            "bare_gemm_tops": useful_ops / t3["bare"] / 1e12,
            "bare_gemm_frac_of_int8_peak": useful_ops / t3["bare"] / 1e12 / INT8_MFMA_PEAK_TOPS,
            "detect_outliers_ms": t_detect * 1e3, "detect_GBs_cache_resident": s1_bytes / t_detect / 1e9,
            "build_aux_ms": t_build * 1e3, "build_aux_GBs_cache_resident": s3_bytes / t_build / 1e9,
            "ms_vendor_int8_gemm_int32_out": vendor_ms, "ms_muxq_linear_graph_replay": graph_ms,
            "ms_muxq_linear_static_list_per_token_x_per_channel_w": static_ms,
            "ms_gelu_then_muxq_linear": unfused_ms,
            "ms_gelu_then_muxq_linear_absmax_from_producer": fused_ms,
            "ms_gelu_with_absmax": gelu_ms, "ms_torch_gelu_tanh": torch_gelu_ms, "mlp": mlp,
            "detect_outliers_cold_ms": t_detect_cold * 1e3, "detect_cold_GBs": s1_bytes / t_detect_cold / 1e9,
            "detect_cold_frac_of_hbm": s1_bytes / t_detect_cold / 1e9 / HBM_PEAK_GBS,
            "build_aux_cold_ms": t_build_cold * 1e3, "build_aux_cold_GBs": s3_bytes / t_build_cold / 1e9,
            "build_aux_cold_frac_of_hbm": s3_bytes / t_build_cold / 1e9 / HBM_PEAK_GBS,
            "note": "the muxq / naive / bare-GEMM legs are medians of event-timed calls run round-robin; "
                    "ms_bare_gemm runs muxq_gemm_i8 on the operand bytes of the GEMM inside muxq_linear "
                    "(Body codes with the call's zero point), ms_bare_gemm_plain_codes on the stage entry "
                    "points' plain codes; detect/build timings are whole entry points (2-3 small launches "
                    "each): warm = X resident in the 256 MB memory-side cache, cold = after a 768 MiB fill",
        }

    cpu, parity, ok = None, None, True
    if args.cpu_rows > 0:
        from oracle import muxq_oracle as orc
        rows = min(args.cpu_rows, M)
        sel = np.arange(rows)
        wpack = orc.quantize_weight(W, case.w_gran)          # offline step, not timed
        t0 = time.perf_counter()
        o = orc.linear(X, wpack=wpack, threshold=case.threshold, e=e, r_cap=r_cap,
                       rows=None if rows == M else sel)
        t_cpu = time.perf_counter() - t0
        cpu = {"value": 2.0 * rows * N * K / t_cpu / 1e12, "unit": "TOP/s", "cores": orc.n_threads(),
               "kind": "oracle", "seconds": t_cpu,
               "sample": f"whole activation-side path on all {M} rows of X (detect, Body/Aux, quantise), "
                         f"then INT32 products, recombination and dequantisation of the first {rows} "
                         f"rows of Y; weights pre-quantised"}
        # the same run is the parity check of the timed GPU result: every element of those rows
        yg = Y_result[:rows].cpu().numpy()
        y32, y16 = o["y32"], o["y16"]
        tol = Y_REL_TOL * float(np.abs(y32).max())
        err = float(np.abs(yg.astype(np.float32) - y32).max())
        mism = int((yg != y16).sum())
        n_ok = int(o["n_used"]) == n_used
        ok = bool(err <= tol and np.isfinite(yg).all() and n_ok)
        parity = {"rows_compared": rows, "elements": int(yg.size), "max_abs_err": err, "tol": tol,
                  "mismatched_fp16": mism, "outlier_channels_oracle": int(o["n_used"]),
                  "outlier_channels_gpu": n_used, "pass": ok}

    out = {
        "metric": "muxq_linear effective INT8 TOPS + % MFMA peak; overhead vs plain INT8 GEMM",
        "value": value, "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config {args.config}: {case.name}, X {M}x{K} fp16 with {case.r} "
                               f"outlier channels, W {K}x{N}, per-{case.w_gran} INT8, exp={e}, "
                               f"threshold={case.threshold}, r_cap={r_cap}",
                   "M": M, "K": K, "N": N},
        "settle_ms": t_settle * 1e3, "settle_calls": settle_calls,
        "ms_per_step_cold_start": t_cold_start * 1e3,
        "frac_of_int8_mfma_peak": value / INT8_MFMA_PEAK_TOPS,
        "roofline": roof, "cpu_baseline": cpu, "parity": parity, "mfma_ceiling": ceiling, "detail": detail,
    }
    print(json.dumps(out))
    if not ok:
        print("bench.py: the GPU result does not match the oracle", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
