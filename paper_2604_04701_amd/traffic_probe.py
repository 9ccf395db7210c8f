"""Workload for the profiler runs (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, --kernel-trace).

Runs a plain device-to-device copy of known size (the calibration dispatch:
`bytes` read and `bytes` written) and then a few muxq_linear calls on one
workload configuration, so that one counter run holds both.  Usage:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -o fetch -- \
        python3 -m paper_2604_04701_amd.traffic_probe --config 5

--setting picks what is called after the copy: the per-tensor layer (default), the
per-vector setting (per-token activation scales, per-channel weight scales), the same
with a static channel list, or the GELU producer followed by the layer that starts from
its channel maxima.  --no-copy leaves the calibration copy out (kernel traces).
"""
import argparse

import torch

from . import binding as B
from . import synth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--case", type=int, default=0)
    ap.add_argument("--iters", type=int, default=3)
    ap.add_argument("--copy-mib", type=int, default=512)
    ap.add_argument("--setting", choices=["tensor", "vector", "vector-static", "gelu"], default="tensor")
    ap.add_argument("--no-copy", action="store_true")
    args = ap.parse_args()
    case = synth.config_cases(args.config)[args.case]
    X, W, _ = synth.make_case(case)
    Xd, Wd = torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda()
    w_gran = case.w_gran if args.setting in ("tensor", "gelu") else "channel"
    w_q, w_scale = B.muxq_quantize_weight(Wd, w_gran)
    ws = B.alloc_workspace(case.M, case.K, case.N, case.r_cap)
    lay = B.workspace_layout(case.M, case.K, case.N, case.r_cap)
    Y = torch.empty((case.M, case.N), dtype=torch.float16, device="cuda")
    kw = dict(threshold=case.threshold, exp=case.exp, r_cap=case.r_cap, out=Y, workspace=ws)
    block = Xg = None
    if args.setting == "vector-static":
        B.muxq_linear(Xd, w_q, w_scale, case.N, w_gran, **kw)
        n_used = int(B.ws_view(ws, lay, "n_outliers", case.M, case.N, case.r_cap)[0].item())
        found = B.ws_view(ws, lay, "outlier_idx", case.M, case.N, case.r_cap)[:n_used].clone()
        block = B.muxq_prepare_static(found, case.K, w_q, case.N, case.r_cap)
    if args.setting == "gelu":
        Xg = torch.empty_like(Xd)
    if not args.no_copy:
        src = torch.empty(args.copy_mib << 20, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(args.iters):
        if not args.no_copy:
            dst.copy_(src)                   # calibration: copy_mib MiB in, copy_mib MiB out
            torch.cuda.synchronize()
        if args.setting == "tensor":
            B.muxq_linear(Xd, w_q, w_scale, case.N, w_gran, **kw)
        elif args.setting == "vector":
            B.muxq_linear(Xd, w_q, w_scale, case.N, w_gran, x_gran="token", **kw)
        elif args.setting == "vector-static":
            B.muxq_linear_static(Xd, w_q, w_scale, case.N, block, w_gran, exp=case.exp, r_cap=case.r_cap,
                                 out=Y, workspace=ws, x_gran="token")
        else:
            B.muxq_gelu_absmax(Xd, ws, lay, out=Xg)
            B.muxq_linear(Xg, w_q, w_scale, case.N, w_gran, absmax_ready=True, **kw)
        if not args.no_copy:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    print(f"traffic_probe: {case.name}, setting {args.setting}, "
          f"{'no copy' if args.no_copy else f'copy {args.copy_mib} MiB'}, {args.iters} iterations")


if __name__ == "__main__":
    main()
