"""Workload for the HBM-traffic counter runs (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE).

Runs a plain device-to-device copy of known size (the calibration dispatch:
`bytes` read and `bytes` written) and then a few muxq_linear calls on one
workload configuration, so that one counter run holds both.  Usage:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -o fetch -- \
        python3 -m paper_2604_04701_amd.traffic_probe --config 5
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
    args = ap.parse_args()
    case = synth.config_cases(args.config)[args.case]
    X, W, _ = synth.make_case(case)
    Xd, Wd = torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda()
    w_q, w_scale = B.muxq_quantize_weight(Wd, case.w_gran)
    ws = B.alloc_workspace(case.M, case.K, case.N, case.r_cap)
    Y = torch.empty((case.M, case.N), dtype=torch.float16, device="cuda")
    src = torch.empty(args.copy_mib << 20, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(args.iters):
        dst.copy_(src)                       # calibration: copy_mib MiB in, copy_mib MiB out
        torch.cuda.synchronize()
        B.muxq_linear(Xd, w_q, w_scale, case.N, case.w_gran, threshold=case.threshold,
                      exp=case.exp, r_cap=case.r_cap, out=Y, workspace=ws)
        torch.cuda.synchronize()
    print(f"traffic_probe: {case.name}, copy {args.copy_mib} MiB, {args.iters} iterations")


if __name__ == "__main__":
    main()
