"""Accuracy of the quantized layer on the GPU, as a stand-in for the perplexity columns of
Tables 1-2 (which need WikiText-2 and the trained GPT-2 weights): the signal-to-
quantisation-noise ratio of Y = X.W computed by the library against the same product in
fp64, for the naive quantiser (Eq. 1-3, r_cap = 0) and for MUXQ (Eq. 4-7), over the
activation widths of Table 1 (IA = 8, 7, 6, 5) and the weight widths of Table 2
(W = 8, 5, 4), per-tensor and per-vector (per-token X, per-channel W).

    python -m paper_2604_04701_amd.accuracy_report --config 2 --case 0

Inputs are the seeded synthetic outlier-bearing activations of the benchmark configurations.
The quantized products run in the HIP library; torch supplies device memory and the fp64
reference product."""
import argparse

import torch

from . import binding as B
from . import synth

WIDTHS = [(8, 8), (7, 8), (6, 8), (5, 8), (8, 5), (8, 4)]          # (IA bits, W bits)
GRANS = [("tensor", "tensor"), ("token", "channel")]                # (activations, weights)


def sqnr_db(y, ref):
    """10 log10( sum ref^2 / sum (y - ref)^2 ) in fp64."""
    y, ref = y.double(), ref.double()
    err = float(((y - ref) ** 2).sum())
    sig = float((ref ** 2).sum())
    return float("inf") if err == 0.0 else 10.0 * torch.log10(torch.tensor(sig / err)).item()


def report(X, W, threshold=6.0, exp=2, r_cap=64, widths=WIDTHS, grans=GRANS):
    """X [M, K], W [K, N]: fp16 tensors on the GPU.  Returns one dict per (granularity, widths)
    with the SQNR of the naive and the MUXQ result in dB and the outlier channels used."""
    M, K = X.shape
    N = W.shape[1]
    ref = X.double() @ W.double()
    ws = B.alloc_workspace(M, K, N, r_cap)
    lay = B.workspace_layout(M, K, N, r_cap)
    rows = []
    for x_gran, w_gran in grans:
        for ia_bits, w_bits in widths:
            w_q, w_scale = B.muxq_quantize_weight(W, w_gran, bits=w_bits)
            y_naive = B.muxq_linear(X, w_q, w_scale, N, w_gran, threshold=threshold, exp=exp, r_cap=0,
                                    x_gran=x_gran, ia_bits=ia_bits)
            y_muxq = B.muxq_linear(X, w_q, w_scale, N, w_gran, threshold=threshold, exp=exp,
                                   r_cap=r_cap, x_gran=x_gran, ia_bits=ia_bits, workspace=ws)
            torch.cuda.synchronize()
            used = int(B.ws_view(ws, lay, "n_outliers", M, N, r_cap)[0].item())
            rows.append(dict(x_gran=x_gran, w_gran=w_gran, ia_bits=ia_bits, w_bits=w_bits,
                             naive_db=sqnr_db(y_naive, ref), muxq_db=sqnr_db(y_muxq, ref),
                             outlier_channels=used))
    return rows


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--case", type=int, default=0)
    ap.add_argument("--exp", type=int, default=None)
    args = ap.parse_args()
    case = synth.config_cases(args.config)[args.case]
    Xh, Wh, _ = synth.make_case(case)
    X, W = torch.from_numpy(Xh).cuda(), torch.from_numpy(Wh).cuda()
    e = case.exp if args.exp is None else args.exp
    rows = report(X, W, threshold=case.threshold, exp=e, r_cap=case.r_cap)
    print(f"{case.name}: X {case.M}x{case.K} with {case.r} outlier channels, W {case.K}x{case.N}, "
          f"exp={e}; SQNR of Y against the fp64 product, dB")
    print("| X scale | W scale | IA | W | naive | MUXQ | gain |")
    print("|---|---|---|---|---|---|---|")
    for r in rows:
        print(f"| per-{r['x_gran']} | per-{r['w_gran']} | {r['ia_bits']} | {r['w_bits']} | "
              f"{r['naive_db']:.2f} | {r['muxq_db']:.2f} | {r['muxq_db'] - r['naive_db']:+.2f} |")


if __name__ == "__main__":
    main()
