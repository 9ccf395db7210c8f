"""Seeded synthetic inputs for the MUXQ linear layer.

Holds none of the method's arithmetic: it only draws activations with a few
large-magnitude channels (the structure Fig. 1 of the paper shows and the
">6" criterion of Sec. III-C relies on) and Gaussian weights, at the shapes of
the GPT-2 projection modules named in Sec. IV-C.  Both the CPU oracle's tests
and the GPU tests/bench take their inputs from here, so the two sides always
see identical bytes.  The data stand in for the WikiText-2 / pretrained GPT-2
activations the paper evaluates on, which are not available offline.

Draw order is fixed: X (standard normal, fp32) -> outlier channel choice ->
per-channel gains -> multiply -> cast to fp16 -> W (0.02 * standard normal,
fp32) -> cast to fp16.
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Case:
    name: str
    M: int
    K: int
    N: int
    r: int                      # planted outlier channels
    gain: Tuple[float, float]   # (lo, hi): U(lo, hi) per channel; lo == hi -> fixed
    seed: int
    w_gran: str = "tensor"      # "tensor" | "channel"
    r_cap: int = 64
    exp: int = 2
    threshold: float = 6.0


def make_x(M: int, K: int, r: int, gain: Tuple[float, float], rng) -> Tuple[np.ndarray, np.ndarray]:
    x = rng.standard_normal((M, K), dtype=np.float32)
    r = min(r, K)
    ch = np.sort(rng.choice(K, size=r, replace=False)) if r > 0 else np.zeros(0, np.int64)
    lo, hi = gain
    g = (np.full(r, lo, np.float32) if lo == hi
         else rng.uniform(lo, hi, size=r).astype(np.float32))
    if r > 0:
        x[:, ch] *= g
    return x.astype(np.float16), ch.astype(np.int64)


def make_w(K: int, N: int, rng, std: float = 0.02) -> np.ndarray:
    w = rng.standard_normal((K, N), dtype=np.float32)
    w *= np.float32(std)
    return w.astype(np.float16)


def make_case(case: Case, with_w: bool = True):
    """Returns (X fp16 [M,K], W fp16 [K,N] or None, planted channel indices)."""
    rng = np.random.default_rng(case.seed)
    X, ch = make_x(case.M, case.K, case.r, case.gain, rng)
    W = make_w(case.K, case.N, rng) if with_w else None
    return X, W, ch


def _layer_set(h: int) -> List[Tuple[int, int]]:
    # c_attn, attention c_proj, c_fc, MLP c_proj of a GPT-2 block (Sec. IV-C).
    return [(h, 3 * h), (h, h), (h, 4 * h), (4 * h, h)]


def config_cases(cfg: int) -> List[Case]:
    """The five workload configurations, numbered 1..5."""
    U = (20.0, 100.0)
    if cfg == 1:
        return [Case("cfg1_768x768", 128, 768, 768, 6, (60.0, 60.0), 0)]
    if cfg == 2:
        return [Case(f"cfg2_{k}x{n}", 1024, k, n, 8, U, 2000 + i)
                for i, (k, n) in enumerate(_layer_set(768))]
    if cfg == 3:
        out = []
        for i, (k, n) in enumerate(_layer_set(1024)):
            for g in ("tensor", "channel"):
                out.append(Case(f"cfg3_{k}x{n}_{g}", 8192, k, n, 12, U, 3000 + i, w_gran=g))
        return out
    if cfg == 4:
        out = []
        for i, (k, n) in enumerate(_layer_set(1280)):
            for r in (1, 4, 16, 64):
                out.append(Case(f"cfg4_{k}x{n}_r{r}", 16384, k, n, r, U,
                                4000 + 10 * i + {1: 0, 4: 1, 16: 2, 64: 3}[r],
                                r_cap=128 if r == 64 else 64))
        return out
    if cfg == 5:
        return [Case("cfg5_4096x16384", 8192, 4096, 16384, 32, (50.0, 50.0), 5000)]
    raise ValueError(f"no such config: {cfg}")
