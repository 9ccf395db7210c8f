"""Seeded, bounded randomised sweeps of the HIP library against the CPU oracle: shapes that
are not multiples of any tile size, both granularities on either side, a bias, exp 0-3,
capacities 0 / 64 / 128 with more outlier channels than capacity, narrower code widths, the
naive entry point and the static-list entry points.  Three views of every draw:
stage by stage through the accumulator export, as a user calls the layer (Y bit-identical,
which runs the plain and staged epilogues), and with a channel list fixed offline."""
import numpy as np
import pytest

import test_gpu_parity as T
from gpu_common import check_case, check_own_scale, check_plain_y, orc, run_gpu, say, synth
from paper_2604_04701_amd.synth import Case

pytestmark = pytest.mark.gpu
U = (20.0, 100.0)


def _draw_shape(rng, Ms, Ks, Ns, budget):
    while True:
        M, K, N = int(rng.choice(Ms)), int(rng.choice(Ks)), int(rng.choice(Ns))
        if M * N * K <= budget:
            return M, K, N


def _draw_opts(rng, K):
    r_cap = min(int(rng.choice([0, 64, 64, 128])), (K + 63) // 64 * 64)
    r = int(rng.integers(0, min(K, max(r_cap, 8) + 10) + 1)) if rng.random() < 0.8 else 0
    kw = dict(w_gran=str(rng.choice(["tensor", "channel"])), x_gran=str(rng.choice(["tensor", "token"])),
              e=int(rng.choice([0, 1, 2, 2, 3])), r_cap=r_cap)
    return r, kw


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_sweep_all_stages(seed):
    rng = np.random.default_rng(seed)
    Ms = [1, 7, 16, 33, 100, 257, 300, 513, 1000, 2049]
    Ks = [8, 64, 72, 200, 256, 328, 512, 1032, 2048, 2112, 4096, 5120]
    Ns = [8, 72, 136, 264, 520, 1096, 1544, 3000]
    for n in range(14):
        M, K, N = _draw_shape(rng, Ms, Ks, Ns, 2.5e9)
        r, kw = _draw_opts(rng, K)
        if rng.random() < 0.3:
            kw["ia_bits"] = int(rng.choice([5, 6, 7]))
        if rng.random() < 0.2:
            kw["w_bits"] = int(rng.choice([4, 5]))
            kw["w_gran"] = "channel"
        bias_seed = int(rng.integers(1, 1000)) if rng.random() < 0.5 else None
        case = Case(f"sweep{seed}_{n}", M, K, N, r, U, int(rng.integers(0, 1 << 30)))
        check_case(case, bias_seed=bias_seed, **kw)


@pytest.mark.parametrize("seed", [21, 22])
def test_sweep_y_as_a_user_calls_it(seed):
    rng = np.random.default_rng(seed)
    Ms = [16, 100, 257, 300, 513, 1000, 1500, 2049, 2690, 3333, 4096]
    Ks = [64, 200, 256, 512, 712, 1032, 1088, 2048, 2112, 4096]
    Ns = [72, 264, 520, 1096, 1544, 3000, 4104, 6152]
    for n in range(12):
        M, K, N = _draw_shape(rng, Ms, Ks, Ns, 1.2e10)
        r, kw = _draw_opts(rng, K)
        bias_seed = int(rng.integers(1, 1000)) if rng.random() < 0.5 else None
        case = Case(f"sweepy{seed}_{n}", M, K, N, r, U, int(rng.integers(0, 1 << 30)))
        if rng.random() < 0.15:
            # the naive entry point against the oracle run without the decomposition
            X, W, _ = synth.make_case(case)
            bias = (np.random.default_rng(bias_seed).standard_normal(N).astype(np.float16)
                    if bias_seed else None)
            say(f"[naive y] {case.name} M={M} K={K} N={N} {kw['w_gran']} bias={bias is not None}")
            g = run_gpu(X, W, w_gran=kw["w_gran"], bias=bias, naive=True, want_acc=False)
            o = orc.linear(X, W, threshold=float("inf"), r_cap=0, w_gran=kw["w_gran"], bias16=bias)
            assert (g["Y"] == o["y16"]).all(), case.name
        else:
            check_plain_y(case, bias_seed=bias_seed, **kw)


@pytest.mark.parametrize("seed", [31, 32])
def test_sweep_static_lists(seed):
    rng = np.random.default_rng(seed)
    Ms = [1, 16, 100, 257, 300, 1000, 2049, 3333]
    Ks = [8, 64, 200, 264, 512, 1032, 2048, 4096]
    Ns = [8, 72, 136, 264, 1096, 4104]
    for n in range(12):
        M, K, N = _draw_shape(rng, Ms, Ks, Ns, 2.5e9)
        r_cap = min(int(rng.choice([0, 64, 128])), (K + 63) // 64 * 64)
        r = int(rng.integers(0, min(K, 40) + 1))
        nl = int(rng.integers(0, min(K, r_cap + 20) + 1))
        raw = sorted(rng.choice(K, size=nl, replace=False).tolist())
        if raw and rng.random() < 0.3:      # entries the rule skips: out of range, not ascending
            raw.insert(int(rng.integers(0, len(raw) + 1)), int(rng.choice([-1, K, K + 5, raw[0]])))
        case = Case(f"sweeps{seed}_{n}", M, K, N, r, U, int(rng.integers(0, 1 << 30)))
        T._check_static(case, raw, str(rng.choice(["tensor", "token"])), str(rng.choice(["tensor", "channel"])),
                        r_cap=r_cap, e=int(rng.choice([1, 2, 3])), with_bias=bool(rng.random() < 0.5))


@pytest.mark.parametrize("seed", [31, 32])
def test_sweep_aux_on_its_own_scale(seed):
    """Aux quantised on the abs-max scale of its own values (the other reading of Eq. 5), one
    activation scale per call or per token: outlier channels from just above the threshold (where
    the two readings differ) to far above it (where they coincide), odd shapes, exp 1-3."""
    rng = np.random.default_rng(seed)
    for n in range(16):
        M = int(rng.integers(1, 700))
        K = 8 * int(rng.integers(2, 280))
        N = 8 * int(rng.integers(1, 160))
        e = int(rng.integers(1, 4))
        X = rng.uniform(-5.0, 5.0, size=(M, K)).astype(np.float32)
        r = int(rng.integers(0, min(9, K // 8)))
        if r:
            ch = np.sort(rng.choice(K, size=r, replace=False))
            top = float(rng.choice([6.5, 7.5, 30.0, 200.0]))
            X[:, ch] = rng.uniform(-top, top, size=(M, r))
            X[int(rng.integers(0, M)), ch] = top
        W = (0.05 * rng.standard_normal((K, N))).astype(np.float16)
        r_cap = min(int(rng.choice([64, 64, 128])), (K + 63) // 64 * 64)
        case = Case(f"own_sweep{seed}_{n}", M, K, N, r, (1.0, 1.0), 0)
        check_own_scale(case, X.astype(np.float16), W, e=e, r_cap=r_cap,
                        w_gran=str(rng.choice(["tensor", "channel"])),
                        x_gran=str(rng.choice(["tensor", "token"])),
                        bias_seed=n if n % 3 == 0 else None)
