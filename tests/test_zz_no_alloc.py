"""muxq_linear_noalloc (intermediates in the library's static device array, no allocation inside
the call) against muxq_linear with a caller's workspace: same Y bit for bit, on two calls in a
row, the second with a smaller input, and a shape beyond the array's size is refused."""
import numpy as np
import pytest
import torch

from gpu_common import orc, say
from paper_2604_04701_amd import binding as B
from paper_2604_04701_amd import synth
from paper_2604_04701_amd.synth import Case

pytestmark = pytest.mark.gpu
U = (20.0, 100.0)


def _both(case, w_gran, with_bias):
    X, W, _ = synth.make_case(case)
    dev = "cuda"
    Xd = torch.from_numpy(X).to(dev)
    w_q, w_scale = B.muxq_quantize_weight(torch.from_numpy(W).to(dev), w_gran)
    bias = (np.random.default_rng(case.seed + 1).standard_normal(case.N).astype(np.float16)
            if with_bias else None)
    bd = torch.from_numpy(bias).to(dev) if with_bias else None
    say(f"[noalloc] {case.name} M={case.M} K={case.K} N={case.N} r={case.r} {w_gran} bias={with_bias}")
    assert B.workspace_bytes(case.M, case.K, case.N, case.r_cap) <= B.lib().muxq_noalloc_max_bytes()
    y_ref = B.muxq_linear(Xd, w_q, w_scale, case.N, w_gran, bias=bd, threshold=case.threshold,
                          exp=case.exp, r_cap=case.r_cap)
    y_out = torch.full((case.M, case.N), float("nan"), dtype=torch.float16, device=dev)
    B.muxq_linear_noalloc(Xd, w_q, w_scale, case.N, w_gran, bias=bd, threshold=case.threshold,
                          exp=case.exp, r_cap=case.r_cap, out=y_out)
    torch.cuda.synchronize()
    assert torch.equal(y_ref, y_out), f"{case.name}: differs from muxq_linear"
    o = orc.linear(X, W, threshold=case.threshold, e=case.exp, r_cap=case.r_cap, w_gran=w_gran, bias16=bias)
    assert (y_out.cpu().numpy() == o["y16"]).all(), f"{case.name}: differs from the oracle"


def test_two_calls_in_a_row_second_one_smaller():
    # the second call finds the first call's intermediates in the array and must not see them
    _both(Case("noalloc_big", 2049, 1032, 1544, 9, U, 901, r_cap=128), "channel", True)
    _both(Case("noalloc_small", 100, 200, 264, 3, U, 902), "tensor", False)
    _both(synth.config_cases(2)[3], "tensor", False)           # 1024 x 3072 -> 768
    _both(Case("noalloc_tiny", 1, 8, 8, 1, U, 903), "tensor", True)


def test_sizes_beyond_the_array_are_refused():
    L = B.lib()
    assert L.muxq_noalloc_max_bytes() == 16 << 20
    case = synth.config_cases(5)[0]
    assert B.workspace_bytes(case.M, case.K, case.N, case.r_cap) > L.muxq_noalloc_max_bytes()
    Xd = torch.zeros((8, case.K), dtype=torch.float16, device="cuda")      # never read: refused first
    fake = torch.zeros(16, dtype=torch.uint8, device="cuda")
    st = L.muxq_linear_noalloc(Xd.data_ptr(), case.M, case.K, case.K, fake.data_ptr(), fake.data_ptr(), 0,
                               case.N, None, 6.0, 2, 64, fake.data_ptr(), case.N, None)
    assert st == 5, st                                                    # MUXQ_ERR_WORKSPACE
    # bad shapes keep their own status
    assert L.muxq_linear_noalloc(Xd.data_ptr(), 0, 768, 768, fake.data_ptr(), fake.data_ptr(), 0, 768, None,
                                 6.0, 2, 64, fake.data_ptr(), 768, None) == 2
