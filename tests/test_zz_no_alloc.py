"""massv_spec_accept_static (scratch space inside the library, for callers that cannot allocate) against
massv_spec_accept on the same inputs: identical integers, on two calls in a row, the second with a smaller input."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2505_10526_amd import synth, binding

pytestmark = pytest.mark.gpu


def both(a, temperature):
    dev = "cuda:0"
    B, Q, V = a.target_logits.shape
    gamma = Q - 1
    t = torch.from_numpy(a.target_logits).to(dev)
    d = torch.from_numpy(a.draft_logits).to(dev) if temperature > 0 and gamma > 0 else None
    x = torch.from_numpy(a.draft_tokens).to(dev) if gamma > 0 else None
    u = torch.from_numpy(a.uniforms).to(dev) if temperature > 0 else None
    n_ref, out_ref = binding.spec_accept(t, d, x, u, temperature)
    n = torch.full((B,), -7, dtype=torch.int32, device=dev)
    out = torch.full((B, Q), -7, dtype=torch.int32, device=dev)
    binding.spec_accept_static(t, d, x, u, temperature, n, out)
    torch.cuda.synchronize()
    assert torch.equal(n, n_ref), (n, n_ref)
    assert torch.equal(out, out_ref), (out, out_ref)
    return n_ref.cpu().numpy()


@pytest.mark.parametrize("temperature", [0.7, 0.0])
def test_two_calls_in_a_row_second_smaller(temperature):
    # the long-context stress shape first (the largest scratch need of the configurations: 1.2 MB), then a small
    # ragged vocabulary whose records land on top of what the first call left behind
    big = synth.accept_inputs(32, 7, 152064, temperature, seed=0, target_std=3.0, corr=0.8)
    small = synth.accept_inputs(3, 5, 4096 + 5, temperature, seed=11, target_std=2.0, noise_std=1.5, peak=4.0)
    both(big, temperature)
    n = both(small, temperature)
    assert n.max() > 0                              # the second case is not all first-token rejections
    both(synth.accept_inputs(5, 0, 1000, temperature, seed=31, target_std=2.0), temperature)     # gamma = 0 draw


def test_sizes_beyond_the_array_are_refused_before_any_launch():
    lib = binding.load()
    limit = lib.massv_spec_accept_static_limit()
    assert limit == 4 << 20
    B, gamma, V = 64, 15, 262144
    assert lib.massv_spec_accept_workspace(B, gamma, V) > limit
    t = torch.zeros(8, device="cuda:0")                              # never touched: the call must fail first
    n = torch.zeros(8, dtype=torch.int32, device="cuda:0")
    rc = lib.massv_spec_accept_static(C.c_void_p(t.data_ptr()), C.c_void_p(t.data_ptr()), C.c_void_p(n.data_ptr()),
                                      C.c_void_p(t.data_ptr()), 1.0, B, gamma, V, C.c_void_p(n.data_ptr()),
                                      C.c_void_p(n.data_ptr()), None)
    assert rc == binding.EUNSUPPORTED
    assert lib.massv_spec_accept_static(None, None, None, None, 0.0, 1, 0, 8, None, None, None) == binding.EINVAL
