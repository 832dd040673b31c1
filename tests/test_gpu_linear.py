"""GPU parity of massv_linear (the compute-bound projection used for the multimodal projector of paper
Section 3.1 and for prefill-sized inputs) against the CPU checker."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2505_10526_amd import synth, binding
from helpers import to_dev, assert_close

pytestmark = pytest.mark.gpu
TOL = 1e-2        # bf16 output of an fp32-accumulated sum: one rounding (2^-9 relative) plus accumulation-order noise

ACTS = {binding.LIN_NONE: lambda v: v, binding.LIN_SILU: O.silu, binding.LIN_GELU_TANH: O.gelu_tanh,
        binding.LIN_GELU_ERF: O.gelu_erf}


def inputs(M, N, K, seed, bias=True, w_std=0.05):
    x = synth.normal((M, K), 1.0, seed, 60, dtype="bf16")
    w = synth.normal((N, K), w_std, seed, 61, dtype="bf16")
    b = synth.normal((N,), 0.5, seed, 62, dtype="bf16") if bias else None
    return x, w, b


def run_gpu(x, w, b, act):
    y = binding.linear(to_dev(x, "bf16"), binding.weight_pack(to_dev(w, "bf16")),
                       None if b is None else to_dev(b, "bf16"), act)
    torch.cuda.synchronize()
    return y.float().cpu().numpy()


@pytest.mark.parametrize("M,N,K", [(300, 272, 128), (260, 528, 64), (1, 16, 64), (17, 4096, 192), (1024, 1024, 512),
                                   (513, 768, 1280)])
def test_ragged_shapes_against_checker(M, N, K):
    """Rows and features that end inside a tile, one k-step, odd numbers of k-steps, one row."""
    x, w, b = inputs(M, N, K, seed=M + N)
    got = run_gpu(x, w, b, binding.LIN_NONE)
    assert_close(got, O.linear(x, w, b), TOL, f"linear {M}x{N}x{K}")


@pytest.mark.parametrize("act", sorted(ACTS))
@pytest.mark.parametrize("bias", [False, True])
def test_bias_and_activations(act, bias):
    x, w, b = inputs(200, 320, 256, seed=7 + act, bias=bias)
    got = run_gpu(x, w, b, act)
    assert_close(got, ACTS[act](O.linear(x, w, b)), TOL, f"act {act} bias {bias}")


def test_prefill_sized_projection_sampled():
    """4096 rows through a 3584 -> 18944 projection (the launch the benchmark times): 3000 sampled outputs, the
    four corners included, each checked against its own dot product."""
    M, N, K = 4096, 18944, 3584
    x, w, _ = inputs(M, N, K, seed=9, bias=False, w_std=0.02)
    got = run_gpu(x, w, None, binding.LIN_NONE)
    rng = np.random.default_rng(9)
    ms = np.concatenate([[0, 0, M - 1, M - 1], rng.integers(0, M, 2996)])
    ns = np.concatenate([[0, N - 1, 0, N - 1], rng.integers(0, N, 2996)])
    ref = np.einsum("ik,ik->i", x[ms].astype(np.float64), w[ns].astype(np.float64))
    assert_close(got[ms, ns], ref, TOL, "sampled outputs")
    assert np.all(np.isfinite(got))


def test_projector_mlp():
    """Two-layer projector (Linear, GELU, Linear) over the image features of a batch: 3 images x 250 features of
    dimension 1280 -> 2048 -> 1536."""
    m, d_vis, d_hid, d_emb = 750, 1280, 2048, 1536
    h = synth.normal((m, d_vis), 1.0, 11, 63, dtype="bf16")
    w1 = synth.normal((d_hid, d_vis), 0.03, 11, 64, dtype="bf16"); b1 = synth.normal((d_hid,), 0.1, 11, 65, dtype="bf16")
    w2 = synth.normal((d_emb, d_hid), 0.03, 11, 66, dtype="bf16"); b2 = synth.normal((d_emb,), 0.1, 11, 67, dtype="bf16")
    ref = O.projector_mlp(h, w1, b1, w2, b2, "bf16")
    mid = binding.linear(to_dev(h, "bf16"), binding.weight_pack(to_dev(w1, "bf16")), to_dev(b1, "bf16"), binding.LIN_GELU_ERF)
    out = binding.linear(mid, binding.weight_pack(to_dev(w2, "bf16")), to_dev(b2, "bf16"), binding.LIN_NONE)
    torch.cuda.synchronize()
    assert_close(out.float().cpu().numpy(), ref, 2e-2, "projector output")


def test_repeatable_bits():
    x, w, b = inputs(700, 512, 320, seed=12)
    a = run_gpu(x, w, b, binding.LIN_GELU_TANH)
    c = run_gpu(x, w, b, binding.LIN_GELU_TANH)
    assert np.array_equal(a, c)


@pytest.mark.parametrize("M,N,K", [(1, 16, 64), (16, 16, 64), (257, 272, 64), (255, 256, 128), (256, 4096 + 16, 192)])
def test_smallest_and_tile_edge_shapes(M, N, K):
    """One row / one feature tile / one k-step; sizes one short of, equal to and one past a 256-wide tile."""
    x, w, b = inputs(M, N, K, seed=100 + M + N + K)
    assert_close(run_gpu(x, w, b, binding.LIN_GELU_TANH), O.gelu_tanh(O.linear(x, w, b)), TOL, f"{M}x{N}x{K}")


@pytest.mark.parametrize("use_mul,use_add,act", [(True, False, binding.LIN_SILU), (False, True, binding.LIN_NONE),
                                                 (True, True, binding.LIN_GELU_TANH)])
def test_multiplier_and_addend_after_the_activation(use_mul, use_add, act):
    """Y = act(X W^T + b) * mul + add: the gated MLP's act(gate) * up, and a projection added to the residual stream."""
    M, N, K = 333, 528, 192
    x, w, b = inputs(M, N, K, seed=31)
    mul = synth.normal((M, N), 1.0, 31, 63, dtype="bf16") if use_mul else None
    add = synth.normal((M, N), 2.0, 31, 64, dtype="bf16") if use_add else None
    y = binding.linear(to_dev(x, "bf16"), binding.weight_pack(to_dev(w, "bf16")), to_dev(b, "bf16"), act,
                       mul=None if mul is None else to_dev(mul, "bf16"), add=None if add is None else to_dev(add, "bf16"))
    torch.cuda.synchronize()
    ref = ACTS[act](O.linear(x, w, b))
    if use_mul:
        ref = ref * mul
    if use_add:
        ref = ref + add
    assert_close(y.float().cpu().numpy(), ref, TOL, "fused epilogue")


def test_addend_may_be_the_output_itself():
    M, N, K = 260, 272, 128
    x, w, _ = inputs(M, N, K, seed=32, bias=False)
    h = synth.normal((M, N), 1.0, 32, 65, dtype="bf16")
    hd = to_dev(h, "bf16")
    binding.linear(to_dev(x, "bf16"), binding.weight_pack(to_dev(w, "bf16")), None, binding.LIN_NONE, out=hd, add=hd)
    torch.cuda.synchronize()
    assert_close(hd.float().cpu().numpy(), O.linear(x, w) + h, TOL, "residual add in place")


def test_rmsnorm_rows():
    for dtype, tol in (("bf16", 8e-3), ("f32", 2e-6)):
        x = synth.normal((300, 1536), 1.0, 33, 66, dtype=dtype)
        g = synth.normal((1536,), 0.1, 33, 67, dtype=dtype, mean=1.0)
        y = binding.rmsnorm(to_dev(x, dtype), to_dev(g, dtype), 1e-6)
        torch.cuda.synchronize()
        assert_close(y.float().cpu().numpy(), O.rmsnorm(x, g, 1e-6), tol, f"rmsnorm {dtype}")
