"""A whole decoder layer of the prompt pass (paper Section 2.2: image positions, then text, fill the cache) composed from
the library's prefill-side entry points -- rmsnorm, linear (with bias / multiplier / addend), rope_append,
prefill_attention -- against the CPU checker's layer over the same rows, and the cache it leaves against what the
verify step then reads."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2505_10526_amd import binding, synth
from helpers import to_dev, i32, round_up, pad_rows, v_blocked_to_rows, k_cache_to_rows, assert_close

pytestmark = pytest.mark.gpu
TOL = 2e-2

# a layer whose widths the compute-bound projection accepts (K % 64 == 0, N % 16 == 0)
SHAPE = synth.LayerShape(512, 8, 2, 64, 1024, 4096, synth.ACT_SILU, True, dtype="bf16")
SHAPE_GEGLU = synth.LayerShape(512, 4, 4, 128, 768, 4096, synth.ACT_GELU_TANH, False, dtype="bf16", rope_theta=1e4)


def prompt_layer_gpu(s, w, x, pos, kd, vd, kv_len, n_new):
    """One layer over the [B, L, H] rows of a prompt, entry point by entry point."""
    B, L, H = x.shape
    M = B * L
    nq, nkv, d = s.n_q_heads, s.n_kv_heads, s.head_dim
    dev = lambda a: None if a is None else to_dev(a, "bf16")
    pack = lambda a: binding.weight_pack(to_dev(a, "bf16"))
    wqkv = pack(np.concatenate([w["wq"], w["wk"], w["wv"]], axis=0))
    bqkv = dev(np.concatenate([w["bq"], w["bk"], w["bv"]])) if w.get("bq") is not None else None
    act = binding.LIN_SILU if s.act == synth.ACT_SILU else binding.LIN_GELU_TANH
    x2 = x.view(M, H)
    xn = binding.rmsnorm(x2, dev(w["ln1"]), s.norm_eps)
    qkv = binding.linear(xn, wqkv, bqkv)
    q = binding.rope_append(qkv.view(B, L, -1), pos, kv_len, n_new, kd, vd, nq, s.rope_theta)
    o = binding.prefill_attention(q, kd, vd, kv_len, n_new)
    h = binding.linear(o.view(M, nq * d), pack(w["wo"]), add=x2)
    hn = binding.rmsnorm(h, dev(w["ln2"]), s.norm_eps)
    up = binding.linear(hn, pack(w["wu"]))
    gated = binding.linear(hn, pack(w["wg"]), act=act, mul=up)
    y = binding.linear(gated, pack(w["wd"]), add=h)
    return y.view(B, L, H)


@pytest.mark.parametrize("s,seed", [(SHAPE, 1), (SHAPE_GEGLU, 2)], ids=["swiglu_bias_gqa", "geglu_mha_d128"])
def test_prompt_layer_against_the_checker(s, seed):
    B, L = 2, 150
    kv_len = np.array([0, 37], dtype=np.int32)           # a fresh prompt and one continuing a cached piece
    n_img = np.array([64, 20], dtype=np.int32)
    w = synth.layer_weights(s, seed, std=0.05)
    kv = synth.kv_cache(s, B, L, kv_len, n_img, seed, junk_tail=False)
    x = synth.hidden_states(s, B, L, seed)
    pos = synth.positions(kv.kv_len, kv.n_img, L)
    y_ref, k_ref, v_ref = O.verify_layer(s, w, x, pos, kv.k, kv.v, kv.kv_len)
    lm = round_up(kv.l_max, 32)
    kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), "bf16"))
    vd = binding.v_cache_pack(to_dev(pad_rows(kv.v, lm), "bf16"))
    y = prompt_layer_gpu(s, w, to_dev(x, "bf16"), i32(pos), kd, vd, i32(kv_len), i32([L, L]))
    torch.cuda.synchronize()
    assert_close(y.float().cpu().numpy(), y_ref, TOL, "layer output")
    kg = k_cache_to_rows(kd).float().cpu().numpy()
    vg = v_blocked_to_rows(vd).float().cpu().numpy()
    for b in range(B):
        L0 = int(kv_len[b])
        assert_close(kg[b, :, L0:L0 + L], k_ref[b, :, L0:L0 + L], TOL, "appended keys")
        assert_close(vg[b, :, L0:L0 + L], v_ref[b, :, L0:L0 + L], TOL, "appended values")
        assert np.array_equal(kg[b, :, :L0], kv.k[b, :, :L0]) and np.array_equal(vg[b, :, :L0], kv.v[b, :, :L0])


def test_prompt_pass_then_verify_step_on_the_same_cache():
    """The prompt layer fills the cache; the verify layer of the same weights then scores gamma + 1 further positions
    on it.  Against the checker run the same way (its layer over the prompt rows, then over the new rows)."""
    s, seed = SHAPE, 3
    B, L, Q = 2, 96, 6
    kv_len0 = np.array([0, 0], dtype=np.int32)
    w = synth.layer_weights(s, seed, std=0.05)
    l_max = round_up(L + Q + 8, 32)
    zeros = np.zeros((B, s.n_kv_heads, l_max, s.head_dim))
    x_p, x_v = synth.hidden_states(s, B, L, seed), synth.hidden_states(s, B, Q, seed + 1)
    pos_p = np.tile(np.arange(L, dtype=np.int32), (B, 1))
    pos_v = np.tile(np.arange(L, L + Q, dtype=np.int32), (B, 1))
    _, k1, v1 = O.verify_layer(s, w, x_p, pos_p, zeros, zeros, kv_len0)
    y_ref, _, _ = O.verify_layer(s, w, x_v, pos_v, k1, v1, kv_len0 + L)
    kd = binding.k_cache_pack(to_dev(zeros, "bf16"))
    vd = binding.v_cache_pack(to_dev(zeros, "bf16"))
    prompt_layer_gpu(s, w, to_dev(x_p, "bf16"), i32(pos_p), kd, vd, i32(kv_len0), i32([L, L]))
    cfg = binding.LayerConfig(s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.mlp, s.act, s.qkv_bias, s.norm_eps, s.rope_theta)
    wd = binding.pack_layer_weights({k: (None if v is None else to_dev(v, "bf16")) for k, v in w.items()})
    xd = to_dev(x_v, "bf16")
    binding.verify_layer(cfg, wd, xd, i32(pos_v), kd, vd, i32(kv_len0 + L))
    torch.cuda.synchronize()
    assert_close(xd.float().cpu().numpy(), y_ref, TOL, "verify layer after the prompt pass")
