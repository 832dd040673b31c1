"""Pins for the layer half of the CPU checker: attention, rotary embedding,
normalisation, activations, projections.  None of these tests uses a GPU."""
import math

import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2505_10526_amd import synth


# ---------------------------------------------------------------------------
# attention: brute force, closed forms, invariants
# ---------------------------------------------------------------------------
def brute_attention(q, k, v, kv_len, scale):
    """Scalar loops straight from the definition: query i of sequence b sees
    cache rows 0..kv_len[b]+i; head h reads KV head h // G."""
    B, Q, n_q, d = q.shape
    n_kv = k.shape[1]
    G = n_q // n_kv
    out = np.zeros((B, Q, n_q, d))
    for b in range(B):
        for i in range(Q):
            for h in range(n_q):
                g = h // G
                last = int(kv_len[b]) + i
                scores = []
                for j in range(last + 1):
                    acc = 0.0
                    for c in range(d):
                        acc += float(q[b, i, h, c]) * float(k[b, g, j, c])
                    scores.append(acc * scale)
                mx = max(scores)
                ws = [math.exp(s - mx) for s in scores]
                z = sum(ws)
                for c in range(d):
                    acc = 0.0
                    for j in range(last + 1):
                        acc += ws[j] * float(v[b, g, j, c])
                    out[b, i, h, c] = acc / z
    return out


def small_case(seed, B=2, Q=3, n_q=4, n_kv=2, d=8, kv_len=(5, 11)):
    rng = np.random.default_rng(seed)
    L_max = max(kv_len) + Q + 2
    q = rng.standard_normal((B, Q, n_q, d))
    k = rng.standard_normal((B, n_kv, L_max, d))
    v = rng.standard_normal((B, n_kv, L_max, d))
    return q, k, v, np.array(kv_len, dtype=np.int32)


@pytest.mark.parametrize("seed", [0, 1])
def test_attention_matches_brute_force(seed):
    q, k, v, kv_len = small_case(seed)
    scale = 1.0 / math.sqrt(q.shape[-1])
    got = O.attention(q, k, v, kv_len)
    want = brute_attention(q, k, v, kv_len, scale)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_attention_explicit_scale_is_used():
    q, k, v, kv_len = small_case(3)
    got = O.attention(q, k, v, kv_len, scale=0.37)
    want = brute_attention(q, k, v, kv_len, 0.37)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_attention_constant_values_returned_exactly():
    q, k, v, kv_len = small_case(4)
    v[:] = 0.0
    v[:, 0] = 2.5
    v[:, 1] = -1.25
    out = O.attention(q, k, v, kv_len)
    G = q.shape[2] // k.shape[1]
    for h in range(q.shape[2]):
        # also pins the grouped-head mapping: head h reads KV head h // G
        np.testing.assert_allclose(out[:, :, h], 2.5 if h // G == 0 else -1.25, rtol=1e-14)


def test_attention_constant_keys_give_mean_of_visible_values():
    q, k, v, kv_len = small_case(5)
    k[:] = 0.3            # equal scores => uniform weights over the visible rows
    out = O.attention(q, k, v, kv_len)
    B, Q, n_q, d = q.shape
    G = n_q // k.shape[1]
    for b in range(B):
        for i in range(Q):
            n_vis = int(kv_len[b]) + i + 1        # the count pins "inclusive of itself"
            for h in range(n_q):
                np.testing.assert_allclose(out[b, i, h], v[b, h // G, :n_vis].mean(axis=0),
                                           rtol=1e-12, atol=1e-14)


def test_attention_is_causal():
    q, k, v, kv_len = small_case(6)
    base = O.attention(q, k, v, kv_len)
    B, Q = q.shape[:2]
    for b in range(B):
        for i in range(Q):
            k2, v2 = k.copy(), v.copy()
            k2[b, :, int(kv_len[b]) + i + 1:] += 100.0
            v2[b, :, int(kv_len[b]) + i + 1:] -= 100.0
            out = O.attention(q, k2, v2, kv_len)
            assert np.array_equal(out[b, :i + 1], base[b, :i + 1])
            if i + 1 < Q:
                assert not np.allclose(out[b, i + 1:], base[b, i + 1:])


def test_attention_parallel_equals_sequential_decode():
    """Scoring all new positions in one pass equals one-query-at-a-time decoding
    with a growing cache (Section 2.1: the gamma+1 conditionals are computed in
    parallel with one forward call)."""
    q, k, v, kv_len = small_case(7)
    par = O.attention(q, k, v, kv_len)
    B, Q = q.shape[:2]
    for i in range(Q):
        step = O.attention(q[:, i:i + 1], k, v, kv_len + i)
        np.testing.assert_allclose(step[:, 0], par[:, i], rtol=1e-13, atol=1e-15)


def test_attention_against_torch_sdpa_special_case():
    """With one sequence, one query and G = 1 the definition reduces to plain
    softmax attention; cross-check that case with the library routine."""
    rng = np.random.default_rng(8)
    L, d, H = 37, 16, 3
    q = rng.standard_normal((1, 1, H, d))
    k = rng.standard_normal((1, H, L + 1, d))
    v = rng.standard_normal((1, H, L + 1, d))
    got = O.attention(q, k, v, np.array([L], dtype=np.int32))
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)
    want = torch.nn.functional.scaled_dot_product_attention(
        tq, torch.from_numpy(k), torch.from_numpy(v)).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------------------
# rotary embedding
# ---------------------------------------------------------------------------
def test_rope_position_zero_is_identity_and_norm_preserved():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 3, 4, 16))
    assert np.allclose(O.rope(x, np.zeros((2, 3), dtype=np.int32), 1e4), x, atol=0, rtol=0)
    pos = np.array([[5, 6, 7], [100, 2000, 30000]])
    y = O.rope(x, pos, 1e6)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)


def test_rope_inner_product_depends_on_relative_position_only():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((1, 1, 1, 32))
    k = rng.standard_normal((1, 1, 1, 32))
    def dot(m, n):
        a = O.rope(q, np.array([[m]]), 1e4)
        b = O.rope(k, np.array([[n]]), 1e4)
        return float(np.sum(a * b))
    assert abs(dot(17, 5) - dot(112, 100)) < 1e-10
    assert abs(dot(17, 5) - dot(12, 0)) < 1e-10
    assert abs(dot(17, 5) - dot(5, 17)) > 1e-3       # sign of the offset matters


def test_rope_explicit_pair_rotation():
    """d = 4, pairs (0,2) and (1,3); frequencies theta^0 = 1 and theta^(-1/2)."""
    theta, pos = 100.0, 3
    x = np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 1, 1, 4)
    y = O.rope(x, np.array([[pos]]), theta)[0, 0, 0]
    a0, a1 = pos * 1.0, pos * theta ** -0.5
    want = [1 * math.cos(a0) - 3 * math.sin(a0), 2 * math.cos(a1) - 4 * math.sin(a1),
            3 * math.cos(a0) + 1 * math.sin(a0), 4 * math.cos(a1) + 2 * math.sin(a1)]
    np.testing.assert_allclose(y, want, rtol=1e-13)


# ---------------------------------------------------------------------------
# norm, activations, projections, storage rounding
# ---------------------------------------------------------------------------
def test_rmsnorm_against_torch_and_by_hand():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 64))
    g = rng.standard_normal(64)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-6).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-6), want, rtol=1e-12)
    # [3, 4]: mean square 12.5
    np.testing.assert_allclose(O.rmsnorm(np.array([3.0, 4.0]), np.array([2.0, 0.5]), 0.0),
                               [6 / math.sqrt(12.5), 2 / math.sqrt(12.5)], rtol=1e-15)


def test_activations_against_torch():
    x = np.linspace(-9, 9, 1001)
    tx = torch.from_numpy(x)
    np.testing.assert_allclose(O.silu(x), torch.nn.functional.silu(tx).numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(O.gelu_tanh(x), torch.nn.functional.gelu(tx, approximate="tanh").numpy(),
                               rtol=1e-11, atol=1e-14)
    assert O.silu(np.array([0.0]))[0] == 0.0 and abs(O.silu(np.array([1.0]))[0] - 1 / (1 + math.exp(-1))) < 1e-15


def test_linear_is_x_times_w_transposed_plus_bias():
    rng = np.random.default_rng(3)
    x, w, b = rng.standard_normal((3, 7)), rng.standard_normal((5, 7)), rng.standard_normal(5)
    y = O.linear(x, w, b)
    for m in range(3):
        for n in range(5):
            assert abs(y[m, n] - (sum(x[m, k] * w[n, k] for k in range(7)) + b[n])) < 1e-12


def test_gated_mlp_by_loops():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 6))
    wg, wu, wd = rng.standard_normal((9, 6)), rng.standard_normal((9, 6)), rng.standard_normal((6, 9))
    for act, f in ((O.ACT_SILU, lambda z: z / (1 + math.exp(-z))),
                   (O.ACT_GELU_TANH, lambda z: 0.5 * z * (1 + math.tanh(math.sqrt(2 / math.pi) * (z + 0.044715 * z ** 3))))):
        got = O.gated_mlp(x, wg, wu, wd, act)
        for m in range(2):
            hcol = [f(float(wg[j] @ x[m])) * float(wu[j] @ x[m]) for j in range(9)]
            for n in range(6):
                assert abs(got[m, n] - sum(wd[n, j] * hcol[j] for j in range(9))) < 1e-11


def test_round_bf16_against_torch_and_ties_to_even():
    rng = np.random.default_rng(5)
    a = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_bf16(a), want)
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: goes to the even mantissa (1.0);
    # 1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6: goes to 1 + 2^-6.
    assert O.round_bf16(np.array([1 + 2.0 ** -8]))[0] == 1.0
    assert O.round_bf16(np.array([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6
    assert np.array_equal(synth.bf16_representable(a).astype(np.float64), want)


# ---------------------------------------------------------------------------
# the whole layer: composition checks
# ---------------------------------------------------------------------------
def tiny_layer_case(dtype="f32", B=2, Q=3, seed=0):
    s = synth.LayerShape(32, 4, 2, 8, 48, 64, synth.ACT_SILU, True, dtype=dtype)
    w = synth.layer_weights(s, seed, std=0.2)
    kv = synth.kv_cache(s, B, Q, [6, 9], [2, 4], seed)
    x = synth.hidden_states(s, B, Q, seed)
    pos = synth.positions(kv.kv_len, kv.n_img, Q, compress_image=True)
    return s, w, kv, x, pos


def test_layer_composition_against_torch_float64():
    """Rebuild the layer from library routines (torch float64 matmul, rms_norm,
    silu, softmax) and explicit per-query masks; a dropped residual, a swapped
    gate/up, a missing bias or a wrong cache row shows up here."""
    s, w, kv, x, pos = tiny_layer_case()
    y, kc, vc = O.verify_layer(s, w, x, pos, kv.k, kv.v, kv.kv_len)
    T = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    B, Q, H = x.shape
    d, nq, nkv = s.head_dim, s.n_q_heads, s.n_kv_heads
    tx = T(x)
    xn = torch.nn.functional.rms_norm(tx, (H,), T(w["ln1"]), eps=s.norm_eps)
    q = (xn @ T(w["wq"]).T + T(w["bq"])).reshape(B, Q, nq, d)
    k = (xn @ T(w["wk"]).T + T(w["bk"])).reshape(B, Q, nkv, d)
    v = (xn @ T(w["wv"]).T + T(w["bv"])).reshape(B, Q, nkv, d)
    inv = s.rope_theta ** (-torch.arange(0, d // 2, dtype=torch.float64) * 2 / d)
    ang = T(pos)[..., None, None] * inv
    def rot(t):
        a, b = t[..., :d // 2], t[..., d // 2:]
        return torch.cat([a * ang.cos() - b * ang.sin(), b * ang.cos() + a * ang.sin()], -1)
    q, k = rot(q), rot(k)
    kc2, vc2 = T(kv.k).clone(), T(kv.v).clone()
    attn = torch.zeros(B, Q, nq, d, dtype=torch.float64)
    for b in range(B):
        L = int(kv.kv_len[b])
        kc2[b, :, L:L + Q] = k[b].permute(1, 0, 2).float().double()
        vc2[b, :, L:L + Q] = v[b].permute(1, 0, 2).float().double()
        for h in range(nq):
            sc = (q[b, :, h] @ kc2[b, h // 2, :L + Q].T) / math.sqrt(d)      # [Q, L+Q]
            mask = torch.arange(L + Q)[None, :] > (L + torch.arange(Q))[:, None]
            sc = sc.masked_fill(mask, float("-inf"))
            attn[b, :, h] = torch.softmax(sc, -1) @ vc2[b, h // 2, :L + Q]
    h1 = tx + attn.reshape(B, Q, nq * d) @ T(w["wo"]).T
    hn = torch.nn.functional.rms_norm(h1, (H,), T(w["ln2"]), eps=s.norm_eps)
    want = h1 + (torch.nn.functional.silu(hn @ T(w["wg"]).T) * (hn @ T(w["wu"]).T)) @ T(w["wd"]).T
    np.testing.assert_allclose(y, want.float().double().numpy(), rtol=1e-6, atol=1e-6)
    for b in range(B):
        L = int(kv.kv_len[b])
        np.testing.assert_allclose(kc[b, :, :L + Q], kc2[b, :, :L + Q].numpy(), rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(vc[b, :, :L + Q], vc2[b, :, :L + Q].numpy(), rtol=1e-6, atol=1e-7)
        assert np.array_equal(kc[b, :, L + Q:], np.asarray(kv.k, dtype=np.float64)[b, :, L + Q:])


def test_layer_stores_on_bf16_grid():
    s, w, kv, x, pos = tiny_layer_case("bf16")
    y, kc, vc = O.verify_layer(s, w, x, pos, kv.k, kv.v, kv.kv_len)
    for a in (y, kc, vc):
        assert np.array_equal(O.round_bf16(a), a)


def test_lm_head_is_norm_then_projection():
    """Scalar loops (no matrix product, no broadcasting) and a hand-valued case: a transposed w_lm, a norm applied
    after the projection or a dropped gain would each fail one of them."""
    rng = np.random.default_rng(9)
    M, H, V, eps = 4, 16, 10, 1e-6
    x, g, w = rng.standard_normal((M, H)), rng.standard_normal(H), rng.standard_normal((V, H))
    got = O.lm_head_logits(x, g, w, eps)
    got_plain = O.lm_head_logits(x, None, w, eps)
    assert got.shape == (M, V)
    for m in range(M):
        ms = 0.0
        for k in range(H):
            ms += float(x[m, k]) ** 2
        rstd = 1.0 / math.sqrt(ms / H + eps)
        for v in range(V):
            acc, acc_plain = 0.0, 0.0
            for k in range(H):
                acc += float(x[m, k]) * rstd * float(g[k]) * float(w[v, k])
                acc_plain += float(x[m, k]) * float(w[v, k])
            assert abs(got[m, v] - acc) <= 1e-12 * max(1.0, abs(acc))
            assert abs(got_plain[m, v] - acc_plain) <= 1e-12 * max(1.0, abs(acc_plain))
    # by hand: x = (3, 4), mean square 12.5, eps = 0 -> x / sqrt(12.5); gains (2, 1); rows of w_lm (1, 0), (0, 1), (1, 1)
    r = math.sqrt(12.5)
    hand = O.lm_head_logits(np.array([[3.0, 4.0]]), np.array([2.0, 1.0]), np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]]), 0.0)
    np.testing.assert_allclose(hand, [[6.0 / r, 4.0 / r, 10.0 / r]], rtol=1e-15)
