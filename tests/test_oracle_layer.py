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
    parallel in a single forward pass of the target)."""
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


def test_rope_multi_with_equal_ids_is_the_one_id_rotation():
    """Text positions carry three equal ids: every section turns by the same position."""
    rng = np.random.default_rng(40)
    x = rng.standard_normal((2, 5, 3, 16))
    pos = rng.integers(0, 5000, (2, 5))
    for sections in ([8, 0, 0], [2, 3, 3], [0, 4, 4], [1, 1, 6]):
        np.testing.assert_allclose(O.rope_multi(x, np.stack([pos, pos, pos]), sections, 1e6), O.rope(x, pos, 1e6), rtol=1e-13)


def test_rope_multi_explicit_rotation_by_section():
    """d = 8, theta = 10^4: pair frequencies 1, 0.1, 0.01, 0.001.  Sections (1, 2, 1): pair 0 turns by the temporal
    id, pairs 1 and 2 by the height id, pair 3 by the width id -- each at its OWN frequency."""
    x = np.arange(1.0, 9.0).reshape(1, 1, 1, 8)
    t, h, w = 2, 3, 5
    y = O.rope_multi(x, np.array([[[t]], [[h]], [[w]]]), [1, 2, 1], 1e4)[0, 0, 0]
    ang = [t * 1.0, h * 0.1, h * 0.01, w * 0.001]
    want = [x[0, 0, 0, j] * math.cos(ang[j]) - x[0, 0, 0, j + 4] * math.sin(ang[j]) for j in range(4)] + \
           [x[0, 0, 0, j + 4] * math.cos(ang[j]) + x[0, 0, 0, j] * math.sin(ang[j]) for j in range(4)]
    np.testing.assert_allclose(y, want, rtol=1e-12)


def test_rope_multi_each_id_moves_only_its_own_section():
    rng = np.random.default_rng(41)
    x = rng.standard_normal((1, 1, 2, 32))
    sections = [4, 6, 6]
    base = np.array([[[7]], [[11]], [[13]]])
    y0 = O.rope_multi(x, base, sections, 1e4)
    bounds = [(0, 4), (4, 10), (10, 16)]
    for c in range(3):
        p = base.copy(); p[c] += 100
        moved = np.abs(O.rope_multi(x, p, sections, 1e4) - y0).max(axis=(0, 1, 2))       # per feature
        pairs = np.maximum(moved[:16], moved[16:])
        lo, hi = bounds[c]
        assert np.all(pairs[lo:hi] > 1e-6) and np.all(np.delete(pairs, np.arange(lo, hi)) == 0)
    with pytest.raises(ValueError):
        O.rope_multi(x, base, [4, 6, 5], 1e4)


def test_rope_append_by_loops():
    """The prompt-pass step between projection and attention, against per-element loops: head split, rotation of
    queries and keys, rows [kv_len, kv_len + n_new) of the caches written, everything else untouched."""
    rng = np.random.default_rng(42)
    B, L, nq, nkv, d, lmax = 2, 5, 4, 2, 8, 16
    qkv = rng.standard_normal((B, L, (nq + 2 * nkv) * d))
    pos = rng.integers(0, 50, (B, L))
    kv_len, n_new = [3, 0], [5, 2]
    k0, v0 = rng.standard_normal((B, nkv, lmax, d)), rng.standard_normal((B, nkv, lmax, d))
    q, k1, v1 = O.rope_append(qkv, pos, kv_len, n_new, k0, v0, nq, nkv, d, 1e4, "f32")
    f32 = lambda a: np.asarray(a, dtype=np.float32).astype(np.float64)          # the fp32 storage grid
    half = d // 2
    def turn(vec, p):
        out = np.empty(d)
        for j in range(half):
            a = p * 1e4 ** (-2.0 * j / d)
            out[j] = vec[j] * math.cos(a) - vec[j + half] * math.sin(a)
            out[j + half] = vec[j + half] * math.cos(a) + vec[j] * math.sin(a)
        return out
    kw, vw = k0.copy(), v0.copy()
    for b in range(B):
        for i in range(L):
            row = qkv[b, i]
            for h in range(nq):
                want = turn(row[h * d:(h + 1) * d], pos[b, i]) if i < n_new[b] else np.zeros(d)
                np.testing.assert_allclose(q[b, i, h], f32(want), rtol=1e-15, atol=0)
            if i < n_new[b]:
                for g in range(nkv):
                    kw[b, g, kv_len[b] + i] = turn(row[(nq + g) * d:(nq + g + 1) * d], pos[b, i])
                    vw[b, g, kv_len[b] + i] = row[(nq + nkv + g) * d:(nq + nkv + g + 1) * d]
    written = np.zeros_like(k0, dtype=bool)
    for b in range(B):
        written[b, :, kv_len[b]:kv_len[b] + n_new[b]] = True
    np.testing.assert_allclose(k1, np.where(written, f32(kw), kw), rtol=1e-15, atol=0)
    np.testing.assert_allclose(v1, np.where(written, f32(vw), vw), rtol=0, atol=0)
    # head norms come before the rotation, storage rounding after it
    gq, gk = rng.standard_normal(d), rng.standard_normal(d)
    q2, k2, _ = O.rope_append(qkv, pos, kv_len, n_new, k0, v0, nq, nkv, d, 1e4, "bf16", q_norm=gq, k_norm=gk, eps=1e-6)
    hq = qkv[0, 1, d:2 * d]
    want = O.round_bf16(turn(hq * gq / math.sqrt(np.mean(hq ** 2) + 1e-6), pos[0, 1]))
    np.testing.assert_allclose(q2[0, 1, 1], want, rtol=0, atol=0)
    hk = qkv[0, 1, (nq + 1) * d:(nq + 2) * d]
    want = O.round_bf16(turn(hk * gk / math.sqrt(np.mean(hk ** 2) + 1e-6), pos[0, 1]))
    np.testing.assert_allclose(k2[0, 1, kv_len[0] + 1], want, rtol=0, atol=0)


def test_rope_append_feeds_prefill_attention_like_the_layer_does():
    """Projection rows -> rope_append -> prefill_attention gives what verify_layer's own attention block gives on
    the same rows (same cache, same positions): the two paths through the checker agree."""
    rng = np.random.default_rng(43)
    s = synth.TINY
    B, Q = 2, 4
    nq, nkv, d = s.n_q_heads, s.n_kv_heads, s.head_dim
    kv = synth.kv_cache(s, B, Q, [9, 20], [4, 6], 43, junk_tail=False)
    qkv = rng.standard_normal((B, Q, (nq + 2 * nkv) * d))
    pos = synth.positions(kv.kv_len, kv.n_img, Q)
    q, k1, v1 = O.rope_append(qkv, pos, kv.kv_len, [Q, Q], kv.k, kv.v, nq, nkv, d, s.rope_theta, "f32")
    got = O.prefill_attention(q, k1, v1, kv.kv_len, [Q, Q])
    qh = O.rope(qkv[..., :nq * d].reshape(B, Q, nq, d), pos, s.rope_theta)
    np.testing.assert_allclose(got, O.attention(qh, k1, v1, kv.kv_len), rtol=1e-5, atol=1e-6)   # q goes through fp32 storage


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



# ---------------------------------------------------------------------------
# variants of the Gemma 3 family: sliding window, query/key norm, block-output norms
# ---------------------------------------------------------------------------
def brute_window_attention(q, k, v, kv_len, scale, W):
    """Scalar loops: the query at cache row r sees rows max(0, r - W + 1) .. r."""
    B, Q, n_q, d = q.shape
    G = n_q // k.shape[1]
    out = np.zeros((B, Q, n_q, d))
    for b in range(B):
        for i in range(Q):
            r = int(kv_len[b]) + i
            rows = [j for j in range(r + 1) if r - j < W]
            for h in range(n_q):
                sc = [scale * sum(float(q[b, i, h, c]) * float(k[b, h // G, j, c]) for c in range(d)) for j in rows]
                mx = max(sc)
                ws = [math.exp(t - mx) for t in sc]
                for c in range(d):
                    out[b, i, h, c] = sum(wt * float(v[b, h // G, j, c]) for wt, j in zip(ws, rows)) / sum(ws)
    return out


@pytest.mark.parametrize("W", [1, 2, 4, 7, 12, 100])
def test_window_attention_matches_brute_force(W):
    q, k, v, kv_len = small_case(3)
    got = O.attention(q, k, v, kv_len, window=W)
    want = brute_window_attention(q, k, v, kv_len, 1.0 / math.sqrt(q.shape[-1]), W)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_window_special_cases():
    q, k, v, kv_len = small_case(4)
    B, Q = q.shape[:2]
    full = O.attention(q, k, v, kv_len)
    assert np.array_equal(O.attention(q, k, v, kv_len, window=0), full)
    np.testing.assert_allclose(O.attention(q, k, v, kv_len, window=int(kv_len.max()) + Q), full, rtol=1e-14)
    one = O.attention(q, k, v, kv_len, window=1)                   # only the own row: its value, whatever the key
    for b in range(B):
        for i in range(Q):
            for h in range(q.shape[2]):
                np.testing.assert_allclose(one[b, i, h], v[b, h // 2, kv_len[b] + i], rtol=1e-14)
    # a change to a key outside every window is invisible, one inside is not
    k2 = k.copy(); k2[:, :, 0] += 5.0
    W = 3
    assert np.array_equal(O.attention(q, k2, v, kv_len, window=W), O.attention(q, k, v, kv_len, window=W))
    k3 = k.copy(); k3[0, :, kv_len[0] - 1] += 5.0
    assert not np.allclose(O.attention(q, k3, v, kv_len, window=W)[0, 0], O.attention(q, k, v, kv_len, window=W)[0, 0])


def gemma_layer_case(dtype="f32", seed=0):
    s = synth.LayerShape(32, 4, 2, 8, 48, 64, synth.ACT_GELU_TANH, False, rope_theta=1e4, dtype=dtype,
                         window=5, qk_norm=True, post_norms=True)
    w = synth.layer_weights(s, seed, std=0.2)
    kv = synth.kv_cache(s, 2, 3, [6, 9], [2, 4], seed)
    x = synth.hidden_states(s, 2, 3, seed)
    pos = synth.positions(kv.kv_len, kv.n_img, 3, compress_image=True)
    return s, w, kv, x, pos


def test_gemma_style_layer_against_torch_float64():
    """The layer with window, query/key norm and block-output norms rebuilt from torch float64 routines and
    explicit band masks: a norm applied after instead of before the rotation, a norm on the wrong operand,
    an off-by-one window edge or a missing output norm shows up here."""
    s, w, kv, x, pos = gemma_layer_case()
    y, kc, vc = O.verify_layer(s, w, x, pos, kv.k, kv.v, kv.kv_len)
    T = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    rms = lambda t, g: torch.nn.functional.rms_norm(t, (t.shape[-1],), T(g), eps=s.norm_eps)
    B, Q, H = x.shape
    d, nq, nkv, W = s.head_dim, s.n_q_heads, s.n_kv_heads, s.window
    tx = T(x)
    xn = rms(tx, w["ln1"])
    q = rms((xn @ T(w["wq"]).T).reshape(B, Q, nq, d), w["q_norm"])
    k = rms((xn @ T(w["wk"]).T).reshape(B, Q, nkv, d), w["k_norm"])
    v = (xn @ T(w["wv"]).T).reshape(B, Q, nkv, d)
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
        rows = (L + torch.arange(Q))[:, None]
        cols = torch.arange(L + Q)[None, :]
        mask = (cols > rows) | (rows - cols >= W)
        for h in range(nq):
            sc = (q[b, :, h] @ kc2[b, h // 2, :L + Q].T) / math.sqrt(d)
            attn[b, :, h] = torch.softmax(sc.masked_fill(mask, float("-inf")), -1) @ vc2[b, h // 2, :L + Q]
    h1 = tx + rms(attn.reshape(B, Q, nq * d) @ T(w["wo"]).T, w["post_attn_norm"])
    hn = rms(h1, w["ln2"])
    mlp = (torch.nn.functional.gelu(hn @ T(w["wg"]).T, approximate="tanh") * (hn @ T(w["wu"]).T)) @ T(w["wd"]).T
    want = h1 + rms(mlp, w["post_mlp_norm"])
    np.testing.assert_allclose(y, want.float().double().numpy(), rtol=1e-6, atol=1e-6)
    for b in range(B):
        L = int(kv.kv_len[b])
        np.testing.assert_allclose(kc[b, :, :L + Q], kc2[b, :, :L + Q].numpy(), rtol=1e-6, atol=1e-7)


def test_query_key_norm_removes_projection_scale():
    """With the head norms on (and eps negligible) the layer's output does not change when the query or
    key projection is scaled by a constant; without them it does."""
    s, w, kv, x, pos = gemma_layer_case()
    s.norm_eps = 1e-30
    y0, _, _ = O.verify_layer(s, w, x, pos, kv.k, kv.v, kv.kv_len)
    w2 = dict(w, wq=w["wq"] * 3.0)
    y1, _, _ = O.verify_layer(s, w2, x, pos, kv.k, kv.v, kv.kv_len)
    np.testing.assert_allclose(y1, y0, rtol=0, atol=1e-6)
    w3 = dict(w2, q_norm=None); w4 = dict(w, q_norm=None)
    y3, _, _ = O.verify_layer(s, w3, x, pos, kv.k, kv.v, kv.kv_len)
    y4, _, _ = O.verify_layer(s, w4, x, pos, kv.k, kv.v, kv.kv_len)
    assert np.max(np.abs(y3 - y4)) > 1e-3


def test_gelu_erf_and_projector_against_torch():
    """Exact GELU against the library routine; the two-layer projector (Section 3.1) rebuilt from torch float64
    matmuls, with the hidden activation stored in bf16 in between."""
    x = np.linspace(-6, 6, 101)
    np.testing.assert_allclose(O.gelu_erf(x), torch.nn.functional.gelu(torch.from_numpy(x)).numpy(), rtol=1e-12, atol=1e-15)
    rng = np.random.default_rng(5)
    h = synth.bf16_representable(rng.standard_normal((7, 12)).astype(np.float32))
    w1 = synth.bf16_representable((rng.standard_normal((20, 12)) * 0.3).astype(np.float32)); b1 = synth.bf16_representable(rng.standard_normal(20).astype(np.float32))
    w2 = synth.bf16_representable((rng.standard_normal((5, 20)) * 0.3).astype(np.float32)); b2 = synth.bf16_representable(rng.standard_normal(5).astype(np.float32))
    T = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    mid = torch.nn.functional.gelu(T(h) @ T(w1).T + T(b1)).to(torch.bfloat16).double()
    want = (mid @ T(w2).T + T(b2)).numpy()
    np.testing.assert_allclose(O.projector_mlp(h, w1, b1, w2, b2, "bf16"), want, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------------------
# prompt-pass attention (Section 2.2: image positions ahead of the text)
# ---------------------------------------------------------------------------
def prefill_case(seed=0, B=2, Lq=9, n_q=4, n_kv=2, d=8, kv_len=(0, 3), n_new=(9, 5)):
    rng = np.random.default_rng(seed)
    L_max = max(a + b for a, b in zip(kv_len, n_new)) + 2
    q = rng.standard_normal((B, Lq, n_q, d))
    k = rng.standard_normal((B, n_kv, L_max, d))
    v = rng.standard_normal((B, n_kv, L_max, d))
    return q, k, v, np.array(kv_len), np.array(n_new)


def brute_prefill(q, k, v, kv_len, n_new, scale, W=0, n_bidir=None):
    """Scalar loops, no matrix products: weights exp(s_j - max) over the visible rows, normalised."""
    B, Lq, n_q, d = q.shape
    G = n_q // k.shape[1]
    out = np.zeros_like(q)
    for b in range(B):
        for i in range(int(n_new[b])):
            r = int(kv_len[b]) + i
            for h in range(n_q):
                vis = []
                for j in range(int(kv_len[b]) + int(n_new[b])):
                    causal = j <= r
                    if n_bidir is not None and r < n_bidir[b] and j < n_bidir[b]:
                        causal = True
                    if causal and (W == 0 or j > r - W):
                        vis.append(j)
                s = [scale * sum(q[b, i, h, c] * k[b, h // G, j, c] for c in range(d)) for j in vis]
                mx = max(s)
                e = [math.exp(t - mx) for t in s]
                z = sum(e)
                for c in range(d):
                    out[b, i, h, c] = sum(e[t] * v[b, h // G, j, c] for t, j in enumerate(vis)) / z
    return out


@pytest.mark.parametrize("W", [0, 1, 3, 100])
def test_prefill_attention_matches_brute_force(W):
    q, k, v, kv_len, n_new = prefill_case()
    got = O.prefill_attention(q, k, v, kv_len, n_new, window=W)
    np.testing.assert_allclose(got, brute_prefill(q, k, v, kv_len, n_new, 1 / math.sqrt(8), W), rtol=1e-12, atol=1e-14)
    assert np.all(got[1, 5:] == 0)                               # rows past n_new[b] are not positions
    nb = np.array([4, 6])                                        # image block of 4 / 6 rows, the second straddles the cached piece
    got = O.prefill_attention(q, k, v, kv_len, n_new, window=W, n_bidir=nb)
    np.testing.assert_allclose(got, brute_prefill(q, k, v, kv_len, n_new, 1 / math.sqrt(8), W, nb), rtol=1e-12, atol=1e-14)


def test_prefill_attention_against_library_causal_attention():
    """A fresh prompt (nothing cached, every row a position) is plain causal attention: torch's
    scaled_dot_product_attention in float64 with the KV heads repeated over their query-head groups."""
    import torch
    q, k, v, _, _ = prefill_case(seed=3, B=2, Lq=12, n_q=6, n_kv=2, d=16, kv_len=(0, 0), n_new=(12, 12))
    got = O.prefill_attention(q, k[:, :, :12], v[:, :, :12], [0, 0], [12, 12])
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)
    tk = torch.from_numpy(k[:, :, :12]).repeat_interleave(3, dim=1)
    tv = torch.from_numpy(v[:, :, :12]).repeat_interleave(3, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
    # image block of 5 rows attending within itself: an explicit boolean mask
    mask = torch.tril(torch.ones(12, 12, dtype=torch.bool))
    mask[:5, :5] = True
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask).permute(0, 2, 1, 3).numpy()
    got = O.prefill_attention(q, k[:, :, :12], v[:, :, :12], [0, 0], [12, 12], n_bidir=[5, 5])
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


def test_prefill_attention_closed_forms_and_invariants():
    q, k, v, kv_len, n_new = prefill_case(seed=4)
    # equal keys: every visible row has the same weight, so the output is the mean of the visible value rows --
    # this pins the COUNT of visible rows (kv_len + i + 1) and the mapping of query heads to KV heads
    k_const = np.broadcast_to(k[:, :, :1], k.shape)
    got = O.prefill_attention(q, k_const, v, kv_len, n_new)
    for b in range(2):
        for i in range(int(n_new[b])):
            r = int(kv_len[b]) + i
            for h in range(4):
                np.testing.assert_allclose(got[b, i, h], v[b, h // 2, :r + 1].mean(0), rtol=1e-12)
    # causality: rows after a query's own row do not influence it
    k2, v2 = k.copy(), v.copy()
    k2[:, :, 6:] += 100.0
    v2[:, :, 6:] -= 50.0
    a, b_ = O.prefill_attention(q, k, v, kv_len, n_new), O.prefill_attention(q, k2, v2, kv_len, n_new)
    assert np.array_equal(a[0, :6], b_[0, :6])                   # sequence 0: rows 0..5
    assert np.array_equal(a[1, :3], b_[1, :3])                   # sequence 1 starts at row 3: rows 3..5
    assert not np.allclose(a[0, 6:], b_[0, 6:])
    # the prompt fed in two pieces equals the prompt fed at once (Section 2.1: a position conditions on all earlier ones,
    # however they got into the cache)
    whole = O.prefill_attention(q[:1], k[:1], v[:1], [0], [9])
    first = O.prefill_attention(q[:1, :4], k[:1], v[:1], [0], [4])
    second = O.prefill_attention(q[:1, 4:], k[:1], v[:1], [4], [5])
    np.testing.assert_allclose(np.concatenate([first[:, :4], second[:, :5]], 1), whole, rtol=1e-13)
    # and the verify pass is the same definition with gamma+1 new positions
    np.testing.assert_allclose(O.prefill_attention(q[:, :5], k, v, kv_len, [5, 5]), O.attention(q[:, :5], k, v, kv_len), rtol=1e-13)
