"""CPU checker for the target-model verify step of speculative decoding.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
GPU library is compared against.  It is imported by the tests, by the smoke
check and by the benchmark's CPU-baseline leg; the product never calls it, and
it shares no code with the GPU kernels.

Everything is evaluated in float64 with NumPy.  Inputs are float arrays (their
values may lie on the bfloat16 grid); where the step *stores* a tensor in
bfloat16 (rows appended to the KV cache, the layer's output) the value is
rounded to that grid, nothing else is rounded.

What the paper fixes (Section 2.1, "Speculative Decoding"):
  * the target scores the gamma drafted tokens plus one more position in a
    single parallel forward, position i conditioning on everything before it;
  * drafted token x_i is accepted with probability min(1, p_i(x_i)/q_i(x_i)),
    tokens are examined in order and the first rejection ends the iteration;
  * on rejection a replacement is drawn from norm(max(p_i - q_i, 0));
  * at temperature 0 a token is accepted iff it equals argmax p_i and a
    rejected token is replaced by argmax p_i.
  * Eq. (TVD): TVD(P,Q) = 1/2 sum_x |P(x) - Q(x)|  (Section 6, "Distribution
    Analysis").
What it leaves open, and the reading taken here:
  R1  The verify forward receives the last emitted token followed by the gamma
      drafts (gamma+1 query positions); the cache holds everything earlier.
      Query i attends to cache rows [0, kv_len + i] inclusive.
  R2  When all gamma drafts are accepted one further token is emitted from
      p_{gamma+1} (arg-max at temperature 0), as in the algorithm of Leviathan
      et al. that Section 2.1 cites; each step emits n+1 in [1, gamma+1] tokens.
  R3  One temperature T divides target and draft logits; T = 0 is the greedy
      branch.  No top-p / top-k truncation in verification.
  R4  uniforms[b, i] (i < gamma) decides draft i whether or not it is reached;
      uniforms[b, gamma] drives the one inverse-CDF draw.
  R5  Accept iff p >= q or u*q < p (no division; u in [0,1)).
  R6  arg-max ties: lowest index.
  R7  Inverse CDF: ascending token id, smallest k with cumsum_k > u * total.
      total == 0 (p == q everywhere): draw from p_i instead.  If rounding lets no
      k cross, the largest index with positive mass.
  R8  Layer internals (the paper only speaks of a single forward pass of the target): pre-norm decoder
      layer, RMSNorm y = x*g/sqrt(mean(x^2)+eps), grouped-query attention with
      head h reading KV head h // (n_q/n_kv), rotary embedding in the
      half-split pairing (j, j + d/2) with angle pos * theta^(-2j/d), gated MLP
      down(act(gate(x)) * up(x)) with act = SiLU or tanh-GELU.

  R13 Variants of the layer used by the Gemma 3 targets of Section 5 ("Models"),
      which the paper names but does not describe; taken from that model
      family's public description: (a) sliding-window layers, where a query at
      cache row r sees rows max(0, r-W+1) .. r only; (b) RMSNorm over head_dim
      of every query and key head (own gain vectors) after the projection and
      before the rotary embedding; (c) an RMSNorm of the attention block's and
      of the MLP block's output before each is added to the residual stream.
      All are optional and off for the Qwen-shaped configurations.
  R14 Prompt pass (Section 2.2): the image features are ordinary positions of the
      sequence placed ahead of the text, attended causally like any other
      position.  Optionally (off by default) the leading image block attends
      within itself in both directions, as the Gemma 3 family's public
      description has it; the paper does not say.
  R15 Rotary position ids of the prompt pass.  Section 2.2 puts the m image
      features ahead of the text as ordinary positions; Section 5 ("Models")
      names the Qwen2.5-VL targets, whose public description numbers an image
      position by three ids (temporal, height, width) and gives each rotary
      pair j one of them: with sections (s_t, s_h, s_w), s_t + s_h + s_w = d/2,
      pairs [0, s_t) turn by the temporal id, the next s_h by the height id, the
      last s_w by the width id, each by id * theta^(-2j/d) with j the pair's own
      index.  Text positions carry three equal ids, which is the one-id rotation
      of R8.  The paper itself does not describe this; the position ids are an
      input either way (R10).

Pins (tests/test_oracle_*.py): brute-force attention loops, closed forms for
constant keys / values, causality and grouped-head invariants, equivalence of
the parallel pass with one-query-at-a-time decoding, library special cases for
norm / activations / matmul, rotary invariants, the temperature-0
longest-prefix invariant, E[accept] = 1 - TVD, chi-square of emitted tokens
against the target distribution, inverse-CDF exact histograms.
The whole layer and lm_head at 7B shapes have no external pin beyond the
composition of these pinned parts.
"""
from __future__ import annotations

import math
import numpy as np

ACT_SILU = 0
ACT_GELU_TANH = 1


# ----------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------
def round_bf16(a):
    """Nearest bfloat16 (ties to even) of each value, returned as float64."""
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(a))


def _store(a, dtype):
    if dtype == "bf16":
        return round_bf16(a)
    if dtype == "f32":
        return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# layer pieces (reading R8)
# ----------------------------------------------------------------------------
def rmsnorm(x, g, eps):
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)


def linear(x, w, b=None):
    """y = x W^T (+ b);  w is [out, in]."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T
    if b is not None:
        y = y + np.asarray(b, dtype=np.float64)
    return y


def rope(x, pos, theta):
    """Rotate x[..., d] by angle pos * theta^(-2j/d) in the pairs (j, j+d/2).

    x: [B, Q, heads, d]; pos: [B, Q] integer position ids."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    j = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * j / d)
    ang = np.asarray(pos, dtype=np.float64)[..., None, None] * inv_freq   # [B,Q,1,half]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def rope_multi(x, pos3, sections, theta):
    """Rotary embedding with three position ids per row (R15).

    x: [B, Q, heads, d]; pos3: [3, B, Q] (temporal, height, width ids); sections: three pair counts summing to
    d/2.  Pair j = (j, j + d/2) turns by pos3[c(j)] * theta^(-2j/d), c(j) = the section j falls in."""
    x = np.asarray(x, dtype=np.float64)
    pos3 = np.asarray(pos3, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    st, sh, sw = (int(v) for v in sections)
    if st + sh + sw != half or min(st, sh, sw) < 0:
        raise ValueError("sections must be non-negative and sum to d/2")
    comp = np.array([0] * st + [1] * sh + [2] * sw)                   # component of each pair
    j = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * j / d)
    ids = np.moveaxis(pos3, 0, -1)[..., comp]                          # [B, Q, half]: the id each pair turns by
    ang = (ids * inv_freq)[:, :, None, :]                              # [B, Q, 1, half]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def rope_append(qkv, pos, kv_len, n_new, k_cache, v_cache, n_q, n_kv, d, theta, dtype, sections=None,
                q_norm=None, k_norm=None, eps=1e-6):
    """Prompt-pass step between the q/k/v projection and the attention (Section 2.2; R14, R15): split the projected
    rows into heads, optionally normalise query and key heads (R13), rotate queries and keys by their position ids,
    and write keys and values of the first n_new[b] rows of sequence b into the caches at rows kv_len[b] + i.

    qkv: [B, L, (n_q + 2 n_kv) d] (query heads, key heads, value heads); pos: [B, L], or [3, B, L] with sections.
    Returns (q [B, L, n_q, d] on the storage grid -- rows at and past n_new[b] are zero --, k_cache, v_cache)."""
    qkv = np.asarray(qkv, dtype=np.float64)
    B, L, _ = qkv.shape
    k_cache = np.array(k_cache, dtype=np.float64)
    v_cache = np.array(v_cache, dtype=np.float64)
    q = qkv[..., :n_q * d].reshape(B, L, n_q, d)
    k = qkv[..., n_q * d:(n_q + n_kv) * d].reshape(B, L, n_kv, d)
    v = qkv[..., (n_q + n_kv) * d:].reshape(B, L, n_kv, d)
    if q_norm is not None:
        q = rmsnorm(q, q_norm, eps)
    if k_norm is not None:
        k = rmsnorm(k, k_norm, eps)
    if sections is None:
        q, k = rope(q, pos, theta), rope(k, pos, theta)
    else:
        q, k = rope_multi(q, pos, sections, theta), rope_multi(k, pos, sections, theta)
    q_out = np.zeros((B, L, n_q, d))
    for b in range(B):
        L0, n = int(kv_len[b]), int(n_new[b])
        q_out[b, :n] = _store(q[b, :n], dtype)
        k_cache[b, :, L0:L0 + n] = _store(k[b, :n].transpose(1, 0, 2), dtype)
        v_cache[b, :, L0:L0 + n] = _store(v[b, :n].transpose(1, 0, 2), dtype)
    return q_out, k_cache, v_cache


def silu(x):
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(-x))


def gelu_tanh(x):
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def gelu_erf(x):
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * (1.0 + np.vectorize(math.erf)(x / math.sqrt(2.0)))


def projector_mlp(h, w1, b1, w2, b2, dtype="bf16"):
    """Multimodal projector of Section 3.1 in its usual two-layer form: vision features [m, d_vis] ->
    Linear, GELU, Linear -> [m, d_emb].  The hidden activation is stored in `dtype` between the two maps."""
    mid = _store(gelu_erf(linear(h, w1, b1)), dtype)
    return linear(mid, w2, b2)


def gated_mlp(x, wg, wu, wd, act):
    a = silu if act == ACT_SILU else gelu_tanh
    return linear(a(linear(x, wg)) * linear(x, wu), wd)


def softmax(z, axis=-1):
    z = np.asarray(z, dtype=np.float64)
    z = z - np.max(z, axis=axis, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=axis, keepdims=True)


def attention(q, k_cache, v_cache, kv_len, scale=None, window=0):
    """Grouped-query causal attention of the Q new positions (reading R1).

    q: [B, Q, n_q, d]; k_cache, v_cache: [B, n_kv, L_max, d] whose rows
    [0, kv_len[b] + Q) are valid (the new positions are already appended);
    kv_len: [B] lengths before the step.  window W > 0: the query at cache row r
    sees rows max(0, r - W + 1) .. r only (R13a).  Returns [B, Q, n_q, d] float64.
    """
    q = np.asarray(q, dtype=np.float64)
    k_cache = np.asarray(k_cache, dtype=np.float64)
    v_cache = np.asarray(v_cache, dtype=np.float64)
    B, Q, n_q, d = q.shape
    n_kv = k_cache.shape[1]
    G = n_q // n_kv
    if scale is None or scale == 0:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros_like(q)
    for b in range(B):
        L = int(kv_len[b])
        for h in range(n_q):
            g = h // G
            for i in range(Q):
                n_vis = L + i + 1
                lo = max(0, n_vis - int(window)) if window else 0
                s = scale * (k_cache[b, g, lo:n_vis] @ q[b, i, h])
                out[b, i, h] = softmax(s) @ v_cache[b, g, lo:n_vis]
    return out


def prefill_attention(q, k_cache, v_cache, kv_len, n_new, scale=None, window=0, n_bidir=None):
    """Attention of the prompt pass that fills the cache (Section 2.2: the m projected image features V_1..V_m
    enter the sequence ahead of the text tokens and the language model conditions on all of them): many new
    positions per sequence instead of gamma+1, otherwise the definition of `attention`.

    q: [B, L_q, n_q, d], of which rows i < n_new[b] are sequence b's new positions; k_cache, v_cache:
    [B, n_kv, L_max, d] with rows [0, kv_len[b] + n_new[b]) valid (the new positions already appended; kv_len[b] > 0
    when the prompt is fed in several pieces).  The query at cache row r = kv_len[b] + i sees rows 0 .. r (reading R1).
    window W > 0: rows max(0, r - W + 1) .. r only (R13a).  n_bidir[b] = m (R14, optional): the first m rows are an
    image-token block whose members see the whole block, i.e. a query at row r < m sees rows 0 .. m-1.
    Returns [B, L_q, n_q, d] float64; rows i >= n_new[b] are zero."""
    q = np.asarray(q, dtype=np.float64)
    k_cache = np.asarray(k_cache, dtype=np.float64)
    v_cache = np.asarray(v_cache, dtype=np.float64)
    B, Lq, n_q, d = q.shape
    G = n_q // k_cache.shape[1]
    if scale is None or scale == 0:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros_like(q)
    for b in range(B):
        L, n = int(kv_len[b]), int(n_new[b])
        m = int(n_bidir[b]) if n_bidir is not None else 0
        for i in range(n):
            r = L + i
            hi = max(r + 1, min(m, L + n)) if r < m else r + 1        # one past the last visible row
            lo = max(0, r + 1 - int(window)) if window else 0
            for h in range(n_q):
                g = h // G
                s = scale * (k_cache[b, g, lo:hi] @ q[b, i, h])
                out[b, i, h] = softmax(s) @ v_cache[b, g, lo:hi]
    return out


def verify_layer(shape, w, x, pos, k_cache, v_cache, kv_len):
    """One decoder layer over the Q new positions of every sequence.

    shape: object with hidden, n_q_heads, n_kv_heads, head_dim, mlp, act,
    norm_eps, rope_theta, dtype and optionally window.  w: dict of ln1, wq, wk,
    wv, bq, bk, bv, wo, ln2, wg, wu, wd and optionally q_norm, k_norm [d],
    post_attn_norm, post_mlp_norm [H] (R13).  x: [B, Q, H].  Returns (x_out,
    k_cache, v_cache) with the new rows written at [kv_len[b], kv_len[b] + Q) on
    the storage grid."""
    x = np.asarray(x, dtype=np.float64)
    B, Q, H = x.shape
    nq, nkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    k_cache = np.array(k_cache, dtype=np.float64)
    v_cache = np.array(v_cache, dtype=np.float64)

    xn = rmsnorm(x, w["ln1"], shape.norm_eps)
    q = linear(xn, w["wq"], w.get("bq")).reshape(B, Q, nq, d)
    k = linear(xn, w["wk"], w.get("bk")).reshape(B, Q, nkv, d)
    v = linear(xn, w["wv"], w.get("bv")).reshape(B, Q, nkv, d)
    if w.get("q_norm") is not None:
        q = rmsnorm(q, w["q_norm"], shape.norm_eps)
    if w.get("k_norm") is not None:
        k = rmsnorm(k, w["k_norm"], shape.norm_eps)
    q = rope(q, pos, shape.rope_theta)
    k = rope(k, pos, shape.rope_theta)
    for b in range(B):
        L = int(kv_len[b])
        k_cache[b, :, L:L + Q] = _store(k[b].transpose(1, 0, 2), shape.dtype)
        v_cache[b, :, L:L + Q] = _store(v[b].transpose(1, 0, 2), shape.dtype)
    o = attention(q, k_cache, v_cache, kv_len, window=getattr(shape, "window", 0))
    a = linear(o.reshape(B, Q, nq * d), w["wo"])
    if w.get("post_attn_norm") is not None:
        a = rmsnorm(a, w["post_attn_norm"], shape.norm_eps)
    h = x + a
    hn = rmsnorm(h, w["ln2"], shape.norm_eps)
    f = gated_mlp(hn, w["wg"], w["wu"], w["wd"], shape.act)
    if w.get("post_mlp_norm") is not None:
        f = rmsnorm(f, w["post_mlp_norm"], shape.norm_eps)
    y = h + f
    return _store(y, shape.dtype), k_cache, v_cache


def lm_head_logits(x, final_norm, w_lm, eps):
    """logits = RMSNorm(x) W_lm^T (no norm when final_norm is None); x: [M, H]."""
    xn = np.asarray(x, dtype=np.float64) if final_norm is None else rmsnorm(x, final_norm, eps)
    return linear(xn, w_lm)


# ----------------------------------------------------------------------------
# acceptance (Section 2.1)
# ----------------------------------------------------------------------------
def first_argmax(row):
    return int(np.argmax(np.asarray(row)))       # np.argmax returns the first maximum (R6)


def inverse_cdf(r, u):
    """Smallest k with sum_{x<=k} r_x > u * sum_x r_x (R7); also the relative
    distance of u*total from the two cumulative values that bracket it."""
    r = np.asarray(r, dtype=np.float64)
    c = np.cumsum(r)
    total = c[-1]
    thr = float(u) * total
    hit = np.nonzero(c > thr)[0]
    if hit.size:
        k = int(hit[0])
    else:
        k = int(np.nonzero(r > 0)[0][-1])
    below = c[k - 1] if k > 0 else 0.0
    margin = min(abs(c[k] - thr), abs(thr - below) if k > 0 else np.inf) / total
    return k, float(margin)


def tvd(p, q):
    """Eq. (TVD): half the L1 distance between two distributions."""
    return 0.5 * float(np.sum(np.abs(np.asarray(p, dtype=np.float64) - np.asarray(q, dtype=np.float64))))


def tvd_rows(target_logits, draft_logits, temperature):
    """Eq. (TVD) for every row: the distance between softmax(target/T) and softmax(draft/T) (Section 6)."""
    t = np.asarray(target_logits, dtype=np.float64)
    d = np.asarray(draft_logits, dtype=np.float64)
    return np.array([tvd(softmax(t[r] / temperature), softmax(d[r] / temperature)) for r in range(t.shape[0])])


def embed_tokens(table, tokens):
    """Input rows of the first layer for fed-back tokens (Section 2.1's loop): row m is table[tokens[m]];
    a token outside the vocabulary gives a zero row."""
    table = np.asarray(table)
    out = np.zeros((len(tokens), table.shape[1]), dtype=table.dtype)
    for m, tok in enumerate(np.asarray(tokens).tolist()):
        if 0 <= tok < table.shape[0]:
            out[m] = table[tok]
    return out


def commit_tokens(n_accepted, out_tokens, kv_len):
    """Bookkeeping between two iterations of Section 2.1's loop: sequence b keeps n_b drafts and the final
    token.  Returns (last_token, new kv_len)."""
    n = np.asarray(n_accepted)
    out = np.asarray(out_tokens)
    last = np.array([out[b, n[b]] for b in range(len(n))], dtype=np.int32)
    return last, (np.asarray(kv_len) + n + 1).astype(np.int32)


def residual(p, q):
    """max(p - q, 0) without normalisation; p itself when that is identically 0 (R7)."""
    r = np.maximum(np.asarray(p, dtype=np.float64) - np.asarray(q, dtype=np.float64), 0.0)
    return r if r.sum() > 0.0 else np.asarray(p, dtype=np.float64)


def spec_accept(target_logits, draft_logits, draft_tokens, uniforms, temperature,
                return_final_mass=False):
    """Sequential accept / reject / resample for every sequence of the batch.

    target_logits [B, gamma+1, V], draft_logits [B, gamma, V] (ignored at T=0),
    draft_tokens [B, gamma] (a value outside [0, V) is rejected at either
    temperature), uniforms [B, gamma+1] (ignored at T=0).  gamma = 0
    is the drafting loop's own sampling step: one token drawn from the single
    row's distribution, nothing to verify.
    Returns n_accepted [B] int32, out_tokens [B, gamma+1] int32 (accepted
    drafts, the final token, then -1), and margin [B, 2]: the smallest relative
    distance from flipping of (0) any evaluated accept comparison with p < q,
    |u - p/q| / max(u, p/q), and (1) the inverse-CDF draw, as a fraction of the
    total mass (both inf at T=0).  With return_final_mass the unnormalised mass
    vector the final token was drawn from is returned per sequence as well.
    """
    t = np.asarray(target_logits, dtype=np.float64)
    B, Q, V = t.shape
    gamma = Q - 1
    x = np.asarray(draft_tokens).reshape(B, gamma)
    n_acc = np.zeros(B, dtype=np.int32)
    out = np.full((B, Q), -1, dtype=np.int32)
    margin = np.full((B, 2), np.inf)
    masses = []
    greedy = (temperature == 0)
    if not greedy:
        dl = np.asarray(draft_logits, dtype=np.float64) if gamma > 0 else None
        u = np.asarray(uniforms, dtype=np.float64).reshape(B, Q)
    for b in range(B):
        n = 0
        for i in range(gamma):
            tok = int(x[b, i])
            if not (0 <= tok < V):
                ok = False          # not a token of the vocabulary: p_i and q_i are not defined for it
            elif greedy:
                ok = (tok == first_argmax(t[b, i]))
            else:
                p = softmax(t[b, i] / temperature)[tok]
                q = softmax(dl[b, i] / temperature)[tok]
                ok = (p >= q) or (u[b, i] * q < p)
                if p < q:
                    ratio = p / q
                    margin[b, 0] = min(margin[b, 0], abs(u[b, i] - ratio) / max(u[b, i], ratio))
            if not ok:
                break
            out[b, n] = tok
            n += 1
        if greedy:
            final = first_argmax(t[b, n])
        else:
            p = softmax(t[b, n] / temperature)
            r = residual(p, softmax(dl[b, n] / temperature)) if n < gamma else p
            final, margin[b, 1] = inverse_cdf(r, u[b, gamma])
            if return_final_mass:
                masses.append(r)
        out[b, n] = final
        n_acc[b] = n
    if return_final_mass:
        return n_acc, out, margin, masses
    return n_acc, out, margin
