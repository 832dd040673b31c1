"""Seeded synthetic inputs for the speculative-decoding verify step.

This module only draws random tensors of the right shapes; it contains none of
the method's arithmetic (no softmax, no attention, no acceptance rule) so that
it can feed both the GPU library and the CPU checker without coupling them.

The paper evaluates on multimodal prompts (an image prefix followed by text,
speculation length gamma = 5, temperatures 0 and 1; Section 5, "Inference
Settings").  Those prompts and the trained models are not available, so every
tensor here is synthetic: Gaussian weights and activations with the layer
geometry of the 7B / 12B targets the paper names (Section 5, "Models"), a KV
cache whose leading rows stand for image tokens (Section 2.2), and draft logits
obtained by perturbing the target logits.

All arrays are NumPy float32/int32.  In "bf16" mode every float value is
rounded so that it is exactly representable in bfloat16; the arrays stay
float32 so that both consumers can widen them without loss.
"""
from __future__ import annotations

from dataclasses import dataclass, field
import numpy as np

ACT_SILU = 0
ACT_GELU_TANH = 1


def bf16_representable(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), keep float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = u >> np.uint32(16)                   # one temporary, updated in place (the big weight matrices are ~1 GB each)
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r &= np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(a.shape)


@dataclass
class LayerShape:
    """Geometry of one decoder layer plus the vocabulary projection."""
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp: int
    vocab: int
    act: int = ACT_SILU
    qkv_bias: bool = True
    norm_eps: float = 1e-6
    rope_theta: float = 1e6
    dtype: str = "bf16"          # "bf16" or "f32"
    # Variants of the Gemma 3 family (the 12B / 27B targets of Section 5): sliding-window attention over the
    # last `window` cache rows (0 = all), RMSNorm of every query / key head, RMSNorm of each block's output.
    window: int = 0
    qk_norm: bool = False
    post_norms: bool = False

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# Shapes used throughout tests and the benchmark.
TINY = LayerShape(256, 4, 2, 64, 688, 4096, ACT_SILU, True, dtype="f32")
TINY_BF16 = LayerShape(256, 4, 2, 64, 704, 4096, ACT_SILU, True, dtype="bf16")
QWEN7B = LayerShape(3584, 28, 4, 128, 18944, 152064, ACT_SILU, True)
GEMMA12B = LayerShape(3840, 16, 8, 256, 15360, 262144, ACT_GELU_TANH, False)
# Drafter-sized shapes (Section 5, "Models": a small language model of the target's family drafts for it).
# The drafter's vocabulary is taken equal to the target's so that both logit rows index the same tokens.
TINY_DRAFT_BF16 = LayerShape(128, 2, 1, 64, 352, 4096, ACT_SILU, True, dtype="bf16")
QWEN1P5B = LayerShape(1536, 12, 2, 128, 8960, 152064, ACT_SILU, True)
# A local (sliding-window) layer of the Gemma3-12B-shaped target with that family's extra norms.
GEMMA12B_LOCAL = LayerShape(3840, 16, 8, 256, 15360, 262144, ACT_GELU_TANH, False, rope_theta=1e4,
                            window=1024, qk_norm=True, post_norms=True)
TINY_GEMMA = LayerShape(256, 4, 2, 64, 688, 4096, ACT_GELU_TANH, False, rope_theta=1e4, dtype="f32",
                        window=48, qk_norm=True, post_norms=True)
TINY_GEMMA_BF16 = LayerShape(256, 4, 2, 64, 704, 4096, ACT_GELU_TANH, False, rope_theta=1e4, dtype="bf16",
                             window=48, qk_norm=True, post_norms=True)


def _rng(seed, *stream):
    return np.random.default_rng([int(seed), *[int(s) for s in stream]])


def _finish(a, dtype):
    a = a.astype(np.float32, copy=False)
    return bf16_representable(a) if dtype == "bf16" else a


def normal(shape, std, seed, *stream, dtype="bf16", mean=0.0):
    g = _rng(seed, *stream)
    a = g.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return _finish(a, dtype)


def layer_weights(shape: LayerShape, seed: int, layer: int = 0, std: float = 0.02, threads: int = 1):
    """Weights of one decoder layer: every linear map N(0, std), norm gains near 1.

    Gains are 1 + 0.1 N(0,1) rather than exactly 1 so that a missing gain
    multiplication changes the result.
    """
    s, dt = shape, shape.dtype
    H, d = s.hidden, s.head_dim
    nq, nkv, F = s.n_q_heads * d, s.n_kv_heads * d, s.mlp
    # name -> (shape, std, stream id, mean); every tensor has its own random stream, so the draws are independent of
    # the order (and of the number of threads) they are made in
    spec = {
        "ln1": ((H,), 0.1, 0, 1.0), "wq": ((nq, H), std, 1, 0.0), "wk": ((nkv, H), std, 2, 0.0),
        "wv": ((nkv, H), std, 3, 0.0), "wo": ((H, nq), std, 4, 0.0), "ln2": ((H,), 0.1, 5, 1.0),
        "wg": ((F, H), std, 6, 0.0), "wu": ((F, H), std, 7, 0.0), "wd": ((H, F), std, 8, 0.0),
    }
    if s.qkv_bias:
        spec.update(bq=((nq,), std, 9, 0.0), bk=((nkv,), std, 10, 0.0), bv=((nkv,), std, 11, 0.0))
    if s.qk_norm:
        spec.update(q_norm=((d,), 0.1, 12, 1.0), k_norm=((d,), 0.1, 13, 1.0))
    if s.post_norms:
        spec.update(post_attn_norm=((H,), 0.1, 14, 1.0), post_mlp_norm=((H,), 0.1, 15, 1.0))

    def draw(item):
        name, (shp, sd, stream, mean) = item
        return name, normal(shp, sd, seed, layer, stream, dtype=dt, mean=mean)

    w = {"bq": None, "bk": None, "bv": None}
    if threads > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(threads) as pool:
            w.update(dict(pool.map(draw, sorted(spec.items(), key=lambda kv: -int(np.prod(kv[1][0]))))))
    else:
        w.update(dict(map(draw, spec.items())))
    return w


def lm_head_weights(shape: LayerShape, seed: int, std: float = 0.02):
    dt = shape.dtype
    return {
        "final_norm": normal((shape.hidden,), 0.1, seed, 1000, 0, dtype=dt, mean=1.0),
        "w_lm": normal((shape.vocab, shape.hidden), std, seed, 1000, 1, dtype=dt),
    }


def embedding_table(shape: LayerShape, seed: int, std: float = 1.0):
    """Input embedding rows, one per vocabulary entry: N(0, std)."""
    return normal((shape.vocab, shape.hidden), std, seed, 1000, 2, dtype=shape.dtype)


@dataclass
class KVState:
    """Cached keys/values in the logical layout [B, n_kv, L_max, d] (float32
    values on the storage grid), lengths before the step, image-prefix sizes."""
    k: np.ndarray
    v: np.ndarray
    kv_len: np.ndarray      # int32 [B]
    n_img: np.ndarray       # int32 [B]
    l_max: int


def kv_cache(shape: LayerShape, batch: int, n_query: int, kv_len, n_img, seed: int,
             layer: int = 0, std: float = 1.0, img_scale: float = 1.5,
             hot_keys: int = 0, l_max: int | None = None, junk_tail: bool = True) -> KVState:
    """Cached prefix: rows [0, n_img[b]) are image-token positions (Section 2.2:
    projected image features precede the text tokens), drawn with a larger
    spread so that a kernel skipping or duplicating the prefix is caught.

    `hot_keys` rows per (b, head) get their key scaled by 8 to force the running
    maximum of a streaming softmax to move late in the stream.
    Rows at and beyond kv_len[b] hold large finite junk: the step overwrites
    rows [kv_len, kv_len + n_query) and must never read anything beyond.
    """
    kv_len = np.broadcast_to(np.asarray(kv_len, dtype=np.int32), (batch,)).copy()
    n_img = np.broadcast_to(np.asarray(n_img, dtype=np.int32), (batch,)).copy()
    if l_max is None:
        l_max = int(kv_len.max()) + n_query
    dt = shape.dtype
    nkv, d = shape.n_kv_heads, shape.head_dim
    k = normal((batch, nkv, l_max, d), std, seed, layer, 20, dtype="f32")
    v = normal((batch, nkv, l_max, d), std, seed, layer, 21, dtype="f32")
    g = _rng(seed, layer, 22)
    for b in range(batch):
        k[b, :, : n_img[b]] *= np.float32(img_scale)
        v[b, :, : n_img[b]] *= np.float32(img_scale)
        if hot_keys:
            for h in range(nkv):
                rows = g.choice(int(kv_len[b]), size=min(hot_keys, int(kv_len[b])), replace=False)
                k[b, h, rows] *= np.float32(8.0)
        if junk_tail:
            k[b, :, kv_len[b]:] = np.float32(777.0)
            v[b, :, kv_len[b]:] = np.float32(-555.0)
    return KVState(_finish(k, dt), _finish(v, dt), kv_len, n_img, l_max)


def hidden_states(shape: LayerShape, batch: int, n_query: int, seed: int):
    return normal((batch, n_query, shape.hidden), 1.0, seed, 30, dtype=shape.dtype)


def queries(shape: LayerShape, batch: int, n_query: int, seed: int, std: float = 1.0):
    return normal((batch, n_query, shape.n_q_heads, shape.head_dim), std, seed, 31,
                  dtype=shape.dtype)


def positions(kv_len, n_img, n_query: int, compress_image: bool = False):
    """Rotary position ids of the new tokens.  By default the cache row index;
    with compress_image the image prefix counts as half its length, standing
    for multimodal rotary schemes where ids and cache rows differ."""
    kv_len = np.asarray(kv_len, dtype=np.int64)
    base = kv_len - (np.asarray(n_img, dtype=np.int64) // 2 if compress_image else 0)
    return (base[:, None] + np.arange(n_query)[None, :]).astype(np.int32)


@dataclass
class AcceptInputs:
    target_logits: np.ndarray   # float32 [B, gamma+1, V]
    draft_logits: np.ndarray    # float32 [B, gamma, V]
    draft_tokens: np.ndarray    # int32 [B, gamma]
    uniforms: np.ndarray        # float32 [B, gamma+1] in [0, 1)
    temperature: float


def draft_tokens_from(draft_logits: np.ndarray, temperature: float, seed: int) -> np.ndarray:
    """Tokens the drafter would propose (Section 2.1): the arg-max of its logits
    at temperature 0, otherwise a draw from its distribution.  The draw uses
    Gumbel perturbation of the scaled logits followed by arg-max, which needs no
    normalisation; ties resolve to the lowest index (np.argmax)."""
    B, G, V = draft_logits.shape
    out = np.empty((B, G), dtype=np.int32)
    g = _rng(seed, 41)
    for b in range(B):
        for i in range(G):
            row = draft_logits[b, i].astype(np.float64)
            if temperature > 0:
                row = row / temperature + g.gumbel(size=V)
            out[b, i] = int(np.argmax(row))
    return out


def accept_inputs(batch: int, gamma: int, vocab: int, temperature: float, seed: int,
                  target_std: float = 1.0, noise_std: float = 1.0, corr: float | None = None,
                  peak: float = 1.0, target_logits: np.ndarray | None = None) -> AcceptInputs:
    """Target and draft logits, draft tokens and uniforms for one accept call.

    corr=None: draft = target + N(0, noise_std).  corr=c: draft =
    c*target + sqrt(1-c^2) N(0, target_std) (same marginal, correlation c).
    `peak` multiplies the target logits before the draft is derived, giving a
    sharper distribution and hence longer accepted prefixes.
    """
    Q = gamma + 1
    if target_logits is None:
        t = normal((batch, Q, vocab), target_std, seed, 50, dtype="f32")
    else:
        t = np.array(target_logits, dtype=np.float32).reshape(batch, Q, vocab)
    if peak != 1.0:
        t = (t * np.float32(peak)).astype(np.float32)
    if corr is None:
        d = t[:, :gamma] + normal((batch, gamma, vocab), noise_std, seed, 51, dtype="f32")
    else:
        d = np.float32(corr) * t[:, :gamma] + np.float32(np.sqrt(1.0 - corr * corr)) * \
            normal((batch, gamma, vocab), target_std * peak, seed, 51, dtype="f32")
    d = np.ascontiguousarray(d, dtype=np.float32)
    u = _rng(seed, 52).random((batch, Q), dtype=np.float32)
    u = np.minimum(u, np.float32(1.0 - 2 ** -24))
    x = draft_tokens_from(d, temperature, seed)
    return AcceptInputs(np.ascontiguousarray(t), d, x, u, float(temperature))
