"""ctypes binding of libmassv_verify.so (see include/massv_verify.h).

Argument marshalling only: tensors are torch CUDA tensors whose device
pointers are handed to the C ABI; every step of the verify path runs in the
library's HIP kernels.  There is no CPU or PyTorch fallback: if the shared
library is missing, `load()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmassv_verify.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, ELAUNCH = 0, -1, -2, -3, -4
F32, BF16 = 0, 1
ACT_SILU, ACT_GELU_TANH = 0, 1
V_BLOCK = 32
MAX_ROWS = 64

EXPORTS = [
    "massv_status_string", "massv_abi_version",
    "massv_verify_attention_workspace", "massv_verify_attention", "massv_v_cache_pack", "massv_k_cache_pack",
    "massv_verify_layer_workspace", "massv_verify_layer", "massv_verify_layers",
    "massv_lm_head_logits_workspace", "massv_lm_head_logits",
    "massv_spec_accept_workspace", "massv_spec_accept", "massv_trace_kernel", "massv_weight_pack",
    "massv_spec_tvd_workspace", "massv_spec_tvd", "massv_embed_tokens", "massv_commit_tokens",
    "massv_linear_workspace", "massv_linear",
    "massv_lm_head_greedy_accept_workspace", "massv_lm_head_greedy_accept",
    "massv_spec_accept_static_limit", "massv_spec_accept_static", "massv_prefill_attention", "massv_rope_append", "massv_linear_ex", "massv_rmsnorm",
    "massv_lm_head_accept_workspace", "massv_lm_head_accept",
]
K_QKV, K_ATTENTION, K_ATTN_COMBINE, K_OPROJ, K_GATEUP, K_DOWN, K_LMHEAD, K_ACCEPT_STATS, K_RESIDUAL_MASS, K_LINEAR, K_PREFILL_ATTENTION = range(11)
LIN_NONE, LIN_SILU, LIN_GELU_TANH, LIN_GELU_ERF = range(4)


class AttnDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_query", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("l_max", C.c_int32),
                ("scale", C.c_float), ("dtype", C.c_int32), ("window", C.c_int32)]


class LayerDesc(C.Structure):
    _fields_ = [("attn", AttnDesc), ("hidden", C.c_int32), ("mlp", C.c_int32), ("act", C.c_int32),
                ("qkv_bias", C.c_int32), ("norm_eps", C.c_float), ("rope_theta", C.c_float)]


WEIGHT_FIELDS = ["ln1", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "ln2", "wg", "wu", "wd",
                 "q_norm", "k_norm", "post_attn_norm", "post_mlp_norm"]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class MassvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load():
    """Load the shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_10526_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    lib.massv_status_string.restype = C.c_char_p
    lib.massv_status_string.argtypes = [C.c_int]
    lib.massv_abi_version.restype = C.c_int
    lib.massv_abi_version.argtypes = []
    lib.massv_verify_attention_workspace.restype = sz
    lib.massv_verify_attention_workspace.argtypes = [C.POINTER(AttnDesc)]
    lib.massv_verify_attention.restype = C.c_int
    lib.massv_verify_attention.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.massv_prefill_attention.restype = C.c_int
    lib.massv_prefill_attention.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, vp]
    lib.massv_rope_append.restype = C.c_int
    lib.massv_rope_append.argtypes = [C.POINTER(AttnDesc), vp, vp, i32, C.POINTER(C.c_int32), f32, vp, vp, f32, vp, vp, vp, vp, vp, vp]
    lib.massv_v_cache_pack.restype = C.c_int
    lib.massv_v_cache_pack.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
    lib.massv_k_cache_pack.restype = C.c_int
    lib.massv_k_cache_pack.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
    lib.massv_verify_layer_workspace.restype = sz
    lib.massv_verify_layer_workspace.argtypes = [C.POINTER(LayerDesc)]
    lib.massv_verify_layer.restype = C.c_int
    lib.massv_verify_layer.argtypes = [C.POINTER(LayerDesc), C.POINTER(LayerWeights), vp, vp, vp, vp, vp,
                                       vp, sz, vp]
    lib.massv_verify_layers.restype = C.c_int
    lib.massv_verify_layers.argtypes = [C.POINTER(LayerDesc), C.POINTER(LayerWeights), i32, vp, vp,
                                        C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), vp,
                                        C.POINTER(C.c_int32), C.POINTER(C.c_float), vp, sz, vp]
    lib.massv_lm_head_logits_workspace.restype = sz
    lib.massv_lm_head_logits_workspace.argtypes = [i32, i32, i32, i32]
    lib.massv_lm_head_logits.restype = C.c_int
    lib.massv_lm_head_logits.argtypes = [vp, vp, vp, vp, i32, i32, i32, f32, i32, vp, sz, vp]
    lib.massv_spec_accept_workspace.restype = sz
    lib.massv_spec_accept_workspace.argtypes = [i32, i32, i32]
    lib.massv_spec_accept.restype = C.c_int
    lib.massv_spec_accept.argtypes = [vp, vp, vp, vp, f32, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.massv_spec_accept_static_limit.restype = sz
    lib.massv_spec_accept_static_limit.argtypes = []
    lib.massv_spec_accept_static.restype = C.c_int
    lib.massv_spec_accept_static.argtypes = [vp, vp, vp, vp, f32, i32, i32, i32, vp, vp, vp]
    lib.massv_weight_pack.restype = C.c_int
    lib.massv_weight_pack.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.massv_trace_kernel.restype = C.c_int
    lib.massv_trace_kernel.argtypes = [C.c_int, vp, vp]
    lib.massv_spec_tvd_workspace.restype = sz
    lib.massv_spec_tvd_workspace.argtypes = [i32, i32]
    lib.massv_spec_tvd.restype = C.c_int
    lib.massv_spec_tvd.argtypes = [vp, vp, f32, i32, i32, vp, vp, sz, vp]
    lib.massv_linear_workspace.restype = sz
    lib.massv_linear_workspace.argtypes = [i32, i32, i32, i32]
    lib.massv_linear.restype = C.c_int
    lib.massv_linear.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]
    lib.massv_linear_ex.restype = C.c_int
    lib.massv_linear_ex.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]
    lib.massv_rmsnorm.restype = C.c_int
    lib.massv_rmsnorm.argtypes = [vp, vp, vp, i32, i32, f32, i32, vp]
    lib.massv_lm_head_greedy_accept_workspace.restype = sz
    lib.massv_lm_head_greedy_accept_workspace.argtypes = [i32, i32, i32, i32, i32]
    lib.massv_lm_head_greedy_accept.restype = C.c_int
    lib.massv_lm_head_greedy_accept.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, f32, i32, vp, vp, vp, sz, vp]
    lib.massv_lm_head_accept_workspace.restype = sz
    lib.massv_lm_head_accept_workspace.argtypes = [i32, i32, i32, i32, i32]
    lib.massv_lm_head_accept.restype = C.c_int
    lib.massv_lm_head_accept.argtypes = [vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, f32, i32, vp, vp, vp, vp, sz, vp]
    lib.massv_commit_tokens.restype = C.c_int
    lib.massv_commit_tokens.argtypes = [vp, vp, vp, vp, i32, i32, vp]
    lib.massv_embed_tokens.restype = C.c_int
    lib.massv_embed_tokens.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().massv_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise MassvError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


_workspaces: dict = {}


def workspace(nbytes: int, device) -> torch.Tensor:
    """A reusable scratch buffer of at least nbytes on `device`."""
    key = (torch.device(device).index or 0)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty(max(int(nbytes), 1 << 20), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def _need(t, name, dtype=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}")


# ---------------------------------------------------------------------------
# verify_attention
# ---------------------------------------------------------------------------
def attn_desc(batch, n_query, n_q_heads, n_kv_heads, head_dim, l_max, dtype, scale=0.0, window=0) -> AttnDesc:
    return AttnDesc(batch, n_query, n_q_heads, n_kv_heads, head_dim, l_max, scale, dtype, window)


def v_cache_pack(v_row_major: torch.Tensor) -> torch.Tensor:
    """[B, n_kv, L_max, d] row-major values -> the library's blocked value-cache
    layout [B, n_kv, L_max/32, d, 32] (done by the library's own kernel)."""
    _need(v_row_major, "v")
    B, n_kv, L, d = v_row_major.shape
    out = torch.empty((B, n_kv, L // V_BLOCK, d, V_BLOCK), dtype=v_row_major.dtype, device=v_row_major.device)
    _check(load().massv_v_cache_pack(_ptr(v_row_major), _ptr(out), B, n_kv, L, d,
                                     dtype_code(v_row_major), _stream()), "massv_v_cache_pack")
    return out


def k_cache_pack(k_row_major: torch.Tensor) -> torch.Tensor:
    """[B, n_kv, L_max, d] row-major keys -> the library's key-cache layout for that dtype (bf16: rows
    blocked in matrix-operand order, fp32: unchanged), done by the library's own kernel.  The result keeps
    the shape [B, n_kv, L_max, d]; only the order of the elements in memory differs."""
    _need(k_row_major, "k")
    B, n_kv, L, d = k_row_major.shape
    out = torch.empty_like(k_row_major)
    _check(load().massv_k_cache_pack(_ptr(k_row_major), _ptr(out), B, n_kv, L, d,
                                     dtype_code(k_row_major), _stream()), "massv_k_cache_pack")
    return out


def verify_attention(q, k_cache, v_cache, kv_len, scale=0.0, out=None, ws=None, window=0):
    """q [B,Q,n_q,d]; k_cache [B,n_kv,L_max,d] in the key-cache layout (k_cache_pack); v_cache blocked
    [B,n_kv,L_max/32,d,32];
    kv_len int32 [B]; window > 0: sliding-window attention over the last `window` rows.
    Returns out [B,Q,n_q,d]."""
    lib = load()
    for t, n in ((q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache")):
        _need(t, n, q.dtype)
    _need(kv_len, "kv_len", torch.int32)
    B, Q, n_q, d = q.shape
    n_kv, l_max = k_cache.shape[1], k_cache.shape[2]
    desc = attn_desc(B, Q, n_q, n_kv, d, l_max, dtype_code(q), scale, window)
    if out is None:
        out = torch.empty_like(q)
    need = lib.massv_verify_attention_workspace(C.byref(desc))
    if ws is None:
        ws = workspace(need, q.device)
    _check(lib.massv_verify_attention(C.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(kv_len),
                                      _ptr(out), _ptr(ws), ws.numel(), _stream()), "massv_verify_attention")
    return out


def prefill_attention(q, k_cache, v_cache, kv_len, n_new, n_bidir=None, scale=0.0, out=None, window=0):
    """q [B,L_q,n_q,d]; caches as for verify_attention; kv_len, n_new (and n_bidir) int32 [B].
    Returns out [B,L_q,n_q,d]; rows i >= n_new[b] are left as they were (zeros for a fresh `out`)."""
    for t, n in ((q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache")):
        _need(t, n, q.dtype)
    for t, n in ((kv_len, "kv_len"), (n_new, "n_new")) + (((n_bidir, "n_bidir"),) if n_bidir is not None else ()):
        _need(t, n, torch.int32)
    B, Lq, n_q, d = q.shape
    n_kv, l_max = k_cache.shape[1], k_cache.shape[2]
    desc = attn_desc(B, Lq, n_q, n_kv, d, l_max, dtype_code(q), scale, window)
    if out is None:
        out = torch.zeros_like(q)
    _check(load().massv_prefill_attention(C.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(kv_len),
                                          _ptr(n_new), _ptr(n_bidir), _ptr(out), _stream()), "massv_prefill_attention")
    return out


def rope_append(qkv, pos, kv_len, n_new, k_cache, v_cache, n_q, rope_theta, sections=None, q_norm=None, k_norm=None,
                norm_eps=1e-6, q_out=None):
    """qkv [B,L_q,(n_q+2n_kv)d]; pos int32 [B,L_q], or [3,B,L_q] with `sections` (three pair counts, host ints);
    caches as for verify_attention (written in place at rows kv_len[b] .. kv_len[b]+n_new[b]-1).
    Returns q_out [B,L_q,n_q,d]; rows i >= n_new[b] are left as they were (zeros for a fresh `q_out`)."""
    for t, n in ((qkv, "qkv"), (k_cache, "k_cache"), (v_cache, "v_cache")):
        _need(t, n, qkv.dtype)
    for t, n in ((pos, "pos"), (kv_len, "kv_len"), (n_new, "n_new")):
        _need(t, n, torch.int32)
    B, Lq, width = qkv.shape
    n_kv, l_max, d = k_cache.shape[1], k_cache.shape[2], k_cache.shape[3]
    if width != (n_q + 2 * n_kv) * d:
        raise ValueError("qkv width does not match the head counts")
    n_pos = 1 if sections is None else 3
    if tuple(pos.shape) != ((B, Lq) if n_pos == 1 else (3, B, Lq)):
        raise ValueError("pos has the wrong shape")
    sec = None if sections is None else (C.c_int32 * 3)(*[int(v) for v in sections])
    desc = attn_desc(B, Lq, n_q, n_kv, d, l_max, dtype_code(qkv), 0.0, 0)
    if q_out is None:
        q_out = torch.zeros((B, Lq, n_q, d), dtype=qkv.dtype, device=qkv.device)
    _check(load().massv_rope_append(C.byref(desc), _ptr(qkv), _ptr(pos), n_pos, sec, float(rope_theta), _ptr(q_norm),
                                    _ptr(k_norm), float(norm_eps), _ptr(kv_len), _ptr(n_new), _ptr(q_out), _ptr(k_cache),
                                    _ptr(v_cache), _stream()), "massv_rope_append")
    return q_out


# ---------------------------------------------------------------------------
# verify_layer / lm_head_logits
# ---------------------------------------------------------------------------
@dataclass
class LayerConfig:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp: int
    act: int = ACT_SILU
    qkv_bias: bool = True
    norm_eps: float = 1e-6
    rope_theta: float = 1e6
    scale: float = 0.0
    window: int = 0


def layer_desc(cfg: LayerConfig, batch, n_query, l_max, dtype) -> LayerDesc:
    a = attn_desc(batch, n_query, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, l_max, dtype, cfg.scale, cfg.window)
    return LayerDesc(a, cfg.hidden, cfg.mlp, cfg.act, int(bool(cfg.qkv_bias)), cfg.norm_eps, cfg.rope_theta)


MATRIX_FIELDS = ["wq", "wk", "wv", "wo", "wg", "wu", "wd"]


def weight_pack(w: torch.Tensor) -> torch.Tensor:
    """Row-major [N, K] projection matrix -> the library's streaming layout (same shape and dtype on
    the torch side; the element order is the library's).  Done by the library's own kernel."""
    _need(w, "w")
    N, K = w.shape
    out = torch.empty_like(w)
    _check(load().massv_weight_pack(_ptr(w), _ptr(out), N, K, dtype_code(w), _stream()), "massv_weight_pack")
    return out


def pack_layer_weights(w: dict) -> dict:
    """Copy of a layer's weight dict with every projection matrix in streaming layout."""
    return {k: (weight_pack(v) if (k in MATRIX_FIELDS and v is not None) else v) for k, v in w.items()}


def layer_weights(w: dict) -> LayerWeights:
    """dict of CUDA tensors (keys ln1, wq, ... wd; matrices already in streaming layout, see
    pack_layer_weights; biases may be None) -> struct of device pointers.  The caller keeps the
    tensors alive."""
    lw = LayerWeights()
    for name in WEIGHT_FIELDS:
        t = w.get(name)
        if t is not None:
            _need(t, name)
        setattr(lw, name, None if t is None else t.data_ptr())
    return lw


def verify_layer_workspace(desc: LayerDesc) -> int:
    return load().massv_verify_layer_workspace(C.byref(desc))


def verify_layer(cfg: LayerConfig, w, x, pos, k_cache, v_cache, kv_len, ws=None, desc=None, lw=None):
    """One decoder layer over the new positions; x [B,Q,H] is updated in place
    and the caches receive the new rows.  `w` is a dict of tensors (matrices in
    streaming layout, see pack_layer_weights) or a prebuilt LayerWeights."""
    lib = load()
    _need(x, "x")
    _need(pos, "pos", torch.int32)
    _need(kv_len, "kv_len", torch.int32)
    _need(k_cache, "k_cache", x.dtype)
    _need(v_cache, "v_cache", x.dtype)
    B, Q, _ = x.shape
    if desc is None:
        desc = layer_desc(cfg, B, Q, k_cache.shape[2], dtype_code(x))
    if lw is None:
        lw = w if isinstance(w, LayerWeights) else layer_weights(w)
    if ws is None:
        ws = workspace(lib.massv_verify_layer_workspace(C.byref(desc)), x.device)
    _check(lib.massv_verify_layer(C.byref(desc), C.byref(lw), _ptr(x), _ptr(pos), _ptr(k_cache), _ptr(v_cache),
                                  _ptr(kv_len), _ptr(ws), ws.numel(), _stream()), "massv_verify_layer")
    return x


class LayerStack:
    """Marshalled arguments of massv_verify_layers for a fixed stack of layers: arrays of weight
    structs and cache pointers built once.  Keeps the tensors alive."""

    def __init__(self, weights: list, k_caches: list, v_caches: list, windows=None, rope_thetas=None):
        """windows / rope_thetas: optional per-layer sliding-window sizes and rotary bases (stacks that
        interleave local and global layers); None = the descriptor's values for every layer."""
        n = len(weights)
        assert n == len(k_caches) == len(v_caches) and n >= 1
        assert windows is None or len(windows) == n
        assert rope_thetas is None or len(rope_thetas) == n
        self.windows = None if windows is None else (C.c_int32 * n)(*[int(v) for v in windows])
        self.rope_thetas = None if rope_thetas is None else (C.c_float * n)(*[float(v) for v in rope_thetas])
        self.n = n
        self._keep = (weights, k_caches, v_caches)
        lws = [w if isinstance(w, LayerWeights) else layer_weights(w) for w in weights]
        self.weights = (LayerWeights * n)(*lws)
        self.k = (C.c_void_p * n)(*[t.data_ptr() for t in k_caches])
        self.v = (C.c_void_p * n)(*[t.data_ptr() for t in v_caches])


def verify_layers(cfg: LayerConfig, stack: LayerStack, x, pos, kv_len, l_max, ws=None, desc=None):
    """All layers of `stack` over the new positions (one library call); x [B,Q,H] updated in place."""
    lib = load()
    _need(x, "x")
    _need(pos, "pos", torch.int32)
    _need(kv_len, "kv_len", torch.int32)
    B, Q, _ = x.shape
    if desc is None:
        desc = layer_desc(cfg, B, Q, l_max, dtype_code(x))
    if ws is None:
        ws = workspace(lib.massv_verify_layer_workspace(C.byref(desc)), x.device)
    _check(lib.massv_verify_layers(C.byref(desc), stack.weights, stack.n, _ptr(x), _ptr(pos), stack.k, stack.v,
                                   _ptr(kv_len), stack.windows, stack.rope_thetas, _ptr(ws), ws.numel(), _stream()),
           "massv_verify_layers")
    return x


def lm_head_logits(x, final_norm, w_lm, norm_eps=1e-6, out=None, ws=None):
    """x [M,H] (or [B,Q,H]); w_lm [V,H] in streaming layout (weight_pack); returns float32 logits [M,V]."""
    lib = load()
    _need(x, "x")
    _need(w_lm, "w_lm", x.dtype)
    H = x.shape[-1]
    M = x.numel() // H
    V = w_lm.shape[0]
    if out is None:
        out = torch.empty((M, V), dtype=torch.float32, device=x.device)
    need = lib.massv_lm_head_logits_workspace(M, H, V, dtype_code(x))
    if ws is None:
        ws = workspace(need, x.device)
    _check(lib.massv_lm_head_logits(_ptr(x), _ptr(final_norm), _ptr(w_lm), _ptr(out), M, H, V,
                                    float(norm_eps), dtype_code(x), _ptr(ws), ws.numel(), _stream()),
           "massv_lm_head_logits")
    return out


# ---------------------------------------------------------------------------
# spec_accept
# ---------------------------------------------------------------------------
def spec_accept(target_logits, draft_logits, draft_tokens, uniforms, temperature,
                n_accepted=None, out_tokens=None, ws=None):
    """target_logits [B,gamma+1,V] f32, draft_logits [B,gamma,V] f32 (None at T=0),
    draft_tokens [B,gamma] i32, uniforms [B,gamma+1] f32 (None at T=0).
    gamma = 0 (draft_logits, draft_tokens None) draws one token per sequence.
    Returns (n_accepted [B] i32, out_tokens [B,gamma+1] i32)."""
    lib = load()
    _need(target_logits, "target_logits", torch.float32)
    if draft_tokens is not None:
        _need(draft_tokens, "draft_tokens", torch.int32)
    if draft_logits is not None:
        _need(draft_logits, "draft_logits", torch.float32)
    if uniforms is not None:
        _need(uniforms, "uniforms", torch.float32)
    B, Q, V = target_logits.shape
    gamma = Q - 1
    dev = target_logits.device
    if n_accepted is None:
        n_accepted = torch.empty((B,), dtype=torch.int32, device=dev)
    if out_tokens is None:
        out_tokens = torch.empty((B, Q), dtype=torch.int32, device=dev)
    need = lib.massv_spec_accept_workspace(B, gamma, V)
    if ws is None:
        ws = workspace(need, dev)
    _check(lib.massv_spec_accept(_ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens), _ptr(uniforms),
                                 float(temperature), B, gamma, V, _ptr(n_accepted), _ptr(out_tokens),
                                 _ptr(ws), ws.numel(), _stream()), "massv_spec_accept")
    return n_accepted, out_tokens


def spec_accept_static(target_logits, draft_logits, draft_tokens, uniforms, temperature, n_accepted, out_tokens):
    """massv_spec_accept_static: as spec_accept, scratch space inside the library; the caller passes every
    tensor, outputs included (this wrapper allocates nothing either)."""
    _need(target_logits, "target_logits", torch.float32)
    _need(n_accepted, "n_accepted", torch.int32)
    _need(out_tokens, "out_tokens", torch.int32)
    B, Q, V = target_logits.shape
    _check(load().massv_spec_accept_static(_ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens), _ptr(uniforms),
                                           float(temperature), B, Q - 1, V, _ptr(n_accepted), _ptr(out_tokens),
                                           _stream()), "massv_spec_accept_static")
    return n_accepted, out_tokens


def lm_head_greedy_accept(x, final_norm, w_lm, draft_tokens, norm_eps=1e-6, n_accepted=None, out_tokens=None, ws=None):
    """x [B,Q,H]; w_lm [V,H] in streaming layout; draft_tokens [B,Q-1] i32 (None when Q == 1).
    Temperature-0 verification without materialising the logits.  Returns (n_accepted, out_tokens)."""
    lib = load()
    _need(x, "x")
    _need(w_lm, "w_lm", x.dtype)
    if draft_tokens is not None:
        _need(draft_tokens, "draft_tokens", torch.int32)
    B, Q, H = x.shape
    V = w_lm.shape[0]
    dev = x.device
    if n_accepted is None:
        n_accepted = torch.empty((B,), dtype=torch.int32, device=dev)
    if out_tokens is None:
        out_tokens = torch.empty((B, Q), dtype=torch.int32, device=dev)
    if ws is None:
        ws = workspace(lib.massv_lm_head_greedy_accept_workspace(B, Q - 1, H, V, dtype_code(x)), dev)
    _check(lib.massv_lm_head_greedy_accept(_ptr(x), _ptr(final_norm), _ptr(w_lm), _ptr(draft_tokens), B, Q - 1, H, V,
                                           float(norm_eps), dtype_code(x), _ptr(n_accepted), _ptr(out_tokens),
                                           _ptr(ws), ws.numel(), _stream()), "massv_lm_head_greedy_accept")
    return n_accepted, out_tokens


def lm_head_accept(x, final_norm, w_lm, draft_logits, draft_tokens, uniforms, temperature, norm_eps=1e-6,
                   logits=None, n_accepted=None, out_tokens=None, ws=None):
    """x [B,Q,H]; w_lm [V,H] in streaming layout; draft_logits [B,Q-1,V] f32, draft_tokens [B,Q-1] i32 (None when
    Q == 1), uniforms [B,Q] f32 (None at T = 0).  Vocabulary projection and accept rule in one call; at T > 0 the
    logits are written to `logits` [B*Q, V].  Returns (n_accepted, out_tokens, logits or None)."""
    lib = load()
    _need(x, "x")
    _need(w_lm, "w_lm", x.dtype)
    B, Q, H = x.shape
    V = w_lm.shape[0]
    dev = x.device
    if n_accepted is None:
        n_accepted = torch.empty((B,), dtype=torch.int32, device=dev)
    if out_tokens is None:
        out_tokens = torch.empty((B, Q), dtype=torch.int32, device=dev)
    if logits is None and temperature > 0:
        logits = torch.empty((B * Q, V), dtype=torch.float32, device=dev)
    if ws is None:
        ws = workspace(lib.massv_lm_head_accept_workspace(B, Q - 1, H, V, dtype_code(x)), dev)
    _check(lib.massv_lm_head_accept(_ptr(x), _ptr(final_norm), _ptr(w_lm), _ptr(draft_logits), _ptr(draft_tokens),
                                    _ptr(uniforms), float(temperature), B, Q - 1, H, V, float(norm_eps), dtype_code(x),
                                    _ptr(logits), _ptr(n_accepted), _ptr(out_tokens), _ptr(ws), ws.numel(), _stream()),
           "massv_lm_head_accept")
    return n_accepted, out_tokens, logits


def spec_tvd(target_logits, draft_logits, temperature, tvd=None, ws=None):
    """target_logits, draft_logits [rows,V] f32 -> tvd [rows] f64."""
    lib = load()
    _need(target_logits, "target_logits", torch.float32)
    _need(draft_logits, "draft_logits", torch.float32)
    if target_logits.dim() != 2 or target_logits.shape != draft_logits.shape:
        raise ValueError("spec_tvd: both logit arrays must be [rows, V]")
    rows, V = target_logits.shape
    dev = target_logits.device
    if tvd is None:
        tvd = torch.empty((rows,), dtype=torch.float64, device=dev)
    else:
        _need(tvd, "tvd", torch.float64)
    if ws is None:
        ws = workspace(lib.massv_spec_tvd_workspace(rows, V), dev)
    _check(lib.massv_spec_tvd(_ptr(target_logits), _ptr(draft_logits), float(temperature), rows, V,
                              _ptr(tvd), _ptr(ws), ws.numel(), _stream()), "massv_spec_tvd")
    return tvd


def linear(x, w_packed, bias=None, act=LIN_NONE, out=None, ws=None, mul=None, add=None):
    """x [M,K] row-major; w_packed [N,K] in streaming layout (weight_pack); bias [N] or None -> y [M,N]
    = act(x w^T + bias) * mul + add, with mul / add [M,N] row-major or None (`add` may be `out`)."""
    lib = load()
    _need(x, "x")
    _need(w_packed, "w", x.dtype)
    M, K = x.shape
    N = w_packed.shape[0]
    for t, n in ((bias, "bias"), (mul, "mul"), (add, "add")):
        if t is not None:
            _need(t, n, x.dtype)
            if n != "bias" and tuple(t.shape) != (M, N):
                raise ValueError(f"{n} must be [M, N]")
    if out is None:
        out = torch.empty((M, N), dtype=x.dtype, device=x.device)
    else:
        _need(out, "out", x.dtype)
    if ws is None:
        ws = workspace(lib.massv_linear_workspace(M, N, K, dtype_code(x)), x.device)
    if mul is None and add is None:
        _check(lib.massv_linear(_ptr(x), _ptr(w_packed), _ptr(bias), _ptr(out), M, N, K, int(act), dtype_code(x),
                                _ptr(ws), ws.numel(), _stream()), "massv_linear")
    else:
        _check(lib.massv_linear_ex(_ptr(x), _ptr(w_packed), _ptr(bias), _ptr(mul), _ptr(add), _ptr(out), M, N, K, int(act),
                                   dtype_code(x), _ptr(ws), ws.numel(), _stream()), "massv_linear_ex")
    return out


def rmsnorm(x, gain, eps=1e-6, out=None):
    """x [M,H] row-major, gain [H] -> y [M,H] = x * gain / sqrt(mean(x^2) + eps), any number of rows."""
    _need(x, "x")
    _need(gain, "gain", x.dtype)
    M, H = x.shape
    if out is None:
        out = torch.empty_like(x)
    else:
        _need(out, "out", x.dtype)
    _check(load().massv_rmsnorm(_ptr(x), _ptr(gain), _ptr(out), M, H, float(eps), dtype_code(x), _stream()), "massv_rmsnorm")
    return out


def commit_tokens(n_accepted, out_tokens, kv_len, last_token=None):
    """kv_len [B] += n_accepted + 1 (in place); returns last_token [B] = out_tokens[b, n_accepted[b]]."""
    for t, n in ((n_accepted, "n_accepted"), (out_tokens, "out_tokens"), (kv_len, "kv_len")):
        _need(t, n, torch.int32)
    B, Q = out_tokens.shape
    if last_token is None:
        last_token = torch.empty((B,), dtype=torch.int32, device=kv_len.device)
    else:
        _need(last_token, "last_token", torch.int32)
    _check(load().massv_commit_tokens(_ptr(n_accepted), _ptr(out_tokens), _ptr(kv_len), _ptr(last_token), B, Q - 1,
                                      _stream()), "massv_commit_tokens")
    return last_token


def embed_tokens(table, tokens, x=None):
    """table [V,H], tokens [M] i32 -> x [M,H] of the table's dtype."""
    lib = load()
    _need(table, "table", table.dtype)
    _need(tokens, "tokens", torch.int32)
    V, H = table.shape
    M = tokens.numel()
    if x is None:
        x = torch.empty((M, H), dtype=table.dtype, device=table.device)
    else:
        _need(x, "x", table.dtype)
    _check(lib.massv_embed_tokens(_ptr(table), _ptr(tokens), _ptr(x), M, H, V, dtype_code(table), _stream()),
           "massv_embed_tokens")
    return x


# ---------------------------------------------------------------------------
# one-shot kernel timing
# ---------------------------------------------------------------------------
def trace_kernel(kernel_id: int, start: "torch.cuda.Event", stop: "torch.cuda.Event"):
    """Ask the library to record `start` / `stop` around the next launch of one
    kernel (K_* ids) made from this thread.  Both events must have been created
    with enable_timing=True and recorded once (torch creates the HIP event on
    first use)."""
    _check(load().massv_trace_kernel(int(kernel_id), C.c_void_p(start.cuda_event), C.c_void_p(stop.cuda_event)),
           "massv_trace_kernel")
