"""The C ABI without a GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2505_10526_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "massv_verify.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        build.build(verbose=False)
    return binding.load()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(massv_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    assert binding.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert binding.status_string(code)
    assert lib.massv_abi_version() >= 1


def test_struct_sizes_match_header():
    assert C.sizeof(binding.AttnDesc) == 36
    assert C.sizeof(binding.LayerDesc) == 36 + 24
    assert C.sizeof(binding.LayerWeights) == 16 * C.sizeof(C.c_void_p)


FAKE = C.c_void_p(0x1000)      # never dereferenced: every call below must fail validation first


def test_spec_accept_argument_checks(lib):
    f = lib.massv_spec_accept
    ws = lib.massv_spec_accept_workspace(2, 5, 1000)
    assert ws > 0
    assert lib.massv_spec_accept_workspace(0, 5, 1000) == 0
    ok_args = lambda **kw: [kw.get("t", FAKE), kw.get("d", FAKE), kw.get("x", FAKE), kw.get("u", FAKE),
                            kw.get("T", 1.0), kw.get("B", 2), kw.get("g", 5), kw.get("V", 1000),
                            kw.get("n", FAKE), kw.get("o", FAKE), kw.get("ws", FAKE), kw.get("wsb", ws), None]
    assert f(*ok_args(t=None)) == binding.EINVAL
    assert f(*ok_args(d=None)) == binding.EINVAL            # T > 0 needs draft logits
    assert f(*ok_args(u=None)) == binding.EINVAL
    assert f(*ok_args(T=-0.5)) == binding.EINVAL
    assert f(*ok_args(T=float("nan"))) == binding.EINVAL
    assert f(*ok_args(B=0)) == binding.EINVAL
    assert f(*ok_args(g=-1)) == binding.EINVAL
    assert f(*ok_args(x=None)) == binding.EINVAL            # gamma > 0 needs draft tokens
    assert f(*ok_args(g=0, d=None, x=None, u=None)) == binding.EINVAL     # sampling at T > 0 needs a uniform
    assert lib.massv_spec_accept_workspace(2, 0, 1000) > 0
    assert f(*ok_args(g=99)) == binding.EUNSUPPORTED
    assert f(*ok_args(wsb=ws - 1)) == binding.EWORKSPACE
    assert f(*ok_args(ws=None)) == binding.EWORKSPACE


def test_spec_tvd_and_embed_argument_checks(lib):
    f = lib.massv_spec_tvd
    ws = lib.massv_spec_tvd_workspace(6, 1000)
    assert ws > 0 and lib.massv_spec_tvd_workspace(0, 1000) == 0
    assert f(None, FAKE, 1.0, 6, 1000, FAKE, FAKE, ws, None) == binding.EINVAL
    assert f(FAKE, None, 1.0, 6, 1000, FAKE, FAKE, ws, None) == binding.EINVAL
    assert f(FAKE, FAKE, 1.0, 6, 1000, None, FAKE, ws, None) == binding.EINVAL
    assert f(FAKE, FAKE, 0.0, 6, 1000, FAKE, FAKE, ws, None) == binding.EINVAL      # undefined at T = 0
    assert f(FAKE, FAKE, float("inf"), 6, 1000, FAKE, FAKE, ws, None) == binding.EINVAL
    assert f(FAKE, FAKE, 1.0, 0, 1000, FAKE, FAKE, ws, None) == binding.EINVAL
    assert f(FAKE, FAKE, 1.0, 40000, 1000, FAKE, FAKE, 1 << 40, None) == binding.EUNSUPPORTED
    assert f(FAKE, FAKE, 1.0, 6, 1000, FAKE, FAKE, ws - 1, None) == binding.EWORKSPACE
    g = lib.massv_embed_tokens
    assert g(None, FAKE, FAKE, 4, 64, 100, binding.BF16, None) == binding.EINVAL
    assert g(FAKE, None, FAKE, 4, 64, 100, binding.BF16, None) == binding.EINVAL
    assert g(FAKE, FAKE, None, 4, 64, 100, binding.BF16, None) == binding.EINVAL
    assert g(FAKE, FAKE, FAKE, 0, 64, 100, binding.BF16, None) == binding.EINVAL
    assert g(FAKE, FAKE, FAKE, 4, 64, 100, 7, None) == binding.EINVAL
    assert g(FAKE, FAKE, FAKE, 4, 63, 100, binding.BF16, None) == binding.EUNSUPPORTED


def test_attention_argument_checks(lib):
    f = lib.massv_verify_attention
    good = binding.attn_desc(2, 6, 28, 4, 128, 2080, binding.BF16)
    need = lib.massv_verify_attention_workspace(C.byref(good))
    assert need > 0
    call = lambda d, q=FAKE, wsb=need: f(C.byref(d), q, FAKE, FAKE, FAKE, FAKE, FAKE, wsb, None)
    assert call(good, q=None) == binding.EINVAL
    assert call(good, wsb=need - 1) == binding.EWORKSPACE
    bad = binding.attn_desc(2, 6, 28, 5, 128, 2080, binding.BF16)        # 28 % 5 != 0
    assert call(bad) == binding.EINVAL and lib.massv_verify_attention_workspace(C.byref(bad)) == 0
    assert call(binding.attn_desc(2, 6, 28, 4, 128, 2070, binding.BF16)) == binding.EINVAL     # l_max % 32
    assert call(binding.attn_desc(2, 6, 28, 4, 96, 2080, binding.BF16)) == binding.EUNSUPPORTED
    assert call(binding.attn_desc(2, 12, 28, 4, 128, 2080, binding.BF16)) == binding.EUNSUPPORTED  # 84 stacked rows
    assert call(binding.attn_desc(2, 6, 28, 4, 128, 2080, 7)) == binding.EINVAL
    assert call(binding.attn_desc(2, 6, 28, 4, 128, 2080, binding.BF16, scale=-1.0)) == binding.EINVAL


def test_cache_pack_argument_checks(lib):
    for f in (lib.massv_k_cache_pack, lib.massv_v_cache_pack):
        assert f(None, FAKE, 2, 4, 64, 128, binding.BF16, None) == binding.EINVAL
        assert f(FAKE, None, 2, 4, 64, 128, binding.BF16, None) == binding.EINVAL
        assert f(FAKE, FAKE, 0, 4, 64, 128, binding.BF16, None) == binding.EINVAL
        assert f(FAKE, FAKE, 2, 4, 64, 128, 7, None) == binding.EINVAL
        assert f(FAKE, FAKE, 2, 4, 70, 128, binding.BF16, None) == binding.EINVAL        # rows in blocks of 32
    assert lib.massv_k_cache_pack(FAKE, FAKE, 2, 4, 64, 124, binding.BF16, None) == binding.EINVAL   # 8-feature chunks


def test_key_cache_layout_formula():
    """The element offset stated in the header for bf16 keys, written out here, against the un-blocking that the
    GPU tests use to read a cache back (tests/helpers.py): both must describe the same permutation."""
    import torch
    from helpers import k_cache_to_rows
    B, n_kv, L, d = 2, 3, 96, 64
    rows = torch.arange(B * n_kv * L * d, dtype=torch.float32).reshape(B, n_kv, L, d)
    packed = torch.empty(B * n_kv * L * d, dtype=torch.float32)
    b, g, j, c = torch.meshgrid(torch.arange(B), torch.arange(n_kv), torch.arange(L), torch.arange(d), indexing="ij")
    off = ((b * n_kv + g) * L + 32 * (j // 32)) * d + (((j // 4) % 2 * (d // 8) + c // 8) * 16 + 4 * ((j % 32) // 8) + j % 4) * 8 + c % 8
    assert torch.equal(torch.sort(off.reshape(-1)).values, torch.arange(B * n_kv * L * d))      # a permutation
    packed[off.reshape(-1)] = rows.reshape(-1)
    assert torch.equal(k_cache_to_rows(packed.reshape(B, n_kv, L, d), blocked=True), rows)


def test_negative_window_is_rejected(lib):
    d = binding.attn_desc(2, 6, 28, 4, 128, 2080, binding.BF16, window=-1)
    assert lib.massv_verify_attention_workspace(C.byref(d)) == 0
    assert lib.massv_verify_attention(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == binding.EINVAL


def test_layer_and_lm_head_argument_checks(lib):
    cfg = binding.LayerConfig(3584, 28, 4, 128, 18944)
    d = binding.layer_desc(cfg, 8, 6, 2080, binding.BF16)
    need = lib.massv_verify_layer_workspace(C.byref(d))
    assert need > 0
    w = binding.LayerWeights(*([0x1000] * 12))
    f = lib.massv_verify_layer
    assert f(C.byref(d), C.byref(w), None, FAKE, FAKE, FAKE, FAKE, FAKE, need, None) == binding.EINVAL
    assert f(C.byref(d), C.byref(w), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, need - 1, None) == binding.EWORKSPACE
    w2 = binding.LayerWeights(*([0x1000] * 12)); w2.bq = None
    assert f(C.byref(d), C.byref(w2), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, need, None) == binding.EINVAL
    big = binding.layer_desc(cfg, 16, 6, 2080, binding.BF16)             # M = 96 rows
    assert f(C.byref(big), C.byref(w), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == binding.EUNSUPPORTED
    odd = binding.layer_desc(binding.LayerConfig(3584, 28, 4, 128, 18950), 1, 6, 2080, binding.BF16)
    assert f(C.byref(odd), C.byref(w), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == binding.EUNSUPPORTED

    g = lib.massv_lm_head_logits
    need = lib.massv_lm_head_logits_workspace(48, 3584, 152064, binding.BF16)
    assert need >= 48 * 3584 * 2
    assert g(None, FAKE, FAKE, FAKE, 48, 3584, 152064, 1e-6, binding.BF16, FAKE, need, None) == binding.EINVAL
    assert g(FAKE, FAKE, FAKE, FAKE, 48, 3584, 152064, 1e-6, binding.BF16, FAKE, need - 1, None) == binding.EWORKSPACE
    assert g(FAKE, FAKE, FAKE, FAKE, 65, 3584, 152064, 1e-6, binding.BF16, FAKE, 1 << 30, None) == binding.EUNSUPPORTED
    assert g(FAKE, FAKE, FAKE, FAKE, 48, 3584, 152065, 1e-6, binding.BF16, FAKE, 1 << 30, None) == binding.EUNSUPPORTED
    assert g(FAKE, FAKE, FAKE, FAKE, 0, 3584, 152064, 1e-6, binding.BF16, FAKE, need, None) == binding.EINVAL


def test_linear_argument_checks(lib):
    f = lib.massv_linear
    ws = lib.massv_linear_workspace(300, 272, 128, binding.BF16)
    assert ws >= 304 * 128 * 2
    assert lib.massv_linear_workspace(300, 272, 100, binding.BF16) == 0
    ok = lambda **kw: [kw.get("x", FAKE), kw.get("w", FAKE), kw.get("b", None), kw.get("y", FAKE), kw.get("M", 300),
                       kw.get("N", 272), kw.get("K", 128), kw.get("act", 0), kw.get("dt", binding.BF16), kw.get("ws", FAKE),
                       kw.get("wsb", ws), None]
    assert f(*ok(x=None)) == binding.EINVAL
    assert f(*ok(w=None)) == binding.EINVAL
    assert f(*ok(y=None)) == binding.EINVAL
    assert f(*ok(M=0)) == binding.EINVAL
    assert f(*ok(act=9)) == binding.EINVAL
    assert f(*ok(K=96)) == binding.EUNSUPPORTED          # k-steps of 64
    assert f(*ok(N=270)) == binding.EUNSUPPORTED
    assert f(*ok(dt=binding.F32)) == binding.EUNSUPPORTED
    assert f(*ok(wsb=ws - 1)) == binding.EWORKSPACE
    assert f(*ok(ws=None)) == binding.EWORKSPACE


def test_linear_ex_and_rmsnorm_argument_checks(lib):
    f = lib.massv_linear_ex
    ws = lib.massv_linear_workspace(300, 272, 128, binding.BF16)
    ok = lambda **kw: [kw.get("x", FAKE), kw.get("w", FAKE), None, kw.get("mul", FAKE), kw.get("add", None), kw.get("y", FAKE),
                       kw.get("M", 300), kw.get("N", 272), kw.get("K", 128), kw.get("act", 1), binding.BF16, kw.get("ws", FAKE),
                       kw.get("wsb", ws), None]
    assert f(*ok(x=None)) == binding.EINVAL
    assert f(*ok(y=None)) == binding.EINVAL
    assert f(*ok(act=-1)) == binding.EINVAL
    assert f(*ok(K=96)) == binding.EUNSUPPORTED
    assert f(*ok(wsb=ws - 1)) == binding.EWORKSPACE
    g = lib.massv_rmsnorm
    okn = lambda **kw: [kw.get("x", FAKE), kw.get("g", FAKE), kw.get("y", FAKE), kw.get("M", 4), kw.get("H", 256),
                        kw.get("eps", 1e-6), kw.get("dt", binding.BF16), None]
    for name in ("x", "g", "y"):
        assert g(*okn(**{name: None})) == binding.EINVAL
    assert g(*okn(M=0)) == binding.EINVAL
    assert g(*okn(H=0)) == binding.EINVAL
    assert g(*okn(eps=-1.0)) == binding.EINVAL
    assert g(*okn(dt=7)) == binding.EINVAL


def test_lm_head_greedy_accept_argument_checks(lib):
    f = lib.massv_lm_head_greedy_accept
    ws = lib.massv_lm_head_greedy_accept_workspace(8, 5, 3584, 152064, binding.BF16)
    assert ws > 0
    assert lib.massv_lm_head_greedy_accept_workspace(8, 5, 3584, 152064, binding.F32) == 0
    ok = lambda **kw: [kw.get("x", FAKE), FAKE, kw.get("w", FAKE), kw.get("d", FAKE), kw.get("B", 8), kw.get("g", 5), kw.get("H", 3584),
                       kw.get("V", 152064), 1e-6, kw.get("dt", binding.BF16), kw.get("n", FAKE), kw.get("o", FAKE), kw.get("ws", FAKE),
                       kw.get("wsb", ws), None]
    assert f(*ok(x=None)) == binding.EINVAL
    assert f(*ok(w=None)) == binding.EINVAL
    assert f(*ok(d=None)) == binding.EINVAL
    assert f(*ok(n=None)) == binding.EINVAL
    assert f(*ok(B=0)) == binding.EINVAL
    assert f(*ok(dt=binding.F32)) == binding.EUNSUPPORTED
    assert f(*ok(B=11)) == binding.EUNSUPPORTED            # 66 rows
    assert f(*ok(g=16, B=1)) == binding.EUNSUPPORTED
    assert f(*ok(V=152065)) == binding.EUNSUPPORTED
    assert f(*ok(wsb=ws - 1)) == binding.EWORKSPACE


def test_lm_head_accept_argument_checks(lib):
    f = lib.massv_lm_head_accept
    ws = lib.massv_lm_head_accept_workspace(8, 5, 3584, 152064, binding.BF16)
    assert ws >= lib.massv_lm_head_greedy_accept_workspace(8, 5, 3584, 152064, binding.BF16)
    assert lib.massv_lm_head_accept_workspace(8, 5, 3584, 152064, binding.F32) == 0
    ok = lambda **kw: [kw.get("x", FAKE), FAKE, kw.get("w", FAKE), kw.get("dl", FAKE), kw.get("d", FAKE), kw.get("u", FAKE),
                       kw.get("T", 0.7), kw.get("B", 8), kw.get("g", 5), kw.get("H", 3584), kw.get("V", 152064), kw.get("eps", 1e-6),
                       kw.get("dt", binding.BF16), kw.get("lg", FAKE), kw.get("n", FAKE), kw.get("o", FAKE), kw.get("ws", FAKE),
                       kw.get("wsb", ws), None]
    assert f(*ok(x=None)) == binding.EINVAL
    assert f(*ok(w=None)) == binding.EINVAL
    assert f(*ok(lg=None)) == binding.EINVAL               # T > 0: the residual draw reads the logits
    assert f(*ok(u=None)) == binding.EINVAL
    assert f(*ok(dl=None)) == binding.EINVAL
    assert f(*ok(d=None)) == binding.EINVAL
    assert f(*ok(n=None)) == binding.EINVAL
    assert f(*ok(o=None)) == binding.EINVAL
    assert f(*ok(T=-1.0)) == binding.EINVAL
    assert f(*ok(T=float("nan"))) == binding.EINVAL
    assert f(*ok(T=float("inf"))) == binding.EINVAL
    assert f(*ok(eps=-1.0)) == binding.EINVAL
    assert f(*ok(B=0)) == binding.EINVAL
    assert f(*ok(T=0.0, x=None)) == binding.EINVAL         # T = 0 goes through the greedy call's checks
    assert f(*ok(dt=binding.F32)) == binding.EUNSUPPORTED
    assert f(*ok(B=11)) == binding.EUNSUPPORTED            # 66 rows
    assert f(*ok(V=152065)) == binding.EUNSUPPORTED
    assert f(*ok(wsb=ws - 1)) == binding.EWORKSPACE
    assert f(*ok(ws=None)) == binding.EWORKSPACE


def test_spec_accept_static_argument_checks(lib):
    f = lib.massv_spec_accept_static
    limit = lib.massv_spec_accept_static_limit()
    assert limit == 4 << 20
    ok = lambda **kw: [kw.get("t", FAKE), kw.get("d", FAKE), kw.get("x", FAKE), kw.get("u", FAKE), kw.get("T", 1.0),
                       kw.get("B", 2), kw.get("g", 5), kw.get("V", 1000), kw.get("n", FAKE), kw.get("o", FAKE), None]
    assert f(*ok(t=None)) == binding.EINVAL
    assert f(*ok(d=None)) == binding.EINVAL
    assert f(*ok(u=None)) == binding.EINVAL
    assert f(*ok(n=None)) == binding.EINVAL
    assert f(*ok(T=-0.5)) == binding.EINVAL
    assert f(*ok(B=0)) == binding.EINVAL
    assert f(*ok(g=99)) == binding.EUNSUPPORTED
    # a call whose partial results do not fit the fixed array is refused before anything is looked up or launched
    assert lib.massv_spec_accept_workspace(256, 7, 262144) > limit
    assert f(*ok(B=256, g=7, V=262144)) == binding.EUNSUPPORTED


def test_prefill_attention_argument_checks(lib):
    f = lib.massv_prefill_attention
    def desc(**kw):
        return binding.AttnDesc(kw.get("B", 2), kw.get("Q", 64), kw.get("nq", 28), kw.get("nkv", 4), kw.get("d", 128),
                                kw.get("lmax", 256), 0.0, kw.get("dt", binding.BF16), kw.get("window", 0))
    args = lambda d, **kw: [C.byref(d) if d is not None else None, kw.get("q", FAKE), kw.get("k", FAKE), kw.get("v", FAKE),
                            kw.get("kv", FAKE), kw.get("nn", FAKE), None, kw.get("o", FAKE), None]
    assert f(*args(None)) == binding.EINVAL
    for name in ("q", "k", "v", "kv", "nn", "o"):
        assert f(*args(desc(), **{name: None})) == binding.EINVAL
    assert f(*args(desc(Q=0))) == binding.EINVAL
    assert f(*args(desc(Q=257))) == binding.EINVAL          # more new positions than the cache has rows
    assert f(*args(desc(nq=28, nkv=3))) == binding.EINVAL   # query heads must divide over the KV heads
    assert f(*args(desc(window=-1))) == binding.EINVAL
    assert f(*args(desc(d=96))) in (binding.EINVAL, binding.EUNSUPPORTED)


def test_rope_append_argument_checks(lib):
    f = lib.massv_rope_append
    def desc(**kw):
        return binding.AttnDesc(kw.get("B", 2), kw.get("Q", 64), 28, 4, kw.get("d", 128), kw.get("lmax", 256), 0.0,
                                kw.get("dt", binding.BF16), 0)
    sec = lambda *v: (C.c_int32 * 3)(*v)
    args = lambda d, **kw: [C.byref(d) if d is not None else None, kw.get("qkv", FAKE), kw.get("pos", FAKE), kw.get("n_pos", 1),
                            kw.get("sec", None), kw.get("theta", 1e6), None, None, 1e-6, kw.get("kv", FAKE), kw.get("nn", FAKE),
                            kw.get("q", FAKE), kw.get("k", FAKE), kw.get("v", FAKE), None]
    assert f(*args(None)) == binding.EINVAL
    for name in ("qkv", "pos", "kv", "nn", "q", "k", "v"):
        assert f(*args(desc(), **{name: None})) == binding.EINVAL
    assert f(*args(desc(Q=0))) == binding.EINVAL
    assert f(*args(desc(Q=257))) == binding.EINVAL
    assert f(*args(desc(), theta=0.0)) == binding.EINVAL
    assert f(*args(desc(), n_pos=2)) == binding.EINVAL
    assert f(*args(desc(), n_pos=3)) == binding.EINVAL                       # three ids need the sections
    assert f(*args(desc(), n_pos=3, sec=sec(16, 24, 23))) == binding.EINVAL   # must sum to d/2
    assert f(*args(desc(), n_pos=3, sec=sec(70, -6, 0))) == binding.EINVAL
    assert f(*args(desc(d=96))) == binding.EUNSUPPORTED


def test_binding_refuses_to_run_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="missing"):
        binding.load()
