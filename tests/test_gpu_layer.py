"""GPU parity of verify_layer and lm_head_logits against the CPU checker."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2505_10526_amd import synth, binding
from helpers import DEV, to_dev, i32, round_up, pad_rows, assert_close, max_rel_err, v_blocked_to_rows, k_cache_to_rows

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
TOL_F32 = 5e-5      # fp32 path; sums of up to 688 products, fp32 accumulation in a different order


def cfg_of(s):
    return binding.LayerConfig(s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.mlp, s.act, s.qkv_bias,
                               s.norm_eps, s.rope_theta, window=s.window)


def run_layer(s, B, Q, kv_len, n_img, seed, kv_std=1.0, compress=True, w_std=0.02):
    w = synth.layer_weights(s, seed, std=w_std)
    kv = synth.kv_cache(s, B, Q, kv_len, n_img, seed, std=kv_std, hot_keys=1)
    x = synth.hidden_states(s, B, Q, seed)
    pos = synth.positions(kv.kv_len, kv.n_img, Q, compress_image=compress)
    y_ref, k_ref, v_ref = O.verify_layer(s, w, x, pos, kv.k, kv.v, kv.kv_len)
    lm = round_up(kv.l_max, 32)
    kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), s.dtype))
    vd = binding.v_cache_pack(to_dev(pad_rows(kv.v, lm), s.dtype))
    wd = binding.pack_layer_weights({k: (None if v is None else to_dev(v, s.dtype)) for k, v in w.items()})
    xd = to_dev(x, s.dtype)
    binding.verify_layer(cfg_of(s), wd, xd, i32(pos), kd, vd, i32(kv.kv_len))
    torch.cuda.synchronize()
    tol = TOL_BF16 if s.dtype == "bf16" else TOL_F32
    assert_close(xd.float().cpu().numpy(), y_ref, tol, "layer output")
    kg = k_cache_to_rows(kd).float().cpu().numpy()
    vg = v_blocked_to_rows(vd).float().cpu().numpy()
    for b in range(B):
        L = int(kv.kv_len[b])
        assert_close(kg[b, :, L:L + Q], k_ref[b, :, L:L + Q], tol, "appended keys")
        assert_close(vg[b, :, L:L + Q], v_ref[b, :, L:L + Q], tol, "appended values")
        # the cached prefix is untouched
        assert np.array_equal(kg[b, :, :L], kv.k[b, :, :L])
        assert np.array_equal(vg[b, :, :L], kv.v[b, :, :L])
    return xd


def test_tiny_fp32_layer():
    """Config 1: hidden 256, 4/2 heads, d=64, SwiGLU 688, fp32, KV prefix 256 (64 image rows)."""
    run_layer(synth.TINY, 1, 6, [256], [64], seed=0, kv_std=0.02)
    run_layer(synth.TINY, 2, 6, [256, 100], [64, 30], seed=1, kv_std=1.0, w_std=0.05)


def test_tiny_bf16_layer():
    run_layer(synth.TINY_BF16, 1, 6, [256], [64], seed=2, w_std=0.05)
    run_layer(synth.TINY_BF16, 3, 4, [40, 0, 95], [8, 0, 64], seed=3, w_std=0.05)


def test_qwen7b_layer_b1():
    """Config 2: one Qwen2.5-VL-7B-shaped layer, B=1, gamma=5, KV 1024 (700 image rows)."""
    run_layer(synth.QWEN7B, 1, 6, [1024], [700], seed=4)


def test_qwen7b_layer_b8_ragged():
    """Config 3's layer shape: B=8 (M=48), ragged lengths.  Shorter caches than 1024-2048 keep the
    checker's run time in seconds; the full lengths are covered by the attention tests."""
    rng = np.random.default_rng(5)
    run_layer(synth.QWEN7B, 8, 6, rng.integers(100, 400, 8), rng.integers(20, 100, 8), seed=5)


def test_qwen7b_layer_b8_full_lengths():
    """Config 3's layer at its real sizes: B=8, gamma=5, per-sequence lengths U[1024, 2048] with 256-1024
    image rows -- the launch configuration bench.py times (same tile counts, K slabs and attention splits)."""
    rng = np.random.default_rng(0)
    run_layer(synth.QWEN7B, 8, 6, rng.integers(1024, 2049, 8), rng.integers(256, 1025, 8), seed=10)


def test_gemma12b_layer_b4_full_length():
    """Config 4 at its real sizes: B=4, KV length 4096 with 256 leading image rows."""
    run_layer(synth.GEMMA12B, 4, 6, [4096] * 4, [256] * 4, seed=11)


def test_qwen7b_layer_max_rows():
    """The largest row count the bf16 kernels take: B=8, gamma=7 -> M = 64 rows (four 16-row tiles),
    56 stacked query rows per KV head."""
    rng = np.random.default_rng(15)
    run_layer(synth.QWEN7B, 8, 8, rng.integers(40, 300, 8), rng.integers(8, 40, 8), seed=15)


def test_single_row_and_single_sequence():
    """Degenerate sizes: one query position (plain decoding), one sequence."""
    run_layer(synth.TINY_BF16, 1, 1, [33], [5], seed=16, w_std=0.05)
    run_layer(synth.TINY, 1, 1, [0], [0], seed=17, w_std=0.05)
    run_layer(synth.QWEN7B, 1, 1, [70], [20], seed=18)


def test_gemma12b_layer_b4():
    """Config 4's layer: hidden 3840, 16/8 heads, d=256, GeGLU 15360, no bias, B=4 (M=24)."""
    run_layer(synth.GEMMA12B, 4, 6, [300, 256, 50, 411], [256, 200, 10, 256], seed=6)


@pytest.mark.parametrize("shape,M", [(synth.TINY, 6), (synth.TINY_BF16, 6), (synth.TINY_BF16, 48)])
def test_lm_head_small(shape, M):
    lw = synth.lm_head_weights(shape, 7, std=0.05)
    x = synth.normal((M, shape.hidden), 1.0, 7, 60, dtype=shape.dtype)
    ref = O.lm_head_logits(x, lw["final_norm"], lw["w_lm"], shape.norm_eps)
    got = binding.lm_head_logits(to_dev(x, shape.dtype), to_dev(lw["final_norm"], shape.dtype),
                                 binding.weight_pack(to_dev(lw["w_lm"], shape.dtype)), shape.norm_eps)
    assert_close(got.cpu().numpy(), ref, TOL_BF16 if shape.dtype == "bf16" else TOL_F32, "logits")
    ref2 = O.lm_head_logits(x, None, lw["w_lm"], shape.norm_eps)
    got2 = binding.lm_head_logits(to_dev(x, shape.dtype), None, binding.weight_pack(to_dev(lw["w_lm"], shape.dtype)))
    assert_close(got2.cpu().numpy(), ref2, TOL_BF16 if shape.dtype == "bf16" else TOL_F32, "logits no norm")


@pytest.mark.parametrize("shape,M", [(synth.QWEN7B, 6), (synth.QWEN7B, 48), (synth.GEMMA12B, 24)])
def test_lm_head_full_vocab(shape, M):
    """lm_head at the real vocabulary (152064 / 262144 rows)."""
    lw = synth.lm_head_weights(shape, 8)
    x = synth.normal((M, shape.hidden), 1.0, 8, 60, dtype=shape.dtype)
    ref = O.lm_head_logits(x, lw["final_norm"], lw["w_lm"], shape.norm_eps)
    got = binding.lm_head_logits(to_dev(x, shape.dtype), to_dev(lw["final_norm"], shape.dtype),
                                 binding.weight_pack(to_dev(lw["w_lm"], shape.dtype)), shape.norm_eps)
    assert_close(got.cpu().numpy(), ref, TOL_BF16, "logits")


def run_stack(s, n_layers, B, Q, kv_len, n_img, seed, w_std=0.02):
    """n_layers layers through ONE massv_verify_layers call against the checker's layer-by-layer chain."""
    ws_h = [synth.layer_weights(s, seed, layer=l, std=w_std) for l in range(n_layers)]
    kvs = [synth.kv_cache(s, B, Q, kv_len, n_img, seed, layer=l, hot_keys=1) for l in range(n_layers)]
    x = synth.hidden_states(s, B, Q, seed)
    pos = synth.positions(kvs[0].kv_len, kvs[0].n_img, Q, compress_image=True)
    y_ref = x
    k_refs, v_refs = [], []
    for l in range(n_layers):
        y_ref, k_ref, v_ref = O.verify_layer(s, ws_h[l], y_ref, pos, kvs[l].k, kvs[l].v, kvs[l].kv_len)
        k_refs.append(k_ref); v_refs.append(v_ref)
    lm = round_up(kvs[0].l_max, 32)
    kds = [binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), s.dtype)) for kv in kvs]
    vds = [binding.v_cache_pack(to_dev(pad_rows(kv.v, lm), s.dtype)) for kv in kvs]
    wds = [binding.pack_layer_weights({k: (None if v is None else to_dev(v, s.dtype)) for k, v in w.items()}) for w in ws_h]
    stack = binding.LayerStack(wds, kds, vds)
    xd = to_dev(x, s.dtype)
    binding.verify_layers(cfg_of(s), stack, xd, i32(pos), i32(kvs[0].kv_len), lm)
    torch.cuda.synchronize()
    tol = TOL_BF16 if s.dtype == "bf16" else TOL_F32 * n_layers
    assert_close(xd.float().cpu().numpy(), y_ref, tol, "stack output")
    for l in range(n_layers):
        kg = k_cache_to_rows(kds[l]).float().cpu().numpy()
        vg = v_blocked_to_rows(vds[l]).float().cpu().numpy()
        for b in range(B):
            L = int(kvs[l].kv_len[b])
            assert_close(kg[b, :, L:L + Q], k_refs[l][b, :, L:L + Q], tol, f"layer {l} appended keys")
            assert_close(vg[b, :, L:L + Q], v_refs[l][b, :, L:L + Q], tol, f"layer {l} appended values")


def test_layer_stack_tiny():
    run_stack(synth.TINY, 3, 2, 6, [256, 100], [64, 30], seed=12, w_std=0.05)
    run_stack(synth.TINY_BF16, 3, 2, 6, [256, 100], [64, 30], seed=13, w_std=0.05)


def test_layer_stack_qwen7b_two_layers():
    """Two Qwen2.5-VL-7B-shaped layers, B=8 (M=48), in one call: the fused norm between layers."""
    rng = np.random.default_rng(14)
    run_stack(synth.QWEN7B, 2, 8, 6, rng.integers(100, 400, 8), rng.integers(20, 100, 8), seed=14)


CHAIN_LAYERS = 28


@pytest.fixture(scope="module")
def chain(request):
    """The headline workload at its real depth and sizes: 28 Qwen2.5-VL-7B-shaped layers, B=8, gamma=5 (M=48),
    per-sequence lengths U[1024, 2048] with 256-1024 image rows, every layer with its own weights and cache.
    Three runs against the checker's layer-by-layer chain:
      stepwise   layer l alone, fed the checker's output of layer l-1 (identical inputs on both sides);
      sequential the library's own output fed forward, one massv_verify_layer call per layer;
      one_call   the same through ONE massv_verify_layers call over all 28 layers.
    The host holds one layer's weights at a time (the next layer's are drawn while the checker works)."""
    from concurrent.futures import ThreadPoolExecutor
    capman = request.config.pluginmanager.getplugin("capturemanager")

    def say(msg):                                    # progress lines from the work itself: this runs for minutes
        with capman.global_and_fixture_disabled():
            print(msg, flush=True)

    s, N, B, Q, seed = synth.QWEN7B, CHAIN_LAYERS, 8, 6, 50
    rng = np.random.default_rng(0)
    kv_len, n_img = rng.integers(1024, 2049, B), rng.integers(256, 1025, B)
    x = synth.hidden_states(s, B, Q, seed)
    pos = synth.positions(kv_len, n_img, Q)
    lm = round_up(int(kv_len.max()) + Q, 32)
    pool = ThreadPoolExecutor(1)
    draw = lambda l: (synth.layer_weights(s, seed, layer=l, threads=6),
                      synth.kv_cache(s, B, Q, kv_len, n_img, seed, layer=l, hot_keys=1))
    nxt = pool.submit(draw, 0)
    wds, kds, vds = [], [], []
    y_ref, x_seq = x, to_dev(x, s.dtype)
    r = dict(stepwise=[], sequential=[], ref_max=[], layers=N)
    kvl_d, pos_d = i32(kv_len), i32(pos)
    for l in range(N):
        w, kv = nxt.result()
        if l + 1 < N:
            nxt = pool.submit(draw, l + 1)
        kds.append(binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), s.dtype)))
        vds.append(binding.v_cache_pack(to_dev(pad_rows(kv.v, lm), s.dtype)))
        wds.append(binding.pack_layer_weights({k: (None if v is None else to_dev(v, s.dtype)) for k, v in w.items()}))
        x_step = to_dev(y_ref, s.dtype)              # the checker's previous output: on the bf16 grid already
        y_ref, _, _ = O.verify_layer(s, w, y_ref, pos, kv.k, kv.v, kv.kv_len)
        del w, kv
        binding.verify_layer(cfg_of(s), wds[l], x_step, pos_d, kds[l], vds[l], kvl_d)
        binding.verify_layer(cfg_of(s), wds[l], x_seq, pos_d, kds[l], vds[l], kvl_d)     # rewrites the same cache rows
        torch.cuda.synchronize()
        for name, t in (("stepwise", x_step), ("sequential", x_seq)):
            got = t.float().cpu().numpy()
            assert np.all(np.isfinite(got)), f"layer {l} ({name}): non-finite output"
            r[name].append(max_rel_err(got, y_ref))
        r["ref_max"].append(float(np.max(np.abs(y_ref))))
        if l % 4 == 3:
            say(f"[chain] layer {l + 1}/{N}: stepwise {r['stepwise'][-1]:.2e}, sequential {r['sequential'][-1]:.2e}, "
                f"max |ref| {r['ref_max'][-1]:.1f}")
    pool.shutdown()
    stack = binding.LayerStack(wds, kds, vds)
    xd = to_dev(x, s.dtype)
    binding.verify_layers(cfg_of(s), stack, xd, pos_d, kvl_d, lm)      # rows kv_len .. kv_len+Q-1 are rewritten first
    torch.cuda.synchronize()
    r["one_call"] = max_rel_err(xd.float().cpu().numpy(), y_ref)
    say("[chain] stepwise error of each layer (max |err| / max |ref|): " + " ".join(f"{e:.2e}" for e in r["stepwise"]))
    say("[chain] sequential error after each layer: " + " ".join(f"{e:.2e}" for e in r["sequential"]))
    say("[chain] max |ref| after each layer: " + " ".join(f"{m:.1f}" for m in r["ref_max"]))
    say(f"[chain] one call over {N} layers: {r['one_call']:.3e}")
    return r


def test_every_layer_of_the_full_depth_stack_meets_the_bound(chain):
    """Each of the 28 layers, at the activation statistics of its own depth and with identical inputs on both
    sides, is within the bf16 bound."""
    assert max(chain["stepwise"]) <= TOL_BF16, chain["stepwise"]


def test_full_depth_chain_stays_consistent(chain):
    """Both sides feeding their own output forward: the library rounds the operands of every projection to bf16,
    the checker rounds only what the step stores, so the two drift apart with depth.  This is a guard against a
    defect that compounds (a wrong residual path, a stale workspace between layers), not the parity bound: the
    one call over all layers must agree with the layer-at-a-time run (same arithmetic, same inputs up to the fused
    norm between layers) and the drift must stay of the size that per-layer errors adding up explain."""
    seq, one = chain["sequential"][-1], chain["one_call"]
    assert abs(one - seq) <= 1e-2, (one, seq)
    budget = float(np.sum(np.array(chain["stepwise"]) * np.array(chain["ref_max"])) / chain["ref_max"][-1])
    assert one <= budget, (one, budget)


@pytest.mark.xfail(strict=False, reason="free-running 28-layer chain: bf16 operand rounding compounds with depth; "
                                        "the measured curve is reported, the bound is not raised")
def test_full_depth_chain_meets_the_single_layer_bound(chain):
    assert chain["one_call"] <= TOL_BF16, chain["one_call"]


def test_layer_repeatable_bits():
    s = synth.QWEN7B
    w = binding.pack_layer_weights({k: (None if v is None else to_dev(v, s.dtype)) for k, v in synth.layer_weights(s, 9).items()})
    kv = synth.kv_cache(s, 2, 6, [64, 200], [10, 50], 9, junk_tail=False)
    pos = i32(synth.positions(kv.kv_len, kv.n_img, 6))
    outs = []
    for _ in range(2):
        lm = round_up(kv.l_max, 32)
        kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), s.dtype))
        vd = binding.v_cache_pack(to_dev(np.nan_to_num(pad_rows(kv.v, lm)), s.dtype))
        x = to_dev(synth.hidden_states(s, 2, 6, 9), s.dtype)
        binding.verify_layer(cfg_of(s), w, x, pos, kd, vd, i32(kv.kv_len))
        outs.append((x.clone(), kd.clone(), vd.clone()))
    for a, b in zip(*outs):
        assert torch.equal(torch.nan_to_num(a.float()), torch.nan_to_num(b.float()))


@pytest.mark.parametrize("s", [synth.TINY, synth.TINY_BF16], ids=["f32", "bf16"])
def test_embed_tokens_gathers_rows(s):
    table = synth.embedding_table(s, 5)
    tokens = np.array([0, s.vocab - 1, 17, 17, -3, s.vocab, 1234], dtype=np.int32)
    ref = O.embed_tokens(table, tokens)
    got = binding.embed_tokens(to_dev(table, s.dtype), i32(tokens))
    assert np.array_equal(got.float().cpu().numpy(), ref)


# ---------------------------------------------------------------------------
# layer variants of the Gemma 3 targets: sliding window, query/key head norms, block-output norms
# ---------------------------------------------------------------------------
def test_gemma_style_tiny_layers():
    run_layer(synth.TINY_GEMMA, 2, 6, [256, 100], [64, 30], seed=31, w_std=0.05)
    run_layer(synth.TINY_GEMMA_BF16, 3, 4, [140, 0, 95], [8, 0, 64], seed=32, w_std=0.05)


def test_gemma12b_local_layer():
    """One Gemma3-12B-shaped sliding-window layer: d=256 heads with query/key norms, window 1024 over KV 4096,
    block-output norms, tanh-GELU MLP."""
    run_layer(synth.GEMMA12B_LOCAL, 4, 6, [4096, 3000, 1024, 500], [256, 256, 256, 100], seed=33)


def test_each_gemma_variant_alone():
    """Each optional step switched on by itself (a step wired to the wrong switch fails here)."""
    import dataclasses
    base = synth.TINY_BF16
    for kw in (dict(window=20), dict(qk_norm=True), dict(post_norms=True)):
        run_layer(dataclasses.replace(base, **kw), 2, 6, [100, 37], [30, 5], seed=34, w_std=0.05)


def test_layer_stack_interleaves_local_and_global_layers():
    """Four layers in one call, windows (24, 24, 0, 24) and rotary bases (1e4, 1e4, 1e6, 1e4) given per layer."""
    import dataclasses
    for base in (synth.TINY_GEMMA, synth.TINY_GEMMA_BF16):
        windows, thetas = [24, 24, 0, 24], [1e4, 1e4, 1e6, 1e4]
        shapes = [dataclasses.replace(base, window=w, rope_theta=t) for w, t in zip(windows, thetas)]
        B, Q, seed = 2, 6, 35
        ws_h = [synth.layer_weights(s, seed, layer=l, std=0.05) for l, s in enumerate(shapes)]
        kvs = [synth.kv_cache(base, B, Q, [200, 61], [64, 30], seed, layer=l, hot_keys=1) for l in range(4)]
        x = synth.hidden_states(base, B, Q, seed)
        pos = synth.positions(kvs[0].kv_len, kvs[0].n_img, Q, compress_image=True)
        y_ref = x
        for l in range(4):
            y_ref, _, _ = O.verify_layer(shapes[l], ws_h[l], y_ref, pos, kvs[l].k, kvs[l].v, kvs[l].kv_len)
        lm = round_up(kvs[0].l_max, 32)
        kds = [binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), base.dtype)) for kv in kvs]
        vds = [binding.v_cache_pack(to_dev(pad_rows(kv.v, lm), base.dtype)) for kv in kvs]
        wds = [binding.pack_layer_weights({k: (None if v is None else to_dev(v, base.dtype)) for k, v in w.items()}) for w in ws_h]
        stack = binding.LayerStack(wds, kds, vds, windows=windows, rope_thetas=thetas)
        xd = to_dev(x, base.dtype)
        binding.verify_layers(cfg_of(base), stack, xd, i32(pos), i32(kvs[0].kv_len), lm)
        torch.cuda.synchronize()
        tol = TOL_BF16 if base.dtype == "bf16" else TOL_F32 * 4
        assert_close(xd.float().cpu().numpy(), y_ref, tol, "interleaved stack output")


# ---------------------------------------------------------------------------
# vocabulary projection fused with the temperature-0 accept rule (no logits written)
# ---------------------------------------------------------------------------
def greedy_case(s, B, gamma, seed, head_std=0.05, duplicate_rows=False):
    Q = gamma + 1
    head = synth.lm_head_weights(s, seed, std=head_std)
    if duplicate_rows:                                   # every logit appears twice: ties must go to the lower token id
        head["w_lm"][s.vocab // 2:] = head["w_lm"][: s.vocab // 2]
    x = synth.hidden_states(s, B, Q, seed)
    logits = O.lm_head_logits(x.reshape(B * Q, -1), head["final_norm"], head["w_lm"], s.norm_eps).reshape(B, Q, -1)
    # drafts: the checker's arg-max for a random-length prefix of every sequence, something else after it
    rng = np.random.default_rng(seed)
    drafts = np.argmax(logits[:, :gamma], axis=-1).astype(np.int32)
    for b in range(B):
        keep = int(rng.integers(0, gamma + 1))
        if keep < gamma:
            drafts[b, keep] = (drafts[b, keep] + 1 + int(rng.integers(0, s.vocab - 1))) % s.vocab
    xd = to_dev(x, s.dtype)
    norm, w = to_dev(head["final_norm"], s.dtype), binding.weight_pack(to_dev(head["w_lm"], s.dtype))
    return xd, norm, w, i32(drafts), logits, drafts


@pytest.mark.parametrize("s,B,gamma,dup", [(synth.TINY_BF16, 3, 5, False), (synth.TINY_BF16, 8, 5, True), (synth.TINY_BF16, 1, 0, False),
                                           (synth.TINY_BF16, 4, 15, False), (synth.QWEN7B, 8, 5, False), (synth.QWEN7B, 2, 3, True)],
                         ids=["tiny", "tiny-ties", "tiny-gamma0", "tiny-gamma15", "qwen7b", "qwen7b-ties"])
def test_lm_head_greedy_accept(s, B, gamma, dup):
    xd, norm, w, dtok, logits_ref, drafts = greedy_case(s, B, gamma, seed=41 + B + gamma, duplicate_rows=dup)
    n_f, out_f = binding.lm_head_greedy_accept(xd, norm, w, dtok if gamma else None, s.norm_eps)
    # the two separate calls on the same inputs: identical integers, ties included
    lg = binding.lm_head_logits(xd, norm, w, s.norm_eps).reshape(B, gamma + 1, -1)
    n_2, out_2 = binding.spec_accept(lg, None, dtok if gamma else None, None, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(n_f, n_2) and torch.equal(out_f, out_2)
    if dup:
        assert int(out_f.max()) < s.vocab // 2
        return
    # the checker, wherever its arg-max is clear of the bf16 path's error
    top = np.sort(logits_ref, axis=-1)[..., -2:]
    clear = (top[..., 1] - top[..., 0]) > 5e-3 * np.max(np.abs(logits_ref))
    n_o, out_o, _ = O.spec_accept(logits_ref, None, drafts, None, 0.0)
    for b in range(B):
        if clear[b].all():
            assert int(n_f[b]) == n_o[b] and np.array_equal(out_f[b].cpu().numpy(), out_o[b])
    if gamma <= 5:
        assert clear.all(axis=1).sum() >= 1                 # the comparison with the checker is not vacuous
    if gamma >= 5 and B >= 3:
        assert len(set(n_o.tolist())) > 1


# ---------------------------------------------------------------------------
# vocabulary projection + accept rule in one call at T > 0 (row statistics formed in the projection's epilogue)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("s,B,gamma,T,noise", [(synth.TINY_BF16, 3, 5, 1.0, 0.3), (synth.TINY_BF16, 1, 0, 0.7, 0.3),
                                               (synth.TINY_BF16, 4, 15, 1.0, 0.1), (synth.QWEN7B, 8, 5, 1.0, 0.5),
                                               (synth.QWEN7B, 8, 5, 0.7, 1.5), (synth.QWEN7B, 2, 3, 0.0, 1.0)],
                         ids=["tiny", "tiny-gamma0", "tiny-gamma15", "qwen7b", "qwen7b-T0.7", "qwen7b-T0"])
def test_lm_head_accept_one_call(s, B, gamma, T, noise):
    Q, seed = gamma + 1, 70 + B + gamma
    T = float(np.float32(T))
    head = synth.lm_head_weights(s, seed, std=0.05)
    xd = to_dev(synth.hidden_states(s, B, Q, seed), s.dtype)
    norm, w = to_dev(head["final_norm"], s.dtype), binding.weight_pack(to_dev(head["w_lm"], s.dtype))
    lg = binding.lm_head_logits(xd, norm, w, s.norm_eps)                   # the separate calls: logits first
    tl = lg.cpu().numpy().reshape(B, Q, -1)
    a = synth.accept_inputs(B, gamma, s.vocab, T, seed, noise_std=noise, target_logits=tl)   # drafts from the GPU's own logits
    dl = torch.from_numpy(a.draft_logits).cuda() if gamma else None
    dt = torch.from_numpy(a.draft_tokens).cuda() if gamma else None
    u = torch.from_numpy(a.uniforms).cuda()
    n_2, out_2 = binding.spec_accept(lg.view(B, Q, -1), dl if T > 0 else None, dt, u if T > 0 else None, T)
    n_f, out_f, lg_f = binding.lm_head_accept(xd, norm, w, dl, dt, u if T > 0 else None, T, s.norm_eps)
    torch.cuda.synchronize()
    if T > 0:
        assert torch.equal(lg_f, lg)                                        # the same projection arithmetic
    # the checker on the same fp32 logits
    n_o, out_o, margin = O.spec_accept(tl, a.draft_logits, a.draft_tokens, a.uniforms, T)
    clear = np.all(margin > 1e-5, axis=1)
    assert clear.sum() >= 0.5 * B, "pick another seed: too few decisions clear of rounding"
    for b in range(B):
        if clear[b]:
            for n_g, out_g in ((n_2, out_2), (n_f, out_f)):
                assert int(n_g[b]) == n_o[b] and np.array_equal(out_g[b].cpu().numpy(), out_o[b]), (b, out_g[b], out_o[b])
    if gamma >= 5 and T > 0:
        assert n_o.max() > 0                                                # drafts do get accepted in this case
