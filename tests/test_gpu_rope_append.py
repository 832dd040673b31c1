"""GPU parity of massv_rope_append (the prompt-pass step between the q/k/v projection and prefill_attention, paper
Section 2.2) against the CPU checker: head split, optional head norms, rotation by one or by three position ids
per row (sectioned pairs, the numbering the Qwen2.5-VL targets of Section 5 use for image positions), append of
the first n_new rows to the caches."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2505_10526_amd import binding, synth
from helpers import to_dev, i32, round_up, pad_rows, v_blocked_to_rows, k_cache_to_rows, assert_close

pytestmark = pytest.mark.gpu

# the rotation is formed in double on both sides; what differs is one storage rounding
TOL = {"bf16": 8e-3, "f32": 2e-6}


def run_case(s, kv_len, n_new, Lq, seed, sections=None, norms=False, theta=None):
    rng = np.random.default_rng(seed)
    B = len(kv_len)
    nq, nkv, d = s.n_q_heads, s.n_kv_heads, s.head_dim
    theta = theta or s.rope_theta
    l_max = round_up(max(int(a) + int(n) for a, n in zip(kv_len, n_new)) + 5, 32)
    conv = synth.bf16_representable if s.dtype == "bf16" else (lambda a: np.asarray(a, np.float32).astype(np.float64))
    qkv = conv(rng.standard_normal((B, Lq, (nq + 2 * nkv) * d)))
    k0 = conv(rng.standard_normal((B, nkv, l_max, d)))
    v0 = conv(rng.standard_normal((B, nkv, l_max, d)))
    if sections is None:
        pos = rng.integers(0, 30000, (B, Lq)).astype(np.int32)
    else:                        # image-like rows: a shared temporal id, a grid of height / width ids; then text rows
        pos = np.empty((3, B, Lq), dtype=np.int32)
        for b in range(B):
            n_img = Lq // 2
            side = max(1, int(np.sqrt(max(n_img, 1))))
            t0 = int(rng.integers(0, 2000))
            for i in range(Lq):
                if i < n_img:
                    pos[:, b, i] = (t0, t0 + i // side, t0 + i % side)
                else:
                    pos[:, b, i] = t0 + side + (i - n_img)
    gq = conv(1.0 + 0.1 * rng.standard_normal(d)) if norms else None
    gk = conv(1.0 + 0.1 * rng.standard_normal(d)) if norms else None
    q_ref, k_ref, v_ref = O.rope_append(qkv, pos, kv_len, n_new, k0, v0, nq, nkv, d, theta, s.dtype, sections=sections,
                                        q_norm=gq, k_norm=gk, eps=s.norm_eps)
    kd = binding.k_cache_pack(to_dev(k0, s.dtype))
    vd = binding.v_cache_pack(to_dev(v0, s.dtype))
    q = binding.rope_append(to_dev(qkv, s.dtype), i32(pos), i32(kv_len), i32(n_new), kd, vd, nq, theta, sections=sections,
                            q_norm=None if gq is None else to_dev(gq, s.dtype), k_norm=None if gk is None else to_dev(gk, s.dtype),
                            norm_eps=s.norm_eps)
    torch.cuda.synchronize()
    qg = q.float().cpu().numpy()
    kg = k_cache_to_rows(kd).float().cpu().numpy()
    vg = v_blocked_to_rows(vd).float().cpu().numpy()
    tol = TOL[s.dtype]
    for b in range(B):
        L0, n = int(kv_len[b]), int(n_new[b])
        if n:
            assert_close(qg[b, :n], q_ref[b, :n], tol, f"queries of sequence {b}")
            assert_close(kg[b, :, L0:L0 + n], k_ref[b, :, L0:L0 + n], tol, f"keys of sequence {b}")
            assert np.array_equal(vg[b, :, L0:L0 + n], v_ref[b, :, L0:L0 + n]), "values are copied, not rounded again"
        assert not qg[b, n:].any(), "rows past n_new are not written"
        keep = np.ones(l_max, dtype=bool)
        keep[L0:L0 + n] = False
        assert np.array_equal(kg[b][:, keep], k0[b][:, keep]) and np.array_equal(vg[b][:, keep], v0[b][:, keep])
    return qg, kg, vg


def test_tiny_fp32_one_id():
    run_case(synth.TINY, [0, 7], [9, 4], 9, seed=1)


def test_tiny_fp32_three_ids():
    run_case(synth.TINY, [3, 0], [10, 10], 10, seed=2, sections=[8, 12, 12])


@pytest.mark.parametrize("sections", [None, [16, 24, 24], [64, 0, 0]])
def test_qwen7b_shape_ragged(sections):
    """28/4 heads, d = 128: ragged n_new (one sequence with nothing to do), caches partly filled, rows that straddle a
    32-row block of the blocked key cache."""
    run_case(synth.QWEN7B, [0, 30, 500, 64], [300, 70, 0, 1], 300, seed=3, sections=sections)


def test_equal_ids_give_the_one_id_result():
    s = synth.QWEN7B
    rng = np.random.default_rng(4)
    B, Lq = 2, 40
    pos = rng.integers(0, 5000, (B, Lq)).astype(np.int32)
    qkv = to_dev(synth.bf16_representable(rng.standard_normal((B, Lq, (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim))), "bf16")
    outs = []
    for p, sec in ((pos, None), (np.stack([pos, pos, pos]), [16, 24, 24])):
        kd = torch.zeros((B, s.n_kv_heads, 64, s.head_dim), dtype=torch.bfloat16, device="cuda")
        vd = torch.zeros_like(kd)
        q = binding.rope_append(qkv, i32(p), i32([0, 5]), i32([Lq, Lq]), kd, vd, s.n_q_heads, s.rope_theta, sections=sec)
        outs.append((q, kd, vd))
    torch.cuda.synchronize()
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_gemma12b_shape_with_head_norms():
    run_case(synth.GEMMA12B, [0, 100], [130, 33], 130, seed=5, norms=True)


def test_feeds_prefill_attention():
    """Projection rows -> rope_append -> prefill_attention on the device against the same chain of checker calls."""
    s = synth.QWEN7B
    rng = np.random.default_rng(6)
    kv_len, n_new, Lq = [0, 40], [200, 150], 200
    B, nq, nkv, d = 2, s.n_q_heads, s.n_kv_heads, s.head_dim
    l_max = 256
    qkv = synth.bf16_representable(rng.standard_normal((B, Lq, (nq + 2 * nkv) * d)))
    k0 = synth.bf16_representable(rng.standard_normal((B, nkv, l_max, d)))
    v0 = synth.bf16_representable(rng.standard_normal((B, nkv, l_max, d)))
    pos = np.stack([np.arange(Lq) + int(L) for L in kv_len]).astype(np.int32)
    q_ref, k_ref, v_ref = O.rope_append(qkv, pos, kv_len, n_new, k0, v0, nq, nkv, d, s.rope_theta, "bf16")
    o_ref = O.prefill_attention(q_ref, k_ref, v_ref, kv_len, n_new)
    kd, vd = binding.k_cache_pack(to_dev(k0, "bf16")), binding.v_cache_pack(to_dev(v0, "bf16"))
    q = binding.rope_append(to_dev(qkv, "bf16"), i32(pos), i32(kv_len), i32(n_new), kd, vd, nq, s.rope_theta)
    out = binding.prefill_attention(q, kd, vd, i32(kv_len), i32(n_new))
    torch.cuda.synchronize()
    og = out.float().cpu().numpy()
    for b in range(B):
        assert_close(og[b, :n_new[b]], o_ref[b, :n_new[b]], 2e-2, f"attention output of sequence {b}")


def test_rows_that_would_pass_the_end_of_the_cache_are_dropped():
    """kv_len + n_new <= l_max is the caller's duty; a violation is clamped, never written past the cache."""
    s = synth.QWEN7B
    rng = np.random.default_rng(7)
    B, Lq, l_max = 2, 48, 64
    nq, nkv, d = s.n_q_heads, s.n_kv_heads, s.head_dim
    qkv = to_dev(synth.bf16_representable(rng.standard_normal((B, Lq, (nq + 2 * nkv) * d))), "bf16")
    pos = i32(np.tile(np.arange(Lq, dtype=np.int32), (B, 1)))
    guard = 4 * l_max * d                                   # elements behind each cache that must stay as they are
    kbuf = torch.full((B * nkv * l_max * d + guard,), 7.0, dtype=torch.bfloat16, device="cuda")
    vbuf = torch.full((B * nkv * l_max * d + guard,), 7.0, dtype=torch.bfloat16, device="cuda")
    kd = kbuf[:B * nkv * l_max * d].view(B, nkv, l_max, d)
    vd = vbuf[:B * nkv * l_max * d].view(B, nkv, l_max, d)
    q = binding.rope_append(qkv, pos, i32([40, 64]), i32([Lq, Lq]), kd, vd, nq, s.rope_theta)
    torch.cuda.synchronize()
    assert torch.all(kbuf[B * nkv * l_max * d:] == 7.0) and torch.all(vbuf[B * nkv * l_max * d:] == 7.0)
    kr = k_cache_to_rows(kd).float().cpu().numpy()
    assert np.all(kr[0, :, :40] == 7.0) and np.all(kr[0, :, 40:] != 7.0)       # 24 rows fit, the rest are dropped
    assert np.all(kr[1] == 7.0)                                              # a full cache takes nothing
    assert q[0, :24].abs().sum() > 0 and not q[0, 24:].any() and not q[1].any()
