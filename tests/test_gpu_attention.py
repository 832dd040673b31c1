"""GPU parity of verify_attention against the CPU checker (paper Section 2.1:
gamma+1 positions scored in one parallel pass over the KV cache whose prefix
holds image-token then text positions)."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2505_10526_amd import synth, binding
from helpers import DEV, to_dev, i32, round_up, pad_rows, assert_close

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2      # max |err| / max |ref|, the bound set for bf16 activations
TOL_F32 = 2e-5       # fp32 path: fp32 accumulation over <= 300 keys of O(1) values


def run_case(shape, B, Q, kv_len, n_img, seed, std=1.0, hot_keys=0, l_max=None, q_std=1.0, nan_tail=False, window=0):
    kv = synth.kv_cache(shape, B, Q, kv_len, n_img, seed, std=std, hot_keys=hot_keys)
    # the step's own rows: new keys / values at [kv_len, kv_len+Q)
    newk = synth.normal((B, shape.n_kv_heads, Q, shape.head_dim), std, seed, 77, dtype=shape.dtype)
    newv = synth.normal((B, shape.n_kv_heads, Q, shape.head_dim), std, seed, 78, dtype=shape.dtype)
    for b in range(B):
        L = int(kv.kv_len[b])
        kv.k[b, :, L:L + Q] = newk[b]
        kv.v[b, :, L:L + Q] = newv[b]
        if nan_tail:
            kv.k[b, :, L + Q:] = np.nan
            kv.v[b, :, L + Q:] = np.nan
    q = synth.queries(shape, B, Q, seed, std=q_std)
    ref = O.attention(q, kv.k, kv.v, kv.kv_len, window=window)
    lm = round_up(l_max or kv.l_max, 32)
    kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), shape.dtype))
    vd = binding.v_cache_pack(to_dev(pad_rows(kv.v, lm), shape.dtype))
    out = binding.verify_attention(to_dev(q, shape.dtype), kd, vd, i32(kv.kv_len), window=window)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), ref


def test_tiny_fp32_config():
    """B=1, gamma=5, KV prefix 256 (64 image rows), 4 q / 2 kv heads, d=64, K,V ~ N(0, 0.02)."""
    got, ref = run_case(synth.TINY, 1, 6, [256], [64], seed=0, std=0.02)
    assert_close(got, ref, TOL_F32, "tiny fp32")


def test_tiny_fp32_rescale_variant():
    """Same shape with K,V ~ N(0,1) and a few keys scaled by 8: the running maximum moves late."""
    got, ref = run_case(synth.TINY, 2, 6, [256, 300], [64, 10], seed=1, std=1.0, hot_keys=3)
    assert_close(got, ref, TOL_F32, "tiny fp32 hot keys")


@pytest.mark.parametrize("kv_len", [[0], [1], [26], [27], [31], [32], [250], [256], [1000]])
def test_bf16_ragged_lengths_d64(kv_len):
    """Block boundaries of 32 keys, an empty cache, lengths that end inside / at a block."""
    s = synth.LayerShape(256, 4, 2, 64, 704, 4096, dtype="bf16")
    got, ref = run_case(s, 1, 6, kv_len, [min(kv_len[0], 64)], seed=2, hot_keys=2 if kv_len[0] > 4 else 0, nan_tail=True)
    assert_close(got, ref, TOL_BF16, f"bf16 d64 kv_len={kv_len}")


def test_qwen7b_shape_single_sequence():
    """28 q / 4 kv heads, d=128, gamma=5, KV 1024 (700 image rows)."""
    got, ref = run_case(synth.QWEN7B, 1, 6, [1024], [700], seed=3, hot_keys=2)
    assert_close(got, ref, TOL_BF16, "qwen7b B=1")


def test_qwen7b_shape_ragged_batch():
    """B=8, per-sequence lengths in [1024, 2048] with 256-1024 leading image rows; one
    allocation size for all, rows past each sequence's end hold NaN."""
    rng = np.random.default_rng(4)
    kv_len = rng.integers(1024, 2049, 8)
    n_img = rng.integers(256, 1025, 8)
    got, ref = run_case(synth.QWEN7B, 8, 6, kv_len, n_img, seed=4, hot_keys=2, nan_tail=True)
    assert_close(got, ref, TOL_BF16, "qwen7b B=8 ragged")


def test_gemma12b_shape():
    """16 q / 8 kv heads, d=256, B=4 (two sequences checked against the checker at full length 4096)."""
    got, ref = run_case(synth.GEMMA12B, 2, 6, [4096, 4000], [256, 256], seed=5, hot_keys=2, nan_tail=True)
    assert_close(got, ref, TOL_BF16, "gemma12b")


def test_long_context_gamma7():
    """gamma=7 (56 stacked query rows), KV 8192 with 1280 image rows."""
    got, ref = run_case(synth.QWEN7B, 2, 8, [8192, 5000], [1280, 1280], seed=6, hot_keys=3, nan_tail=True)
    assert_close(got, ref, TOL_BF16, "long context")


def test_parallel_pass_equals_sequential_decode_on_gpu():
    """The Q-query pass equals Q single-query calls with a growing cache (Section 2.1)."""
    s = synth.QWEN7B
    B, Q = 2, 6
    kv = synth.kv_cache(s, B, Q, [300, 77], [100, 10], 7, junk_tail=False)
    q = synth.queries(s, B, Q, 7)
    lm = round_up(kv.l_max, 32)
    kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), "bf16"))
    vd = binding.v_cache_pack(to_dev(pad_rows(kv.v, lm), "bf16"))
    qd = to_dev(q, "bf16")
    par = binding.verify_attention(qd, kd, vd, i32(kv.kv_len)).float().cpu().numpy()
    for i in range(Q):
        one = binding.verify_attention(qd[:, i:i + 1].contiguous(), kd, vd, i32(kv.kv_len + i)).float().cpu().numpy()
        # same keys, same per-row arithmetic up to how the key range is cut into splits
        np.testing.assert_allclose(one[:, 0], par[:, i], rtol=2e-2, atol=2e-3)


def test_repeatable_bits_and_pack_roundtrip():
    s = synth.QWEN7B
    kv = synth.kv_cache(s, 2, 6, [500, 333], [100, 100], 8, junk_tail=False)
    q = to_dev(synth.queries(s, 2, 6, 8), "bf16")
    lm = round_up(kv.l_max, 32)
    kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), "bf16"))
    vrow = to_dev(np.nan_to_num(pad_rows(kv.v, lm)), "bf16")
    vd = binding.v_cache_pack(vrow)
    from helpers import v_blocked_to_rows, k_cache_to_rows
    assert torch.equal(v_blocked_to_rows(vd), vrow)
    krow = to_dev(np.nan_to_num(pad_rows(kv.k, lm)), "bf16")
    assert torch.equal(k_cache_to_rows(binding.k_cache_pack(krow)), krow)
    a = binding.verify_attention(q, kd, vd, i32(kv.kv_len))
    b = binding.verify_attention(q, kd, vd, i32(kv.kv_len))
    assert torch.equal(a, b)


# ---------------------------------------------------------------------------
# sliding-window layers of the Gemma 3 targets (Section 5, "Models")
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("window", [1, 2, 6, 31, 32, 33, 64, 100, 300, 5000])
def test_window_bf16_d128_ragged(window):
    """Windows smaller than the query count, at and around block boundaries, larger than the cache;
    ragged lengths including an empty cache."""
    got, ref = run_case(synth.QWEN7B, 4, 6, [0, 37, 250, 1000], [0, 10, 64, 300], seed=21, hot_keys=2, nan_tail=True,
                        window=window)
    assert_close(got, ref, TOL_BF16, f"window {window}")


@pytest.mark.parametrize("window", [5, 48, 200])
def test_window_fp32_and_d64(window):
    got, ref = run_case(synth.TINY, 2, 6, [256, 30], [64, 10], seed=22, hot_keys=2, window=window)
    assert_close(got, ref, TOL_F32, f"fp32 window {window}")
    s = synth.LayerShape(256, 4, 2, 64, 704, 4096, dtype="bf16")
    got, ref = run_case(s, 3, 4, [300, 2, 95], [64, 0, 64], seed=23, hot_keys=2, nan_tail=True, window=window)
    assert_close(got, ref, TOL_BF16, f"bf16 d64 window {window}")


def test_window_gemma12b_local_layer_shape():
    """16 q / 8 kv heads, d=256, KV 4096, window 1024: three quarters of the cache are never read."""
    got, ref = run_case(synth.GEMMA12B_LOCAL, 2, 6, [4096, 3000], [256, 256], seed=24, hot_keys=2, window=1024)
    assert_close(got, ref, TOL_BF16, "gemma local")


def test_window_rows_outside_are_not_read():
    """Rows below every query's window hold NaN: the output must not see them."""
    s, B, Q, W = synth.QWEN7B, 2, 6, 40
    kv = synth.kv_cache(s, B, Q, [500, 90], [100, 20], seed=25, junk_tail=False)
    q = synth.queries(s, B, Q, 25)
    ref = O.attention(q, kv.k, kv.v, kv.kv_len, window=W)
    k, v = kv.k.copy(), kv.v.copy()
    for b in range(B):
        lo = int(kv.kv_len[b]) - W + 1          # the first query's window starts here
        k[b, :, :lo] = np.nan
        v[b, :, : lo // 32 * 32] = np.nan       # values are read in blocks of 32 rows and masked by weight 0
    lm = round_up(kv.l_max, 32)
    out = binding.verify_attention(to_dev(q, s.dtype), binding.k_cache_pack(to_dev(pad_rows(k, lm), s.dtype)),
                                   binding.v_cache_pack(to_dev(pad_rows(v, lm), s.dtype)), i32(kv.kv_len), window=W)
    torch.cuda.synchronize()
    assert_close(out.float().cpu().numpy(), ref, TOL_BF16, "window with NaN outside")


@pytest.mark.parametrize("window", [3, 40, 700])
def test_window_four_row_tiles_and_wide_heads(window):
    """gamma = 7 on the 28/4-head shape stacks 56 rows (four row tiles); d = 256 with gamma = 15 stacks 32."""
    got, ref = run_case(synth.QWEN7B, 2, 8, [900, 65], [300, 10], seed=26, hot_keys=2, nan_tail=True, window=window)
    assert_close(got, ref, TOL_BF16, f"Q=8 window {window}")
    got, ref = run_case(synth.GEMMA12B, 1, 16, [333], [100], seed=27, hot_keys=2, nan_tail=True, window=window)
    assert_close(got, ref, TOL_BF16, f"d=256 Q=16 window {window}")


# ---------------------------------------------------------------------------
# long key streams per wavefront: the launch shapes bench.py times
# ---------------------------------------------------------------------------
def deep_stream_case(shape, B, Q, L, n_img, seed, check_seqs):
    """All B sequences at cache length L go through ONE library call (so the grid, the number of key-range
    splits and the blocks per wavefront are those of the full batch); the checker is run on the sequences in
    check_seqs (all of them: a few seconds).  Keys in the second half of the stream
    and among the new rows are scaled up by growing factors, so the largest score of many rows moves several
    times deep into the stream (the streaming softmax has to re-reference late), while rows that meet those
    keys with a negative product stay diffuse.  Rows past L + Q hold NaN."""
    kv = synth.kv_cache(shape, B, Q, [L] * B, [n_img] * B, seed, junk_tail=False)
    kv.k[:, :, L:L + Q] = synth.normal((B, shape.n_kv_heads, Q, shape.head_dim), 1.0, seed, 77, dtype=shape.dtype)
    kv.v[:, :, L:L + Q] = synth.normal((B, shape.n_kv_heads, Q, shape.head_dim), 1.0, seed, 78, dtype=shape.dtype)
    rng = np.random.default_rng([seed, 79])
    for b in range(B):
        for g in range(shape.n_kv_heads):
            rows = np.sort(rng.choice(np.arange(L // 2, L + Q), size=6, replace=False))
            for t, r in enumerate(rows):
                kv.k[b, g, r] *= np.float32(3.0 + 1.5 * t)
    kv.k = synth.bf16_representable(kv.k)
    q = synth.queries(shape, B, Q, seed)
    lm = round_up(L + Q, 32)
    kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), shape.dtype))
    vd = binding.v_cache_pack(to_dev(pad_rows(kv.v, lm), shape.dtype))
    out = binding.verify_attention(to_dev(q, shape.dtype), kd, vd, i32(kv.kv_len))
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.all(np.isfinite(got))
    sel = list(check_seqs)
    ref = O.attention(q[sel], kv.k[sel], kv.v[sel], kv.kv_len[sel])
    return got[sel], ref


def test_long_context_batched_launch():
    """The long-context stress configuration as the benchmark launches it: B=32, gamma=7 (56 stacked rows, four
    row tiles), KV 8192 with 1280 image rows, 28/4 heads, d=128 -- grid 2 x 4 x 32, 129 key blocks per split,
    about 32 per wavefront on the single-register-set refill path."""
    got, ref = deep_stream_case(synth.QWEN7B, 32, 8, 8192, 1280, seed=30, check_seqs=range(32))
    assert_close(got, ref, TOL_BF16, "long context, B=32")


def test_deep_stream_wide_heads_single_split():
    """Gemma3-12B-shaped heads (16/8, d=256), B=32, KV 4096: one split per (sequence, KV head), 32 key blocks per
    wavefront through the plain d=256 loop; the kernel writes the final output itself (no combine)."""
    got, ref = deep_stream_case(synth.GEMMA12B, 32, 6, 4096, 256, seed=31, check_seqs=range(32))
    assert_close(got, ref, TOL_BF16, "d=256, B=32, one split")


def test_deep_stream_two_register_sets():
    """d=128 with one row tile (8/4 heads, gamma=5: 12 stacked rows), B=64, KV 4096: one split, 32 key blocks per
    wavefront through the loop that keeps the next block's keys and values in a second register set."""
    s = synth.LayerShape(1024, 8, 4, 128, 2048, 4096, dtype="bf16")
    got, ref = deep_stream_case(s, 64, 6, 4096, 256, seed=32, check_seqs=range(64))
    assert_close(got, ref, TOL_BF16, "d=128 one row tile, B=64, one split")
