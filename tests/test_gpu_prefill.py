"""GPU parity of prefill_attention against the CPU checker (paper Section 2.2: the projected image features enter
the sequence ahead of the text tokens; the prompt pass attends over all of them)."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2505_10526_amd import synth, binding
from helpers import to_dev, i32, round_up, pad_rows, assert_close

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
TOL_F32 = 2e-5


def run_case(shape, kv_len, n_new, n_img, seed, Lq=None, window=0, bidir=False, hot_keys=2, check=None):
    """Caches hold kv_len[b] + n_new[b] valid rows (image rows first, drawn wider), NaN beyond; q rows past n_new[b]
    hold NaN as well (they are not positions).  `check`: sequences handed to the checker (default all)."""
    B = len(kv_len)
    kv_len, n_new, n_img = (np.asarray(a, dtype=np.int32) for a in (kv_len, n_new, n_img))
    Lq = Lq or int(n_new.max())
    total = kv_len + n_new
    kv = synth.kv_cache(shape, B, 0, total, n_img, seed, hot_keys=hot_keys, junk_tail=False)
    for b in range(B):
        kv.k[b, :, total[b]:] = np.nan
        kv.v[b, :, total[b]:] = np.nan
    q = synth.queries(shape, B, Lq, seed)
    for b in range(B):
        q[b, n_new[b]:] = np.nan
    nb = n_img if bidir else None
    sel = list(range(B)) if check is None else list(check)
    ref = O.prefill_attention(q[sel], kv.k[sel], kv.v[sel], kv_len[sel], n_new[sel], window=window,
                              n_bidir=None if nb is None else nb[sel])
    lm = round_up(int(total.max()), 32)
    kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), shape.dtype))
    vd = binding.v_cache_pack(to_dev(pad_rows(kv.v, lm), shape.dtype))
    out = binding.prefill_attention(to_dev(q, shape.dtype), kd, vd, i32(kv_len), i32(n_new),
                                    None if nb is None else i32(nb), window=window)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    tol = TOL_BF16 if shape.dtype == "bf16" else TOL_F32
    for j, b in enumerate(sel):
        n = int(n_new[b])
        if n:
            assert_close(got[b, :n], ref[j, :n], tol, f"sequence {b}")
        assert np.all(got[b, n:] == 0), "rows past n_new must not be written"
    return got


def test_tiny_fp32():
    run_case(synth.TINY, [0, 30], [70, 41], [64, 10], seed=0)
    run_case(synth.TINY, [0, 30], [70, 41], [64, 40], seed=1, bidir=True)
    run_case(synth.TINY, [5, 0], [60, 33], [20, 8], seed=2, window=17)


@pytest.mark.parametrize("n_new", [[1], [2], [9], [10], [31], [33], [64], [65], [200], [257]])
def test_bf16_ragged_sizes_d64(n_new):
    """Row-tile and key-block boundaries: G = 2 heads stacked, 64 stacked rows per wave, 256 per workgroup."""
    s = synth.LayerShape(256, 4, 2, 64, 704, 4096, dtype="bf16")
    run_case(s, [0], n_new, [min(n_new[0], 20)], seed=3)
    run_case(s, [37], n_new, [30], seed=4, Lq=n_new[0] + 3)


def test_qwen7b_shape_ragged_batch():
    """28/4 heads, d=128 (7 heads stacked per position): fresh prompts of different lengths with image prefixes,
    one sequence continuing a cached piece, one with nothing to do."""
    run_case(synth.QWEN7B, [0, 0, 300, 0], [700, 1000, 421, 0], [576, 700, 256, 0], seed=5)


def test_qwen7b_shape_image_block_attends_within_itself():
    run_case(synth.QWEN7B, [0, 100], [500, 300], [256, 260], seed=6, bidir=True)


@pytest.mark.parametrize("window", [1, 40, 512])
def test_qwen7b_shape_sliding_window(window):
    run_case(synth.QWEN7B, [0, 64], [600, 333], [256, 100], seed=7, window=window)


def test_gemma12b_shape():
    """16/8 heads, d=256 (two heads stacked), 32 stacked rows per wave; local-layer variant with the image block."""
    run_case(synth.GEMMA12B, [0, 0], [900, 257], [256, 256], seed=8)
    run_case(synth.GEMMA12B, [0, 50], [600, 300], [256, 256], seed=9, window=128, bidir=True)


def test_prompt_fed_in_two_pieces_equals_one_piece():
    """Section 2.1: a position conditions on all earlier ones however they got into the cache."""
    s = synth.QWEN7B
    kv = synth.kv_cache(s, 1, 0, [500], [256], 10, junk_tail=False)
    q = synth.queries(s, 1, 500, 10)
    kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, 512), s.dtype))
    vd = binding.v_cache_pack(to_dev(pad_rows(kv.v, 512), s.dtype))
    qd = to_dev(q, s.dtype)
    whole = binding.prefill_attention(qd, kd, vd, i32([0]), i32([500]))
    a = binding.prefill_attention(qd[:, :200].contiguous(), kd, vd, i32([0]), i32([200]))
    b = binding.prefill_attention(qd[:, 200:].contiguous(), kd, vd, i32([200]), i32([300]))
    torch.cuda.synchronize()
    two = torch.cat([a, b], 1).float().cpu().numpy()
    # same keys per row; only the grouping of rows into waves differs, the arithmetic of a row does not
    np.testing.assert_allclose(two, whole.float().cpu().numpy(), rtol=2e-2, atol=2e-3)
    assert torch.equal(whole, binding.prefill_attention(qd, kd, vd, i32([0]), i32([500])))       # repeatable bits


def test_verify_pass_is_the_short_case():
    """gamma+1 new positions over a long cache: the same numbers as verify_attention up to rounding order."""
    s = synth.QWEN7B
    kv = synth.kv_cache(s, 2, 6, [1000, 333], [700, 100], 11, junk_tail=False)
    q = to_dev(synth.queries(s, 2, 6, 11), s.dtype)
    lm = round_up(kv.l_max, 32)
    kd = binding.k_cache_pack(to_dev(pad_rows(kv.k, lm), s.dtype))
    vd = binding.v_cache_pack(to_dev(np.nan_to_num(pad_rows(kv.v, lm)), s.dtype))
    a = binding.prefill_attention(q, kd, vd, i32(kv.kv_len), i32([6, 6])).float().cpu().numpy()
    b = binding.verify_attention(q, kd, vd, i32(kv.kv_len)).float().cpu().numpy()
    np.testing.assert_allclose(a, b, rtol=2e-2, atol=2e-3)


def test_bench_shape_sampled_rows():
    """The launch the benchmark times: B=8 prompts of 2048 positions (1280 image rows), 28/4 heads, d=128.  The
    checker runs on two of the sequences."""
    run_case(synth.QWEN7B, [0] * 8, [2048] * 8, [1280] * 8, seed=12, check=(0, 7))
