"""Pins for the acceptance half of the CPU checker (Section 2.1 of the paper,
Eq. (TVD) of Section 6).  None of these tests uses a GPU."""
import json
import math
import os

import numpy as np
import pytest
from scipy import stats

from oracle import verify_oracle as O
from paper_2505_10526_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "accept_worked_examples.json")


def logits_of(p):
    with np.errstate(divide="ignore"):
        return np.log(np.asarray(p, dtype=np.float64))


# ---------------------------------------------------------------------------
# softmax / TVD basics
# ---------------------------------------------------------------------------
def test_softmax_invariants():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((7, 513)) * 5
    p = O.softmax(z)
    assert np.all(np.abs(p.sum(-1) - 1) < 1e-12)
    np.testing.assert_allclose(O.softmax(z + 123.456), p, rtol=1e-11)
    np.testing.assert_allclose(O.softmax(np.log([1.0, 2.0, 5.0])), [0.125, 0.25, 0.625], rtol=1e-14)
    # temperature: softmax(z/T) with T=0.5 squares the odds
    np.testing.assert_allclose(O.softmax(np.log([1.0, 3.0]) / 0.5), [0.1, 0.9], rtol=1e-14)


def test_tvd_definition_and_range():
    assert O.tvd([1, 0], [0, 1]) == 1.0
    assert O.tvd([0.3, 0.7], [0.3, 0.7]) == 0.0
    assert abs(O.tvd([0.5, 0.3, 0.2], [0.2, 0.5, 0.3]) - 0.3) < 1e-15


# ---------------------------------------------------------------------------
# worked examples (tests/golden)
# ---------------------------------------------------------------------------
def load_golden():
    with open(GOLDEN) as f:
        return json.load(f)


@pytest.mark.parametrize("case", load_golden()["cases"], ids=lambda c: c["name"][:20])
def test_worked_probabilistic_examples(case):
    p, q = np.array(case["p"]), np.array(case["q"])
    V = len(p)
    assert abs(O.tvd(p, q) - case["tvd"]) < 1e-12
    # a grid of uniforms is an exact quadrature of the accept probability
    n_u = 6000
    us = (np.arange(n_u) + 0.5) / n_u
    for tok in range(V):
        t = np.broadcast_to(logits_of(p), (n_u, 2, V))
        d = np.broadcast_to(logits_of(q), (n_u, 1, V))
        u = np.stack([us, np.full(n_u, 0.5)], axis=1)
        n, out, _ = O.spec_accept(t, d, np.full((n_u, 1), tok), u, 1.0)
        assert abs(n.mean() - case["accept_prob_per_token"][tok]) <= 1.0 / n_u + 1e-12
    if case["residual_normalised"] is not None:
        # force rejection (token with p<q, u close to 1) and sweep the resample uniform
        tok = int(np.argmin(p / q))
        t = np.broadcast_to(logits_of(p), (n_u, 2, V))
        d = np.broadcast_to(logits_of(q), (n_u, 1, V))
        u = np.stack([np.full(n_u, 0.999999), us], axis=1)
        n, out, _ = O.spec_accept(t, d, np.full((n_u, 1), tok), u, 1.0)
        assert np.all(n == 0)
        hist = np.bincount(out[:, 0], minlength=V) / n_u
        np.testing.assert_allclose(hist, case["residual_normalised"], atol=1.5 / n_u)
    rate = float(np.sum(np.minimum(p, q)))
    assert abs(rate - case["expected_accept_rate"]) < 1e-12
    assert abs(rate - (1 - O.tvd(p, q))) < 1e-12


@pytest.mark.parametrize("case", load_golden()["greedy"], ids=lambda c: c["name"][:20])
def test_worked_greedy_examples(case):
    am, x = case["target_argmax"], case["draft_tokens"]
    V, Q = 12, len(am)
    rng = np.random.default_rng(1)
    t = rng.standard_normal((1, Q, V))
    for i, a in enumerate(am):
        t[0, i, a] = 10.0
    n, out, _ = O.spec_accept(t, None, np.array([x]), None, 0.0)
    assert int(n[0]) == case["n_accepted"]
    assert out[0].tolist() == case["out_tokens"]


# ---------------------------------------------------------------------------
# temperature 0: longest matching prefix (Section 2.1, last paragraph)
# ---------------------------------------------------------------------------
def test_greedy_longest_prefix_invariant():
    rng = np.random.default_rng(2)
    B, gamma, V = 300, 5, 6           # tiny vocabulary: matches are frequent
    t = rng.standard_normal((B, gamma + 1, V))
    x = rng.integers(0, V, (B, gamma))
    # make matches frequent without using the checker: copy the row maximum's
    # position (found by sorting) into most draft slots
    best = np.argsort(-t[:, :gamma], axis=-1, kind="stable")[..., 0]
    x = np.where(rng.random((B, gamma)) < 0.75, best, x)
    n, out, _ = O.spec_accept(t, None, x, None, 0.0)
    seen = set()
    for b in range(B):
        am = [max(range(V), key=lambda k: (t[b, i, k], -k)) for i in range(gamma + 1)]
        m = 0
        while m < gamma and x[b, m] == am[m]:
            m += 1
        assert n[b] == m
        assert out[b, :m].tolist() == x[b, :m].tolist()
        assert out[b, m] == am[m]
        assert np.all(out[b, m + 1:] == -1)
        seen.add(m)
    assert seen == set(range(gamma + 1))


def test_greedy_ties_take_lowest_index():
    t = np.zeros((1, 2, 5))
    t[0, 0, [1, 3]] = 2.0
    t[0, 1, [2, 4]] = 7.0
    n, out, _ = O.spec_accept(t, None, np.array([[1]]), None, 0.0)
    assert n[0] == 1 and out[0].tolist() == [1, 2]
    n, out, _ = O.spec_accept(t, None, np.array([[3]]), None, 0.0)
    assert n[0] == 0 and out[0].tolist() == [1, -1]


# ---------------------------------------------------------------------------
# T > 0: closed forms
# ---------------------------------------------------------------------------
def sample_from(p, rng, size):
    return rng.choice(len(p), size=size, p=p)


@pytest.mark.parametrize("V,temperature", [(8, 1.0), (64, 0.7)])
def test_accept_rate_is_one_minus_tvd(V, temperature):
    """E_{x~q} min(1, p(x)/q(x)) = sum_x min(p,q) = 1 - TVD(p,q)."""
    rng = np.random.default_rng(3)
    tl = rng.standard_normal(V) * 2
    dl = tl + rng.standard_normal(V)
    p, q = O.softmax(tl / temperature), O.softmax(dl / temperature)
    N = 120000
    x = sample_from(q, rng, N)
    t = np.broadcast_to(tl, (N, 2, V))
    d = np.broadcast_to(dl, (N, 1, V))
    u = rng.random((N, 2))
    n, _, _ = O.spec_accept(t, d, x[:, None], u, temperature)
    want = 1.0 - O.tvd(p, q)
    sigma = math.sqrt(want * (1 - want) / N)
    assert abs(n.mean() - want) < 4 * sigma


def test_output_distribution_equals_target_chi_square():
    """First emitted token ~ p_1 and the first two jointly ~ p_1 x p_2
    (Section 2.1: the output distribution is the target's)."""
    rng = np.random.default_rng(4)
    V, gamma, N = 16, 2, 150000
    tl = rng.standard_normal((gamma + 1, V)) * 1.5
    dl = tl[:gamma] + rng.standard_normal((gamma, V)) * 1.0
    p = O.softmax(tl)
    q = O.softmax(dl)
    x = np.stack([sample_from(q[i], rng, N) for i in range(gamma)], axis=1)
    u = rng.random((N, gamma + 1))
    n, out, _ = O.spec_accept(np.broadcast_to(tl, (N, gamma + 1, V)),
                              np.broadcast_to(dl, (N, gamma, V)), x, u, 1.0)
    obs = np.bincount(out[:, 0], minlength=V)
    chi = stats.chisquare(obs, p[0] * N)
    assert chi.pvalue > 1e-3, chi
    # joint over two positions, among trials that emitted at least two tokens;
    # conditional on the first token being accepted the second is ~ p_2
    two = out[:, 1] >= 0
    obs2 = np.bincount(out[two, 1], minlength=V)
    chi2 = stats.chisquare(obs2, p[1] * two.sum())
    assert chi2.pvalue > 1e-3, chi2
    assert set(np.unique(n)) == {0, 1, 2}


def test_identical_distributions_always_accept_and_bonus_follows_target():
    rng = np.random.default_rng(5)
    V, gamma, N = 12, 3, 40000
    tl = rng.standard_normal((gamma + 1, V))
    p = O.softmax(tl)
    x = np.stack([sample_from(p[i], rng, N) for i in range(gamma)], axis=1)
    u = rng.random((N, gamma + 1))
    n, out, _ = O.spec_accept(np.broadcast_to(tl, (N, gamma + 1, V)),
                              np.broadcast_to(tl[:gamma], (N, gamma, V)), x, u, 1.0)
    assert np.all(n == gamma)
    assert np.array_equal(out[:, :gamma], x)
    assert stats.chisquare(np.bincount(out[:, gamma], minlength=V), p[gamma] * N).pvalue > 1e-3


def test_disjoint_supports_always_reject_and_residual_is_target():
    V, N = 10, 30000
    p = np.array([0.4, 0.3, 0.2, 0.1, 0, 0, 0, 0, 0, 0])
    q = np.array([0, 0, 0, 0, 0, 0.5, 0.25, 0.125, 0.0625, 0.0625])
    rng = np.random.default_rng(6)
    x = sample_from(q, rng, N)
    u = rng.random((N, 2))
    t = np.broadcast_to(logits_of(p), (N, 2, V))
    d = np.broadcast_to(logits_of(q), (N, 1, V))
    n, out, _ = O.spec_accept(t, d, x[:, None], u, 1.0)
    assert np.all(n == 0)
    obs = np.bincount(out[:, 0], minlength=V)
    assert np.all(obs[4:] == 0)
    assert stats.chisquare(obs[:4], p[:4] * N).pvalue > 1e-3


def test_one_hot_draft():
    """q one-hot on x, p[x] = alpha: accepted with probability alpha; the
    residual is p with x removed."""
    V, N, alpha = 6, 50000, 0.35
    p = np.array([0.05, 0.35, 0.2, 0.1, 0.25, 0.05])
    q = np.zeros(V); q[1] = 1.0
    rng = np.random.default_rng(7)
    u = rng.random((N, 2))
    n, out, _ = O.spec_accept(np.broadcast_to(logits_of(p), (N, 2, V)),
                              np.broadcast_to(logits_of(q), (N, 1, V)),
                              np.ones((N, 1), dtype=np.int32), u, 1.0)
    assert abs(n.mean() - alpha) < 4 * math.sqrt(alpha * (1 - alpha) / N)
    rej = out[n == 0, 0]
    assert np.all(rej != 1)
    want = p.copy(); want[1] = 0; want /= want.sum()
    keep = want > 0
    assert stats.chisquare(np.bincount(rej, minlength=V)[keep], want[keep] * len(rej)).pvalue > 1e-3


def test_rejection_stops_the_chain_and_uniform_mapping():
    """u[b, i] belongs to draft i; u[b, gamma] to the final draw; tokens after
    the first rejection are not examined."""
    p = np.array([0.5, 0.5]); q = np.array([0.9, 0.1])      # token 0: ratio 5/9
    t = np.broadcast_to(logits_of(p), (1, 4, 2))
    d = np.broadcast_to(logits_of(q), (1, 3, 2))
    x = np.array([[0, 0, 1]])
    # u0 accepts (0.5 < 5/9), u1 rejects (0.6 > 5/9): n = 1; residual = [0, 1] -> token 1
    n, out, _ = O.spec_accept(t, d, x, np.array([[0.5, 0.6, 0.0, 0.3]]), 1.0)
    assert n[0] == 1 and out[0].tolist() == [0, 1, -1, -1]
    # both accepted, third token has p > q so it is accepted whatever u2 is; bonus from p with u3
    n, out, _ = O.spec_accept(t, d, x, np.array([[0.5, 0.1, 0.999, 0.3]]), 1.0)
    assert n[0] == 3 and out[0].tolist() == [0, 0, 1, 0]
    n, out, _ = O.spec_accept(t, d, x, np.array([[0.5, 0.1, 0.999, 0.7]]), 1.0)
    assert out[0].tolist() == [0, 0, 1, 1]


def test_token_outside_the_vocabulary_is_rejected():
    """A draft id outside [0, V) is no token: the chain stops there at either temperature and the final token
    comes from that position's rows (residual max(p - q, 0) at T > 0, arg-max at T = 0).  Worked by hand:
    p = (0.5, 0.5), q = (0.9, 0.1) -> residual (0, 0.4) -> token 1 for any u."""
    p = np.array([0.5, 0.5]); q = np.array([0.9, 0.1])
    t = np.broadcast_to(logits_of(p), (1, 3, 2))
    d = np.broadcast_to(logits_of(q), (1, 2, 2))
    for bad in (-1, 2, 10 ** 6):
        n, out, _ = O.spec_accept(t, d, np.array([[1, bad]]), np.array([[0.99, 0.0, 0.5]]), 1.0)
        assert n[0] == 1 and out[0].tolist() == [1, 1, -1]          # token 1 has p > q: accepted whatever u is
        n, out, _ = O.spec_accept(t, d, np.array([[bad, 1]]), np.array([[0.0, 0.0, 0.5]]), 1.0)
        assert n[0] == 0 and out[0].tolist() == [1, -1, -1]
        t0 = np.array([[[0.0, 1.0], [2.0, 1.0], [0.0, 3.0]]])
        n, out, _ = O.spec_accept(t0, None, np.array([[1, bad]]), None, 0.0)
        assert n[0] == 1 and out[0].tolist() == [1, 0, -1]


# ---------------------------------------------------------------------------
# inverse CDF
# ---------------------------------------------------------------------------
def test_inverse_cdf_exact_on_integer_masses():
    r = np.array([0, 3, 0, 1, 4, 0, 2, 0], dtype=np.float64)       # total 10
    assert O.inverse_cdf(r, 0.0)[0] == 1                          # first positive index
    assert O.inverse_cdf(r, 1 - 2 ** -53)[0] == 6                  # last positive index
    us = (np.arange(1000) + 0.5) / 1000
    hist = np.bincount([O.inverse_cdf(r, u)[0] for u in us], minlength=8)
    assert hist.tolist() == [0, 300, 0, 100, 400, 0, 200, 0]
    # boundary: u * total == cumulative value exactly -> strict '>' moves on
    assert O.inverse_cdf(r, 0.3)[0] == 3
    assert O.inverse_cdf(r, 0.4)[0] == 4


def test_inverse_cdf_margin():
    r = np.array([1.0, 1.0, 2.0])
    k, m = O.inverse_cdf(r, 0.30)         # threshold 1.2, between cum 1 and 2
    assert k == 1 and abs(m - 0.05) < 1e-15
    k, m = O.inverse_cdf(r, 0.10)         # threshold 0.4 inside the first bin
    assert k == 0 and abs(m - 0.15) < 1e-15


def test_residual_falls_back_to_p_when_empty():
    p = np.array([0.2, 0.8])
    assert np.array_equal(O.residual(p, p), p)
    np.testing.assert_allclose(O.residual(p, [0.5, 0.5]), [0.0, 0.3], atol=1e-16)


def test_margin_reports_closest_accept_comparison():
    p = np.array([0.5, 0.5]); q = np.array([0.8, 0.2])      # token 0: ratio 0.625
    t = np.broadcast_to(logits_of(p), (1, 2, 2)); d = np.broadcast_to(logits_of(q), (1, 1, 2))
    _, _, m = O.spec_accept(t, d, np.array([[0]]), np.array([[0.6, 0.5]]), 1.0)
    assert abs(m[0, 0] - 0.025 / 0.625) < 1e-12


def test_synthetic_accept_inputs_exercise_every_accept_length():
    a = synth.accept_inputs(64, 5, 512, 1.0, seed=0, target_std=1.0, noise_std=1.0, peak=4.0)
    n, out, _ = O.spec_accept(a.target_logits, a.draft_logits, a.draft_tokens, a.uniforms, 1.0)
    assert set(np.unique(n)) == set(range(6))
    assert np.all((out >= 0).sum(1) == n + 1)


def test_sampling_step_draws_from_the_single_row():
    """gamma = 0 (the drafting loop's own draw, Section 2.1): with V = 4 and weights 1:2:3:4 the token
    is the quartile-like bucket of the uniform, n_accepted is 0; greedy gives the lowest arg-max."""
    logits = np.log(np.array([[[1.0, 2.0, 3.0, 4.0]]]))            # p = .1 .2 .3 .4
    for u, want in ((0.0, 0), (0.05, 0), (0.15, 1), (0.29, 1), (0.31, 2), (0.59, 2), (0.61, 3), (0.999, 3)):
        n, out, _ = O.spec_accept(logits, None, np.zeros((1, 0), np.int32), np.array([[u]]), 1.0)
        assert n[0] == 0 and out[0, 0] == want, (u, out)
    # temperature 0.5 squares the weights: p = 1/30, 4/30, 9/30, 16/30
    for u, want in ((0.03, 0), (0.04, 1), (0.16, 1), (0.17, 2), (0.46, 2), (0.47, 3)):
        _, out, _ = O.spec_accept(logits, None, np.zeros((1, 0), np.int32), np.array([[u]]), 0.5)
        assert out[0, 0] == want, (u, out)
    n, out, _ = O.spec_accept(np.array([[[0.0, 7.0, 7.0, 1.0]]]), None, np.zeros((1, 0), np.int32), None, 0.0)
    assert n[0] == 0 and out[0, 0] == 1


def test_sampling_step_frequencies_follow_softmax():
    rng = np.random.default_rng(3)
    logits = rng.normal(size=(1, 1, 6)) * 1.5
    p = np.exp(logits[0, 0] / 0.8); p /= p.sum()
    draws = 20000
    u = rng.random(draws)
    counts = np.zeros(6)
    big = np.repeat(logits, draws, axis=0)
    _, out, _ = O.spec_accept(big, None, np.zeros((draws, 0), np.int32), u[:, None], 0.8)
    for k in out[:, 0]:
        counts[k] += 1
    chi2 = float(np.sum((counts - draws * p) ** 2 / (draws * p)))
    assert chi2 < 25.7                                            # chi-square, 5 dof, p = 1e-4


def test_tvd_rows_closed_forms():
    """Eq. (TVD) on logits: identical rows give 0, disjoint supports give 1, two-token rows give
    |sigmoid(a/T) - sigmoid(b/T)|, and a shift of either row by a constant changes nothing."""
    t = np.array([[0.0, 1.0, 2.0], [0.0, -np.inf, -np.inf], [3.0, 0.0, -np.inf]])
    d = np.array([[5.0, 6.0, 7.0], [-np.inf, 0.0, 1.0], [-1.0, 0.0, -np.inf]])
    T = 0.7
    got = O.tvd_rows(t, d, T)
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    assert abs(got[0]) < 1e-15
    assert abs(got[1] - 1.0) < 1e-15
    assert abs(got[2] - abs(sig(3.0 / T) - sig(-1.0 / T))) < 1e-14


def test_embed_tokens_gathers_rows():
    table = np.arange(20, dtype=np.float32).reshape(5, 4)
    out = O.embed_tokens(table, [3, 0, 4, 7, -1])
    assert np.array_equal(out[0], table[3]) and np.array_equal(out[1], table[0]) and np.array_equal(out[2], table[4])
    assert not out[3].any() and not out[4].any()


def test_commit_tokens_worked_example():
    """gamma = 3: a sequence that kept 2 drafts emits 3 tokens and its next input is the third."""
    out = np.array([[11, 12, 99, -1], [7, -1, -1, -1], [1, 2, 3, 4]])
    last, kv = O.commit_tokens([2, 0, 3], out, [100, 50, 0])
    assert last.tolist() == [99, 7, 4] and kv.tolist() == [103, 51, 4]
