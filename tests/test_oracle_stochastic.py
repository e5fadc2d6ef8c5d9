"""Pins for the stochastic verification rule (section 2.1) on the oracle (no GPU)."""
import os

import numpy as np
import pytest

from oracle import minions_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    n = 0
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        assert list(orc.philox4x32(w[0:4], w[4:6])) == w[6:10]
        n += 1
    assert n == 3


def test_unit_double_range_and_bits():
    assert orc.unit_double(0, 0) == 0.0
    assert orc.unit_double(0xFFFFFFFF, 0xFFFFFFFF) == 1.0 - 2.0 ** -53
    assert orc.unit_double(0x80000000, 0) == 0.5
    assert orc.unit_double(0, 1 << 6) == 2.0 ** -53            # lowest bit that counts
    assert orc.unit_double(31, 63) == 0.0                      # the dropped low bits
    us = [orc.verify_uniforms(7, 3, b, j) for b in range(20) for j in range(20)]
    flat = np.array(us).ravel()
    assert flat.min() >= 0.0 and flat.max() < 1.0 and len(set(flat.tolist())) == flat.size
    assert abs(flat.mean() - 0.5) < 0.05
    assert orc.verify_uniforms(7, 3, 1, 2) != orc.verify_uniforms(7, 4, 1, 2) != orc.verify_uniforms(8, 4, 1, 2)


def test_sample_cdf_closed_cases():
    assert orc.sample_cdf(np.array([1.0, 1.0, 2.0]), 0.49)[0] == 1
    assert orc.sample_cdf(np.array([1.0, 1.0, 2.0]), 0.50)[0] == 2      # the running sum must exceed the target
    assert orc.sample_cdf(np.array([1.0, 1.0, 2.0]), 0.0)[0] == 0
    assert orc.sample_cdf(np.array([0.0, 1.0, 0.0]), 0.0)[0] == 1       # a token without mass is never drawn
    assert orc.sample_cdf(np.array([0.0, 1.0, 0.0]), 1.0 - 2.0 ** -53)[0] == 1
    v, gap = orc.sample_cdf(np.array([1.0, 3.0]), 0.5)
    assert v == 1 and gap == pytest.approx(0.25)


def _dists(rng, k, V, spread):
    logits = rng.normal(0.0, spread, (k + 1, V))
    q = np.stack([orc.llm_probs(rng.normal(0.0, spread, V), 1.0) for _ in range(k)])
    return logits, q


def test_llm_probs_recovers_a_known_distribution_at_any_temperature():
    """Closed form: scores T * log p (plus any constant) at temperature T are the distribution p itself; and
    at temperature T the odds of two tokens are exp((l_a - l_b) / T)."""
    g = np.random.default_rng(5)
    for T in (0.5, 1.0, 2.0, 7.25):
        p = g.random(37) + 1e-3
        p /= p.sum()
        for shift in (0.0, -31.5, 400.0):
            o = orc.llm_probs(T * np.log(p) + shift, T)
            assert np.allclose(o, p, rtol=1e-12, atol=0.0)
            assert abs(o.sum() - 1.0) < 1e-14
    l = np.array([0.3, -1.2, 2.0, 0.0])
    for T in (0.5, 2.0):
        o = orc.llm_probs(l, T)
        assert np.isclose(o[2] / o[1], np.exp((l[2] - l[1]) / T), rtol=1e-13)
        assert np.isclose(o[0] / o[3], np.exp(0.3 / T), rtol=1e-13)
    # T -> infinity flattens, a masked score has no mass
    assert np.allclose(orc.llm_probs(l, 1e9), 0.25, atol=1e-8)
    assert orc.llm_probs(np.array([0.0, -np.inf, 0.0]), 0.5).tolist() == [0.5, 0.0, 0.5]


def test_emitted_tokens_follow_the_llm_distribution():
    """The rule is lossless: whatever q is, the token emitted at a position is distributed as o there.
    Checked on the first position and, given that the first draft survived, on the second."""
    rng = np.random.default_rng(11)
    V, k, T, N = 5, 3, 0.8, 24000
    logits, q = _dists(rng, k, V, 1.5)
    o0, o1 = orc.llm_probs(logits[0], T), orc.llm_probs(logits[1], T)
    first = np.zeros(V)
    second = np.zeros(V)
    acc_hist = np.zeros(k + 1)
    for t in range(N):
        voted = [int(rng.choice(V, p=q[i])) for i in range(k)]
        a, out, _ = orc.accept_stochastic(voted, logits, q, k, T, seed=99, step=t, b=0)
        assert len(out) == a + 1 and out[:a] == voted[:a]
        if a < k:
            assert out[a] != voted[a]       # a rejected token has no mass left in max(0, o - q)
        first[out[0]] += 1
        acc_hist[a] += 1
        if a >= 1:
            second[out[1]] += 1
    assert np.abs(first / N - o0).max() < 4.0 * np.sqrt(0.25 / N)
    n2 = second.sum()
    assert n2 > N / 10 and np.abs(second / n2 - o1).max() < 4.0 * np.sqrt(0.25 / n2)
    # the chance that the first draft survives is sum_x min(q(x), o(x))
    p_keep = float(np.minimum(q[0], o0).sum())
    assert abs((N - acc_hist[0]) / N - p_keep) < 4.0 * np.sqrt(0.25 / N)


def test_equal_distributions_accept_everything():
    rng = np.random.default_rng(5)
    V, k, T = 17, 6, 1.3
    logits = rng.normal(0.0, 2.0, (k + 1, V))
    q = np.stack([orc.llm_probs(logits[i], T) for i in range(k)])
    for t in range(50):
        voted = [int(rng.integers(V)) for _ in range(k)]
        a, out, _ = orc.accept_stochastic(voted, logits, q, k, T, seed=1, step=t, b=3)
        assert a == k and out[:k] == voted
        _, u = orc.verify_uniforms(1, t, 3, k)
        assert out[k] == orc.sample_cdf(orc.llm_probs(logits[k], T), u)[0]   # bonus token from o_{k+1}


def test_low_temperature_is_the_greedy_rule():
    """With one-hot drafts and T -> 0 the rule keeps a token iff it is the LLM's argmax and replaces
    the first other one by that argmax: the greedy acceptance."""
    rng = np.random.default_rng(8)
    V, k = 23, 5
    for t in range(40):
        logits = rng.normal(0.0, 3.0, (k + 1, V))
        g = orc.greedy_tokens(logits)
        logits[np.arange(k + 1), g] += 0.1   # a clear winner per row: exp(-0.1 / T) vanishes
        voted = [int(g[i]) if rng.random() < 0.7 else int(rng.integers(V)) for i in range(k)]
        q = np.zeros((k, V))
        q[np.arange(k), voted] = 1.0
        a, out, _ = orc.accept_stochastic(voted, logits, q, k, 1e-3, seed=2, step=t, b=0)
        assert (a, out) == orc.accept(voted, g, k)


def test_rejection_probability_is_one_minus_ratio():
    logits = np.log(np.array([[0.25, 0.75], [0.5, 0.5]]))
    q = np.array([[0.5, 0.5]])
    N, kept = 20000, 0
    for t in range(N):
        a, out, _ = orc.accept_stochastic([0], logits, q, 1, 1.0, seed=4, step=t, b=1)
        kept += a
        if a == 0:
            assert out == [1]               # all of max(0, o - q) sits on token 1
    assert abs(kept / N - 0.5) < 4.0 * np.sqrt(0.25 / N)
    # a token the LLM gives at least the SSM's probability is never rejected
    for t in range(200):
        assert orc.accept_stochastic([1], logits, q, 1, 1.0, seed=4, step=t, b=1)[0] == 1


def test_draft_sample_distribution_and_streams():
    """An SSM's draws follow its own q; SSMs and the verifier use different numbers under one seed."""
    rng = np.random.default_rng(21)
    V, T, N = 6, 0.7, 20000
    z = rng.normal(0.0, 1.2, V)
    q = orc.llm_probs(z, T)
    counts = np.zeros(V)
    for step in range(N):
        tok, q32, _ = orc.draft_sample(z, T, seed=5, step=step, ssm=2, b=1, t=3)
        counts[tok] += 1
    assert q32.dtype == np.float32 and np.abs(q32 - q).max() < 1e-7
    assert np.abs(counts / N - q).max() < 4.0 * np.sqrt(0.25 / N)
    us = {orc.verify_uniforms(5, 9, 1, 3, consumer=c) for c in range(0, 6)}
    assert len(us) == 6
    assert orc.verify_uniforms(5, 9, 1, 3) == orc.verify_uniforms(5, 9, 1, 3, consumer=0)
    # a draw on a one-hot distribution is that token whatever the number
    hot = np.full(V, -1e4); hot[4] = 0.0
    assert all(orc.draft_sample(hot, 1.0, 1, s_, 0, 0, 0)[0] == 4 for s_ in range(50))


def test_a_draft_distribution_above_the_llms_everywhere_never_re_emits_the_rejected_token():
    """q = 1.5 o (not a distribution): max(0, o - q) is empty.  A rejected token is then replaced from o without
    that token: the replacement differs from it, is rejected with probability 1 - o/q = 1/3, and follows
    o(v) / (1 - o(x)); with all of o on the token, it stays."""
    g = np.random.default_rng(11)
    V, T, x = 6, 1.0, 2
    logits = np.stack([g.normal(0.0, 1.0, V), g.normal(0.0, 1.0, V)])
    o = orc.llm_probs(logits[0], T)
    q = (1.5 * o)[None, :]
    counts, rejected, n = np.zeros(V), 0, 6000
    for step in range(n):
        a, toks, _ = orc.accept_stochastic([x], logits, q, 1, T, 5, step, 0)
        if a == 0:
            rejected += 1
            assert toks[0] != x
            counts[toks[0]] += 1
    assert abs(rejected / n - 1.0 / 3.0) < 0.02
    want = o.copy(); want[x] = 0.0; want /= want.sum()
    assert np.abs(counts / rejected - want).max() < 0.03
    # all of o on x, q(x) > 1: whatever the uniform number says, x is what comes out, and the next position is reached
    lone = np.full((2, V), -np.inf); lone[0, x] = 0.0; lone[1] = logits[1]
    q1 = np.zeros((1, V)); q1[0, x] = 3.0
    for step in range(50):
        a, toks, _ = orc.accept_stochastic([x], lone, q1, 1, T, 5, step, 0)
        assert a == 1 and toks[0] == x and len(toks) == 2
