"""Pins for the oracle's accept / resample rule (CPU only): what Section 3.1 and Algorithm 1 fix."""
from fractions import Fraction
import itertools

import numpy as np
import pytest
from scipy import stats

import oracle
import workloads as wl


def _rand_probs(rng, shape, V, sharp=1.0):
    z = rng.standard_normal(shape + (V,)) * sharp
    e = np.exp(z - z.max(-1, keepdims=True))
    return (e / e.sum(-1, keepdims=True)).astype(np.float32)


def test_equal_distributions_accept_every_draft():
    """p_d = p_t makes the ratio 1, so every draft is accepted for every u in [0,1) (Section 3.1)."""
    rng = np.random.default_rng(1)
    N, G, V = 64, 5, 50
    p = _rand_probs(rng, (N, G), V)
    toks = rng.integers(0, V, size=(N, G))
    for u in (0.0, 0.5, 1.0 - 2.0 ** -24):
        a, out, n, _ = oracle.accept_resample(p, p.copy(), toks, np.full((N, G), u, np.float32),
                                              np.full(N, u, np.float32))
        assert (a == G).all() and (n == G).all()
        assert np.array_equal(out[:, :G], toks) and (out[:, G] == -1).all()


def test_greedy_equals_argmax_decoding():
    """Greedy verification reproduces token-by-token argmax decoding of the target (Section 3.1:
    the output is unchanged in the greedy setting)."""
    rng = np.random.default_rng(2)
    N, G, V = 200, 4, 12
    logits = rng.standard_normal((N, G, V)).astype(np.float32)
    best = logits.argmax(-1)
    drafts = best.copy()
    wrong = rng.random((N, G)) < 0.3
    drafts[wrong] = (drafts[wrong] + 1 + rng.integers(0, V - 1, size=wrong.sum())) % V
    a, out, n, _ = oracle.accept_resample(None, None, drafts, None, None, greedy=True, logits=logits)
    for b in range(N):
        first_bad = int(np.argmax(drafts[b] != best[b])) if (drafts[b] != best[b]).any() else G
        assert a[b] == first_bad
        # emitted tokens are exactly the argmax continuation
        assert np.array_equal(out[b, :n[b]], best[b, :n[b]])
        assert n[b] == min(first_bad + 1, G)
    # ties resolve to the lowest index
    tie = np.zeros((1, 1, 5), np.float32)
    a, out, n, _ = oracle.accept_resample(None, None, np.array([[3]]), None, None, greedy=True, logits=tie)
    assert a[0] == 0 and out[0, 0] == 0


def test_acceptance_rate_closed_form():
    """P(accept) for x ~ q is sum_x min(p(x), q(x)); emitted count is a+1 after a rejection (Algorithm 1)."""
    rng = np.random.default_rng(3)
    V, n = 16, 200_000
    p = _rand_probs(rng, (), V, 1.5)
    q = _rand_probs(rng, (), V, 1.5)
    u = wl.uniform24(77, (3, n))
    x = np.array([oracle.sample_from_probs(q, u[0, i]) for i in range(n)])
    P = np.broadcast_to(p, (n, 1, V)); Q = np.broadcast_to(q, (n, 1, V))
    a, out, nout, p_tok = oracle.accept_resample(P, Q, x[:, None], u[1][:, None], u[2])
    alpha = float(np.minimum(p.astype(np.float64), q.astype(np.float64)).sum())
    rate = a.mean()
    assert abs(rate - alpha) < 4 * np.sqrt(alpha * (1 - alpha) / n)
    assert (nout == 1).all()                       # gamma = 1: either the draft or one new token
    assert (out[a == 1, 0] == x[a == 1]).all()
    assert np.array_equal(p_tok[:, 0], p[x])


@pytest.mark.parametrize("temp_mode", ["sampled"])
def test_output_distribution_equals_target_chi_square(temp_mode):
    """Losslessness (Section 3.1): over 10^6 seeded trials on a 16-token vocabulary the emitted token
    is distributed as the target p (chi-square p-value > 0.01)."""
    rng = np.random.default_rng(4)
    V, n = 16, 1_000_000
    p = _rand_probs(rng, (), V, 1.2)
    q = _rand_probs(rng, (), V, 1.2)
    u = wl.uniform24(2024, (3, n))
    # drafts x ~ q via the same fixed-point sampler, vectorised by hand for speed: compare with the
    # oracle's scalar routine on a prefix
    k = np.floor(q.astype(np.float64) * 2.0 ** 38).astype(np.uint64)
    cs = np.cumsum(k)
    m = (u[0].astype(np.float64) * 2 ** 24).astype(np.uint64)
    t = (m * np.uint64(int(cs[-1]))) >> np.uint64(24)
    x = np.searchsorted(cs, t, side="right")
    assert all(x[i] == oracle.sample_from_probs(q, u[0, i]) for i in range(2000))
    P = np.broadcast_to(p, (n, 1, V)); Q = np.broadcast_to(q, (n, 1, V))
    a, out, nout, _ = oracle.accept_resample(P, Q, x[:, None], u[1][:, None], u[2])
    emitted = out[:, 0]
    counts = np.bincount(emitted, minlength=V)
    chi = stats.chisquare(counts, p.astype(np.float64) / p.astype(np.float64).sum() * n)
    assert chi.pvalue > 0.01, chi
    # and it is NOT distributed as q (the test has power)
    assert stats.chisquare(counts, q.astype(np.float64) / q.astype(np.float64).sum() * n).pvalue < 1e-6


def _exact_law(p, q):
    """Exact output law of one draft-then-verify position: P(emit y) = q(y) min(1, p/q) + P(rej) res(y)."""
    p = [Fraction(float(v)) for v in p]
    q = [Fraction(float(v)) for v in q]
    acc = [min(pi, qi) for pi, qi in zip(p, q)]
    rej = 1 - sum(acc)
    res = [max(Fraction(0), pi - qi) for pi, qi in zip(p, q)]
    z = sum(res)
    return [a + (rej * r / z if z else 0) for a, r in zip(acc, res)], acc


def test_brute_force_enumeration_tiny():
    """Enumerate every draft sequence and a dense grid of uniforms on V <= 4, gamma <= 2: the frequency
    of each outcome agrees with the analytic law within the grid resolution, and the emitted-token law
    of the first position equals p."""
    rng = np.random.default_rng(5)
    for V, G in ((2, 1), (3, 2), (4, 2)):
        p = _rand_probs(rng, (G,), V)
        q = _rand_probs(rng, (G,), V)
        law0, acc0 = _exact_law(p[0], q[0])
        assert all(abs(float(l) - float(Fraction(float(pp)))) < 1e-6 for l, pp in zip(law0, p[0]))
        grid = 64
        us = ((np.arange(grid) + 0.5) / grid * 2 ** 24).astype(np.int64).astype(np.float32) * np.float32(2.0 ** -24)
        for drafts in itertools.product(range(V), repeat=G):
            cases = list(itertools.product(us, repeat=G))
            n = len(cases)
            d = np.tile(np.array(drafts), (n, 1))
            P = np.broadcast_to(p, (n, G, V)); Q = np.broadcast_to(q, (n, G, V))
            ua = np.array(cases, np.float32)
            a, out, nout, _ = oracle.accept_resample(P, Q, d, ua, np.full(n, 0.25, np.float32))
            # P(a >= j) = prod_{i<j} min(1, p_i(x_i)/q_i(x_i))
            want = 1.0
            for j in range(G):
                want *= min(1.0, float(p[j][drafts[j]]) / float(q[j][drafts[j]]))
                assert abs((a >= j + 1).mean() - want) <= (j + 1) / grid + 1e-9
            assert ((nout == a + 1) | (a == G)).all() and (nout[a == G] == G).all()
        # resampled token law: conditional on rejection at position 0 it is norm(max(0, p - q))
        res = np.maximum(p[0].astype(np.float64) - q[0].astype(np.float64), 0)
        if res.sum() > 0:
            ur = wl.uniform24(9, (4096,))
            toks = [oracle.accept_resample(p[None], q[None], np.array([[int(np.argmax(q[0] - p[0]))] + [0] * (G - 1)]),
                                           np.full((1, G), 1 - 2.0 ** -24, np.float32), np.array([u]))[1][0, 0]
                    for u in ur]
            freq = np.bincount(toks, minlength=V) / len(ur)
            assert np.abs(freq - res / res.sum()).max() < 4 * np.sqrt(0.25 / len(ur))


def test_fixed_point_draw_matches_float64_inverse_cdf():
    """The integer scan picks the same token as a serial float64 inverse CDF except when u falls within
    2^-24 of a CDF step (quantisation of the weights is below 2^-38 per entry)."""
    rng = np.random.default_rng(6)
    V = 1000
    disagreements = 0
    for trial in range(300):
        w = _rand_probs(rng, (), V, 2.0)
        u = wl.uniform24(100 + trial, (1,))[0]
        tok = oracle.fixed_point_draw(w, u)
        cdf = np.cumsum(w.astype(np.float64)) / w.astype(np.float64).sum()
        ref = int(np.searchsorted(cdf, float(u), side="right"))
        if tok != ref:
            disagreements += 1
            assert abs(tok - ref) == 1 and min(abs(cdf[min(tok, ref)] - float(u)), 1.0) < 2.0 ** -23
    assert disagreements <= 2
    # degenerate cases
    assert oracle.fixed_point_draw(np.zeros(5, np.float32), np.float32(0.5)) == -1
    one_hot = np.zeros(7, np.float32); one_hot[4] = 1.0
    for u in (0.0, 0.999):
        assert oracle.fixed_point_draw(one_hot, np.float32(np.floor(u * 2 ** 24) / 2 ** 24)) == 4


def test_zero_probability_edge_cases():
    """q(x) = 0 < p(x) accepts; p(x) = q(x) = 0 rejects and resamples; p <= q everywhere falls back to p."""
    p = np.array([[[0.5, 0.5, 0.0, 0.0]]], np.float32)
    q = np.array([[[0.0, 0.5, 0.0, 0.5]]], np.float32)
    u = np.array([[0.99]], np.float32) * 0 + np.float32(1 - 2.0 ** -24)
    a, out, n, _ = oracle.accept_resample(p, q, np.array([[0]]), u, np.array([0.3], np.float32))
    assert a[0] == 1
    a, out, n, _ = oracle.accept_resample(p, q, np.array([[2]]), u * 0, np.array([0.3], np.float32))
    assert a[0] == 0 and out[0, 0] == 0 and n[0] == 1       # residual mass only on token 0
    a, out, n, _ = oracle.accept_resample(p, q, np.array([[3]]), u * 0, np.array([0.3], np.float32))
    assert a[0] == 0 and out[0, 0] == 0                      # p(3) = 0 < anything*q(3)? u=0: 0 < 0 false
    same = np.array([[[0.25, 0.75]]], np.float32)
    assert oracle.specsample.residual_draw(same[0, 0], same[0, 0], np.float32(0.5)) == 1   # fallback to p


def test_bonus_row_and_bookkeeping_loop():
    """With gamma+1 target rows an extra token is drawn when every draft is accepted; replaying
    Algorithm 1's length bookkeeping drives every branch to exactly the maximum length."""
    rng = np.random.default_rng(8)
    N, G, V = 5, 3, 9
    p = _rand_probs(rng, (N, G + 1), V)
    toks = rng.integers(0, V, size=(N, G))
    a, out, n, _ = oracle.accept_resample(p, p[:, :G].copy(), toks, np.zeros((N, G), np.float32),
                                          np.full(N, 0.5, np.float32))
    assert (a == G).all() and (n == G + 1).all() and (out[:, G] >= 0).all()
    for b in range(N):
        assert out[b, G] == oracle.sample_from_probs(p[b, G], np.float32(0.5))
    # multi-step loop: validated lengths grow by n_out and stop at l
    l, L = 40, np.ones(N, int)
    private_len = np.zeros(N, int)
    step = 0
    while (L < l).any():
        q = _rand_probs(rng, (N, G), V)
        pp = _rand_probs(rng, (N, G), V)
        d = rng.integers(0, V, size=(N, G))
        a, out, n, _ = oracle.accept_resample(pp, q, d, wl.uniform24(step, (N, G)), wl.uniform24(step, (N,), 1))
        assert ((n == a + 1) | ((a == G) & (n == G))).all()
        new_len = oracle.commit_lengths(private_len, a, G)
        assert (new_len - private_len == np.minimum(a + 1, G)).all()
        private_len = new_len
        L = np.minimum(L + n, l)
        step += 1
    assert (L == l).all()


def test_softmax_temperature_closed_forms():
    """p = softmax(logits / T): logits (0, ln 2) give (1/3, 2/3) at T = 1, (1/5, 4/5) at T = 1/2 (the odds 2 are
    raised to the power 1/T) and (1, sqrt 2) / (1 + sqrt 2) at T = 2; a constant added to every logit changes
    nothing; rows are independent.  Dividing by T is what Section 3.1's sampling temperature means: T -> 0
    approaches the greedy choice, so a lower T must sharpen the distribution."""
    ln2 = np.log(2.0)
    z = np.array([0.0, ln2])
    for T, want in ((1.0, [1 / 3, 2 / 3]), (0.5, [1 / 5, 4 / 5]), (2.0, [1 / (1 + 2 ** 0.5), 2 ** 0.5 / (1 + 2 ** 0.5)])):
        got = oracle.softmax_temperature(z, T)
        assert got.dtype == np.float32
        assert np.allclose(got, want, rtol=0, atol=1e-7), (T, got)
        assert np.allclose(oracle.softmax_temperature(z + 123.456, T), want, rtol=0, atol=1e-7)
    # three logits, T = 1/3: odds (1 : 2 : 3) become (1 : 8 : 27)
    got = oracle.softmax_temperature(np.log([1.0, 2.0, 3.0]), 1.0 / 3.0)
    assert np.allclose(got, np.array([1, 8, 27]) / 36.0, atol=1e-7)
    # batched rows are treated independently, along the last axis
    rows = np.array([[0.0, ln2], [ln2, 0.0], [5.0, 5.0]])
    assert np.allclose(oracle.softmax_temperature(rows, 1.0), [[1 / 3, 2 / 3], [2 / 3, 1 / 3], [0.5, 0.5]], atol=1e-7)
    # large logits do not overflow
    assert np.allclose(oracle.softmax_temperature(np.array([1000.0, 1000.0 + ln2]), 1.0), [1 / 3, 2 / 3], atol=1e-7)
