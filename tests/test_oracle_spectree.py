"""Pins of the oracle for within-branch candidate trees (oracle/spectree.py), CPU only: what Section 2.2 /
Section 4.1 (k_config) / the appendix on tree attention fix, and what the mathematics fixes where the paper is
silent (the multi-candidate rule must keep the output law equal to the target's, Section 3.1)."""
from fractions import Fraction

import numpy as np
from scipy import stats

import oracle
import workloads as wl


def _rand_probs(rng, shape, V, sharp=1.0):
    z = rng.standard_normal(shape + (V,)) * sharp
    e = np.exp(z - z.max(-1, keepdims=True))
    return (e / e.sum(-1, keepdims=True)).astype(np.float32)


def _draw_many(q, u):
    """x ~ q for a vector of uniforms by the fixed-point sampler, vectorised (checked against the scalar one)."""
    k = np.floor(q.astype(np.float64) * 2.0 ** 38).astype(np.uint64)
    cs = np.cumsum(k)
    m = (u.astype(np.float64) * 2 ** 24).astype(np.uint64)
    t = (m * np.uint64(int(cs[-1]))) >> np.uint64(24)
    x = np.searchsorted(cs, t, side="right")
    assert all(x[i] == oracle.sample_from_probs(q, u[i]) for i in range(50))
    return x


def test_k_config_tables():
    """(2, 2, 1): 2 + 4 + 4 = 10 draft tokens in three positions (appendix on tree attention); children of a
    node are consecutive; (1, 1, 1) is a chain."""
    parent, depth = oracle.tree_from_k_config((2, 2, 1))
    assert len(parent) == 11 and list(depth) == [0, 1, 1, 2, 2, 2, 2, 3, 3, 3, 3]
    assert list(parent) == [-1, 0, 0, 1, 1, 2, 2, 3, 4, 5, 6]
    parent, depth = oracle.tree_from_k_config((4, 2, 1))
    assert len(parent) == 1 + 4 + 8 + 8 and (np.bincount(depth) == [1, 4, 8, 8]).all()
    assert oracle.path_to(parent, 20) == [0, 4, 12, 20]
    parent, _ = oracle.tree_from_k_config((1, 1, 1, 1))
    assert list(parent) == [-1, 0, 1, 2, 3]


def test_one_candidate_per_position_is_the_chain_rule():
    """k_config of all ones reduces to the single-candidate rule exactly: same accept counts, tokens and p(x),
    with and without the bonus row, sampled and greedy."""
    rng = np.random.default_rng(11)
    N, G, V = 40, 4, 23
    parent, _ = oracle.tree_from_k_config((1,) * G)
    for bonus in (False, True):
        Tp = G + int(bonus)
        p = _rand_probs(rng, (N, Tp), V, 1.5)
        noise = rng.standard_normal((N, G, V)) * 0.7
        lq = np.log(p[:, :G].astype(np.float64)) + noise
        q = (np.exp(lq) / np.exp(lq).sum(-1, keepdims=True)).astype(np.float32)
        u = wl.uniform24(3 + bonus, (2, N, G))
        drafts = wl.draw_tokens(q, u[0])
        u_res = wl.uniform24(5, (N,))
        want = oracle.accept_resample(p, q, drafts, u[1], u_res)
        node_tok = np.concatenate([np.zeros((N, 1), np.int32), drafts], 1)
        u_acc = np.concatenate([np.zeros((N, 1), np.float32), u[1]], 1)
        a, out, n, path, p_tok = oracle.accept_resample_tree(p, q, node_tok, parent, u_acc, u_res)
        assert np.array_equal(a, want[0]) and np.array_equal(out, want[1]) and np.array_equal(n, want[2])
        assert np.array_equal(p_tok[:, 1:], want[3])
        for b in range(N):
            assert list(path[b, :a[b]]) == list(range(1, a[b] + 1))
        assert 0 < want[0].sum() < N * G
        logits = rng.standard_normal((N, Tp, V)).astype(np.float32)
        best = logits.argmax(-1)
        gd = best[:, :G].copy()
        gd[rng.random((N, G)) < 0.3] = 0
        wg = oracle.accept_resample(None, None, gd, None, None, greedy=True, logits=logits)
        tg = oracle.accept_resample_tree(None, None, np.concatenate([np.zeros((N, 1), np.int32), gd], 1), parent, None,
                                         None, greedy=True, logits=logits)
        assert np.array_equal(tg[0], wg[0]) and np.array_equal(tg[1], wg[1]) and np.array_equal(tg[2], wg[2])


def _exact_round_probs(p, q, xs):
    """Acceptance probability of each candidate in turn, given that those before it were rejected, in exact
    rational arithmetic: min(1, p_i(x_i) / q(x_i)) with p_1 = p and p_{i+1} = norm(max(0, p_i - q))."""
    pi = [Fraction(float(v)) for v in p]
    qq = [Fraction(float(v)) for v in q]
    out = []
    for x in xs:
        out.append(min(Fraction(1), pi[x] / qq[x]) if qq[x] else Fraction(1 if pi[x] > 0 else 0))
        res = [max(Fraction(0), a - b) for a, b in zip(pi, qq)]
        z = sum(res)
        if z == 0:
            break
        pi = [r / z for r in res]
    return out, pi


def test_acceptance_probabilities_of_later_candidates_exact():
    """For fixed candidates (x_1, x_2, x_3) at one node, sweeping the uniform of candidate i over a fine grid
    (with the earlier candidates forced to be rejected) accepts it on exactly the fraction min(1, p_i(x_i) /
    q(x_i)) of the grid, p_i being the i-th normalised residual in exact arithmetic; and after k rejections the
    emitted token follows the last residual."""
    rng = np.random.default_rng(12)
    V, k = 5, 3
    parent, _ = oracle.tree_from_k_config((k,))
    grid = 4096
    us = (np.arange(grid, dtype=np.int64) * (2 ** 24 // grid) + 1).astype(np.float32) * np.float32(2.0 ** -24)
    checked = 0
    for trial in range(6):
        p = _rand_probs(rng, (), V, 1.3)
        q = _rand_probs(rng, (), V, 1.3)
        for xs in ((0, 1, 2), (3, 3, 4), (2, 0, 2), (4, 4, 4)):
            want, last = _exact_round_probs(p, q, xs)
            for i in range(len(want)):
                if any(want[j] == 1 for j in range(i)):
                    break                                   # an earlier candidate cannot be rejected
                u_acc = np.zeros((grid, k + 1), np.float32)
                u_acc[:, 1:1 + i] = np.float32(1 - 2.0 ** -24)       # earlier candidates: rejected (u q >= p_j)
                for j in range(i):
                    assert want[j] < 1 - 1e-6
                u_acc[:, 1 + i] = us
                tok = np.tile(np.array([0] + list(xs), np.int32), (grid, 1))
                a, out, n, path, _ = oracle.accept_resample_tree(np.tile(p, (grid, 1, 1)), np.tile(q, (grid, 1, 1)), tok,
                                                                parent, u_acc, np.full(grid, 0.5, np.float32))
                got = np.mean(path[:, 0] == 1 + i)
                assert abs(got - float(want[i])) <= 2.0 / grid, (trial, xs, i, got, float(want[i]))
                checked += 1
        # all rejected: the replacement token follows the k-th residual
        xs = tuple(int(v) for v in np.argsort(q - p)[-k:])              # tokens with q well above p
        want, last = _exact_round_probs(p, q, xs)
        if all(w < 0.999 for w in want) and len(want) == k:
            n = 20000
            ur = wl.uniform24(40 + trial, (n,))
            tok = np.tile(np.array([0] + list(xs), np.int32), (n, 1))
            a, out, _, _, _ = oracle.accept_resample_tree(np.tile(p, (n, 1, 1)), np.tile(q, (n, 1, 1)), tok, parent,
                                                          np.full((n, k + 1), 1 - 2.0 ** -24, np.float32), ur)
            assert (a == 0).all()
            freq = np.bincount(out[:, 0], minlength=V) / n
            assert np.abs(freq - np.array([float(v) for v in last])).max() < 4 * np.sqrt(0.25 / n)
    assert checked >= 30


def test_output_law_with_several_candidates_is_the_target_chi_square():
    """Losslessness with k candidates per position (Section 3.1's guarantee carried to Section 2.2's trees): the
    first emitted token is distributed as the target p at the root whatever q is, for k = 2, 3, 4; the test has
    power against q and against the single-candidate rule applied to the best of k."""
    rng = np.random.default_rng(13)
    for k, V, n in ((2, 16, 200_000), (3, 8, 120_000), (4, 6, 80_000)):
        p = _rand_probs(rng, (), V, 1.2)
        q = _rand_probs(rng, (), V, 1.2)
        parent, _ = oracle.tree_from_k_config((k,))
        u = wl.uniform24(100 + k, (2 * k + 1, n))
        tok = np.zeros((n, k + 1), np.int32)
        u_acc = np.zeros((n, k + 1), np.float32)
        for i in range(k):
            tok[:, 1 + i] = _draw_many(q, u[i])
            u_acc[:, 1 + i] = u[k + i]
        a, out, nout, _, _ = oracle.accept_resample_tree(np.broadcast_to(p, (n, 1, V)), np.broadcast_to(q, (n, 1, V)),
                                                         tok, parent, u_acc, u[2 * k])
        assert (nout == 1).all()
        counts = np.bincount(out[:, 0], minlength=V)
        p64 = p.astype(np.float64) / p.astype(np.float64).sum()
        assert stats.chisquare(counts, p64 * n).pvalue > 0.01, (k, counts, p64 * n)
        q64 = q.astype(np.float64) / q.astype(np.float64).sum()
        assert stats.chisquare(counts, q64 * n).pvalue < 1e-6
        # more candidates are accepted more often than one: P(a = 1) exceeds sum min(p, q)
        assert a.mean() > np.minimum(p64, q64).sum() + 0.02


def test_two_level_tree_joint_law():
    """k_config (2, 2): the first token follows the root's target distribution; given that it was accepted, the
    second emitted token follows the target distribution AT that token (each node carries its own p and q)."""
    rng = np.random.default_rng(14)
    V, n = 6, 150_000
    parent, depth = oracle.tree_from_k_config((2, 2))
    P0, Q0 = _rand_probs(rng, (), V, 1.0), _rand_probs(rng, (), V, 1.0)
    P1, Q1 = _rand_probs(rng, (V,), V, 1.0), _rand_probs(rng, (V,), V, 1.0)      # by first token
    u = wl.uniform24(200, (13, n))
    tok = np.zeros((n, 7), np.int32)
    tok[:, 1], tok[:, 2] = _draw_many(Q0, u[0]), _draw_many(Q0, u[1])
    for c, (par, ui) in enumerate(((1, 2), (1, 3), (2, 4), (2, 5)), start=3):
        for x in range(V):
            sel = tok[:, par] == x
            if sel.any():
                tok[sel, c] = _draw_many(Q1[x], np.concatenate([u[ui][sel], u[ui][:50]]))[:sel.sum()]
    p = np.zeros((n, 3, V), np.float32)
    q = np.zeros((n, 3, V), np.float32)
    p[:, 0], q[:, 0] = P0, Q0
    for node in (1, 2):
        p[:, node], q[:, node] = P1[tok[:, node]], Q1[tok[:, node]]
    u_acc = np.zeros((n, 7), np.float32)
    for i in range(1, 7):
        u_acc[:, i] = u[5 + i]
    a, out, nout, path, _ = oracle.accept_resample_tree(p, q, tok, parent, u_acc, u[12])
    assert ((nout == a + 1) | (a == 2)).all() and (nout[a == 2] == 2).all()
    c1 = np.bincount(out[:, 0], minlength=V)
    assert stats.chisquare(c1, P0.astype(np.float64) / P0.astype(np.float64).sum() * n).pvalue > 0.01
    got, exp = [], []
    for x in range(V):
        sel = (a >= 1) & (out[:, 0] == x)
        got.append(np.bincount(out[sel, 1], minlength=V))
        exp.append(P1[x].astype(np.float64) / P1[x].astype(np.float64).sum() * sel.sum())
    got, exp = np.concatenate(got), np.concatenate(exp)
    assert (exp > 5).all()
    chi = ((got - exp) ** 2 / exp).sum()
    assert stats.chi2.sf(chi, len(got) - V) > 0.01
    # the accepted node is a child of the previous one
    for b in range(0, n, 997):
        prev = 0
        for d in range(a[b]):
            assert parent[path[b, d]] == prev and out[b, d] == tok[b, path[b, d]]
            prev = path[b, d]


def test_tree_forward_is_a_plain_causal_forward_per_path():
    """Tree attention (appendix): a token sees the context and its ancestors only, so its logits are those of
    the last position of an ordinary causal forward over prompt + path, computed here from the TOKENS with no
    cache at all; on a chain the tree forward is the verify forward."""
    w = wl.get_workload("c1").scaled(n_layers=2, d_model=64, n_heads=2, head_dim=32, d_ff=128, vocab=97, S=9, N=2, seed=17)
    m = w.model
    W = wl.Weights(m, w.seed)
    prefix = wl.prefix_tokens(w)
    _, ks, vs = oracle.decode_rows(m, W, prefix)
    ctx = lambda l: [(ks[l], vs[l])] * w.N
    rng = np.random.default_rng(2)
    parent, depth = oracle.tree_from_k_config((2, 2, 1))
    n = len(parent)
    tok = rng.integers(0, m.vocab, (w.N, n)).astype(np.int32)
    for n_rows in (7, n):                                       # without and with the leaves' rows
        got = oracle.tree_forward(m, W, tok, parent, n_rows, ctx, [w.S] * w.N)
        for b in range(w.N):
            for r in range(n_rows):
                seq = np.concatenate([prefix, tok[b, oracle.path_to(parent, r)]])
                want, _, _ = oracle.decode_rows(m, W, seq)
                assert np.abs(got[b, r] - want[-1]).max() < 1e-9
        # siblings differ: the mask is not the chain's
        assert np.abs(got[0, 3] - got[0, 5]).max() > 1e-6
    chain, _ = oracle.tree_from_k_config((1, 1, 1))
    a = oracle.tree_forward(m, W, tok[:, :4], chain, 3, ctx, [w.S] * w.N)
    b = oracle.verify_forward(m, W, tok[:, :3], ctx, [w.S] * w.N)
    assert np.abs(a - b).max() < 1e-12


def test_committed_rows_of_a_walk():
    """Rows that stay in the cache: the root and the accepted nodes that were fed; on a chain their number is the
    chain rule's min(a + 1, T)."""
    parent, _ = oracle.tree_from_k_config((2, 2, 1))
    assert oracle.commit_rows_tree(parent, [2, 6, 10], 3, 7) == [0, 2, 6]          # leaf 10 was not fed
    assert oracle.commit_rows_tree(parent, [2, 6, 10], 3, 11) == [0, 2, 6, 10]     # bonus rows: it was
    assert oracle.commit_rows_tree(parent, [1, -1, -1], 1, 7) == [0, 1]
    assert oracle.commit_rows_tree(parent, [-1, -1, -1], 0, 7) == [0]
    chain, _ = oracle.tree_from_k_config((1, 1, 1, 1))
    for a in range(5):
        for T in (4, 5):
            rows = oracle.commit_rows_tree(chain, list(range(1, 5)), a, T)
            assert len(rows) == int(oracle.commit_lengths(0, a, T))
