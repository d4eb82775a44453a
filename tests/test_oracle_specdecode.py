"""Pins of the oracle for the rounds of Algorithm 1 (oracle/specdecode.py), CPU only."""
import numpy as np

import oracle
import workloads as wl


def _tiny():
    w = wl.get_workload("c1").scaled(n_layers=1, d_model=64, n_heads=2, head_dim=32, d_ff=128, vocab=97, S=9, seed=7)
    return w, wl.Weights(w.model, w.seed)


def _context(m, W, prefix):
    _, ks, vs = oracle.decode_rows(m, W, prefix)
    return [(ks[l], vs[l]) for l in range(m.n_layers)]


def test_draft_equal_to_target_accepts_everything_and_is_plain_sampling():
    """Special case that reduces to a textbook routine: when the draft model IS the target model, q = p at
    every position, u * q < p holds for every u < 1, all gamma drafts of every round are accepted, and the
    validated sequence is ordinary autoregressive sampling in which token t is drawn with u_draft[t]."""
    w, W = _tiny()
    m = w.model
    prefix = wl.prefix_tokens(w)
    ctx = _context(m, W, prefix)
    gamma, max_new, temp = 3, 11, 0.9
    u = wl.uniform24(5, (3, max_new + gamma))
    toks, rounds = oracle.speculative_rounds(m, W, ctx, w.S, m, W, ctx, w.S, first_tok=5, gamma=gamma,
                                             max_new=max_new, temperature=temp, u_draft=u[0], u_acc=u[1], u_res=u[2])
    assert all(r["accepted"] == gamma and len(r["emitted"]) == gamma for r in rounds)
    # independent loop: feed the whole sequence so far through the model, sample the next token
    seq, want = [5], []
    for t in range(max_new):
        logits, _, _ = oracle.decode_rows(m, W, np.array(seq), ctx_kv=lambda l: ctx[l], pos0=w.S)
        q = oracle.softmax_temperature(logits[-1], temp).astype(np.float32)
        tok = int(oracle.sample_from_probs(q, u[0][t]))
        want.append(tok)
        seq.append(tok)
    assert toks == want


def test_round_bookkeeping_with_a_different_draft_model():
    """Each round emits its accepted drafts plus, after a rejection, exactly one replacement; rounds start where
    the previous one ended; the result has max_new tokens; a rejected draft is never emitted in its place."""
    w, W = _tiny()
    m = w.model
    wd = w.scaled(seed=99)
    Wd = wl.Weights(wd.model, wd.seed)
    prefix = wl.prefix_tokens(w)
    ctx_t, ctx_d = _context(m, W, prefix), _context(m, Wd, prefix)
    gamma, max_new = 4, 13
    u = wl.uniform24(6, (3, max_new + gamma))
    toks, rounds = oracle.speculative_rounds(m, W, ctx_t, w.S, m, Wd, ctx_d, w.S, first_tok=11, gamma=gamma,
                                             max_new=max_new, temperature=1.0, u_draft=u[0], u_acc=u[1], u_res=u[2])
    assert len(toks) == max_new
    pos, flat = 0, []
    for r in rounds:
        assert r["start"] == pos
        a = r["accepted"]
        assert 0 <= a <= gamma
        assert len(r["emitted"]) == a + (1 if a < gamma else 0)
        assert r["emitted"][:a] == r["drafts"][:a]
        pos += len(r["emitted"])
        flat += r["emitted"]
    assert flat[:max_new] == toks
    assert any(r["accepted"] < gamma for r in rounds)      # the two models differ: some draft is rejected


# ---------------------------------------------------------------------------------------------------------
# Pins of the REJECTION path (rows kept after a rejection, the next pending token, the roll-back of both caches)
# against something other than the loop itself: a cache-less recomputation and the target's exact law.

class _SharpHead:
    """The same random-init weights with the LM head scaled up, so that next-token distributions are far from
    uniform and the draft model's differ clearly from the target's (inputs only: no arithmetic of the method)."""

    def __init__(self, inner, factor):
        self.inner, self.factor = inner, factor

    def tok_emb(self):
        return self.inner.tok_emb()

    def norm_final(self):
        return self.inner.norm_final()

    def lm_head(self):
        return self.inner.lm_head() * np.float32(self.factor)

    def layer(self, l):
        return self.inner.layer(l)


def _pair(vocab, seed_t, seed_d, factor, S=5):
    w = wl.get_workload("c1").scaled(n_layers=1, d_model=32, n_heads=2, head_dim=16, d_ff=64, vocab=vocab, S=S,
                                     seed=seed_t)
    m = w.model
    Wt = _SharpHead(wl.Weights(m, seed_t), factor)
    Wd = _SharpHead(wl.Weights(m, seed_d), factor)
    return w, m, Wt, Wd


def _no_cache_round(m, Wt, Wd, seq, gamma, temp, u_d, u_a, u_r, L):
    """One round of Algorithm 1 recomputed WITHOUT any cache: `seq` is everything validated so far (prompt, first
    token, emitted tokens; its last entry is the pending token); every model call is a plain causal forward of
    the whole sequence from position 0."""
    drafts, q_rows = [], []
    for j in range(gamma):
        logits, _, _ = oracle.decode_rows(m, Wd, np.array(seq + drafts))
        q = oracle.softmax_temperature(logits[-1], temp)
        drafts.append(int(oracle.sample_from_probs(q, u_d[L + j])))
        q_rows.append(q)
    logits, _, _ = oracle.decode_rows(m, Wt, np.array(seq + drafts[:gamma - 1]))
    p = oracle.softmax_temperature(logits[-gamma:], temp)
    a, toks, n_out, _ = oracle.accept_resample(p[None], np.stack(q_rows)[None], np.array([drafts]),
                                               np.asarray(u_a[L:L + gamma])[None], np.asarray([u_r[L]]))
    return drafts, int(a[0]), [int(t) for t in toks[0][:int(n_out[0])]]


def test_rounds_with_rejections_equal_a_cache_less_replay():
    """Every round of a run that rejects drafts, recomputed from the full token sequence with no KV cache at all,
    proposes the same drafts, accepts the same number and emits the same tokens.  Catches a wrong number of
    rows kept after a rejection (both caches), a wrong pending token and a wrong position offset: each of them
    changes what the next round's models see."""
    w, m, Wt, Wd = _pair(vocab=61, seed_t=21, seed_d=22, factor=10.0)
    prefix = [int(t) for t in wl.prefix_tokens(w)]
    ctx_t, ctx_d = _context(m, Wt, np.array(prefix)), _context(m, Wd, np.array(prefix))
    gamma, max_new, temp, first = 3, 17, 0.8, 7
    u = wl.uniform24(8, (3, max_new + gamma))
    toks, rounds = oracle.speculative_rounds(m, Wt, ctx_t, w.S, m, Wd, ctx_d, w.S, first_tok=first, gamma=gamma,
                                             max_new=max_new, temperature=temp, u_draft=u[0], u_acc=u[1], u_res=u[2])
    hist = [r["accepted"] for r in rounds]
    assert 0 in hist and any(0 < a < gamma for a in hist)           # rejections at the first row and later
    validated = []
    for r in rounds:
        assert r["start"] == len(validated)
        drafts, a, emitted = _no_cache_round(m, Wt, Wd, prefix + [first] + validated, gamma, temp, u[0], u[1], u[2],
                                             len(validated))
        assert (drafts, a, emitted) == (r["drafts"], r["accepted"], r["emitted"]), (r, drafts, a, emitted)
        validated += emitted
    assert validated[:max_new] == toks


def test_commit_lengths_equals_cached_rows_of_the_replay():
    """Algorithm 1's length bookkeeping in cache terms: after every round the rows a branch keeps in its cache are
    all its validated tokens except the newest one (the pending token, whose KV is computed by the next round).
    commit_lengths must give exactly that count when it is fed the accept counts of a replayed run; the count
    itself comes from the emitted token lists, not from a formula."""
    w, m, Wt, Wd = _pair(vocab=61, seed_t=21, seed_d=22, factor=10.0)
    prefix = wl.prefix_tokens(w)
    ctx_t, ctx_d = _context(m, Wt, prefix), _context(m, Wd, prefix)
    seen = set()
    for gamma, Wdraft in ((1, Wd), (2, Wd), (4, Wd), (3, Wt), (1, Wt)):      # draft = target: every draft accepted
        max_new = 15
        u = wl.uniform24(30 + gamma, (3, max_new + gamma))
        cd = ctx_t if Wdraft is Wt else ctx_d
        _, rounds = oracle.speculative_rounds(m, Wt, ctx_t, w.S, m, Wdraft, cd, w.S, first_tok=3, gamma=gamma,
                                              max_new=max_new, temperature=1.0, u_draft=u[0], u_acc=u[1], u_res=u[2])
        cached = np.zeros(1, np.int64)            # private rows in the cache; the first token is pending
        n_validated = 1
        for r in rounds:
            cached = oracle.commit_lengths(cached, np.array([r["accepted"]]), gamma)
            n_validated += len(r["emitted"])
            assert int(cached[0]) == n_validated - 1, (gamma, r)
            seen.add("all" if r["accepted"] == gamma else ("none" if r["accepted"] == 0 else "some"))
    assert seen == {"all", "none", "some"}


def test_tokens_of_rounds_with_rejections_follow_the_target_law():
    """Losslessness across rounds (Section 3.1; Algorithm 1): the first three validated tokens of a branch are
    distributed as three autoregressive draws from the TARGET model, whatever the draft model proposes.  With
    gamma = 2 the three tokens span two or three rounds, so the law depends on what is kept after a rejection.
    Exact law by enumeration on a 4-token vocabulary; chi-square over seeded trials; the test has power against
    the draft model's law."""
    V, gamma, temp, first, n = 4, 2, 1.0, 1, 6000
    w, m, Wt, Wd = _pair(vocab=V, seed_t=31, seed_d=32, factor=60.0, S=3)
    prefix = [int(t) for t in wl.prefix_tokens(w)]

    def law(W):
        out = np.zeros((V, V, V))
        def nxt(seq):
            logits, _, _ = oracle.decode_rows(m, W, np.array(seq))
            return oracle.softmax_temperature(logits[-1], temp).astype(np.float64)
        p1 = nxt(prefix + [first])
        for a in range(V):
            p2 = nxt(prefix + [first, a])
            for b in range(V):
                out[a, b] = p1[a] * p2[b] * nxt(prefix + [first, a, b])
        return out / out.sum()
    law_t, law_d = law(Wt), law(Wd)
    assert np.abs(law_t - law_d).sum() > 0.3                         # the two models differ clearly
    ctx_t, ctx_d = _context(m, Wt, np.array(prefix)), _context(m, Wd, np.array(prefix))
    counts = np.zeros((V, V, V))
    n_rounds = 0
    for trial in range(n):
        u = wl.uniform24(1000 + trial, (3, 3 + gamma))
        toks, rounds = oracle.speculative_rounds(m, Wt, ctx_t, w.S, m, Wd, ctx_d, w.S, first_tok=first, gamma=gamma,
                                                 max_new=3, temperature=temp, u_draft=u[0], u_acc=u[1], u_res=u[2])
        counts[tuple(toks)] += 1
        n_rounds += len(rounds)
    assert n_rounds > 1.5 * n                                        # most runs need a round after a rejection
    keep = law_t.ravel() * n >= 5                                    # pool the rare cells (chi-square validity)
    obs = np.append(counts.ravel()[keep], counts.ravel()[~keep].sum())
    exp = np.append(law_t.ravel()[keep], law_t.ravel()[~keep].sum()) * n
    exp_d = np.append(law_d.ravel()[keep], law_d.ravel()[~keep].sum()) * n
    if exp[-1] == 0:
        obs, exp, exp_d = obs[:-1], exp[:-1], exp_d[:-1]
    from scipy import stats
    assert stats.chisquare(obs, exp).pvalue > 0.01
    chi_d = float((((obs - exp_d) ** 2) / np.maximum(exp_d, 1e-9)).sum())
    assert chi_d > 10 * len(obs)                                     # ... and not as the draft model's
