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
