"""Test oracle for the rounds of Algorithm 1 (paper Section 3.4), one branch at a time, serially.

Test infrastructure only (see oracle/__init__.py).  A branch repeats: the draft model proposes gamma tokens
autoregressively from the validated context; the target model scores them in one forward (Section 3.1);
accepted drafts extend the validated sequence, the first rejection adds the target's replacement token and
ends the round; the draft model continues from the validated sequence.  The scheduling of Section 3.3 (queue,
ready flags, who is verified when) decides WHEN a round runs, never what it produces: uniforms are consumed by
position (draft token j of a round that starts with L validated tokens uses u_draft[L + j], its accept test
u_acc[L + j], the round's replacement u_res[L]), so this serial loop is the plain definition of the result of
any schedule.
"""
import numpy as np

from .transformer import decode_rows
from .specsample import softmax_temperature, sample_from_probs, accept_resample


def _extend(ctx, new):
    """ctx, new: per-layer lists of (K, V) [H][C][dh]; returns their concatenation along C."""
    return [(np.concatenate([ck, nk], 1), np.concatenate([cv, nv], 1)) for (ck, cv), (nk, nv) in zip(ctx, new)]


def speculative_rounds(model_t, W_t, ctx_t, pos_t, model_d, W_d, ctx_d, pos_d, first_tok, gamma, max_new,
                       temperature, u_draft, u_acc, u_res):
    """One branch.  ctx_t / ctx_d: per-layer lists of (K, V) of the context already cached in the target /
    draft model (prefix + private), pos_t / pos_d their lengths.  Returns (tokens [max_new], rounds) where
    rounds is a list of dicts with the round's drafts, accept count, emitted tokens and decision margins."""
    out, rounds = [], []
    pending = int(first_tok)
    while len(out) < max_new:
        L = len(out)
        # drafting: gamma autoregressive steps of the draft model
        drafts, q_rows, new_d = [], [], None
        cur = pending
        for j in range(gamma):
            ctx_j = ctx_d if new_d is None else _extend(ctx_d, new_d)
            logits, kn, vn = decode_rows(model_d, W_d, np.array([cur]), ctx_kv=lambda l: ctx_j[l],
                                         pos0=pos_d + j)
            step = [(kn[l], vn[l]) for l in range(model_d.n_layers)]
            new_d = step if new_d is None else _extend(new_d, step)
            q = softmax_temperature(logits[0], temperature).astype(np.float32)   # the draft's q row is float32
            tok = sample_from_probs(q, u_draft[L + j])
            drafts.append(int(tok))
            q_rows.append(q)
            cur = int(tok)
        # verification: pending + drafts 1..gamma-1 through the target in one pass
        rows = np.array([pending] + drafts[:gamma - 1])
        logits, kn, vn = decode_rows(model_t, W_t, rows, ctx_kv=lambda l: ctx_t[l], pos0=pos_t)
        p = softmax_temperature(logits, temperature).astype(np.float32)
        q_arr = np.stack(q_rows)
        a, toks, n_out, _ = accept_resample(p[None], q_arr[None], np.array([drafts]), np.asarray(u_acc[L:L + gamma])[None],
                                            np.asarray([u_res[L]]))
        a, n_out = int(a[0]), int(n_out[0])
        emitted = [int(t) for t in toks[0][:n_out]]
        qt = np.array([q_arr[j, drafts[j]] for j in range(gamma)], np.float64)
        pt = np.array([p[j, drafts[j]] for j in range(gamma)])
        margin = np.abs(np.asarray(u_acc[L:L + gamma], np.float64) * qt - pt) / np.maximum(pt, 1e-300)
        rounds.append(dict(start=L, drafts=drafts, accepted=a, emitted=emitted, margin=margin[:min(a + 1, gamma)]))
        out += emitted
        keep = min(a + 1, gamma)                     # rows of this round whose KV both models keep
        ctx_t = _extend(ctx_t, [(kn[l][:, :keep], vn[l][:, :keep]) for l in range(model_t.n_layers)])
        ctx_d = _extend(ctx_d, [(k[:, :keep], v[:, :keep]) for k, v in new_d])
        pos_t += keep
        pos_d += keep
        pending = emitted[-1]
    return out[:max_new], rounds
