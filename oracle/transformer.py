"""Plain float64 decoder-only transformer (test infrastructure; see package docstring).

Architecture (the LLaMA family the paper evaluates, Section 4.1 "Models"): pre-norm RMSNorm, multi-head
attention with rotary position embedding (rotate-half pairing (i, i + dh/2), base theta), scale
1/sqrt(dh), causal mask, SwiGLU feed-forward, final RMSNorm, untied LM head, no biases.

The verify phase (Section 3.1; the verify call E of Algorithm 1) asks for the target model's
next-token distribution at each draft position of each branch, given that branch's context.  Branches
do not interact (Section 3: each generation runs in its own branch, independent of the others), so the oracle
simply runs an ordinary causal forward per branch over the new rows against that branch's context KV.
"""
import numpy as np

F64 = np.float64


def rms_norm(x, gain, eps):
    x = np.asarray(x, F64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(gain, F64)


def rope_rotate(x, pos, theta):
    """x: [T][H][dh]; pos: [T] absolute positions.  Rotates the pair (i, i + dh/2) by pos * theta^(-2i/dh)."""
    x = np.asarray(x, F64)
    dh = x.shape[-1]
    half = dh // 2
    inv_freq = F64(theta) ** (-np.arange(half, dtype=F64) * 2.0 / dh)
    ang = np.asarray(pos, F64)[:, None] * inv_freq[None, :]          # [T][half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def _silu(z):
    return z / (1.0 + np.exp(-z))


def layer_rows(model, w, x, ctx_k, ctx_v, pos0):
    """One decoder layer over T new rows.

    x: [T][d] residual stream; ctx_k / ctx_v: [H][C][dh] keys (already rotated) and values of the
    C context tokens; the new rows sit at absolute positions pos0 .. pos0+T-1 and attend to the whole
    context plus, causally, to each other.  Returns (x_out, k_new [H][T][dh], v_new [H][T][dh]).
    """
    T = x.shape[0]
    H, dh = model.n_heads, model.head_dim
    h = rms_norm(x, w["norm_attn"], model.rms_eps)
    q = (h @ np.asarray(w["wq"], F64).T).reshape(T, H, dh)
    k = (h @ np.asarray(w["wk"], F64).T).reshape(T, H, dh)
    v = (h @ np.asarray(w["wv"], F64).T).reshape(T, H, dh)
    pos = pos0 + np.arange(T)
    q = rope_rotate(q, pos, model.rope_theta)
    k = rope_rotate(k, pos, model.rope_theta)
    k_new = np.transpose(k, (1, 0, 2))
    v_new = np.transpose(v, (1, 0, 2))
    K = np.concatenate([np.asarray(ctx_k, F64), k_new], axis=1)     # [H][C+T][dh]
    V = np.concatenate([np.asarray(ctx_v, F64), v_new], axis=1)
    C = K.shape[1] - T
    attn = np.empty((T, H, dh), F64)
    for t in range(T):
        n_keys = C + t + 1                                            # causal: context + rows 0..t
        for hh in range(H):
            s = K[hh, :n_keys] @ q[t, hh] / np.sqrt(F64(dh))
            s = np.exp(s - s.max())
            attn[t, hh] = (s / s.sum()) @ V[hh, :n_keys]
    x = x + attn.reshape(T, H * dh) @ np.asarray(w["wo"], F64).T
    h = rms_norm(x, w["norm_ffn"], model.rms_eps)
    g = h @ np.asarray(w["wgate"], F64).T
    u = h @ np.asarray(w["wup"], F64).T
    x = x + (_silu(g) * u) @ np.asarray(w["wdown"], F64).T
    return x, k_new, v_new


def decode_rows(model, weights, tokens, ctx_kv=None, pos0=0):
    """Ordinary causal forward of one sequence of new tokens against an optional context.

    tokens: int[T].  ctx_kv: None (no context: a plain causal forward from position 0) or a callable
    layer -> (K [H][C][dh], V [H][C][dh]).  Returns (logits [T][V], [k_new per layer], [v_new per layer]).
    """
    return _forward([np.asarray(tokens)], weights, model,
                    (lambda l: [ctx_kv(l)]) if ctx_kv is not None else None, [pos0], single=True)


def verify_forward(model, weights, row_tok, ctx_kv, pos0):
    """The verify phase for all branches.

    row_tok: int[N][T] -- row 0 of a branch is its pending token (validated, KV not yet cached), rows
    1.. are its draft tokens; ctx_kv: callable layer -> list over branches of (K_b [H][C_b][dh],
    V_b [H][C_b][dh]) with C_b = shared + private context length of branch b; pos0[b] = C_b.
    Returns logits [N][T][V] (float64): logits[b][j] is the target's distribution for the token that
    follows row j, i.e. the one that verifies draft token j+1 of branch b.
    """
    row_tok = np.asarray(row_tok)
    logits, _, _ = _forward([row_tok[b] for b in range(row_tok.shape[0])], weights, model, ctx_kv,
                            list(pos0), single=False)
    return logits


def _forward(seqs, weights, model, ctx_kv, pos0, single):
    H, dh = model.n_heads, model.head_dim
    emb = np.asarray(weights.tok_emb(), F64)
    xs = [emb[s] for s in seqs]
    del emb
    ks, vs = [], []
    for l in range(model.n_layers):
        w = weights.layer(l)                      # generated / fetched once per layer, all branches use it
        ctx = ctx_kv(l) if ctx_kv is not None else [(np.zeros((H, 0, dh)), np.zeros((H, 0, dh)))] * len(seqs)
        kl, vl = [], []
        for b in range(len(seqs)):
            xs[b], kn, vn = layer_rows(model, w, xs[b], ctx[b][0], ctx[b][1], pos0[b])
            kl.append(kn)
            vl.append(vn)
        ks.append(kl)
        vs.append(vl)
    g = weights.norm_final()
    lm = np.asarray(weights.lm_head(), F64)
    logits = [rms_norm(x, g, model.rms_eps) @ lm.T for x in xs]
    if single:
        return logits[0], [k[0] for k in ks], [v[0] for v in vs]
    return np.stack(logits), ks, vs
