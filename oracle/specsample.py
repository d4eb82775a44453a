"""Speculative-sampling accept / resample rule in plain numpy (test infrastructure; see package
docstring).

Section 3.1: draft token x_j is accepted with probability min(1, p_t(x_j | .) / p_d(x_j | .)), drafts
are checked left to right, the first rejection ends the check and the target model returns one new
token; Algorithm 1 (verification process) does the bookkeeping: the validated length grows by one per
accepted token and by one for the resampled token, and nothing is emitted beyond the k-th accepted
draft.  The paper attributes losslessness to Leviathan et al. but does not print the distribution of
the resampled token; the only distribution that makes the output law equal to the target's is
norm(max(0, p - q)), which is what is used here (and what the chi-square pin checks).

Readings fixed here, shared as a specification with the HIP library:
  * accept test in the product form, single float32 multiply, strict:  fl32(u * q(x)) < p(x).
    p = q > 0 accepts for every u in [0,1); q = 0 < p accepts; p = q = 0 rejects.
  * uniforms are inputs on the 2^-24 grid, u = m * 2^-24, one per (branch, draft position) plus one per
    branch for the resample / bonus draw, consumed by index.
  * draws use an order-independent fixed-point inverse CDF (fixed_point_draw) so that a parallel scan
    and a serial one give the same token.
  * greedy mode: accept iff the draft equals argmax of the logits (lowest index on ties), otherwise
    emit the argmax.
  * bonus row: if p has gamma+1 rows and every draft is accepted, one more token is drawn from row gamma.
"""
import numpy as np

_SCALE_BITS = 38


def softmax_temperature(logits, temperature):
    """p = softmax(logits / temperature) evaluated in float64, returned rounded to float32."""
    z = np.asarray(logits, np.float64) / np.float64(temperature)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)


def _mantissa24(u):
    m = np.float64(np.float32(u)) * 2.0 ** 24
    assert m == np.floor(m) and 0 <= m < 2 ** 24, "uniform must be m * 2^-24 with 0 <= m < 2^24"
    return int(m)


def fixed_point_draw(weights32, u):
    """Inverse-CDF draw from non-negative float32 weights with an integer (order-independent) scan.

    k_w = trunc(weights_w * 2^38) as an integer; Z = sum k_w; t = (m * Z) >> 24 with u = m * 2^-24;
    the token is the smallest v whose inclusive prefix sum exceeds t.  Returns -1 when Z = 0.
    """
    w = np.asarray(weights32, np.float32)
    k = np.floor(w.astype(np.float64) * 2.0 ** _SCALE_BITS).astype(np.uint64)
    Z = int(k.sum(dtype=np.uint64))
    if Z == 0:
        return -1
    t = (_mantissa24(u) * Z) >> 24
    csum = np.cumsum(k, dtype=np.uint64)
    return int(np.searchsorted(csum, np.uint64(t), side="right"))


def sample_from_probs(q32, u):
    """Draft-side draw x ~ q (Section 3.1: drafts are sampled autoregressively from p_d)."""
    tok = fixed_point_draw(q32, u)
    assert tok >= 0
    return tok


def residual_draw(p32, q32, u):
    """Token from norm(max(0, p - q)); the subtraction is a single float32 operation.  If the residual
    vanishes after quantisation (p <= q everywhere) the draw falls back to p itself."""
    p32 = np.asarray(p32, np.float32)
    q32 = np.asarray(q32, np.float32)
    r = np.maximum(p32 - q32, np.float32(0.0))
    tok = fixed_point_draw(r, u)
    if tok < 0:
        tok = fixed_point_draw(p32, u)
    assert tok >= 0
    return tok


def accept_resample(p, q, draft_tok, u_acc, u_res, greedy=False, logits=None):
    """Accept / reject / resample for every branch.

    p: float32 [N][Tp][V] target distributions, Tp = gamma or gamma+1 (bonus row); q: float32
    [N][gamma][V] draft distributions; draft_tok int [N][gamma]; u_acc float32 [N][gamma]; u_res
    float32 [N].  greedy=True uses `logits` [N][Tp][V] instead of p, q and the uniforms.
    Returns (accept_len [N], out_tok [N][gamma+1] padded with -1, n_out [N], p_tok [N][gamma]).
    """
    draft_tok = np.asarray(draft_tok)
    N, G = draft_tok.shape
    src = np.asarray(logits if greedy else p)
    Tp = src.shape[1]
    assert Tp in (G, G + 1)
    accept_len = np.zeros(N, np.int32)
    out_tok = np.full((N, G + 1), -1, np.int32)
    n_out = np.zeros(N, np.int32)
    p_tok = np.zeros((N, G), np.float32)
    for b in range(N):
        a = 0
        new_tok = -1
        for j in range(G):
            x = int(draft_tok[b, j])
            if greedy:
                best = int(np.argmax(src[b, j]))          # first maximum = lowest index on ties
                ok = (x == best)
            else:
                pj = np.float32(p[b, j, x])
                qj = np.float32(q[b, j, x])
                ok = bool(np.float32(np.float32(u_acc[b, j]) * qj) < pj)
            if ok:
                a += 1
                continue
            new_tok = best if greedy else residual_draw(p[b, j], q[b, j], u_res[b])
            break
        if a == G and Tp == G + 1:                         # bonus row: every draft accepted
            new_tok = int(np.argmax(src[b, G])) if greedy else sample_from_probs(p[b, G], u_res[b])
        accept_len[b] = a
        out_tok[b, :a] = draft_tok[b, :a]
        if new_tok >= 0:
            out_tok[b, a] = new_tok
            n_out[b] = a + 1
        else:
            n_out[b] = a
        if not greedy:                                     # diagnostic p(x_j) for every row, decided or not
            for j in range(G):
                p_tok[b, j] = np.float32(p[b, j, int(draft_tok[b, j])])
    return accept_len, out_tok, n_out, p_tok


def commit_lengths(private_len, accept_len, T):
    """Algorithm 1 bookkeeping in cache terms: rows 0..a (pending token + a accepted drafts) become
    context, capped at the T rows that were actually fed."""
    return np.asarray(private_len) + np.minimum(np.asarray(accept_len) + 1, T)
