"""Within-branch candidate trees (the k_config of Section 4.1; Section 2.2 "Tree Attention"; Appendix "Details
of Tree Attention") -- test oracle, plain numpy (test infrastructure; see the package docstring).

k_config = (k_1, ..., k_G): a draft phase proposes G positions; at position j every candidate of position
j - 1 gets k_j candidate continuations, sampled independently from the draft model's distribution given the
path that leads to them.  (2, 2, 1) is 2 + 4 + 4 = 10 draft tokens.  The target scores all candidates in one
pass with the tree mask of the appendix figure: a token attends to the context and to its ancestors only, i.e.
it sees exactly the sequence context + root-to-itself path, at the positions of that sequence.  So the plain
definition of the forward is: for every path, an ordinary causal forward of that sequence.

Verification walks the tree from the root.  The paper prints no rule for several candidates at a position (it
cites multi-candidate speculative decoding for one); the reading taken here is the multi-round rejection rule
for candidates drawn independently WITH replacement from q, which keeps the output law equal to the target's
(pinned by exact enumeration and chi-square in tests/test_oracle_spectree.py):
  at a node with target distribution p and draft distribution q, the first candidate x_1 is tested as in the
  single-candidate rule, accept iff fl32(u_1 q(x_1)) < p(x_1); after a rejection the target is replaced by the
  normalised residual p_2 = norm(max(0, p - q)), the next candidate is accepted with probability
  min(1, p_2(x_2) / q(x_2)), and so on; when every candidate of the node is rejected, one token is drawn from the
  last residual and the walk ends; an accepted candidate becomes the current node.
Residuals live in fixed point so that a parallel implementation reproduces every decision bit for bit:
  R_2[w] = trunc(max(0, fl32(p_w - q_w)) 2^38)                (the weights of the single-candidate draw)
  Z_i = sum_w R_i[w]                                           (integers: any order of summation)
  candidate i >= 2 is accepted iff  fl64(fl64(fl32(u_i q(x_i))) * fl64(Z_i)) < fl64(R_i[x_i])   (one float64 multiply)
  R_{i+1}[w] = max(0, R_i[w] - trunc(fl64(fl64(q_w) * fl64(Z_i))))
  the final draw is the fixed-point inverse CDF over R_{k+1} with u_res; if a residual sums to zero (p <= q
  everywhere after quantisation) the walk stops testing and the token is drawn from p itself.
With one candidate per position this is exactly accept_resample of specsample.py.
"""
import numpy as np

from .specsample import fixed_point_draw, sample_from_probs, _SCALE_BITS
from . import transformer


def tree_from_k_config(k_config):
    """Level-order node table of a candidate tree.  Node 0 is the root (the pending token: validated, not a
    draft); level j = 1..G holds k_1 * ... * k_j nodes; the children of a node are consecutive and come in the
    order of their parents.  Returns (parent [n], depth [n]) as int arrays, parent[0] = -1."""
    parent, depth = [-1], [0]
    level = [0]
    for j, k in enumerate(k_config, start=1):
        assert k >= 1
        nxt = []
        for node in level:
            for _ in range(k):
                parent.append(node)
                depth.append(j)
                nxt.append(len(parent) - 1)
        level = nxt
    return np.array(parent, np.int32), np.array(depth, np.int32)


def children_of(parent):
    kids = [[] for _ in parent]
    for i, p in enumerate(parent):
        if p >= 0:
            kids[p].append(i)
    return kids


def path_to(parent, node):
    out = []
    while node >= 0:
        out.append(node)
        node = int(parent[node])
    return out[::-1]


def tree_forward(model, weights, node_tok, parent, n_rows, ctx_kv, pos0):
    """Target logits at the first n_rows nodes of every branch's tree (the rows that are fed: every node whose
    children are to be verified, or all nodes when the leaves get a bonus distribution too).

    node_tok: int [N][>= n_rows], entry 0 the pending token; ctx_kv: layer -> list over branches of (K, V) of the
    branch's context; pos0[b] its length.  Every maximal root-to-node path among the fed nodes is run as an
    ordinary causal sequence against the branch's context; the logits of a node are those of its position in any
    path through it.  Returns float64 [N][n_rows][V]."""
    node_tok = np.asarray(node_tok)
    N = node_tok.shape[0]
    kids = children_of(parent[:n_rows])
    ends = [r for r in range(n_rows) if not kids[r]]               # fed nodes without fed children
    paths = [path_to(parent, r) for r in ends]
    seqs, owner = [], []
    for b in range(N):
        for path in paths:
            seqs.append(node_tok[b, path])
            owner.append(b)
    # all paths of one length go through the model together (a layer's weights are asked for once per group);
    # a full tree has a single length
    logits = [None] * len(seqs)
    for length in sorted({len(s) for s in seqs}):
        idx = [i for i, s in enumerate(seqs) if len(s) == length]
        lg, _, _ = transformer._forward([seqs[i] for i in idx], weights, model,
                                        lambda l, idx=idx: [ctx_kv(l)[owner[i]] for i in idx],
                                        [pos0[owner[i]] for i in idx], single=False)
        for k, i in enumerate(idx):
            logits[i] = lg[k]
    out = np.zeros((N, n_rows, logits[0].shape[-1]))
    i = 0
    for b in range(N):
        for path in paths:
            for t, node in enumerate(path):
                out[b, node] = logits[i][t]
            i += 1
    return out


def _fixed(w32):
    return np.floor(np.asarray(w32, np.float32).astype(np.float64) * 2.0 ** _SCALE_BITS).astype(np.uint64)


def _draw_fixed_weights(R, u):
    """Fixed-point inverse CDF over integer weights R (the scan of fixed_point_draw on already quantised weights)."""
    Z = int(R.sum(dtype=np.uint64))
    assert Z > 0
    m = int(np.float64(np.float32(u)) * 2.0 ** 24)
    t = (m * Z) >> 24
    return int(np.searchsorted(np.cumsum(R, dtype=np.uint64), np.uint64(t), side="right"))


def accept_resample_tree(p, q, node_tok, parent, u_acc, u_res, greedy=False, logits=None):
    """Walk of the candidate tree for every branch.

    parent: [n] level-order node table (tree_from_k_config).  p: float32 [N][n_rows][V], the target distribution
    AT node r (what follows the path to r), n_rows = number of nodes that have children (no bonus) or n (bonus:
    a token is also drawn after a fully accepted path); q: float32 [N][n_par][V], the draft distribution at every
    node that has children, from which its children were drawn; node_tok int [N][n] (entry 0 unused); u_acc
    float32 [N][n] (entry i tests node i; entry 0 unused); u_res float32 [N].  greedy: a candidate is accepted iff
    it equals the argmax of `logits` at its parent (lowest index on ties); the first such child in order wins;
    otherwise the argmax is emitted.
    Returns (accept_len [N] = depth reached, out_tok [N][G+1] padded with -1, n_out [N], path [N][G] accepted
    node ids padded with -1, p_tok [N][n] = p at the parent of node i evaluated at its token; entry 0 is 0)."""
    node_tok = np.asarray(node_tok)
    parent = np.asarray(parent)
    N, n = node_tok.shape[0], len(parent)
    kids = children_of(parent)
    depth = np.zeros(n, int)
    for i in range(1, n):
        depth[i] = depth[parent[i]] + 1
    G = int(depth.max())
    src = np.asarray(logits if greedy else p)
    n_rows = src.shape[1]
    n_par = sum(1 for k in kids if k)
    assert n_rows in (n_par, n)
    bonus = n_rows == n and n_par < n
    accept_len = np.zeros(N, np.int32)
    out_tok = np.full((N, G + 1), -1, np.int32)
    n_out = np.zeros(N, np.int32)
    path = np.full((N, max(G, 1)), -1, np.int32)
    p_tok = np.zeros((N, n), np.float32)
    for b in range(N):
        cur, a, new_tok = 0, 0, -1
        while kids[cur]:
            if greedy:
                best = int(np.argmax(src[b, cur]))
                hit = [c for c in kids[cur] if int(node_tok[b, c]) == best]
                if hit:
                    cur = hit[0]
                    out_tok[b, a] = best
                    path[b, a] = cur
                    a += 1
                    continue
                new_tok = best
                break
            P, Q = np.asarray(p[b, cur], np.float32), np.asarray(q[b, cur], np.float32)
            R = Z = None
            chosen = -1
            for i, c in enumerate(kids[cur]):
                x = int(node_tok[b, c])
                uq = np.float32(np.float32(u_acc[b, c]) * Q[x])
                if i == 0:
                    ok = bool(uq < P[x])
                else:
                    ok = bool(np.float64(uq) * np.float64(Z) < np.float64(R[x]))
                if ok:
                    chosen = c
                    break
                if i == 0:
                    R = _fixed(np.maximum(P - Q, np.float32(0.0)))
                else:
                    Qz = np.floor(Q.astype(np.float64) * np.float64(Z)).astype(np.uint64)
                    R = np.where(R > Qz, R - Qz, np.uint64(0)).astype(np.uint64)
                Z = int(R.sum(dtype=np.uint64))
                if Z == 0:
                    break
            if chosen >= 0:
                out_tok[b, a] = int(node_tok[b, chosen])
                path[b, a] = chosen
                cur = chosen
                a += 1
                continue
            new_tok = _draw_fixed_weights(R, u_res[b]) if Z > 0 else sample_from_probs(P, u_res[b])
            break
        else:
            if bonus:                                   # a leaf was reached: every position accepted
                new_tok = int(np.argmax(src[b, cur])) if greedy else sample_from_probs(p[b, cur], u_res[b])
        accept_len[b] = a
        if new_tok >= 0:
            out_tok[b, a] = new_tok
        n_out[b] = a + (1 if new_tok >= 0 else 0)
        if not greedy:
            for i in range(1, n):
                p_tok[b, i] = np.float32(p[b, parent[i], int(node_tok[b, i])])
    return accept_len, out_tok, n_out, path, p_tok


def commit_rows_tree(parent, path_b, accept_len_b, n_rows):
    """Rows of a branch that stay in its cache after the walk, in order: the root and the accepted nodes that
    were fed (Algorithm 1's bookkeeping: the validated tokens except the newest one)."""
    rows = [0] + [int(c) for c in path_b[:accept_len_b]]
    return [r for r in rows if r < n_rows]
