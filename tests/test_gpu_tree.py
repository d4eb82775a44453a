"""GPU parity of within-branch candidate trees (k_config; Section 2.2 "Tree Attention", Section 4.1, appendix on
tree attention) through the C ABI: the tree-walk accept / resample against the oracle bit for bit, the tree-masked
forward against a plain causal forward per path, and the K/V kept after a walk against a recomputation."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads import gen
from workloads.device import UploadingWeights, make_context, to_device, f32, i32
from harness import CachedWeights, check_logits
import paper_2406_18200_amd as sv
from paper_2406_18200_amd.binding import tree_sizes

pytestmark = pytest.mark.gpu


def _probs(rng, shape, V, sharp):
    z = rng.standard_normal(shape + (V,)) * sharp
    e = np.exp(z - z.max(-1, keepdims=True))
    return (e / e.sum(-1, keepdims=True)).astype(np.float32)


def _tree_case(seed, N, k_config, bonus, V, noise=0.7):
    """p at every fed node, q = a perturbed copy at every node with children, children drawn iid from q."""
    rng = np.random.default_rng(seed)
    parent, depth = oracle.tree_from_k_config(k_config)
    n, n_par = tree_sizes(k_config)
    Tp = n if bonus else n_par
    p = _probs(rng, (N, Tp), V, 2.0)
    lq = np.log(p[:, :n_par].astype(np.float64) + 1e-30) + rng.standard_normal((N, n_par, V)) * noise
    e = np.exp(lq - lq.max(-1, keepdims=True))
    q = (e / e.sum(-1, keepdims=True)).astype(np.float32)
    u = wl.uniform24(seed, (2, N, n))
    tok = np.zeros((N, n), np.int32)
    for i in range(1, n):
        tok[:, i] = wl.draw_tokens(q[:, parent[i]], u[0][:, i])
    return parent, p, q, tok, u[1], wl.uniform24(seed + 1, (N,))


@pytest.mark.parametrize("N,k_config,bonus,V", [(7, (2, 2, 1), False, 32000), (5, (4, 2, 1), True, 32000),
                                                (16, (2, 2, 1), True, 1000), (9, (3,), False, 517),
                                                (4, (1, 1, 1, 1), False, 2000), (6, (2, 1, 3), False, 64),
                                                (3, (5, 2), True, 4096), (2, (1,), True, 1)])
def test_tree_walk_probs_mode_is_bit_exact(N, k_config, bonus, V):
    print(f"case N={N} k_config={k_config} bonus={bonus} V={V}", flush=True)
    parent, p, q, tok, u_acc, u_res = _tree_case(300 + N + V, N, k_config, bonus, V)
    want = oracle.accept_resample_tree(p, q, tok, parent, u_acc, u_res)
    for static in (False, True):
        got = sv.accept_resample(f32(p), f32(q), i32(tok[:, 1:]), f32(u_acc[:, 1:]), f32(u_res), kind="probs",
                                 k_config=k_config, static_scratch=static)
        torch.cuda.synchronize()
        a, out, n_out, p_tok, path = [g.cpu().numpy() for g in got]
        assert np.array_equal(a, want[0]) and np.array_equal(out, want[1]) and np.array_equal(n_out, want[2])
        assert np.array_equal(path, want[3][:, :len(k_config)])
        assert np.array_equal(p_tok, want[4][:, 1:])
    if V >= 1000 and max(k_config) > 1:
        # the cases exercise the later rounds: some accepted node is not the first child of its parent
        kids = oracle.children_of(parent)
        assert any(want[3][b, d] >= 0 and want[3][b, d] != kids[parent[want[3][b, d]]][0]
                   for b in range(N) for d in range(len(k_config)))


def test_tree_walk_greedy_and_logits_modes():
    N, k_config, V, temp = 8, (2, 2, 1), 32000, 0.8
    rng = np.random.default_rng(5)
    parent, _ = oracle.tree_from_k_config(k_config)
    n, n_par = tree_sizes(k_config)
    logits = (rng.standard_normal((N, n, V)) * 2.0).astype(np.float32)
    p = oracle.softmax_temperature(logits, temp)
    q = oracle.softmax_temperature(logits[:, :n_par] + (rng.standard_normal((N, n_par, V)) * 0.6).astype(np.float32), temp)
    u = wl.uniform24(77, (2, N, n))
    tok = np.zeros((N, n), np.int32)
    for i in range(1, n):
        tok[:, i] = wl.draw_tokens(q[:, parent[i]], u[0][:, i])
    u_res = wl.uniform24(78, (N,))
    want = oracle.accept_resample_tree(p, q, tok, parent, u[1], u_res)
    got = [g.cpu().numpy() for g in sv.accept_resample(f32(logits), f32(q), i32(tok[:, 1:]), f32(u[1][:, 1:]), f32(u_res),
                                                        kind="logits", temperature=temp, k_config=k_config)]
    assert np.abs(got[3] - want[4][:, 1:]).max() <= 1e-5 * want[4].max()
    same = np.array_equal(got[0], want[0]) and np.array_equal(got[4], want[3][:, :3])
    assert same, (got[0], want[0])                           # (no near-ties for this seed)
    assert (got[1] == want[1]).mean() > 0.9
    # greedy: a candidate is accepted iff it is the argmax at its parent
    best = logits.argmax(-1)
    gtok = tok.copy()
    for b in range(N):
        if b % 2 == 0:
            gtok[b, 2] = best[b, 0]                            # second child of the root is the argmax
            gtok[b, 5 + b % 2] = best[b, 2]
    wg = oracle.accept_resample_tree(None, None, gtok, parent, None, None, greedy=True, logits=logits)
    gg = [g.cpu().numpy() for g in sv.accept_resample(f32(logits), None, i32(gtok[:, 1:]), None, None, kind="logits",
                                                       greedy=True, k_config=k_config)]
    assert np.array_equal(gg[0], wg[0]) and np.array_equal(gg[1], wg[1]) and np.array_equal(gg[2], wg[2])
    assert np.array_equal(gg[4], wg[3][:, :3]) and wg[0].max() >= 2


@pytest.mark.parametrize("N,k_config,bonus,S,R", [(3, (2, 2, 1), False, 100, 9), (16, (2, 2, 1), False, 257, 40),
                                                  (5, (4, 2, 1), False, 70, 0), (2, (2, 2, 1), True, 64, 5),
                                                  (4, (3, 2), True, 0, 33), (6, (1, 1, 1, 1), False, 90, 3)])
def test_tree_step_small_bf16(N, k_config, bonus, S, R):
    """Whole verify step over candidate trees on a small bf16 model with synthetic KV: logits of every fed node
    against an ordinary causal forward of its path; the walk against the oracle's walk on the library's own
    logits; the rows kept in the cache against the oracle's list; then a second, plain step whose logits depend
    on the K/V the first one kept (moved to the front of the in-flight region in every layer)."""
    G = len(k_config)
    w = wl.get_workload("c6" if S == 0 else "c3").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704,
                                                        vocab=2000, N=N, gamma=G, S=S, R=R, R_min=-1, seed=577 + N)
    m, dev = w.model, "cuda:0"
    parent, depth = oracle.tree_from_k_config(k_config)
    n, n_par = tree_sizes(k_config)
    T = n if bonus else n_par
    up = UploadingWeights(m, w.seed, dev, reuse_buffers=False)
    W = CachedWeights(up)
    rng = np.random.default_rng(w.seed)
    q = _probs(rng, (N, n_par), m.vocab, 1.0)
    u = wl.uniform24(w.seed + 3, (2, N, n))
    tok = np.zeros((N, n), np.int32)
    tok[:, 0] = gen.pending_tokens(w)
    for i in range(1, n):
        tok[:, i] = wl.draw_tokens(q[:, parent[i]], u[0][:, i])
    u_res = wl.uniform24(w.seed + 4, (N,))
    kv = [wl.synthetic_kv(w, l) for l in range(m.n_layers)]

    def ctx(l):
        k_s, v_s, k_p, v_p = kv[l]
        return [(np.concatenate([k_s, k_p[b]], 1), np.concatenate([v_s, v_p[b]], 1)) for b in range(N)]
    ref = oracle.tree_forward(m, W, tok, parent, T, ctx, [S + R] * N)
    # library
    c = make_context(m, up.upload_all(), max_branches=N, max_rows_per_branch=T, max_shared=max(S, 1), max_private=R + G + 2,
                     device=dev)
    for l, (k_s, v_s, k_p, v_p) in enumerate(kv):
        c.kv_load(l, *(to_device(a, m, dev) if a.size else None for a in (k_s, v_s, k_p, v_p)))
    plen = torch.full((N,), R, dtype=torch.int32, device=dev)
    logits = torch.empty((N, T, m.vocab), dtype=torch.float32, device=dev)
    acc = dict(q=f32(q), draft_tok=i32(tok[:, 1:]), u_acc=f32(u[1][:, 1:]), u_res=f32(u_res), temperature=w.temperature)
    outs = c.step(i32(tok[:, :T]), S, plen, logits_out=logits, accept=acc, k_config=k_config)
    torch.cuda.synchronize()
    assert c.status() == 0
    got = logits.cpu().numpy()
    worst, err = check_logits(got, ref, m.dtype)
    print(f"tree logits: max abs err {err:.3e}, worst err/bound {worst:.3f}", flush=True)
    assert worst <= 1.0
    # the chain mask would fail this: siblings see different paths
    a, out, n_out, p_tok, path = [o.cpu().numpy() for o in outs]
    p_own = oracle.softmax_temperature(got, w.temperature)
    own = oracle.accept_resample_tree(p_own, q, tok, parent, u[1], u_res)
    margin_ok = np.array_equal(a, own[0]) and np.array_equal(path, own[3][:, :G])
    assert margin_ok, (a, own[0])
    assert np.allclose(p_tok, own[4][:, 1:], rtol=1e-5, atol=1e-12)
    assert (out == own[1]).mean() > 0.9 and np.array_equal(n_out, own[2])
    rows = [oracle.commit_rows_tree(parent, path[b], int(a[b]), T) for b in range(N)]
    assert np.array_equal(plen.cpu().numpy(), [R + len(r) for r in rows])
    # second step: a plain chain of new tokens per branch against context + kept rows, recomputed by the oracle
    kept_kv = []
    for b in range(N):
        _, kn, vn = oracle.decode_rows(m, W, tok[b, rows[b]], ctx_kv=lambda l, b=b: ctx(l)[b], pos0=S + R)
        kept_kv.append((kn, vn))
    T2 = 3
    rows2 = rng.integers(0, m.vocab, (N, T2)).astype(np.int32)

    def ctx2(l):
        base = ctx(l)
        return [(np.concatenate([base[b][0], kept_kv[b][0][l]], 1), np.concatenate([base[b][1], kept_kv[b][1][l]], 1))
                for b in range(N)]
    ref2 = oracle.verify_forward(m, W, rows2, ctx2, [S + R + len(r) for r in rows])
    logits2 = torch.empty((N, T2, m.vocab), dtype=torch.float32, device=dev)
    c.step(i32(rows2), S, plen, logits_out=logits2)
    torch.cuda.synchronize()
    assert c.status() == 0
    worst2, err2 = check_logits(logits2.cpu().numpy(), ref2, m.dtype)
    print(f"step after the walk: max abs err {err2:.3e}, worst err/bound {worst2:.3f}; kept rows {rows}", flush=True)
    assert worst2 <= 1.0
    if max(k_config) > 1:
        assert any(r != list(range(len(r))) for r in rows) or N < 3        # some kept path is not the first rows
    c.close()


def test_tree_arguments_are_validated():
    z = torch.zeros((1, 7, 8), device="cuda")
    d = torch.zeros((1, 10), dtype=torch.int32, device="cuda")
    u = torch.zeros((1, 10), device="cuda")
    with pytest.raises(sv.SeedError) as e:       # 6 target rows fit neither 7 (nodes with children) nor 11
        sv.accept_resample(z[:, :6].contiguous(), z, d, u, torch.zeros(1, device="cuda"), kind="probs", k_config=(2, 2, 1))
    assert e.value.code == -2
    with pytest.raises(sv.SeedError) as e:       # 1 + 9 + 81 nodes: more than 64
        sv.accept_resample(z, z, torch.zeros((1, 90), dtype=torch.int32, device="cuda"), torch.zeros((1, 90), device="cuda"),
                           torch.zeros(1, device="cuda"), kind="probs", k_config=(9, 9))
    assert e.value.code == -3
