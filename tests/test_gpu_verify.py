"""GPU parity of the whole verify step (forward + accept/resample) against the oracle, through the C ABI."""
import numpy as np
import pytest

import workloads as wl
from harness import Case

pytestmark = pytest.mark.gpu


def test_c1_tiny_fp32_true_prefix():
    """Tiny fp32 plumbing case: both sides compute the 64-token prefix themselves."""
    Case(wl.get_workload("c1")).run_oracle().run_gpu().compare()


def test_c1_bonus_row_and_private_context():
    w = wl.get_workload("c1").scaled(R=7, N=4)
    Case(w, bonus=True).run_oracle().run_gpu().compare()


def test_c1_greedy():
    Case(wl.get_workload("c1"), greedy=True).run_oracle().run_gpu().compare()


@pytest.mark.parametrize("N,gamma,S,R", [(3, 4, 100, 0), (5, 3, 70, 9), (16, 6, 257, 40), (1, 1, 33, 0),
                                         (2, 5, 1100, 300),   # <= 16 rows, 13 partials: in-launch merge in passes
                                         (1, 40, 64, 20),     # one branch of 40 rows: two row groups per branch
                                         (3, 7, 200, 150),    # 21 rows (two row tiles), two private key ranges
                                         (20, 1, 70, 9),      # 20 branches of ONE row: a head's in-flight segment is a single score
                                         (3, 8, 100, 40),     # eight rows per branch: the most a wavefront-per-head branch task takes
                                         (2, 9, 100, 40)])    # nine rows per branch: branch tasks in the workgroup-per-head form
def test_small_bf16_synthetic_kv(N, gamma, S, R):
    """Small bf16 model (2 layers, d=256, 4 heads of 64): several MFMA tiles, ragged tails in rows and keys,
    and every shape of the attention launch (one / two row tiles, merge inside / after the launch, several
    key ranges in the shared and the private segment, several row groups per branch)."""
    w = wl.get_workload("c3").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000,
                                     N=N, gamma=gamma, S=S, R=R, seed=77 + N)
    Case(w).run_oracle().run_gpu().compare()


@pytest.mark.parametrize("N,gamma,S,R,R_min", [(5, 3, 0, 300, 3),     # <= 16 rows, no shared prefix at all
                                               (8, 4, 0, 300, 0),     # 32 rows; branch 0 starts from nothing
                                               (3, 7, 90, 200, 1),    # ragged lengths next to a shared prefix
                                               (2, 2, 0, 0, -1)])     # no context whatsoever: in-flight rows only
def test_ragged_private_contexts_without_shared_prefix(N, gamma, S, R, R_min):
    """State-evaluator shape (Section 3.2: different states, i.e. different prompts): branches with private
    contexts of different lengths and an empty shared segment; the degenerate rows that see only themselves."""
    w = wl.get_workload("c6").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000,
                                     N=N, gamma=gamma, S=S, R=R, R_min=R_min, seed=177 + N)
    c = Case(w).run_oracle().run_gpu()
    c.compare()
    if R_min >= 0:
        assert c.plens[0] == R_min and c.plens[-1] == R


@pytest.mark.parametrize("N,gamma", [(4, 4), (3, 5)])
def test_small_bf16_bonus_row(N, gamma):
    """gamma + 1 target rows per branch (the extra token after a fully accepted round), bf16 kernels, ragged
    private contexts: 20 and 18 rows, i.e. a row-group boundary inside a branch."""
    w = wl.get_workload("c6").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000,
                                     N=N, gamma=gamma, S=50, R=30, R_min=2, seed=277 + N)
    Case(w, bonus=True).run_oracle().run_gpu().compare()


@pytest.mark.parametrize("N,gamma,vocab", [(16, 5, 20800), (16, 6, 20800), (16, 8, 20800), (13, 7, 20800),
                                           (16, 6, 10400), (16, 5, 10400),
                                           (8, 5, 20800), (8, 5, 10400), (16, 4, 20800)])   # 40 and 64 rows
def test_wide_projection_form_ragged_k(N, gamma, vocab):
    """65..128 rows with outputs wide enough for the projection form that stages activations by global -> LDS
    loads (gate/up with 600 n-tiles, LM head with 1300 or 650), and a k extent (18 k-tiles) that ends inside a
    weight group and inside a round of groups: five, six and eight row tiles; at three and six row tiles the LM
    heads run the twelve-wavefront shapes (two n-tiles per wavefront at 1300 n-tiles, one at 650); at four row
    tiles there is no such shape and the first form runs."""
    w = wl.get_workload("c4").scaled(n_layers=2, d_model=576, n_heads=9, head_dim=64, d_ff=4800, vocab=vocab,
                                     N=N, gamma=gamma, S=100, R=20, seed=377 + gamma)
    Case(w, branches=[0, N // 2, N - 1]).run_oracle().run_gpu().compare()


@pytest.mark.parametrize("N,gamma,vocab", [(24, 6, 20800),      # 144 rows: nine row tiles, two blocks of five
                                           (64, 6, 10400),      # 384 rows: 24 tiles, four blocks x two shares
                                           (50, 5, 20800),      # 250 rows: ragged last tile and last share
                                           (96, 8, 2000)])      # 768 rows: the most a step takes
def test_more_than_128_rows(N, gamma, vocab):
    """Steps past 128 rows (batch sweep toward the matrix-core ridge): the projections run as row shares of
    three or four tiles that reuse one pass over the weights, the shared attention segment as several
    workgroups per key range.  Same small model as the wide-form cases; a sample of branches on the oracle
    side (first, middle, last)."""
    w = wl.get_workload("c4").scaled(n_layers=2, d_model=576, n_heads=9, head_dim=64, d_ff=4800, vocab=vocab,
                                     N=N, gamma=gamma, S=100, R=20, seed=577 + gamma)
    Case(w, branches=[0, N // 2, N - 1]).run_oracle().run_gpu().compare()


@pytest.mark.parametrize("N,gamma", [(16, 6), (3, 4)])
def test_small_bf16_greedy_verification(N, gamma):
    """Greedy verification (accept while the draft equals the target's argmax) through the bf16 kernels; the
    argmax is taken on each side from its own logits, so branches whose top two logits are within the logits
    tolerance are compared on validity only (the harness marks them)."""
    w = wl.get_workload("c4").scaled(n_layers=2, d_model=512, n_heads=4, head_dim=128, d_ff=1024, vocab=4096,
                                     N=N, gamma=gamma, S=300, R=33, seed=477 + N)
    Case(w, greedy=True).run_oracle().run_gpu().compare()


def test_small_bf16_head128_long_private_context():
    """head_dim 128, 12 rows against 1000 shared and 260 private keys (three private key ranges)."""
    w = wl.get_workload("c3").scaled(n_layers=2, d_model=512, n_heads=4, head_dim=128, d_ff=1024, vocab=4096,
                                     N=3, gamma=4, S=1000, R=260, seed=93)
    Case(w).run_oracle().run_gpu().compare()


def test_small_bf16_true_prefix_head128():
    w = wl.get_workload("c2").scaled(n_layers=2, d_model=512, n_heads=4, head_dim=128, d_ff=1024, vocab=4096,
                                     N=6, gamma=5, S=150, R=11, seed=91)
    Case(w).run_oracle().run_gpu().compare()


def test_perturbed_draft_q_13b_widths_two_layers():
    """13B widths (d=5120, 40 heads, F=13824) at two layers, N=8 x gamma=5, S=4096, with the draft
    distribution a perturbed copy of the target's, built autoregressively by the oracle: realistic
    acceptance rates, so the accept / resample path sees both outcomes."""
    import harness
    w = wl.get_workload("c5").scaled(n_layers=2)
    W = harness.CachedWeights(wl.Weights(w.model, w.seed))
    q = harness.perturbed_q_autoregressive(w, W)
    c = Case(w, q_override=q).run_oracle().run_gpu()
    c.compare()
    assert 0 < c.ref_accept[0].sum() < w.N * w.gamma


def test_results_are_bit_identical_from_run_to_run():
    """No floating-point atomics anywhere: the same step twice gives the same bits (split-K partials are
    summed by the last workgroup in a fixed order)."""
    import torch
    w = wl.get_workload("c3").scaled(n_layers=2, N=16, gamma=6, S=300, R=17)
    c = Case(w).run_oracle().run_gpu(keep_ctx=True)
    first = (c.gpu_logits.copy(), [a.copy() for a in c.gpu_accept])
    for _ in range(3):
        c.dev_plen.fill_(w.R)
        c.dev_logits.zero_()
        import workloads.device as D
        inp = c.inp
        acc = dict(q=D.f32(inp["q"]), draft_tok=D.i32(inp["drafts"]), u_acc=D.f32(inp["u_acc"]), u_res=D.f32(inp["u_res"]),
                   temperature=w.temperature)
        outs = c.ctx.step(D.i32(inp["row_tok"]), w.S, c.dev_plen, logits_out=c.dev_logits, accept=acc)
        torch.cuda.synchronize()
        assert np.array_equal(c.dev_logits.cpu().numpy(), first[0])
        for a, b in zip(outs, first[1]):
            assert np.array_equal(a.cpu().numpy(), b)
    c.ctx.close()


def test_private_capacity_overflow_is_flagged_not_fatal():
    import torch
    import workloads.device as D
    w = wl.get_workload("c1").scaled(N=2, gamma=3)
    c = Case(w).run_oracle().run_gpu(keep_ctx=True)       # max_private = 0: one step fits exactly
    assert c.status == 0
    inp = c.inp
    acc = dict(q=D.f32(inp["q"]), draft_tok=D.i32(inp["drafts"]), u_acc=D.f32(inp["u_acc"]), u_res=D.f32(inp["u_res"]),
               temperature=w.temperature)
    c.ctx.step(D.i32(inp["row_tok"]), w.S, c.dev_plen, accept=acc)     # private_len is now >= 1 > max_private
    torch.cuda.synchronize()
    assert c.ctx.status() & 1
    assert c.ctx.status() == 0                                          # reading clears the word
    c.ctx.close()


def test_token_ids_outside_the_vocabulary_are_flagged_not_indexed():
    """A draft token id outside [0, V) handed to the accept step is never used as an index: it counts as
    rejected, its p(x) reads 0 and bit 2 of the status word is raised; a row token id outside the vocabulary is
    clamped and raises bit 3.  Every kernel exits normally and the other branches are unaffected."""
    import torch
    import workloads.device as D
    w = wl.get_workload("c3").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000,
                                     N=4, gamma=3, S=70, R=5, seed=321)
    c = Case(w).run_oracle().run_gpu(keep_ctx=True)
    c.compare()
    inp, G, V = c.inp, w.gamma, w.model.vocab
    good = [x.copy() for x in c.gpu_accept]
    for bad_id, branch in ((V + 7, 1), (-3, 2), (2 ** 31 - 1, 0)):
        drafts = inp["drafts"].copy()
        drafts[branch, G - 1] = bad_id                       # the last draft is not among the fed rows
        c.dev_plen.fill_(w.R)
        acc = dict(q=D.f32(inp["q"]), draft_tok=D.i32(drafts), u_acc=D.f32(inp["u_acc"]), u_res=D.f32(inp["u_res"]),
                   temperature=w.temperature)
        outs = [o.cpu().numpy() for o in c.ctx.step(D.i32(inp["row_tok"]), w.S, c.dev_plen, accept=acc)]
        torch.cuda.synchronize()
        assert c.ctx.status() == 4
        a, out, n, ptok = outs
        assert a[branch] == min(good[0][branch], G - 1) and ptok[branch, G - 1] == 0.0
        assert n[branch] == a[branch] + 1 and 0 <= out[branch, a[branch]] < V
        others = [b for b in range(w.N) if b != branch]
        for g, o in zip(good, outs):
            assert np.array_equal(g[others], o[others])
    rows = inp["row_tok"].copy()
    rows[3, 1] = V                                           # first id past the end
    c.dev_plen.fill_(w.R)
    c.ctx.step(D.i32(rows), w.S, c.dev_plen)
    torch.cuda.synchronize()
    assert c.ctx.status() == 8 and c.ctx.status() == 0
    c.ctx.close()


def test_empty_and_single_row_steps():
    import torch
    import workloads.device as D
    w = wl.get_workload("c1")
    c = Case(w).run_oracle().run_gpu(keep_ctx=True)
    empty = torch.zeros((0, 4), dtype=torch.int32, device="cuda")
    assert c.ctx.step(empty, w.S, c.dev_plen) is None                   # N = 0: nothing launched, no error
    c.ctx.close()
    Case(w.scaled(N=1, gamma=1)).run_oracle().run_gpu().compare()


def test_two_consecutive_steps_commit_and_reuse_the_cache():
    """KV commit across steps (Algorithm 1: a branch's validated length grows by the accepted tokens plus the
    replacement; the rows that verified them stay in its cache, the rejected rows are dead).  Step 1 is built so
    that branch b accepts exactly b % (gamma + 1) drafts: q = the oracle's p with u = 0.5 where a draft is to be
    accepted, q = one-hot on the draft with u = 0.999 where it is to be rejected.  Step 2 then feeds, per
    branch, the token step 1 emitted last plus new drafts; its logits are checked against an oracle that
    recomputes every branch from its TOKENS (prefix + private + the rows step 1 committed), so a wrong or stale
    cache row, or a wrong committed length, shows up."""
    import torch
    import oracle
    import workloads.device as D
    from workloads import gen
    from harness import check_logits
    w = wl.get_workload("c2").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000,
                                     N=7, gamma=4, S=90, R=5, seed=123)
    m, G, N, T, dev = w.model, w.gamma, w.N, w.gamma, "cuda:0"
    up = D.UploadingWeights(m, w.seed, dev, reuse_buffers=False)
    prefix, private, pending = wl.prefix_tokens(w), gen.private_tokens(w), gen.pending_tokens(w)
    rng = np.random.default_rng(5)
    drafts1 = rng.integers(0, m.vocab, (N, G)).astype(np.int32)
    rows1 = np.concatenate([pending[:, None], drafts1[:, :T - 1]], axis=1).astype(np.int32)
    # oracle, step 1: context KV from tokens
    _, ks, vs = oracle.decode_rows(m, up, prefix)
    pk, pv = [], []
    for b in range(N):
        _, kb, vb = oracle.decode_rows(m, up, private[b], ctx_kv=lambda l: (ks[l], vs[l]), pos0=w.S)
        pk.append(kb)
        pv.append(vb)
    ctx1 = lambda l: [(np.concatenate([ks[l], pk[b][l]], 1), np.concatenate([vs[l], pv[b][l]], 1)) for b in range(N)]
    ref1 = oracle.verify_forward(m, up, rows1, ctx1, [w.S + w.R] * N)
    p1 = oracle.softmax_temperature(ref1, w.temperature)
    want_a = np.array([b % (G + 1) for b in range(N)])
    q = np.zeros((N, G, m.vocab), np.float32)
    u_acc = np.zeros((N, G), np.float32)
    for b in range(N):
        for j in range(G):
            if j < want_a[b]:
                q[b, j], u_acc[b, j] = p1[b, j], 0.5
            else:
                q[b, j, drafts1[b, j]], u_acc[b, j] = 1.0, 0.999
    u_res = wl.uniform24(w.seed + 4, (N,), stream=1)
    # library, step 1
    ctx = D.make_context(m, up.upload_all(), max_branches=N, max_rows_per_branch=T, max_shared=w.S,
                         max_private=w.R + 2 * T, device=dev)
    plen = torch.zeros(N, dtype=torch.int32, device=dev)
    ctx.prefill_shared(D.i32(prefix, dev))
    for lo in range(0, w.R, T):
        ctx.step(D.i32(private[:, lo:lo + T], dev).contiguous(), w.S, plen, flags=sv_flags().SEED_STEP_COMMIT_ALL)
    acc = dict(q=D.f32(q, dev), draft_tok=D.i32(drafts1, dev), u_acc=D.f32(u_acc, dev), u_res=D.f32(u_res, dev),
               temperature=w.temperature)
    logits = torch.empty((N, T, m.vocab), dtype=torch.float32, device=dev)
    a_g, out_g, n_g, _ = [o.cpu().numpy() for o in ctx.step(D.i32(rows1, dev), w.S, plen, logits_out=logits, accept=acc)]
    worst, err = check_logits(logits.cpu().numpy(), ref1, m.dtype)
    assert worst <= 1.0, (worst, err)
    assert np.array_equal(a_g, want_a), (a_g, want_a)
    commit = np.minimum(want_a + 1, T)
    assert np.array_equal(plen.cpu().numpy(), w.R + commit)
    # step 2: the pending token is the replacement (or, after gamma accepts, the last accepted draft)
    pending2 = np.array([out_g[b, want_a[b]] if want_a[b] < G else drafts1[b, G - 1] for b in range(N)], np.int32)
    assert (pending2 >= 0).all()
    drafts2 = rng.integers(0, m.vocab, (N, G)).astype(np.int32)
    rows2 = np.concatenate([pending2[:, None], drafts2[:, :T - 1]], axis=1).astype(np.int32)
    logits2 = torch.empty((N, T, m.vocab), dtype=torch.float32, device=dev)
    ctx.step(D.i32(rows2, dev), w.S, plen, logits_out=logits2)
    torch.cuda.synchronize()
    # oracle, step 2: each branch again from its tokens
    pk2, pv2 = [], []
    for b in range(N):
        toks = np.concatenate([private[b], rows1[b, :commit[b]]])
        _, kb, vb = oracle.decode_rows(m, up, toks, ctx_kv=lambda l: (ks[l], vs[l]), pos0=w.S)
        pk2.append(kb)
        pv2.append(vb)
    ctx2 = lambda l: [(np.concatenate([ks[l], pk2[b][l]], 1), np.concatenate([vs[l], pv2[b][l]], 1)) for b in range(N)]
    ref2 = oracle.verify_forward(m, up, rows2, ctx2, list(w.S + w.R + commit))
    worst, err = check_logits(logits2.cpu().numpy(), ref2, m.dtype)
    assert worst <= 1.0, (worst, err)
    assert ctx.status() == 0
    ctx.close()


def sv_flags():
    import paper_2406_18200_amd as sv
    return sv.binding


def test_subsets_of_branches_by_cache_slot():
    """Verify steps over SUBSETS of a context's branches (the target verifies whichever drafts are queued):
    branch b of a call is cache slot branch_slot[b].  Six branches with private contexts; two calls verify
    slots (4, 1, 5) and (0, 3); logits against the oracle's for exactly those branches, the accept step's
    lengths land in the right slots, the untouched slot 2 keeps its length, and a later full step sees the
    rows the subset steps committed."""
    import torch
    import oracle
    import workloads.device as D
    from workloads import gen
    from harness import check_logits
    w = wl.get_workload("c2").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000,
                                     N=6, gamma=3, S=70, R=6, seed=321)
    m, G, N, T, dev = w.model, w.gamma, w.N, w.gamma, "cuda:0"
    up = D.UploadingWeights(m, w.seed, dev, reuse_buffers=False)
    prefix, private, pending = wl.prefix_tokens(w), gen.private_tokens(w), gen.pending_tokens(w)
    rng = np.random.default_rng(11)
    _, ks, vs = oracle.decode_rows(m, up, prefix)
    committed = [list(private[b]) for b in range(N)]            # tokens whose KV each branch has committed

    def oracle_logits(slots, rows):
        pk, pv = [], []
        for b in slots:
            _, kb, vb = oracle.decode_rows(m, up, np.array(committed[b]), ctx_kv=lambda l: (ks[l], vs[l]), pos0=w.S)
            pk.append(kb)
            pv.append(vb)
        ctx = lambda l: [(np.concatenate([ks[l], pk[i][l]], 1), np.concatenate([vs[l], pv[i][l]], 1))
                         for i in range(len(slots))]
        return oracle.verify_forward(m, up, rows, ctx, [w.S + len(committed[b]) for b in slots])

    ctx = D.make_context(m, up.upload_all(), max_branches=N, max_rows_per_branch=T, max_shared=w.S,
                         max_private=w.R + 3 * T, device=dev)
    plen = torch.zeros(N, dtype=torch.int32, device=dev)
    ctx.prefill_shared(D.i32(prefix, dev))
    for lo in range(0, w.R, T):
        ctx.step(D.i32(private[:, lo:lo + T], dev).contiguous(), w.S, plen, flags=sv_flags().SEED_STEP_COMMIT_ALL)
    for slots in ([4, 1, 5], [0, 3]):
        n = len(slots)
        drafts = rng.integers(0, m.vocab, (n, G)).astype(np.int32)
        rows = np.concatenate([pending[slots][:, None], drafts[:, :T - 1]], axis=1).astype(np.int32)
        ref = oracle_logits(slots, rows)
        p = oracle.softmax_temperature(ref, w.temperature)
        want_a = np.array([(s + 1) % (G + 1) for s in slots])
        q = np.zeros((n, G, m.vocab), np.float32)
        u_acc = np.zeros((n, G), np.float32)
        for i in range(n):
            for j in range(G):
                if j < want_a[i]:
                    q[i, j], u_acc[i, j] = p[i, j], 0.5
                else:
                    q[i, j, drafts[i, j]], u_acc[i, j] = 1.0, 0.999
        acc = dict(q=D.f32(q, dev), draft_tok=D.i32(drafts, dev), u_acc=D.f32(u_acc, dev),
                   u_res=D.f32(wl.uniform24(w.seed + n, (n,), stream=1), dev), temperature=w.temperature)
        logits = torch.empty((n, T, m.vocab), dtype=torch.float32, device=dev)
        before = plen.cpu().numpy().copy()
        a_g, out_g, _, _ = [o.cpu().numpy() for o in ctx.step(D.i32(rows, dev), w.S, plen, logits_out=logits,
                                                             accept=acc, branch_slot=D.i32(np.array(slots), dev))]
        worst, err = check_logits(logits.cpu().numpy(), ref, m.dtype)
        assert worst <= 1.0, (slots, worst, err)
        assert np.array_equal(a_g, want_a), (slots, a_g, want_a)
        after = plen.cpu().numpy()
        commit = np.minimum(want_a + 1, T)
        for b in range(N):
            assert after[b] == before[b] + (commit[slots.index(b)] if b in slots else 0), (b, before, after)
        for i, b in enumerate(slots):
            committed[b] += list(rows[i, :commit[i]])
            pending[b] = out_g[i, want_a[i]] if want_a[i] < G else drafts[i, G - 1]
    # a full step over all six branches (identity slots) sees what the subset steps left in the caches
    drafts = rng.integers(0, m.vocab, (N, G)).astype(np.int32)
    rows = np.concatenate([pending[:, None], drafts[:, :T - 1]], axis=1).astype(np.int32)
    logits = torch.empty((N, T, m.vocab), dtype=torch.float32, device=dev)
    ctx.step(D.i32(rows, dev), w.S, plen, logits_out=logits)
    torch.cuda.synchronize()
    worst, err = check_logits(logits.cpu().numpy(), oracle_logits(list(range(N)), rows), m.dtype)
    assert worst <= 1.0, (worst, err)
    # an out-of-range slot is clamped and flagged, not fatal
    ctx.step(D.i32(rows[:1], dev), w.S, plen, branch_slot=D.i32(np.array([N + 3]), dev))
    torch.cuda.synchronize()
    assert ctx.status() & 2
    ctx.close()


def test_branch_slots_are_refused_where_unsupported():
    """fp32 contexts and the shared-prefix prefill take no branch_slot: an error code, nothing launched."""
    import torch
    import workloads.device as D
    w = wl.get_workload("c1")
    c = Case(w).run_oracle().run_gpu(keep_ctx=True)
    slots = D.i32(np.arange(w.N))
    with pytest.raises(RuntimeError, match="branch_slot"):
        c.ctx.step(D.i32(c.inp["row_tok"]), w.S, c.dev_plen, branch_slot=slots)
    c.ctx.close()
