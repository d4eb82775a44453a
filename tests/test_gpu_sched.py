"""GPU parity of the rounds-scheduled execution (Algorithm 1) against the serial oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads import gen
from workloads.device import UploadingWeights, make_context, f32, i32
import paper_2406_18200_amd as sv

pytestmark = pytest.mark.gpu


def _models():
    wt = wl.get_workload("c2").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000,
                                      N=5, gamma=3, S=40, R=0, seed=201)
    wd = wt.scaled(n_layers=1, d_model=128, n_heads=2, head_dim=64, d_ff=352, seed=202)
    return wt, wd


def _run(wt, wd, up_t, up_d, prefix, first, u, max_new, unit):
    dev, n, G = "cuda:0", wt.N, wt.gamma
    s_t, s_d = torch.cuda.Stream(), torch.cuda.Stream()
    with torch.cuda.stream(s_t):
        tctx = make_context(wt.model, up_t.upload_all(), max_branches=n, max_rows_per_branch=G, max_shared=wt.S,
                            max_private=max_new + 2 * G, device=dev)
        tctx.prefill_shared(i32(prefix, dev))
    with torch.cuda.stream(s_d):
        dctx = make_context(wd.model, up_d.upload_all(), max_branches=n, max_rows_per_branch=max(1, 128 // n),
                            max_shared=wd.S, max_private=max_new + 2 * G, device=dev)
        dctx.prefill_shared(i32(prefix, dev))
    torch.cuda.synchronize()
    plen_t = torch.zeros(n, dtype=torch.int32, device=dev)
    plen_d = torch.zeros(n, dtype=torch.int32, device=dev)
    toks, lens, stats = sv.sched_run(tctx, dctx, first, f32(u[0], dev), f32(u[1], dev), f32(u[2], dev), plen_t, plen_d,
                                     gamma=G, max_new=max_new, temperature=wt.temperature, shared_len_target=wt.S,
                                     shared_len_draft=wd.S, unit_branches=unit)
    assert tctx.status() == 0 and dctx.status() == 0
    # both caches hold exactly the validated context minus the pending token
    keep_t, keep_d = plen_t.cpu().numpy(), plen_d.cpu().numpy()
    assert np.array_equal(keep_t, keep_d)
    tctx.close()
    dctx.close()
    return toks, lens, stats, keep_t


def test_scheduled_rounds_match_the_serial_oracle_for_every_unit_size():
    wt, wd = _models()
    n, G, max_new = wt.N, wt.gamma, 10
    up_t = UploadingWeights(wt.model, wt.seed, "cuda:0", reuse_buffers=False)
    up_d = UploadingWeights(wd.model, wd.seed, "cuda:0", reuse_buffers=False)
    prefix = wl.prefix_tokens(wt)
    first = gen.pending_tokens(wt)
    u = wl.uniform24(wt.seed + 9, (3, n, max_new + G))
    runs = {unit: _run(wt, wd, up_t, up_d, prefix, first, u, max_new, unit) for unit in (0, 2, 1)}
    base = runs[0]
    for unit, (toks, lens, stats, keep) in runs.items():
        assert (lens == max_new).all()
        assert stats["accepted"] <= stats["drafted"] and stats["emitted"] >= n * max_new
        # the schedule decides when a round runs, not what it produces
        assert np.array_equal(toks, base[0]), unit
        assert np.array_equal(keep, base[3]), unit
    assert runs[1][2]["units"] >= runs[0][2]["units"]          # one branch per unit: more verify steps
    print("stats:", {k: v[2] for k, v in runs.items()}, flush=True)
    # oracle: every branch alone, serially, from the same uniforms
    _, ks_t, vs_t = oracle.decode_rows(wt.model, up_t, prefix)
    _, ks_d, vs_d = oracle.decode_rows(wd.model, up_d, prefix)
    ctx_t = [(ks_t[l], vs_t[l]) for l in range(wt.model.n_layers)]
    ctx_d = [(ks_d[l], vs_d[l]) for l in range(wd.model.n_layers)]
    exact = 0
    for b in range(n):
        want, rounds = oracle.speculative_rounds(wt.model, up_t, ctx_t, wt.S, wd.model, up_d, ctx_d, wd.S, first[b], G,
                                                 max_new, wt.temperature, u[0][b], u[1][b], u[2][b])
        got = base[0][b].tolist()
        if got == want:
            exact += 1
            continue
        # a divergence is only acceptable at a decision the oracle itself marks as a near-tie (the library
        # computes in bf16 / fp32, the oracle in float64): the round in which the sequences part must hold an
        # accept test within the logits tolerance of its threshold
        t = next(i for i in range(max_new) if got[i] != want[i])
        r = next(r for r in rounds if r["start"] <= t < r["start"] + len(r["emitted"]))
        assert r["margin"].min() < 5e-2, (b, t, r)
    print(f"branches identical to the oracle: {exact}/{n}", flush=True)
    assert exact >= n - 1


@pytest.mark.parametrize("n,gamma,max_new,unit", [(1, 1, 5, 0), (8, 2, 7, 3), (3, 4, 9, 2)])
def test_scheduled_rounds_edge_shapes(n, gamma, max_new, unit):
    """One branch with one draft per round; more branches than a unit with a ragged last unit; a validated
    length that ends in the middle of a round.  Tokens against the serial oracle."""
    wt, wd = _models()
    wt, wd = wt.scaled(N=n, gamma=gamma, seed=301 + n), wd.scaled(N=n, gamma=gamma, seed=302 + n)
    up_t = UploadingWeights(wt.model, wt.seed, "cuda:0", reuse_buffers=False)
    up_d = UploadingWeights(wd.model, wd.seed, "cuda:0", reuse_buffers=False)
    prefix = wl.prefix_tokens(wt)
    first = gen.pending_tokens(wt)
    u = wl.uniform24(wt.seed + 9, (3, n, max_new + gamma))
    toks, lens, stats, _ = _run(wt, wd, up_t, up_d, prefix, first, u, max_new, unit)
    assert (lens == max_new).all() and (toks >= 0).all()
    _, ks_t, vs_t = oracle.decode_rows(wt.model, up_t, prefix)
    _, ks_d, vs_d = oracle.decode_rows(wd.model, up_d, prefix)
    ctx_t = [(ks_t[l], vs_t[l]) for l in range(wt.model.n_layers)]
    ctx_d = [(ks_d[l], vs_d[l]) for l in range(wd.model.n_layers)]
    exact = 0
    for b in range(n):
        want, rounds = oracle.speculative_rounds(wt.model, up_t, ctx_t, wt.S, wd.model, up_d, ctx_d, wd.S, first[b],
                                                 gamma, max_new, wt.temperature, u[0][b], u[1][b], u[2][b])
        got = toks[b].tolist()
        if got == want:
            exact += 1
            continue
        t = next(i for i in range(max_new) if got[i] != want[i])
        r = next(r for r in rounds if r["start"] <= t < r["start"] + len(r["emitted"]))
        assert r["margin"].min() < 5e-2, (b, t, r)
    assert exact >= n - 1, (exact, n)
