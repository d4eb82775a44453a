"""GPU parity of the draft-model batched decode step (one autoregressive token per branch and call)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads import gen
from workloads.device import UploadingWeights, make_context, f32, i32
from harness import CachedWeights, check_logits
import paper_2406_18200_amd as sv

pytestmark = pytest.mark.gpu


def _run_draft_case(w, n_steps, greedy=False):
    """Teacher-forced by the ORACLE: the token fed at step j+1 is the oracle's draw, so one differing draw
    cannot derail the rest of the comparison.  Checks per step: logits within tolerance; q = softmax(logits
    / T) within the matching relative tolerance; the sampled token inside the oracle's CDF band, widened by
    the measured deviation between the two CDFs (with a random-init model q is nearly uniform over 32000
    tokens, so a CDF step is ~3e-5 wide and a draw is decided by the last digits of the logits: several
    tokens are then valid, what is unique is the band); the token consistent with the library's own q row
    (stateless sampler, bit-exact)."""
    m, dev = w.model, "cuda:0"
    up = UploadingWeights(m, w.seed, dev, reuse_buffers=False)
    W = CachedWeights(up)
    prefix = wl.prefix_tokens(w)
    _, ks, vs = oracle.decode_rows(m, W, prefix)
    ctx = make_context(m, up.upload_all(), max_branches=w.N, max_rows_per_branch=max(1, 128 // w.N), max_shared=w.S,
                       max_private=n_steps, device=dev)
    assert ctx.prefill_shared(i32(prefix, dev)) == w.S
    plen = torch.zeros(w.N, dtype=torch.int32, device=dev)
    cur = gen.pending_tokens(w)
    u = wl.uniform24(w.seed + 4, (n_steps, w.N))
    q_dev = torch.zeros((w.N, n_steps, m.vocab), dtype=torch.float32, device=dev)
    tok_dev = torch.zeros((w.N, n_steps), dtype=torch.int32, device=dev)
    lg_dev = torch.empty((w.N, m.vocab), dtype=torch.float32, device=dev)
    pk = [[np.zeros((m.n_heads, 0, m.head_dim)) for _ in range(m.n_layers)] for _ in range(w.N)]
    pv = [[np.zeros((m.n_heads, 0, m.head_dim)) for _ in range(m.n_layers)] for _ in range(w.N)]
    near_ties = 0
    for j in range(n_steps):
        # oracle: one new row per branch against shared + private context
        ref_logits = np.zeros((w.N, m.vocab))
        for b in range(w.N):
            lg, kn, vn = oracle.decode_rows(m, W, cur[b:b + 1], pos0=w.S + j,
                                            ctx_kv=lambda l: (np.concatenate([ks[l], pk[b][l]], 1),
                                                              np.concatenate([vs[l], pv[b][l]], 1)))
            ref_logits[b] = lg[0]
            for l in range(m.n_layers):
                pk[b][l] = np.concatenate([pk[b][l], kn[l]], 1)
                pv[b][l] = np.concatenate([pv[b][l], vn[l]], 1)
        ref_q = oracle.softmax_temperature(ref_logits, w.temperature)
        if greedy:
            ref_tok = ref_logits.argmax(-1).astype(np.int32)
        else:
            ref_tok = np.array([oracle.sample_from_probs(ref_q[b], u[j, b]) for b in range(w.N)], np.int32)
        # library
        ctx.draft_step(i32(cur, dev), w.S, plen, f32(u[j], dev), w.temperature, q_out=q_dev[:, j], tok_out=tok_dev[:, j],
                       q_stride=q_dev.stride(0), tok_stride=tok_dev.stride(0), logits_out=lg_dev,
                       flags=sv.binding.SEED_STEP_GREEDY if greedy else 0)
        torch.cuda.synchronize()
        got_logits, got_q, got_tok = lg_dev.cpu().numpy(), q_dev[:, j].cpu().numpy(), tok_dev[:, j].cpu().numpy()
        worst, err = check_logits(got_logits, ref_logits, m.dtype)
        assert worst <= 1.0, (j, worst, err)
        atol, rtol = (2e-2, 1e-2) if m.dtype == "bf16" else (1e-5, 1e-4)
        qtol = np.exp((atol + rtol * np.abs(ref_logits).max()) / w.temperature * 2) - 1
        assert (np.abs(got_q - ref_q) <= qtol * ref_q + 1e-12).all(), j
        assert np.abs(got_q.sum(-1) - 1).max() < 1e-4
        # the token follows bit-exactly from the library's own q row (checked with its stateless sampler)
        if not greedy:
            again = sv.sample_probs(q_dev[:, j], f32(u[j], dev)).cpu().numpy()
            assert np.array_equal(again, got_tok)
        for b in range(w.N):
            if got_tok[b] != ref_tok[b]:
                if greedy:
                    top2 = np.sort(ref_logits[b])[-2:]
                    assert top2[1] - top2[0] < 2 * (atol + rtol * abs(top2[1])), (j, b)
                else:
                    cdf = np.cumsum(ref_q[b].astype(np.float64))
                    cdf /= cdf[-1]
                    cdf_g = np.cumsum(got_q[b].astype(np.float64))
                    cdf_g /= cdf_g[-1]
                    delta = np.abs(cdf - cdf_g).max() + 2.0 ** -24
                    assert delta < (1e-3 if m.dtype == "bf16" else 1e-5), delta
                    t = int(got_tok[b])
                    lo = cdf[t - 1] if t > 0 else 0.0
                    assert lo - delta <= float(u[j, b]) <= cdf[t] + delta, (j, b, t, int(ref_tok[b]))
                near_ties += 1
        cur = ref_tok
    assert np.array_equal(plen.cpu().numpy(), np.full(w.N, n_steps))
    assert ctx.status() == 0
    print(f"draws differing from the oracle's (all inside the CDF band): {near_ties} of {n_steps * w.N}", flush=True)
    ctx.close()


def test_c2_draft_model_batched_decode():
    """Draft configuration: 2-layer d=768, 12 heads, V=32000, N=8 branches, 8 autoregressive steps from a
    shared 256-token prefix (true-prefix protocol: both sides compute the prefix KV themselves)."""
    w = wl.get_workload("c2")
    _run_draft_case(w, w.gamma)


def test_draft_fp32_and_greedy():
    w = wl.get_workload("c1").scaled(N=5)
    _run_draft_case(w, 5)
    _run_draft_case(w, 3, greedy=True)
