"""Shared driver for the GPU parity tests: builds one workload's inputs once, runs the oracle and the HIP
library on them and returns both results.  Oracle-side and GPU-side code meet only in the seeded inputs."""
import time

import numpy as np
import torch

import oracle
import workloads as wl
from workloads import gen
from workloads.device import UploadingWeights, make_context, to_device, f32, i32
from paper_2406_18200_amd import binding as B

TOL = {"fp32": (1e-5, 1e-4), "bf16": (2e-2, 1e-2), "bf16w8": (2e-2, 1e-2), "bf16w4": (2e-2, 1e-2)}   # (absolute, relative): |got - ref| <= abs + rel * |ref|


def check_logits(got, ref, dtype):
    atol, rtol = TOL[dtype]
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    worst = float((err / bound).max())
    return worst, float(err.max())


class CachedWeights:
    """Memoises a small model's tensors so repeated oracle calls do not regenerate them."""

    def __init__(self, inner):
        self.inner, self.cache = inner, {}

    def _get(self, key, fn):
        if key not in self.cache:
            self.cache[key] = np.array(fn(), copy=True)
        return self.cache[key]

    def tok_emb(self):
        return self._get("emb", self.inner.tok_emb)

    def norm_final(self):
        return self._get("nf", self.inner.norm_final)

    def lm_head(self):
        return self._get("lm", self.inner.lm_head)

    def layer(self, l):
        if ("layer", l) not in self.cache:
            self.cache[("layer", l)] = {k: np.array(v, copy=True) for k, v in self.inner.layer(l).items()}
        return self.cache[("layer", l)]


def perturbed_q_autoregressive(w, W, branches=None):
    """Draft distributions that are a perturbed copy of the target's (target logits + noise, same
    temperature), built autoregressively with the ORACLE: row j's logits depend on the drafts sampled from
    q_<j.  Synthetic-KV protocol.  One incremental single-row pass per draft position (the rows before it are
    context by then).  branches: the branches to build (default all); the rows of q of the others stay NaN
    (Case fills them through the library: nothing there is compared with the oracle).  Returns q [N][gamma][V]."""
    m, G = w.model, w.gamma
    sel = list(range(w.N)) if branches is None else list(branches)
    pending = gen.pending_tokens(w)
    plens = wl.private_lens(w)
    u = wl.uniform24(w.seed + 3, (w.N, G))
    q = np.full((w.N, G, m.vocab), np.nan, np.float32)
    new_k = {b: None for b in sel}          # K/V of the rows fed so far, per layer
    new_v = {b: None for b in sel}
    cur = {b: int(pending[b]) for b in sel}
    for j in range(G):
        kv = {}

        def ctx_of(b):
            def f(l):
                if l not in kv:
                    kv.clear()              # one layer's synthetic KV at a time
                    kv[l] = wl.synthetic_kv(w, l)
                k_s, v_s, k_p, v_p = kv[l]
                ks = [k_s, k_p[b][:, :plens[b]]] + ([new_k[b][l]] if new_k[b] is not None else [])
                vs = [v_s, v_p[b][:, :plens[b]]] + ([new_v[b][l]] if new_v[b] is not None else [])
                return np.concatenate(ks, 1), np.concatenate(vs, 1)
            return f
        rows = np.array([[cur[b]] for b in sel])
        # (one layer at a time for all selected branches: verify_forward asks for a layer's weights once)
        ctxs = {b: ctx_of(b) for b in sel}
        logits, ks_new, vs_new = oracle.transformer._forward(
            [rows[i] for i in range(len(sel))], W, m, lambda l: [ctxs[b](l) for b in sel],
            [w.S + int(plens[b]) + j for b in sel], single=False)
        for i, b in enumerate(sel):
            q[b, j] = wl.perturbed_draft_q(w, logits[i, 0].astype(np.float32), b, j)
            step_k = [ks_new[l][i] for l in range(m.n_layers)]
            step_v = [vs_new[l][i] for l in range(m.n_layers)]
            if new_k[b] is None:
                new_k[b], new_v[b] = step_k, step_v
            else:
                new_k[b] = [np.concatenate([a, c], 1) for a, c in zip(new_k[b], step_k)]
                new_v[b] = [np.concatenate([a, c], 1) for a, c in zip(new_v[b], step_v)]
            cur[b] = int(wl.draw_tokens(q[b, j][None], u[b, j][None])[0])
    return q


def build_inputs(w, bonus=False, q_override=None):
    """Host-side inputs of one verify step (everything except the model and the KV context).  Branches whose
    rows of q_override are NaN get their q (and drafts) later, from the library's own single-row steps."""
    G = w.gamma
    pending = gen.pending_tokens(w)
    q = np.array(q_override, np.float32, copy=True) if q_override is not None else wl.random_draft_q(w)
    u = wl.uniform24(w.seed + 3, (w.N, G))
    todo = [b for b in range(w.N) if np.isnan(q[b]).any()]
    if todo:
        q[todo] = 1.0 / q.shape[-1]
    drafts = wl.draw_tokens(q, u)
    T = G + 1 if bonus else G
    row_tok = np.concatenate([pending[:, None], drafts[:, :T - 1]], axis=1).astype(np.int32)
    u_acc = wl.uniform24(w.seed + 4, (w.N, G))
    u_res = wl.uniform24(w.seed + 4, (w.N,), stream=1)
    return dict(q=q, drafts=drafts, row_tok=row_tok, u_acc=u_acc, u_res=u_res, T=T, u_draft=u, pending=pending,
                fill_with_library=todo)


def logits_tolerance_on_probs(ref_logits, dtype, temperature):
    """Relative tolerance on a softmax probability that follows from the tolerance on the logits: every logit
    may move by atol + rtol |l|, numerator and normaliser in opposite directions."""
    atol, rtol = TOL[dtype]
    return float(np.exp(2.0 * (atol + rtol * np.abs(ref_logits).max()) / temperature) - 1.0)


def cdf_band(weights64, tok):
    """[F(tok - 1), F(tok)] of the normalised cumulative distribution of non-negative float64 weights."""
    c = np.cumsum(weights64)
    return (c[tok - 1] / c[-1] if tok > 0 else 0.0), c[tok] / c[-1], c / c[-1]


class Case:
    """Runs oracle and GPU on a workload.  branches = subset of branch indices the oracle evaluates (all by
    default); the GPU always runs the full step in its benchmark launch configuration."""

    def __init__(self, w, bonus=False, greedy=False, branches=None, device="cuda:0", log=print, q_override=None):
        self.w, self.bonus, self.greedy, self.device, self.log = w, bonus, greedy, device, log
        self.branches = list(range(w.N)) if branches is None else list(branches)
        self.inp = build_inputs(w, bonus, q_override)
        self.plens = wl.private_lens(w)          # [N] valid private tokens per branch (ragged workloads: differ)
        assert (self.plens == w.R).all() or w.kv_protocol == "synthetic"

    # ---------------------------------------------------------------- oracle side
    def run_oracle(self):
        w, m, inp = self.w, self.w.model, self.inp
        t0 = time.time()
        self.weights = UploadingWeights(m, w.seed, self.device)
        W = self.weights
        sel = self.branches
        if w.kv_protocol == "true_prefix":
            self.prefix = wl.prefix_tokens(w)
            self.private = gen.private_tokens(w)
            _, ks, vs = oracle.decode_rows(m, W, self.prefix)
            pk, pv = {}, {}
            for b in sel:
                if w.R:
                    _, kb, vb = oracle.decode_rows(m, W, self.private[b], ctx_kv=lambda l: (ks[l], vs[l]), pos0=w.S)
                    pk[b], pv[b] = kb, vb

            def ctx(l):
                out = []
                for b in sel:
                    if w.R:
                        out.append((np.concatenate([ks[l], pk[b][l]], 1), np.concatenate([vs[l], pv[b][l]], 1)))
                    else:
                        out.append((ks[l], vs[l]))
                return out
        else:
            self.kv_dev = []

            def ctx(l):
                k_s, v_s, k_p, v_p = wl.synthetic_kv(w, l)
                self.kv_dev.append(tuple(to_device(a, m, self.device) if a.size else None for a in (k_s, v_s, k_p, v_p)))
                return [(np.concatenate([k_s, k_p[b][:, :self.plens[b]]], 1),
                         np.concatenate([v_s, v_p[b][:, :self.plens[b]]], 1)) for b in sel]
        pos0 = [w.S + int(self.plens[b]) for b in sel]
        self.ref_logits = oracle.verify_forward(m, W, inp["row_tok"][sel], ctx, pos0)
        G = w.gamma
        if self.greedy:
            res = oracle.accept_resample(None, None, inp["drafts"][sel], None, None, greedy=True, logits=self.ref_logits.astype(np.float32))
            self.ref_p = None
        else:
            self.ref_p = oracle.softmax_temperature(self.ref_logits, w.temperature)
            res = oracle.accept_resample(self.ref_p, inp["q"][sel], inp["drafts"][sel], inp["u_acc"][sel], inp["u_res"][sel])
        self.ref_accept = res
        self.log(f"oracle done in {time.time() - t0:.1f}s", flush=True)
        return self

    # ---------------------------------------------------------------- HIP side
    def run_gpu(self, keep_ctx=False):
        w, m, inp = self.w, self.w.model, self.inp
        t0 = time.time()
        dev = self.weights.upload_all()
        T = inp["T"]
        ctx = make_context(m, dev, max_branches=w.N, max_rows_per_branch=T, max_shared=max(w.S, 1),
                           max_private=w.R, device=self.device)
        plen = torch.zeros(w.N, dtype=torch.int32, device=self.device)
        if w.kv_protocol == "true_prefix":
            ctx.prefill_shared(i32(self.prefix, self.device))
            if w.R:
                for lo in range(0, w.R, T):       # private prefill in chunks of at most T rows per branch
                    chunk = i32(self.private[:, lo:lo + T], self.device).contiguous()
                    ctx.step(chunk, w.S, plen, flags=B.SEED_STEP_COMMIT_ALL)
        else:
            for l, (k_s, v_s, k_p, v_p) in enumerate(self.kv_dev):
                ctx.kv_load(l, k_s, v_s, k_p, v_p)
            plen += i32(self.plens, self.device)   # a shorter branch simply ignores the rest of its slot
        if inp["fill_with_library"]:
            self._fill_q_with_library(ctx, plen)
        logits = torch.empty((w.N, T, m.vocab), dtype=torch.float32, device=self.device)
        acc = dict(q=None if self.greedy else f32(inp["q"], self.device), draft_tok=i32(inp["drafts"], self.device),
                   u_acc=None if self.greedy else f32(inp["u_acc"], self.device),
                   u_res=None if self.greedy else f32(inp["u_res"], self.device),
                   temperature=w.temperature, greedy=self.greedy)
        flags = B.SEED_STEP_GREEDY if self.greedy else 0
        outs = ctx.step(i32(inp["row_tok"], self.device), w.S, plen, flags=flags, logits_out=logits, accept=acc)
        torch.cuda.synchronize()
        self.status = ctx.status()
        self.gpu_logits = logits.cpu().numpy()
        self.gpu_accept = [o.cpu().numpy() if o is not None else None for o in outs]
        self.gpu_plen = plen.cpu().numpy()
        self.log(f"gpu done in {time.time() - t0:.1f}s", flush=True)
        if keep_ctx:
            self.ctx, self.dev_plen, self.dev_logits = ctx, plen, logits
        else:
            ctx.close()
        return self

    def _fill_q_with_library(self, ctx, plen):
        """q of the branches the oracle does not evaluate: perturbed copies of the LIBRARY's own target logits,
        one step per draft position (the oracle's branches are fed their oracle-made drafts)."""
        w, m, inp = self.w, self.w.model, self.inp
        todo, G = inp["fill_with_library"], w.gamma
        rows = inp["pending"][:, None].astype(np.int32)
        for j in range(G):
            # position j's target logits: a step over the pending token and the drafts so far, nothing committed
            lg = torch.empty((w.N, j + 1, m.vocab), dtype=torch.float32, device=self.device)
            ctx.step(i32(rows, self.device), w.S, plen, logits_out=lg)
            ell = lg[:, j].cpu().numpy()
            for b in todo:
                inp["q"][b, j] = wl.perturbed_draft_q(w, ell[b], b, j)
                inp["drafts"][b, j] = wl.draw_tokens(inp["q"][b, j][None], inp["u_draft"][b, j][None])[0]
            rows = np.concatenate([rows, inp["drafts"][:, j:j + 1]], axis=1).astype(np.int32)
        T = inp["T"]
        inp["row_tok"] = np.concatenate([inp["pending"][:, None], inp["drafts"][:, :T - 1]], axis=1).astype(np.int32)

    # ---------------------------------------------------------------- comparison
    def compare(self):
        w, inp, sel = self.w, self.inp, self.branches
        G, T = w.gamma, inp["T"]
        worst, max_err = check_logits(self.gpu_logits[sel], self.ref_logits, w.model.dtype)
        self.log(f"logits: max abs err {max_err:.3e}, worst err/bound {worst:.3f}", flush=True)
        assert self.status == 0
        assert worst <= 1.0, (worst, max_err)
        a_w, out_w, n_w, ptok_w = self.ref_accept
        a_g, out_g, n_g, ptok_g = [x[sel] if x is not None else None for x in self.gpu_accept]
        dt = w.model.dtype
        gl = self.gpu_logits[sel]
        if self.greedy:
            # argmax decided on each side from its own logits: identical unless the top two logits are within tolerance
            top2 = np.sort(self.ref_logits, axis=-1)[..., -2:]
            clear_rows = (top2[..., 1] - top2[..., 0]) > 2 * (TOL[dt][0] + TOL[dt][1] * np.abs(top2[..., 1]))
            clear = clear_rows[:, :G].all(axis=1)
            # decisions and emitted tokens follow bit-exactly from the library's own logits (lowest index on ties)
            own = oracle.accept_resample(None, None, inp["drafts"][sel], None, None, greedy=True, logits=gl)
            assert np.array_equal(a_g, own[0]) and np.array_equal(out_g, own[1]) and np.array_equal(n_g, own[2])
        else:
            T_ = w.temperature
            qtok = np.take_along_axis(inp["q"][sel], inp["drafts"][sel][..., None], -1)[..., 0]
            ptol = logits_tolerance_on_probs(self.ref_logits, dt, T_)     # what the logits tolerance allows on p(x)
            rel = np.abs(ptok_g - ptok_w) / np.maximum(ptok_w, 1e-30)
            self.log(f"p_tok: max rel err {rel.max():.3e} (allowed by the logits tolerance: {ptol:.3e})", flush=True)
            assert rel.max() <= ptol
            # (i) the kernel's p(x) is the softmax of ITS OWN logits to 1e-5 (row statistics + exp2 path)
            p_own = oracle.softmax_temperature(gl, T_)
            ptok_own = np.take_along_axis(p_own[:, :G], inp["drafts"][sel][..., None], -1)[..., 0]
            assert (np.abs(ptok_g - ptok_own) <= 1e-5 * ptok_own + 1e-12).all()
            # (ii) decisions follow bit-exactly from the kernel's own p(x)
            host_ok = (inp["u_acc"][sel] * qtok) < ptok_g
            host_a = np.array([int(np.argmin(np.append(host_ok[i], False))) for i in range(len(sel))])
            assert np.array_equal(a_g, host_a)
            # (iii) equal to the oracle's: a decision can differ only where u*q lies between the two values of
            # p(x), i.e. within the MEASURED deviation of p(x) (near-tie; rare)
            margin = np.abs(inp["u_acc"][sel] * qtok - ptok_w) / np.maximum(ptok_w, 1e-30)
            self.log(f"minimum accept margin {margin.min():.3e}", flush=True)
            clear = (margin > 2 * rel.max() + 1e-6).all(axis=1)
        self.log(f"branches with clear decisions: {int(clear.sum())}/{len(sel)}; accepted {a_w.tolist()}", flush=True)
        assert np.array_equal(a_g[clear], a_w[clear])
        assert np.array_equal(n_g[clear], n_w[clear])
        n_new = n_same = 0
        for i in range(len(sel)):
            a = int(a_g[i])
            assert (out_g[i, n_g[i]:] == -1).all() and np.array_equal(out_g[i, :a], inp["drafts"][sel][i, :a])
            assert n_g[i] == a + 1 if (a < G or T == G + 1) else n_g[i] == G
            if n_g[i] == a:
                continue                                   # every draft accepted, no bonus row: nothing new
            tok = int(out_g[i, a])
            assert 0 <= tok < w.model.vocab
            n_new += 1
            if self.greedy:
                if clear[i] and clear_rows[i, a]:
                    assert tok == out_w[i, a]
                continue
            # the new token (replacement after the first rejection, or the bonus token) against the CDF of the
            # distribution it is drawn from: (iv-a) built from the library's own logits, to 1e-5; (iv-b) the
            # oracle's, widened by the measured distance between the two CDFs, which the logits tolerance bounds
            def weights(p):
                return np.maximum(p[i, a].astype(np.float64) - inp["q"][sel][i, a].astype(np.float64), 0) if a < G \
                    else p[i, a].astype(np.float64)
            ur = float(inp["u_res"][sel][i])
            lo, hi, cdf_own = cdf_band(weights(p_own), tok)
            assert lo - 1e-5 <= ur <= hi + 1e-5, (sel[i], a, tok, lo, ur, hi)
            if clear[i]:
                lo, hi, cdf_ref = cdf_band(weights(self.ref_p), tok)
                delta = float(np.abs(cdf_ref - cdf_own).max()) + 1e-5
                mass = float(weights(self.ref_p).sum())              # small residual mass magnifies the deviation
                assert delta <= 2 * ptol / max(mass, 1e-30) + 1e-5, (delta, mass)
                assert lo - delta <= ur <= hi + delta, (sel[i], a, tok, int(out_w[i, a]), lo, ur, hi, delta)
                n_same += int(tok == out_w[i, a])
        self.log(f"new tokens checked against the CDF band: {n_new} ({n_same} equal to the oracle's draw)", flush=True)
        # Algorithm 1 bookkeeping on the device
        want_len = oracle.commit_lengths(self.plens.copy(), self.gpu_accept[0], T)
        assert np.array_equal(self.gpu_plen, want_len)
        return worst, max_err
