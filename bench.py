#!/usr/bin/env python3
"""Benchmark of the batched target-model verify step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: embedding gather, every
decoder layer (RMSNorm, QKV projection, rotary + KV append, tree-KV attention, O projection, SwiGLU FFN),
final norm, LM head and the fused accept / resample, for N branches x gamma draft tokens.  Inputs (weights,
KV cache, draft distributions, uniforms) are resident in HBM before the timed region starts.

Prints ONE JSON line.  The top level is the HEADLINE workload: c4, the largest verify batch (7B shapes, 16
branches x 6 drafts = 96 rows, 2048-token shared prefix + 128 private tokens per branch):
  metric / value -- verified draft tokens/s per target verify step (N * gamma / step time)
  step           -- whole-step figures: algorithmic bytes / time against the 8 TB/s HBM peak, useful flops
  roofline       -- the dominant kernel, the weight-streaming projection: algorithmic weight bytes per launch /
                    its launch duration (HIP events around every launch on the library's stream, in a pass of
                    its own; the cost of an event pair, calibrated on a kernel of known duration, is subtracted and both
                    figures are given), `achievable` = a pure streaming read measured in the same run
  other_workloads -- the same measurement for c5 (13B, 40 rows) and c3 (7B, 12 rows)
  draft_step     -- workload c2: gamma batched autoregressive steps of the small draft model (draft tokens/s)
  batch_sweep    -- c7 / c8: the headline shapes with 64 / 128 branches (384 / 768 rows), useful MFMA fraction
  cpu_baseline   -- the float64 numpy oracle timed on this host's cores on a bounded sample of the headline
                    workload: three of its sixteen branches at full depth (branches are independent), nothing
                    extrapolated.
`--workload X --no-others` measures X alone (the form the profiles under profiles/ are taken with); c7 and c8
(64 and 128 branches x 6 drafts: 384 and 768 rows) are the batch sweep past the matrix-core ridge.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16

# HBM bytes per projection launch from rocprofv3 --pmc runs of this file (FETCH_SIZE, WRITE_SIZE scaled by a
# copy kernel of known size): the figures of the summaries under profiles/, not measured in this run.
PROFILED_TRAFFIC_BYTES = {"c3": (106.4e6, "profiles/gemm_kernel_c3.md"),
                          "c4": (132.5e6, "profiles/verify_step_c4_c5.md"),
                          "c5": (177.7e6, "profiles/verify_step_c4_c5.md"),
                          "c6": (112.0e6, "profiles/verify_step_c6.md")}


def wl_private_lens(w):
    import workloads
    return workloads.private_lens(w)


def algorithmic_bytes(w):
    """Bytes one verify step must move: every weight once, the KV context once, logits and q once."""
    m = w.model
    es = 4 if m.dtype == "fp32" else 2
    # one-byte weights: e4m3 codes (+ a scale per row); four-bit weights: MXFP4 codes + a scale byte per 32
    weights = int(m.params * {"bf16w8": 1.0, "bf16w4": 0.53125}.get(m.dtype, es))
    kv_tok = 2 * m.n_heads * m.head_dim * es * m.n_layers
    kv = (w.S + int(wl_private_lens(w).sum())) * kv_tok
    M = w.N * w.gamma
    other = M * m.vocab * 4 * 2 + w.N * w.gamma * m.vocab * 4 + M * kv_tok   # logits w+r, q read, new KV
    return weights + kv + other, weights


def useful_flops(w):
    m = w.model
    M = w.N * w.gamma
    gemm = 2.0 * M * m.params
    attn = 4.0 * w.gamma * float((w.S + wl_private_lens(w) + (w.gamma + 1) / 2).sum()) * m.n_heads * m.head_dim * m.n_layers
    return gemm + attn


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline(w, inp, branches):
    """The oracle as it stands on `branches` of the workload at full depth: forward over their rows, softmax,
    accept / resample.  Weights and synthetic KV are generated layer by layer as the oracle asks for them; the
    time spent generating them (input preparation, not the method) is measured and left out."""
    import numpy as np
    import oracle
    import workloads as wl
    W = wl.Weights(w.model, w.seed, reuse_buffers=True)
    gen_s = [0.0]

    def timed(fn):
        def f(*a):
            t = time.perf_counter()
            r = fn(*a)
            gen_s[0] += time.perf_counter() - t
            return r
        return f

    class Gen:
        tok_emb, norm_final, lm_head, layer = (staticmethod(timed(getattr(W, n))) for n in
                                               ("tok_emb", "norm_final", "lm_head", "layer"))
    plens = wl.private_lens(w)
    kv_of = timed(lambda l: wl.synthetic_kv(w, l))

    def ctx(l):
        k_s, v_s, k_p, v_p = kv_of(l)
        t = time.perf_counter()
        out = [(np.concatenate([k_s, k_p[b][:, :plens[b]]], 1), np.concatenate([v_s, v_p[b][:, :plens[b]]], 1))
               for b in branches]
        gen_s[0] += time.perf_counter() - t
        return out
    sel = list(branches)
    t0 = time.perf_counter()
    logits = oracle.verify_forward(w.model, Gen, inp["row_tok"][sel], ctx, [w.S + int(plens[b]) for b in sel])
    p = oracle.softmax_temperature(logits, w.temperature)
    oracle.accept_resample(p, inp["q"][sel], inp["drafts"][sel], inp["u_acc"][sel], inp["u_res"][sel])
    total = time.perf_counter() - t0
    t = total - gen_s[0]
    return {"value": len(sel) * w.gamma / t, "unit": "tokens/s", "cores": host_threads(), "kind": "oracle",
            "seconds": t,
            "sample": f"float64 numpy oracle on branches {sel} of the {w.N} of workload {w.name} ({len(sel) * w.gamma} of "
                      f"{w.N * w.gamma} rows), all {w.model.n_layers} layers + LM head + accept: {t:.1f} s of oracle "
                      f"arithmetic ({gen_s[0]:.1f} s of seeded input generation left out); nothing extrapolated"}


def scheduled(args):
    """End-to-end rounds-scheduled execution (paper Section 3.3 / Algorithm 1) on synthetic models: target =
    the workload's model, draft = the c2-shaped model with the same vocabulary, both random-init; for each
    unit size (branches drafted and verified together) the validated tokens per second of the whole run."""
    import numpy as np
    import torch
    import workloads as wl
    from workloads import gen
    from workloads.device import UploadingWeights, make_context, i32
    import paper_2406_18200_amd as sv
    dev = "cuda:0"
    wt = wl.get_workload(args.workload)
    if args.layers:
        wt = wt.scaled(n_layers=args.layers)
    wd = wl.get_workload("c2").scaled(N=wt.N, gamma=wt.gamma, S=wt.S, vocab=wt.model.vocab)
    n, G, L = wt.N, wt.gamma, args.scheduled
    prefix = wl.prefix_tokens(wt)
    first = gen.pending_tokens(wt)
    s_t, s_d = torch.cuda.Stream(), torch.cuda.Stream()
    with torch.cuda.stream(s_t):
        up = UploadingWeights(wt.model, wt.seed, dev)
        tctx = make_context(wt.model, up.upload_all(), max_branches=n, max_rows_per_branch=G, max_shared=wt.S,
                            max_private=L + 2 * G, device=dev)
        del up
        torch.cuda.empty_cache()
        tctx.prefill_shared(i32(prefix, dev))
    with torch.cuda.stream(s_d):
        upd = UploadingWeights(wd.model, wd.seed, dev, reuse_buffers=False)
        dctx = make_context(wd.model, upd.upload_all(), max_branches=n, max_rows_per_branch=max(1, 128 // n),
                            max_shared=wd.S, max_private=L + 2 * G, device=dev)
        dctx.prefill_shared(i32(prefix, dev))
    torch.cuda.synchronize()
    ud, ua, ur = sv.uniform_philox(wt.seed + 9, (3, n, L + G), device=dev)     # generated on the device: never crosses the host link
    units = sorted({n, max(1, (n + 1) // 2), 1}, reverse=True)
    results, ref = {}, None
    for unit in units:
        best = None
        for rep in range(3):                              # first repetition warms up
            plen_t = torch.zeros(n, dtype=torch.int32, device=dev)
            plen_d = torch.zeros(n, dtype=torch.int32, device=dev)
            toks, lens, st = sv.sched_run(tctx, dctx, first, ud, ua, ur, plen_t, plen_d, gamma=G, max_new=L,
                                          temperature=wt.temperature, shared_len_target=wt.S, shared_len_draft=wd.S,
                                          unit_branches=unit)
            assert (lens == L).all()
            if rep and (best is None or st["wall_ms"] < best["wall_ms"]):
                best = st
        ref = toks if ref is None else ref
        best["same_tokens_as_first_unit_size"] = bool(np.array_equal(toks, ref))
        best["tokens_per_s"] = n * L / (best["wall_ms"] * 1e-3)
        results[f"unit_{unit}"] = best
    print(json.dumps({"metric": "validated tokens/s, rounds-scheduled execution (Algorithm 1), end to end",
                      "unit": "tokens/s", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"{wt.name} target + c2-shaped draft model, N={n} branches, gamma={G}, "
                                             f"{L} validated tokens per branch, shared prefix S={wt.S}"},
                      "results": results}), flush=True)


def describe(w, greedy=False):
    m = w.model
    return (f"{w.name}: {m.n_layers}-layer d={m.d_model} H={m.n_heads} F={m.d_ff} V={m.vocab} decoder, N={w.N} branches x "
            f"gamma={w.gamma} drafts, shared prefix S={w.S}, private R={w.R}"
            + (f" (ragged, {w.R_min}..{w.R})" if w.R_min >= 0 else "") + f", temperature {w.temperature}"
            + (" (greedy)" if greedy else ""))


def timed_loop(fn, steps, warmup):
    """W untimed calls, then exactly K timed ones between two events on the current stream (the library's),
    with a device synchronisation on both sides.  Returns (ms per call, wall ms per call)."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps, (time.perf_counter() - t0) * 1e3 / steps


def read_ceiling_gbs(dev, gib=4):
    """A pure streaming read of a buffer much larger than the last-level cache, timed in this run."""
    import torch
    import paper_2406_18200_amd as sv
    buf = torch.empty(gib << 30, dtype=torch.uint8, device=dev)
    buf.zero_()
    ms, _ = timed_loop(lambda: sv.binding.hbm_read_probe(buf), 10, 3)
    n = buf.numel()
    del buf
    torch.cuda.empty_cache()
    return n / (ms * 1e-3) / 1e9


def measure_verify(w, args, dev, with_inputs=False):
    """Builds the workload on the device, times the verify step, then the projection launches in a pass of
    their own.  Returns the result dict (and the host-side inputs for the CPU baseline)."""
    import numpy as np
    import torch
    import workloads as wl
    from workloads import gen
    from workloads.device import UploadingWeights, make_context, f32, i32, to_device
    m = w.model
    G, N, T = w.gamma, w.N, w.gamma
    t_setup = time.time()
    # ---- synthetic inputs, resident on the device -------------------------------------------------
    up = UploadingWeights(m, w.seed, dev, device_quantize=True)
    dw = up.upload_all()
    ctx = make_context(m, dw, max_branches=N, max_rows_per_branch=T, max_shared=max(w.S, 1), max_private=w.R, device=dev)
    del dw, up
    torch.cuda.empty_cache()
    for l in range(m.n_layers):
        k_s, v_s, k_p, v_p = wl.synthetic_kv(w, l)
        ctx.kv_load(l, *(to_device(a, m, dev) if a.size else None for a in (k_s, v_s, k_p, v_p)))
    q = None if w.q_kind == "perturbed" else wl.random_draft_q(w)
    pending = gen.pending_tokens(w)
    plen0 = i32(wl.private_lens(w), dev)        # all R, or ragged (state-evaluator shape)
    plen = plen0.clone()
    if q is None:
        # q_j = softmax((target logits_j + noise) / temp), drafts sampled autoregressively (timing run: the
        # target logits come from the library itself, one step per draft position)
        q = np.zeros((N, G, m.vocab), np.float32)
        drafts = np.zeros((N, G), np.int32)
        u_d = wl.uniform24(w.seed + 3, (N, G))
        rows = pending[:, None].astype(np.int32)
        for j in range(G):
            lg = torch.empty((N, j + 1, m.vocab), dtype=torch.float32, device=dev)
            ctx.step(i32(rows, dev), w.S, plen, logits_out=lg)        # pending token + drafts so far, nothing committed
            ell = lg[:, j].cpu().numpy()
            for b in range(N):
                q[b, j] = wl.perturbed_draft_q(w, ell[b], b, j)
            drafts[:, j] = wl.draw_tokens(q[:, j], u_d[:, j])
            rows = np.concatenate([rows, drafts[:, j:j + 1]], axis=1).astype(np.int32)
    else:
        drafts = wl.draw_tokens(q, wl.uniform24(w.seed + 3, (N, G)))
    row_tok = np.concatenate([pending[:, None], drafts[:, :T - 1]], axis=1).astype(np.int32)
    u_acc = wl.uniform24(w.seed + 4, (N, G))
    u_res = wl.uniform24(w.seed + 4, (N,), stream=1)
    inp = dict(q=q, drafts=drafts, row_tok=row_tok, u_acc=u_acc, u_res=u_res)
    d_row = i32(row_tok, dev)
    acc = dict(q=None if args.greedy else f32(q, dev), draft_tok=i32(drafts, dev),
               u_acc=None if args.greedy else f32(u_acc, dev), u_res=None if args.greedy else f32(u_res, dev),
               temperature=w.temperature, greedy=args.greedy)
    flags = 2 if args.greedy else 0
    torch.cuda.synchronize()
    print(f"[bench] setup {time.time() - t_setup:.1f}s; workload {w.name}: N={N} gamma={G} S={w.S} R={w.R} "
          f"L={m.n_layers} d={m.d_model}", file=sys.stderr, flush=True)
    outs = [None]

    def one_step():
        plen.copy_(plen0)                    # every step sees the same context lengths
        outs[0] = ctx.step(d_row, w.S, plen, flags=flags, accept=acc)

    if args.copy_probe_mb:
        src = torch.empty(args.copy_probe_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ms_per_step, wall_ms = timed_loop(one_step, args.steps, args.warmup)
    accepted = int(outs[0][0].sum().item())
    assert ctx.status() == 0

    # ---- dominant kernel: separate pass with HIP events around every projection launch ---------------
    ev_us = ctx.profile_overhead(500) * 1e3
    ctx.profile_enable(True)
    for _ in range(args.steps):
        one_step()
    launches, gemm_ms, gemm_bytes = ctx.profile_read()
    ctx.profile_enable(False)
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    raw_us = gemm_ms * 1e3 / max(launches, 1)
    kern_us = max(raw_us - ev_us, 1e-3)
    bytes_per_launch = gemm_bytes / max(launches, 1)
    gemm_gbs = bytes_per_launch / (kern_us * 1e-6) / 1e9
    total_bytes, weight_bytes = algorithmic_bytes(w)
    step_gbs = total_bytes / (ms_per_step * 1e-3) / 1e9
    flops = useful_flops(w)
    traffic = PROFILED_TRAFFIC_BYTES.get(w.name, (None, None))
    res = {
        "value": N * G / (ms_per_step * 1e-3), "ms_per_step": ms_per_step,
        "config": {"workload": describe(w, args.greedy), "global_batch": N * G, "seq_len": w.S + w.R + G,
                   "parallelism": "single-gpu"},
        "step": {"algorithmic_bytes": total_bytes, "hbm_GBs": step_gbs, "hbm_frac": step_gbs / HBM_PEAK_GBS,
                 "useful_tflops": flops / (ms_per_step * 1e-3) / 1e12,
                 "mfma_frac": flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                 "mfma_frac_ceiling_at_hbm_peak": min(1.0, N * G / (MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9))),
                 "accepted_tokens": accepted, "wall_ms_per_step": wall_ms},
        "roofline": {"bound": "hbm", "kernel": "gemm_kernel / gemm_wide_kernel (weight-streaming projection)",
                     "achieved": gemm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gemm_gbs / HBM_PEAK_GBS,
                     "traffic": traffic[0], "traffic_source": traffic[1],
                     "launches_per_step": launches / args.steps, "bytes_per_launch": bytes_per_launch,
                     "avg_launch_us": kern_us, "avg_launch_us_between_events": raw_us, "event_pair_us": ev_us,
                     "frac_between_events": bytes_per_launch / (raw_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                     "kernel_share_of_step": kern_us * launches / args.steps / (ms_per_step * 1e3)},
    }
    return (res, inp) if with_inputs else res


def measure_draft(args, dev):
    """Workload c2: gamma autoregressive seed_draft_step calls for N branches of the small draft model from a
    shared prefix (true-prefix protocol: the library computes the prefix KV itself)."""
    import torch
    import workloads as wl
    from workloads import gen
    from workloads.device import UploadingWeights, make_context, f32, i32
    w = wl.get_workload("c2")
    m, N, G = w.model, w.N, w.gamma
    up = UploadingWeights(m, w.seed, dev, reuse_buffers=False)
    ctx = make_context(m, up.upload_all(), max_branches=N, max_rows_per_branch=max(1, 128 // N), max_shared=w.S,
                       max_private=G + 1, device=dev)
    del up
    ctx.prefill_shared(i32(wl.prefix_tokens(w), dev))
    plen = torch.zeros(N, dtype=torch.int32, device=dev)
    u = f32(wl.uniform24(w.seed + 4, (G, N)), dev)
    q = torch.zeros((N, G, m.vocab), dtype=torch.float32, device=dev)
    tok = torch.zeros((G + 1, N), dtype=torch.int32, device=dev)   # row j feeds step j, which writes row j + 1
    tok[0] = i32(gen.pending_tokens(w), dev)

    def draft_round():
        plen.zero_()
        for j in range(G):
            ctx.draft_step(tok[j], w.S, plen, u[j], w.temperature, q_out=q[:, j], tok_out=tok[j + 1],
                           q_stride=q.stride(0), tok_stride=1)
    ms, wall = timed_loop(draft_round, max(10, args.steps), max(3, args.warmup))
    assert ctx.status() == 0
    ctx.close()
    es = 2
    weights = m.params * es
    kv_tok = 2 * m.n_heads * m.head_dim * es * m.n_layers
    step_bytes = weights + (w.S + N * (G - 1) / 2) * kv_tok + N * m.vocab * 4 * 3      # logits w + r, q row written
    us_step = ms * 1e3 / G
    return {"config": {"workload": f"c2: {m.n_layers}-layer d={m.d_model} H={m.n_heads} F={m.d_ff} V={m.vocab} draft model, "
                                   f"N={N} branches x {G} autoregressive steps, shared prefix S={w.S}, temperature {w.temperature}"},
            "metric": "draft tokens/s", "value": N * G / (ms * 1e-3), "unit": "tokens/s", "us_per_draft_step": us_step,
            "wall_us_per_draft_step": wall * 1e3 / G, "algorithmic_bytes_per_step": step_bytes,
            "hbm_frac": step_bytes / (us_step * 1e-6) / 1e9 / HBM_PEAK_GBS,
            "note": "87 MB of weights: resident in the 256 MB last-level cache after the first step; latency-bound"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c4", choices=["c2", "c3", "c4", "c5", "c6", "c7", "c8"],
                    help="the headline workload (default c4: the largest verify batch)")
    ap.add_argument("--no-others", action="store_true", help="measure the headline workload only (profiling runs)")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only; "
                    "the reported number is then NOT the benchmark configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--w8", action="store_true", help="also time c3 and c5 with the projection matrices as one-byte "
                    "e4m3 codes + per-row scales (context dtype bf16w8): reported under fp8_weights, never as the headline")
    ap.add_argument("--w4", action="store_true", help="the same with MXFP4 weights (E2M1 codes + a power-of-two scale per "
                    "32 inputs, context dtype bf16w4): reported under fp4_weights")
    ap.add_argument("--greedy", action="store_true")
    ap.add_argument("--copy-probe-mb", type=int, default=0, help="also launch a plain device-to-device copy "
                    "of this many MiB (three times) before the timed region: the known-size kernel against "
                    "which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--scheduled", type=int, default=0, metavar="L",
                    help="instead of the verify-step benchmark: run Algorithm 1 end to end (rounds-scheduled "
                         "execution, L validated tokens per branch, draft model of the c2 shape) for several unit "
                         "sizes and print one JSON line with validated tokens/s for each")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    if args.scheduled:
        if args.workload == "c4" and "--workload" not in sys.argv:
            args.workload = "c3"
        return scheduled(args)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    if args.workload == "c2":                       # the draft-model step alone (profiling runs)
        print(json.dumps(measure_draft(args, dev)), flush=True)
        return
    w = wl.get_workload(args.workload)
    if args.layers:
        w = w.scaled(n_layers=args.layers)
    head, inp = measure_verify(w, args, dev, with_inputs=True)
    out = {"metric": "verified draft tokens/s per target verify step", "value": head["value"], "unit": "tokens/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32" if w.model.dtype == "fp32" else "bf16", "data": "synthetic", "config": head["config"],
           "step": head["step"], "roofline": head["roofline"]}
    if not args.no_others:
        out["roofline"]["achievable"] = read_ceiling_gbs(dev)
        out["roofline"]["achievable_note"] = "pure streaming read of 4 GiB (seed_hbm_read_probe), GB/s, this run"
        others = {}
        for name in ("c5", "c3"):
            if name == w.name:
                continue
            wo = wl.get_workload(name)
            if args.layers:
                wo = wo.scaled(n_layers=args.layers)
            r = measure_verify(wo, args, dev)
            r.update(metric=out["metric"], unit="tokens/s")
            others[name] = r
        out["other_workloads"] = others
        out["draft_step"] = measure_draft(args, dev)
        # batch sweep past 128 rows (64 and 128 branches): where the step turns from memory- to MFMA-bound
        if w.name == "c4" and not args.layers:
            sweep = {}
            few = argparse.Namespace(**{**vars(args), "steps": max(5, args.steps // 5), "warmup": max(2, args.warmup // 5)})
            for name in ("c7", "c8"):
                r = measure_verify(wl.get_workload(name), few, dev)
                sweep[name] = {"rows": r["config"]["global_batch"], "value": r["value"], "unit": "tokens/s",
                               "ms_per_step": r["ms_per_step"], "steps": few.steps, "warmup": few.warmup,
                               "useful_mfma_frac": r["step"]["mfma_frac"], "useful_tflops": r["step"]["useful_tflops"],
                               "config": r["config"]}
            out["batch_sweep"] = sweep
    if args.w8:
        out["fp8_weights"] = {}
        for name in ("c3", "c5"):
            r = measure_verify(wl.get_workload(name).scaled(dtype="bf16w8"), args, dev)
            r.update(metric=out["metric"], unit="tokens/s", note="weights as e4m3 codes + per-row scales; a different "
                     "precision from the bf16 headline (tests/test_gpu_w8.py and test_gpu_w4.py print the formats' error against the bf16 weights)")
            out["fp8_weights"][name] = r
    if args.w4:
        out["fp4_weights"] = {}
        for name in ("c3", "c5"):
            r = measure_verify(wl.get_workload(name).scaled(dtype="bf16w4"), args, dev)
            r.update(metric=out["metric"], unit="tokens/s", note="weights as MXFP4 codes + block scales; a different "
                     "precision from the bf16 headline (tests/test_gpu_w8.py and test_gpu_w4.py print the formats' error against the bf16 weights)")
            out["fp4_weights"][name] = r
    if not args.no_cpu_baseline:
        sample = [0, w.N // 2, w.N - 1] if w.N > 3 else list(range(w.N))
        out["cpu_baseline"] = cpu_baseline(w, inp, sorted(set(sample)))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
