#!/usr/bin/env python3
"""Benchmark of the batched target-model verify step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: embedding gather, every
decoder layer (RMSNorm, QKV projection, rotary + KV append, tree-KV attention, O projection, SwiGLU FFN),
final norm, LM head and the fused accept / resample, for N branches x gamma draft tokens.  Inputs (weights,
KV cache, draft distributions, uniforms) are resident in HBM before the timed region starts.

Prints ONE JSON line: metric = verified draft tokens/s per target verify step (N * gamma / step time), plus
  roofline     -- the weight-streaming projection kernel: algorithmic weight bytes / its measured duration
                  (HIP events around every launch, taken in a separate pass) against the 8 TB/s HBM peak
  cpu_baseline -- the float64 numpy oracle timed on this host's cores on a bounded sample of the same
                  workload (one and two decoder layers + LM head + accept), extrapolated to all layers.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per projection launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE scaled by a copy
# kernel of known size); see profiles/.  None until measured for that workload.
MEASURED_TRAFFIC_BYTES = {"c3": 106.3e6,     # profiles/gemm_kernel_c3.md: 2 x 51,667 KiB fetched + 521 KiB written
                          "c4": 135.7e6,     # profiles/verify_step_c4_c5.md: 2 x 61,258 KiB + 9,981 KiB
                          "c5": 177.7e6,     # profiles/verify_step_c4_c5.md: 2 x 84,570 KiB + 4,399 KiB
                          "c6": 112.0e6}     # profiles/verify_step_c6.md: 2 x 53,528 KiB + 2,347 KiB


def wl_private_lens(w):
    import workloads
    return workloads.private_lens(w)


def algorithmic_bytes(w):
    """Bytes one verify step must move: every weight once, the KV context once, logits and q once."""
    m = w.model
    es = 2 if m.dtype == "bf16" else 4
    weights = m.params * es
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


def cpu_baseline(w, inp):
    """Oracle on a bounded sample: same widths, N, gamma, S, R; 4 and 20 decoder layers; extrapolated."""
    import numpy as np
    import oracle
    import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    # two depths of the same model (same widths, N, gamma, context), ~10 s of oracle arithmetic together
    L_small, L_big = min(4, w.model.n_layers), min(20, w.model.n_layers)
    wb = w.scaled(n_layers=L_big)
    W = wl.Weights(wb.model, wb.seed)
    cache = {"emb": W.tok_emb(), "nf": W.norm_final(), "lm": W.lm_head(),
             "layers": [W.layer(l) for l in range(L_big)], "kv": [wl.synthetic_kv(wb, l) for l in range(L_big)]}

    class Pre:       # pre-generated tensors: the timed region holds only the oracle's own arithmetic
        tok_emb = staticmethod(lambda: cache["emb"])
        norm_final = staticmethod(lambda: cache["nf"])
        lm_head = staticmethod(lambda: cache["lm"])
        layer = staticmethod(lambda l: cache["layers"][l])

    def ctx(l):
        k_s, v_s, k_p, v_p = cache["kv"][l]
        return [(np.concatenate([k_s, k_p[b][:, :plens[b]]], 1), np.concatenate([v_s, v_p[b][:, :plens[b]]], 1))
                for b in range(w.N)]
    plens = wl.private_lens(w)
    times = {}
    for L in sorted({L_small, L_big}):
        ws = w.scaled(n_layers=L)
        t0 = time.perf_counter()
        logits = oracle.verify_forward(ws.model, Pre, inp["row_tok"], ctx, [ws.S + int(r) for r in plens])
        p = oracle.softmax_temperature(logits, ws.temperature)
        oracle.accept_resample(p, inp["q"], inp["drafts"], inp["u_acc"], inp["u_res"])
        times[L] = time.perf_counter() - t0
    if L_big > L_small:
        per_layer = max((times[L_big] - times[L_small]) / (L_big - L_small), 1e-9)
    else:
        per_layer = times[L_big] / L_big
    fixed = max(times[L_small] - per_layer * L_small, 0.0)
    full = fixed + per_layer * w.model.n_layers
    return {"value": w.N * w.gamma / full, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"float64 numpy oracle, full widths/N/gamma/context, timed at {L_small} and {L_big} layers "
                      f"({times[L_small]:.2f}s, {times[L_big]:.2f}s) + LM head + accept, extrapolated to "
                      f"{w.model.n_layers} layers ({full:.1f}s per step)"}


def scheduled(args):
    """End-to-end rounds-scheduled execution (paper Section 3.3 / Algorithm 1) on synthetic models: target =
    the workload's model, draft = the c2-shaped model with the same vocabulary, both random-init; for each
    unit size (branches drafted and verified together) the validated tokens per second of the whole run."""
    import numpy as np
    import torch
    import workloads as wl
    from workloads import gen
    from workloads.device import UploadingWeights, make_context, f32, i32
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3", choices=["c3", "c4", "c5", "c6"])
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only; "
                    "the reported number is then NOT the benchmark configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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

    import numpy as np
    import torch
    import workloads as wl
    from workloads import gen
    from workloads.device import UploadingWeights, make_context, f32, i32, to_device
    if args.scheduled:
        return scheduled(args)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    w = wl.get_workload(args.workload)
    if args.layers:
        w = w.scaled(n_layers=args.layers)
    m = w.model
    G, N, T = w.gamma, w.N, w.gamma
    t_setup = time.time()

    # ---- synthetic inputs, resident on the device -------------------------------------------------
    up = UploadingWeights(m, w.seed, dev)
    dw = up.upload_all()
    ctx = make_context(m, dw, max_branches=N, max_rows_per_branch=T, max_shared=max(w.S, 1), max_private=w.R, device=dev)
    del dw, up
    torch.cuda.empty_cache()
    for l in range(m.n_layers):
        k_s, v_s, k_p, v_p = wl.synthetic_kv(w, l)
        ctx.kv_load(l, *(to_device(a, m, dev) if a.size else None for a in (k_s, v_s, k_p, v_p)))
    if w.q_kind == "perturbed":
        q = None      # built below from the target's own logits
    else:
        q = wl.random_draft_q(w)
    pending = gen.pending_tokens(w)
    plen0 = i32(wl.private_lens(w), dev)        # all R, or ragged (state-evaluator shape)
    plen = plen0.clone()
    if q is None:
        # q_j = softmax((target logits_j + noise) / temp), drafts sampled autoregressively (timing run: the
        # target logits come from the library itself, one single-row step per draft position)
        q = np.zeros((N, G, m.vocab), np.float32)
        drafts = np.zeros((N, G), np.int32)
        u_d = wl.uniform24(w.seed + 3, (N, G))
        cur = pending.copy()
        lg = torch.empty((N, 1, m.vocab), dtype=torch.float32, device=dev)
        for j in range(G):
            ctx.step(i32(cur[:, None], dev), w.S, plen, flags=4, logits_out=lg)   # COMMIT_ALL: keep the row
            ell = lg.cpu().numpy()[:, 0]
            for b in range(N):
                q[b, j] = wl.perturbed_draft_q(w, ell[b], b, j)
            drafts[:, j] = wl.draw_tokens(q[:, j], u_d[:, j])
            cur = drafts[:, j].copy()
        plen.copy_(plen0)
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

    def one_step():
        plen.copy_(plen0)                    # every step sees the same context lengths
        return ctx.step(d_row, w.S, plen, flags=flags, accept=acc)

    if args.copy_probe_mb:
        src = torch.empty(args.copy_probe_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        outs = one_step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        outs = one_step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = e0.elapsed_time(e1) / args.steps
    accepted = int(outs[0].sum().item())

    # ---- dominant kernel: separate pass with HIP events around every projection launch ---------------
    ctx.profile_enable(True)
    for _ in range(args.steps):
        one_step()
    launches, gemm_ms, gemm_bytes = ctx.profile_read()
    ctx.profile_enable(False)
    gemm_gbs = gemm_bytes / (gemm_ms * 1e-3) / 1e9 if gemm_ms > 0 else 0.0

    total_bytes, weight_bytes = algorithmic_bytes(w)
    tokens_per_s = N * G / (ms_per_step * 1e-3)
    step_gbs = total_bytes / (ms_per_step * 1e-3) / 1e9
    flops = useful_flops(w)
    out = {
        "metric": "verified draft tokens/s per target verify step",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if m.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {m.n_layers}-layer d={m.d_model} H={m.n_heads} F={m.d_ff} V={m.vocab} "
                               f"decoder, N={N} branches x gamma={G} drafts, shared prefix S={w.S}, "
                               f"private R={w.R}" + (f" (ragged, {w.R_min}..{w.R})" if w.R_min >= 0 else "") + f", temperature {w.temperature}" + (" (greedy)" if args.greedy else ""),
                   "global_batch": N * G, "seq_len": w.S + w.R + G, "parallelism": "single-gpu"},
        "step": {"algorithmic_bytes": total_bytes, "hbm_GBs": step_gbs, "hbm_frac": step_gbs / HBM_PEAK_GBS,
                 "useful_tflops": flops / (ms_per_step * 1e-3) / 1e12,
                 "mfma_frac": flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                 "accepted_tokens": accepted, "wall_ms_per_step": wall_ms / args.steps},
        "roofline": {"bound": "hbm", "kernel": "gemm_kernel / gemm_wide_kernel (weight-streaming projection)",
                     "achieved": gemm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gemm_gbs / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
                     "launches_per_step": launches / args.steps,
                     "avg_launch_us": gemm_ms * 1e3 / max(launches, 1),
                     "bytes_per_launch": gemm_bytes / max(launches, 1),
                     "kernel_share_of_step": gemm_ms / args.steps / ms_per_step},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
