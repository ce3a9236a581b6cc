#!/usr/bin/env python3
"""Benchmark of the verification step (Alg. 2 step 2 + KV append / rollback, Sec. IV-C) on one MI355X.

One step = one fsv_verify() call on the 8B-shape, batch-16 workload (ragged gamma 1..8, contexts
512..4096, paged KV, temperature 0.8): target forward over every request's pending token and
drafts, acceptance tests, correction / bonus token, rollback.  All inputs are resident in HBM
before the timed region.  Prints ONE JSON line: metric / value / ms_per_step, a `roofline` object for the dominant
kernel (gate|up GEMM: algorithmic bytes over its measured duration against the 8 TB/s HBM peak, plus counter-measured
traffic) and a `cpu_baseline` object (the oracle timed on one request of the same workload).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "verify_c3_8b_b16_hbm_traffic.txt")


def counter_traffic(workload: str, seed: int, rows: int):
    """HBM bytes one launch of the dominant kernel (gate|up GEMM) moves, from the tracked rocprofv3 --pmc summary.

    The summary carries one machine-readable line ("# bench: key=value ...") with the mean FETCH_SIZE / WRITE_SIZE counts
    per dispatch of that kernel, the KiB each count stands for (from the same counters on a plain copy of known size) and
    the workload, seed and row count it was taken on.  Returns None when the file is missing or was taken on another
    workload: the figure is never a constant of this script."""
    try:
        with open(TRAFFIC_PROFILE) as f:
            line = next(l for l in f if l.startswith("# bench:"))
        kv = dict(t.split("=", 1) for t in line[len("# bench:"):].split())
        if kv["workload"] != workload or int(kv["seed"]) != seed or int(kv["rows"]) != rows:
            return None
        return (float(kv["fetch_counts"]) * float(kv["fetch_kib_per_count"]) +
                float(kv["write_counts"]) * float(kv["write_kib_per_count"])) * 1024.0
    except (OSError, StopIteration, KeyError, ValueError):
        return None


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def cpu_baseline(cfg, wl, req, weights, seed, budget_rows=9):
    """The oracle, as it stands, verifying ONE request of the same workload on the host cores.

    The request's drafts and draft laws are produced by stepping the oracle itself (untimed), so the
    oracle consumes nothing the GPU library computed; only its verify call is timed.
    """
    import torch
    from oracle import oracle
    from paper_2601_00644_amd import synth
    # the request with the most drafts that still fits the row budget (about 10-30 s of CPU work at 8B shapes)
    cand = [b for b in range(req.batch) if 1 <= int(req.gammas[b]) + 1 <= budget_rows]
    if not cand:
        cand = [int(np.argmin(req.gammas))]
    b = max(cand, key=lambda i: (int(req.gammas[i]), -int(req.seq_lens[i])))
    L, g, o = int(req.seq_lens[b]), int(req.gammas[b]), int(req.draft_offsets[b])
    t0 = time.time()
    wn = synth.weights_to_numpy(cfg, weights)
    k, v = synth.make_kv_context(cfg, L, seed, b, device="cuda")
    kc, vc = oracle.new_cache(cfg, L + g + 1)
    kc[:, :L] = synth.kv_to_f64(k)
    vc[:, :L] = synth.kv_to_f64(v)
    del k, v
    log(f"cpu_baseline: request {b} (L={L}, gamma={g}); host copies ready in {time.time() - t0:.1f}s")
    tok, T = int(req.last_token[b]), float(req.temperature[b])
    q = np.zeros((g, cfg.vocab), np.float32)
    d = np.zeros(g, np.int32)
    k2, v2 = kc.copy(), vc.copy()
    for i in range(g):
        lg = oracle.forward(cfg, wn, k2, v2, L + i, np.array([tok], np.int32))[0]
        qi = synth.draft_law(torch.from_numpy(lg), T, wl.sigma, seed, o + i)
        tok = synth.draw_from(qi, float(req.u_draft[o + i]))
        q[i], d[i] = qi.numpy(), tok
    del k2, v2
    log(f"cpu_baseline: drafts stepped by the oracle in {time.time() - t0:.1f}s; timing its verify call")
    t1 = time.time()
    r = oracle.verify(cfg, wn, kc, vc, L, int(req.last_token[b]), d, q, req.u_accept[o:o + g], float(req.u_sample[b]), T)
    dt = time.time() - t1
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    log(f"cpu_baseline: {g} drafts verified in {dt:.2f}s (tau={r.sample.tau}) on {cores} threads")
    return {"value": g / dt, "unit": "verified draft tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"ONE request of the batch, not scaled to the batch: request {b} alone (context {L}, gamma {g}, "
                      f"{g + 1} rows) verified in {dt:.2f} s; the value is its {g} drafts over that time"}


def sampler_bench(args, torch, fv, synth):
    """The accept / resample step alone (fsv_sample) at the sampling configuration: batch 64, ragged gamma 1..16,
    vocabulary 152064, bf16 logits ~ N(0,3), draft laws from logits noised with sigma 0.7, temperature 0.7."""
    V, B, sigma, T = 152064, 64, 0.7, 0.7
    log("workload c4_sampler: generating logits and draft laws on the device")
    case = synth.make_sampler_case(B, 1, 16, V, sigma, T, args.seed, logits_dtype="bf16", device="cuda")
    G, M = int(case.draft_offsets[-1]), int(case.draft_offsets[-1]) + B
    cfg = synth.ModelCfg("sampler", 0, 0, 0, 0, 0, 0, V, "bf16")
    ctx = fv.Context(cfg, None, B, 16, sampler_only=True)
    t = lambda a: torch.as_tensor(np.ascontiguousarray(a), device="cuda")
    batch = fv.DeviceBatch(None, None, t(case.draft_offsets), t(case.draft_tokens), case.draft_probs, t(case.u_accept),
                           t(case.u_sample), t(case.temperature), None, None, None, 0, None,
                           np.ascontiguousarray(case.draft_offsets), np.ascontiguousarray(case.temperature))
    if args.top_p < 1.0:
        batch.top_p_host = np.full(B, args.top_p, np.float32)
        batch.top_p = t(batch.top_p_host)
    res = fv.DeviceResult.alloc(B)
    for _ in range(args.warmup):
        ctx.sample(case.logits, batch, res)
    torch.cuda.synchronize()
    ctx.profile_read()
    # every eighth call carries event pairs (an event-carrying dispatch leaves the GPU idle for some microseconds around it)
    ctx.profile_enable(["sample_stats", "sample_nucleus", "sample_decide"], every=8)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        ctx.sample(case.logits, batch, res)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    dom = prof["sample_stats"]
    dom_ms, dom_bytes = dom["total_ms"] / dom["launches"], dom["bytes"] / dom["launches"]
    tau = res.accepted_len.cpu().numpy()
    out = {"metric": "verified draft tokens/sec on 1 MI355X (rejection sampling alone, vocabulary 152064, batch 64)",
           "value": G / (ms * 1e-3), "unit": "verified draft tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": "c4_sampler", "batch": B, "drafts": G, "rows": M, "vocab": V, "temperature": T,
                      "top_p": args.top_p,
                      "draft_noise_sigma": sigma, "accepted_drafts": int(tau.sum())},
           "roofline": {"bound": "hbm", "kernel": "k_row_stats (one pass over every logits row)",
                        "achieved": dom_bytes / (dom_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": dom_bytes / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                        "launches": dom["launches"], "avg_us": dom_ms * 1e3, "bytes_per_launch": dom_bytes},
           "kernels": {k: {"launches": v["launches"], "avg_us": round(v["total_ms"] / v["launches"] * 1e3, 2),
                           "GBps": round(v["bytes"] / max(v["total_ms"], 1e-9) / 1e6, 1)} for k, v in prof.items()}}
    print(json.dumps(out), flush=True)


def gemm_sweep(args, torch, fv, synth):
    """The GEMM kernel alone (fsv_linear on the 8B gate|up matrix, 4096 -> 28672) over a sweep of row counts:
    achieved weight-stream GB/s and bf16 MFMA TFLOP/s per launch, from events carried by the dispatch."""
    import dataclasses
    cfg = dataclasses.replace(synth.MODELS["llama8b"], n_layers=4, vocab=32000, name="llama8b_4layers")
    log("workload gemm_sweep: 4 layers of 8B-shape weights")
    weights = synth.make_weights(cfg, args.seed, device="cuda")
    rows = [8, 16, 32, 64, 97, 128, 256, 512, 1024, 2048]
    ctx = fv.Context(cfg, weights, max_batch=128, max_gamma=15, max_pages_per_req=1, max_rows=max(rows))
    del weights
    torch.cuda.empty_cache()
    K, N = cfg.d_model, 2 * cfg.d_ffn
    table = []
    for M in rows:
        x = torch.randn((M, K), device="cuda").to(torch.bfloat16)
        for l in range(cfg.n_layers):
            ctx.linear(fv.W_GATE_UP, l, x, N)
        torch.cuda.synchronize()
        ctx.profile_read()
        ctx.profile_enable(["gemm_gate_up"])
        for _ in range(args.steps):
            for l in range(cfg.n_layers):          # a different matrix every launch: nothing stays in the caches
                ctx.linear(fv.W_GATE_UP, l, x, N)
        torch.cuda.synchronize()
        p = ctx.profile_read()["gemm_gate_up"]
        ctx.profile_enable(False)
        us = p["total_ms"] / p["launches"] * 1e3
        table.append({"rows": M, "avg_us": round(us, 2), "weight_GBps": round(N * K * 2 / us / 1e3, 1),
                      "mfma_TFLOPs": round(2.0 * M * N * K / us / 1e6, 1),
                      "frac_hbm_peak": round(N * K * 2 / us / 1e3 / HBM_PEAK_GBS, 3),
                      "frac_mfma_peak": round(2.0 * M * N * K / us / 1e6 / 2500.0, 3)})
        log(str(table[-1]))
    print(json.dumps({"metric": "weight-streaming GEMM alone, 8B gate|up matrix (28672 x 4096 bf16), per launch",
                      "config": {"workload": "gemm_sweep"}, "dtype": "bf16", "data": "synthetic", "sweep": table}), flush=True)


def serve_loop(args, torch, fv, synth):
    """Alg. 2 in a loop at the 8B shapes: 16 persistent sessions, the stride of every session picked each round from a
    lognormal link-rate trace and its acceptance average, drafts from the synthetic edge model, fsv_verify, state update.
    The cloud term of the latency model is FITTED from measured verification times (T_cloud = T_base + K delta_cloud,
    Sec. IV-B); the report is the effective token generation rate (Sec. III) under that model."""
    from paper_2601_00644_amd import serve
    cfg = synth.MODELS["llama8b"]
    S, kmax, rounds, seed = 16, 8, args.steps, args.seed
    log("workload serve_8b: weights")
    weights = synth.make_weights(cfg, seed, device="cuda")
    lm = fv.LatencyModel(alpha_edge=0.012, beta=0.002, bits_per_token=17.0, header_bits=320.0, t_prop=0.020, t_base=0.006,
                         delta_cloud=0.0, t_down=0.005)
    req = synth.make_requests(synth.WORKLOADS["c3_8b_b16"], cfg, seed)
    MP = (4096 + rounds * (kmax + 1) + 15) // 16 + 1
    srv = serve.Server(cfg, weights, S, S * MP, kmax, MP, lm, mu=0.1, temperature=0.8, sigma=0.7, seed=seed)
    for s in range(S):
        k, v = synth.make_kv_context(cfg, int(req.seq_lens[s]), seed, s, device="cuda")
        srv.open_session(s, k, v, int(req.last_token[s]))
        del k, v
    log("sessions restored; fitting T_cloud(K) from fixed-stride rounds")
    pts = []
    for K in (1, 2, 4, 6, 8, 1, 2, 4, 6, 8):
        saved = srv.model
        srv.model = fv.LatencyModel(alpha_edge=0.0, beta=0.0, bits_per_token=0.0, header_bits=0.0, t_prop=1.0, t_base=0.0,
                                    delta_cloud=0.0, t_down=0.0)      # a link on which the longest stride always wins
        out = srv.round(np.full(S, 1e9), k_max=K)
        srv.model = saved
        pts.append((K, out["cloud_ms"] * 1e-3))
    ks, ts = np.array([p[0] for p in pts[5:]], float), np.array([p[1] for p in pts[5:]], float)   # second sweep: warm
    delta, base = np.polyfit(ks, ts, 1)
    lm.t_base, lm.delta_cloud = float(base), float(max(delta, 0.0))
    log(f"fit: T_cloud(K) = {base * 1e3:.3f} ms + K * {delta * 1e3:.4f} ms  (measured {[round(t * 1e3, 3) for t in ts]} ms at K = {ks.tolist()})")
    for ss in srv.sessions:
        ss.emitted, ss.gamma_hat = 0, 0.8
    hist, t_model, emitted, drafted, accepted, cloud = {}, 0.0, 0, 0, 0, []
    for rnd in range(rounds):
        rates = serve.lognormal_rates(S, 2.0e3, 1.5, seed, 10_000 + rnd)
        out = srv.round(rates, k_max=kmax)
        cloud.append(out["cloud_ms"])
        for j, s in enumerate(out["sessions"]):
            K, tau = int(out["K"][j]), int(out["tau"][j])
            hist[K] = hist.get(K, 0) + 1
            t_model += fv.policy_step_time(lm, float(rates[s]), K, out["cloud_ms"] * 1e-3)
            emitted += tau + 1
            drafted += K
            accepted += tau
    out = {"metric": "effective token generation rate per session under the latency model, cloud term measured",
           "value": emitted / t_model, "unit": "tokens/s per session", "config": {"workload": "serve_8b", "sessions": S,
           "rounds": rounds, "k_max": kmax, "rate_median_bps": 2.0e3, "rate_sigma": 1.5},
           "t_cloud_fit_ms": {"t_base": base * 1e3, "delta_cloud": delta * 1e3},
           "stride_histogram": {str(k): hist[k] for k in sorted(hist)}, "acceptance": accepted / max(drafted, 1),
           "mean_cloud_ms": float(np.mean(cloud)), "tokens_per_round": emitted / rounds,
           "cloud_tokens_per_s_all_sessions": emitted / (sum(cloud) * 1e-3), "dtype": "bf16", "data": "synthetic"}
    print(json.dumps(out), flush=True)
    srv.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3_8b_b16")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pages", default=None, choices=["interleaved", "permuted", "contiguous"],
                    help="page-table layout of the KV sessions (default: the workload's own, interleaved)")
    ap.add_argument("--top-p", type=float, default=1.0,
                    help="nucleus mass applied to the target law of every request (1 = off, the configurations' setting)")
    ap.add_argument("--adapters", type=int, default=0,
                    help="serve an evolved target: load this many random LoRA adapters (rank --rank) and spread the requests over "
                         "them and the base target (0 = base target only, the configurations' setting)")
    ap.add_argument("--rank", type=int, default=16)
    ap.add_argument("--breakdown", action="store_true", help="also time every kernel class (one extra untimed pass)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies, the known-size reference the HBM counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (requests are independent, so a multi-GPU deployment shards by "
              "request and needs no exchange); rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2601_00644_amd import flexverify as fv
    from paper_2601_00644_amd import synth, workload

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    if args.workload == "c4_sampler":
        return sampler_bench(args, torch, fv, synth)
    if args.workload == "gemm_sweep":
        return gemm_sweep(args, torch, fv, synth)
    if args.workload == "serve_8b":
        return serve_loop(args, torch, fv, synth)
    wl = synth.WORKLOADS[args.workload]
    if args.pages:
        from dataclasses import replace
        wl = replace(wl, pages=args.pages)
    cfg = synth.MODELS[wl.model]
    log(f"workload {wl.name}: model {cfg.name}, generating weights on the device")
    weights = synth.make_weights(cfg, args.seed, device="cuda")
    w = workload.build(wl, args.seed, weights=weights, log=log)
    req, ctx = w.req, w.ctx
    B, G, M = req.batch, w.drafts, w.drafts + req.batch
    res = fv.DeviceResult.alloc(B)
    if args.top_p < 1.0:
        w.batch.top_p_host = np.full(B, args.top_p, np.float32)
        w.batch.top_p = torch.as_tensor(w.batch.top_p_host, device="cuda")

    if args.adapters > 0:
        ctx.lora_load([synth.make_lora(cfg, args.rank, args.seed, a, device="cuda") for a in range(args.adapters)])
        w.batch.adapter = torch.as_tensor(np.arange(B, dtype=np.int32) % (args.adapters + 1) - 1, device="cuda")

    def step():
        ctx.verify(w.batch, res)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_read()
    # event pairs around the dominant kernel only, every eighth of its 32 launches a step: an event-carrying dispatch
    # leaves the GPU idle for about ten microseconds around it (kernel trace: no gap between the other launches), and
    # the step is what is being timed
    ctx.profile_enable(["gemm_gate_up"], every=8)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # per-step spread (one event a step)
    torch.cuda.synchronize()
    e0.record()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    per_step = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)])
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    tau = res.accepted_len.cpu().numpy()
    dom = prof["gemm_gate_up"]
    dom_ms = dom["total_ms"] / dom["launches"]
    dom_bytes = dom["bytes"] / dom["launches"]
    shape = {"llama8b": "8B", "llama1b": "1B"}.get(wl.model, cfg.name)
    # The gate|up GEMM against both roofs: weight bytes over the HBM peak, and 2 * rows * N * K flop over the dense bf16
    # matrix-core peak.  The larger fraction names the bound (HBM up to a few hundred rows, the matrix cores beyond).
    dom_flop = 2.0 * M * (dom_bytes / 2.0)
    hbm_frac = dom_bytes / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
    mfma_frac = dom_flop / (dom_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS
    if hbm_frac >= mfma_frac:
        roofline = {"bound": "hbm", "kernel": "k_gemm<.,SwiGLU> (gate|up projection, weight streaming)",
                    "achieved": hbm_frac * HBM_PEAK_GBS, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_frac,
                    "traffic": counter_traffic(wl.name, args.seed, M)}
    else:
        roofline = {"bound": "mfma", "kernel": "k_gemm<.,SwiGLU> (gate|up projection, several row blocks per weight strip)",
                    "achieved": mfma_frac * MFMA_BF16_PEAK_TFLOPS, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": mfma_frac, "traffic": counter_traffic(wl.name, args.seed, M)}
    roofline.update({"launches": dom["launches"], "avg_us": dom_ms * 1e3, "bytes_per_launch": dom_bytes,
                     "flop_per_launch": dom_flop, "hbm_frac": hbm_frac, "mfma_frac": mfma_frac})
    out = {"metric": f"verified draft tokens/sec on 1 MI355X ({shape} shapes, batch {B})", "value": G / (ms * 1e-3),
           "unit": "verified draft tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": wl.name, "model_shape": cfg.name, "batch": B, "drafts": G, "rows": M,
                      "kv_tokens": int(req.seq_lens.sum()), "temperature": wl.temperature, "top_p": args.top_p, "draft_noise_sigma": wl.sigma,
                      "adapters": args.adapters, "adapter_rank": args.rank if args.adapters else 0,
                      "accepted_drafts": int(tau.sum()), "emitted_tokens": int(tau.sum()) + B},
           "roofline": roofline,
           "ms_per_step_p10_p50_p90": [float(np.percentile(per_step, p)) for p in (10, 50, 90)],
           "emitted_tokens_per_s": (int(tau.sum()) + B) / (ms * 1e-3)}
    # whole-step algorithmic bytes: weights once + KV of every cached position + logits
    wbytes = sum(v.numel() * v.element_size() for k, v in weights.items() if k != "embed")
    kvbytes = float((req.seq_lens + req.gammas + 1).sum()) * cfg.n_layers * cfg.n_kv_heads * cfg.head_dim * 2 * 2
    out["step_bytes"] = {"weights": wbytes, "kv": kvbytes, "step_GBps": (wbytes + kvbytes) / (ms * 1e-3) / 1e9,
                         "step_frac_of_hbm_peak": (wbytes + kvbytes) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    if args.breakdown:
        ctx.profile_enable(True)
        step()
        torch.cuda.synchronize()
        bd = ctx.profile_read()
        ctx.profile_enable(False)
        out["kernels"] = {k: {"launches": v["launches"], "ms": round(v["total_ms"], 4),
                              "GBps": round(v["bytes"] / max(v["total_ms"], 1e-9) / 1e6, 1)} for k, v in bd.items()}
    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, wl, req, weights, args.seed)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
