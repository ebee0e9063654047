#!/usr/bin/env python3
"""Benchmark of the CopySpec copy-and-verify step on one MI355X.

One "step" is one pass of the whole hot path over one batch: match scan + draft gather,
one target-model forward over the pending token plus k drafts of every stream against its
KV cache, greedy argmax + accept rule, KV length rollback and history append (cs_step).

Default workload (the one the headline metric is quoted on): Llama-style 8B shape, bf16,
batch 8 streams, each a 2048-token document followed by 16384 tokens of history that
re-contains document spans (18432 tokens; the last one is pending, 18431 are cached),
gamma = 3, k = 10.  Weights, KV contents and token histories are seeded synthetic data.

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build is single-GPU.
`--prefill N` times prompt ingestion instead (a separate line, not the headline metric).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_workload(args):
    import numpy as np
    import torch
    import synth
    from paper_2502_08923_amd import binding as cs

    shape = {"8b": synth.LLAMA_8B, "1b": synth.LLAMA_1B}[args.shape]
    if args.layers:
        shape = shape.with_layers(args.layers)
    B, k, gamma = args.batch, args.k, args.gamma
    dev = "cuda:0"
    t0 = time.time()
    w = synth.model_weights(shape, synth.seed_for(4), threads=16)
    log(f"[bench] weights generated in {time.time() - t0:.1f}s")
    t0 = time.time()
    model = cs.Model(w, max_batch=B, max_k=k, device=dev)
    del w
    log(f"[bench] model uploaded in {time.time() - t0:.1f}s")

    hists = [synth.history_cfg4(b, vocab=shape.vocab, doc=args.doc, hist=args.hist, k=k)["tokens"]
             for b in range(B)]
    n = args.doc + args.hist
    L = n - 1
    cap = n + 64 * (k + 1) + 64
    kv = cs.KV(model, B, cap)
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.seed_for(4) + 17)
    t0 = time.time()
    for layer in range(shape.n_layers):
        for b in range(B):
            kr = torch.randn((shape.n_kv_heads, L, shape.head_dim), generator=gen, device=dev,
                             dtype=torch.float32).to(torch.bfloat16)
            vr = torch.randn((shape.n_kv_heads, L, shape.head_dim), generator=gen, device=dev,
                             dtype=torch.float32).to(torch.bfloat16)
            kv.load(layer, b, 0, kr, vr)
    log(f"[bench] KV cache filled in {time.time() - t0:.1f}s")
    stride = ((n + 64 * (k + 1) + 3) // 4) * 4
    hist = np.zeros((B, stride), dtype=np.int32)
    for b in range(B):
        hist[b, :n] = hists[b]
    st = {
        "shape": shape, "model": model, "kv": kv, "B": B, "k": k, "gamma": gamma, "n": n, "L": L,
        "hist": torch.from_numpy(hist).to(dev),
        "hist_len0": torch.full((B,), n, dtype=torch.int32, device=dev),
        "kv_len0": torch.full((B,), L, dtype=torch.int32, device=dev),
        "room0": torch.full((B,), 1 << 20, dtype=torch.int32, device=dev),
        "hists": hists,
    }
    st["hist_len"] = st["hist_len0"].clone()
    st["room"] = st["room0"].clone()
    st["out"] = tuple(torch.empty(B, dtype=torch.int32, device=dev) for _ in range(3))
    return st


def one_step(st, cs):
    """Rewind the state (async, tiny) and run one whole step."""
    st["hist_len"].copy_(st["hist_len0"])
    st["room"].copy_(st["room0"])
    st["kv"].set_len_dev(st["kv_len0"], st["L"])
    return cs.cs_step(st["model"], st["kv"], st["hist"], st["hist_len"], st["room"], st["gamma"],
                      st["k"], "rightmost", out=st["out"])


def algorithmic_bytes(st):
    """Bytes the method itself must move per step (weights once, KV once, history once)."""
    sh, B, k, L = st["shape"], st["B"], st["k"], st["L"]
    d, hd, H, KVH, F, V = sh.d_model, sh.head_dim, sh.n_heads, sh.n_kv_heads, sh.d_ff, sh.vocab
    per_layer_w = ((H + 2 * KVH) * hd * d + d * H * hd + 2 * F * d + d * F) * 2
    attn_launch = B * (L + k + 1) * KVH * hd * 2 * 2          # K and V, bf16, one layer
    return {
        "gemm_step": sh.n_layers * per_layer_w + V * d * 2,
        "attn_launch": attn_launch,
        "attn_step": sh.n_layers * attn_launch,
        "lm_head_launch": V * d * 2,
        "argmax_launch": B * (k + 1) * V * 4,
        "scan_launch": B * st["n"] * 4,
        "gemm_flops_step": 2 * B * (k + 1) * (sh.n_layers * per_layer_w // 2 + V * d),
    }


def bench_scan(cs, torch, synth, log):
    """Configuration 2 (64 x 32768 int32) and a 1 GiB variant for steady-state bandwidth."""
    import numpy as np
    dev = "cuda:0"
    res = {}
    hs = np.stack([synth.history_cfg2(s)["tokens"] for s in range(64)])
    d_hist = torch.from_numpy(hs).to(dev)
    d_len = torch.full((64,), 32768, dtype=torch.int32, device=dev)

    def timed(d_hist, d_len, iters):
        cs.cs_find_match_batch_dev(d_hist, d_len, 3, 10)
        torch.cuda.synchronize()
        cs.cs_profile_enable(["scan"])
        cs.cs_profile_reset()
        t0 = time.perf_counter()
        for _ in range(iters):
            cs.cs_find_match_batch_dev(d_hist, d_len, 3, 10)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / iters
        ms, nl = cs.cs_profile_read("scan")
        cs.cs_profile_enable([])
        return wall, ms / nl * 1e-3

    wall, kern = timed(d_hist, d_len, 200)
    tokens = 64 * 32768
    # cold: a 1 GiB fill between calls evicts the 8 MB of histories from L2 and the 256 MB cache
    evict = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    cs.cs_profile_enable(["scan"])
    cs.cs_profile_reset()
    for i in range(10):
        evict.fill_(float(i))
        cs.cs_find_match_batch_dev(d_hist, d_len, 3, 10)
    torch.cuda.synchronize()
    ms, nl = cs.cs_profile_read("scan")
    cs.cs_profile_enable([])
    cold = ms / nl * 1e-3
    del evict
    res["cfg2"] = {"tokens": tokens, "call_us": wall * 1e6, "kernel_us": kern * 1e6,
                   "kernel_us_cold": cold * 1e6,
                   "gtokens_per_s_call": tokens / wall / 1e9,
                   "gtokens_per_s_kernel": tokens / kern / 1e9,
                   "kernel_GBps": tokens * 4 / kern / 1e9, "kernel_GBps_cold": tokens * 4 / cold / 1e9}
    nb = 8192
    big = d_hist.repeat(nb // 64, 1).contiguous()
    big_len = torch.full((nb,), 32768, dtype=torch.int32, device=dev)
    wall, kern = timed(big, big_len, 20)
    tokens = nb * 32768
    res["scaled_1GiB"] = {"tokens": tokens, "call_us": wall * 1e6, "kernel_us": kern * 1e6,
                          "gtokens_per_s_kernel": tokens / kern / 1e9,
                          "kernel_GBps": tokens * 4 / kern / 1e9,
                          "hbm_frac": tokens * 4 / kern / 1e9 / HBM_PEAK_GBS}
    del big
    return res


def cpu_baseline(st, args):
    """The CPU oracle timed on a bounded sample of the same workload: `cpu_streams` of the B
    streams, `cpu_layers` decoder layers at full width and full context, plus the scan, the
    lm_head, the argmax and the accept rule; the layer time is scaled to the full depth and
    the stream time to the full batch."""
    import synth
    from oracle import copyspec_oracle as orc
    sh = st["shape"]
    nl, ns = min(args.cpu_layers, sh.n_layers), min(args.cpu_streams, st["B"])
    sub = sh.with_layers(nl)
    w = synth.model_weights(sub, synth.seed_for(4), threads=8)
    L, k = st["L"], st["k"]
    t_scan = t_layers = t_head = 0.0
    for b in range(ns):
        okv = orc.KVCache(sub, L + k + 1)
        for layer in range(nl):
            kr, vr = synth.random_kv(sub, L, synth.seed_for(4), layer, b)
            okv.load(layer, kr, vr)
        okv.truncate(L)
        h = st["hists"][b]
        t0 = time.perf_counter()
        _, _, draft = orc.find_match_np(h, st["gamma"], k)
        t_scan += time.perf_counter() - t0
        # layers (return_hidden skips the lm_head) and lm_head timed separately
        t0 = time.perf_counter()
        hidden = orc.forward_block(w, okv, [int(h[-1])] + draft, return_hidden=True)
        t_layers += time.perf_counter() - t0
        t0 = time.perf_counter()
        logits = hidden @ orc._f64(w["lm_head"]).T
        am = [orc.argmax_first(r) for r in logits]
        orc.accept_prefix(am, draft)
        t_head += time.perf_counter() - t0
        del okv
    t_stream = (t_scan + t_layers / nl * sh.n_layers + t_head) / ns
    t_step = t_stream * st["B"]
    return {"value": st["B"] * k / t_step, "unit": "tokens/s",
            "cores": int(os.environ.get("OMP_NUM_THREADS") or os.cpu_count()),
            "kind": "oracle",
            "sample": f"{ns} of {st['B']} streams, {nl} of {sh.n_layers} layers + lm_head + scan at "
                      f"full width and context (L={L}); measured {t_scan + t_layers + t_head:.1f}s "
                      f"(scan {t_scan * 1e3:.1f} ms, layers {t_layers:.1f}s, head {t_head:.1f}s), "
                      f"scaled to {sh.n_layers} layers x {st['B']} streams"}


def bench_prefill(args):
    """Prompt ingestion alone (`--prefill N`): one stream, an N-token prompt through cs_prefill,
    `steps` times into the same cache.  The projections of a prompt block are compute-bound, so
    the roofline object is the MFMA one (all projection launches, HIP events)."""
    import torch
    import synth
    from paper_2502_08923_amd import binding as cs
    shape = {"8b": synth.LLAMA_8B, "1b": synth.LLAMA_1B}[args.shape]
    if args.layers:
        shape = shape.with_layers(args.layers)
    n = args.prefill
    model = cs.Model(synth.model_weights(shape, synth.seed_for(4), threads=16), max_batch=1, max_k=args.k)
    kv = cs.KV(model, 1, n + 64)
    prompt = synth.history_cfg4(0, vocab=shape.vocab, doc=args.doc, hist=max(n - args.doc, 0) + 64,
                                k=args.k)["tokens"][:n].tolist()
    for _ in range(max(args.warmup, 1)):
        cs.cs_prefill(model, kv, 0, prompt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        cs.cs_prefill(model, kv, 0, prompt)
    torch.cuda.synchronize()
    t = (time.perf_counter() - t0) / args.steps
    classes = ["gemm", "attn", "attn_merge"]
    cs.cs_profile_enable(classes)
    cs.cs_profile_reset()
    for _ in range(args.steps):
        cs.cs_prefill(model, kv, 0, prompt)
    torch.cuda.synchronize()
    prof = {c: cs.cs_profile_read(c) for c in classes}
    cs.cs_profile_enable([])
    d, hd, H, KVH, F = shape.d_model, shape.head_dim, shape.n_heads, shape.n_kv_heads, shape.d_ff
    rows = n - 1                                          # the last prompt token stays pending
    gemm_flops = 2.0 * rows * shape.n_layers * ((H + 2 * KVH) * hd * d + d * H * hd + 2 * F * d + d * F)
    attn_flops = 4.0 * hd * H * shape.n_layers * rows * (rows + 1) / 2      # causal QK^T and PV
    gemm_s = prof["gemm"][0] / args.steps * 1e-3
    attn_s = prof["attn"][0] / args.steps * 1e-3
    out = {
        "metric": f"prompt tokens/sec/GPU ({args.shape.upper()} shape, {n}-token prompt)",
        "value": rows / t, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": max(args.warmup, 1),
        "ms_per_step": t * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"llama-{args.shape} shape x{shape.n_layers} layers, one stream, {n}-token prompt "
                               f"ingested by cs_prefill (one whole prompt per step)", "prompt": n},
        "roofline": {"bound": "mfma", "kernel": "k_gemm_dma (all projections of the prompt blocks)",
                     "achieved": gemm_flops / gemm_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_flops / gemm_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "flops_per_step": gemm_flops, "ms_per_step": gemm_s * 1e3},
        "kernels": {"attention": {"bound": "mfma", "ms_per_step": attn_s * 1e3,
                                  "achieved_TFLOPs": attn_flops / attn_s / 1e12,
                                  "frac": attn_flops / attn_s / 1e12 / MFMA_BF16_PEAK_TFLOPS},
                    "attn_merge": {"ms_per_step": prof["attn_merge"][0] / args.steps}},
        "cpu_baseline": None,
    }
    print(json.dumps(out), flush=True)


def measured_traffic(kernel: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE +
    WRITE_SIZE, each scaled by what the same counter reads for a 1 GiB device copy), or None.
    bench.py cannot collect hardware counters itself; the summary says how they were taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_llama8b_b8_k10.txt")
    try:
        for line in open(path):
            if line.startswith(f"TRAFFIC {kernel} "):
                return float(line.split()[2])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--shape", default="8b", choices=["8b", "1b"])
    ap.add_argument("--layers", type=int, default=0, help="override depth (debug only; invalid as a result)")
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--k", type=int, default=10)
    ap.add_argument("--gamma", type=int, default=3)
    ap.add_argument("--doc", type=int, default=2048)
    ap.add_argument("--hist", type=int, default=16384)
    ap.add_argument("--cpu-layers", type=int, default=16)
    ap.add_argument("--cpu-streams", type=int, default=2)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-scan", action="store_true")
    ap.add_argument("--prefill", type=int, default=0,
                    help="time the ingestion of an N-token prompt (one stream) instead of the step")
    ap.add_argument("--calib-copy", action="store_true",
                    help="only run a 1 GiB device copy (yardstick for the HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    from paper_2502_08923_amd import binding as cs
    cs.load_library()
    torch.cuda.set_device(0)

    if args.calib_copy:
        # plain device copy of known size: the yardstick for the FETCH_SIZE / WRITE_SIZE counters
        n = 1 << 28                                       # 1 GiB of float32 read, 1 GiB written
        x = torch.empty(n, dtype=torch.float32, device="cuda:0").normal_()
        y = torch.empty_like(x)
        for _ in range(5):
            y.copy_(x)
        torch.cuda.synchronize()
        print(json.dumps({"calib_copy_bytes_read": n * 4, "calib_copy_bytes_written": n * 4}))
        return

    if args.prefill:
        bench_prefill(args)
        return

    st = build_workload(args)
    B, k = st["B"], st["k"]
    for _ in range(args.warmup):
        one_step(st, cs)
    torch.cuda.synchronize()

    # timed region: exactly `steps` whole steps, inputs resident in HBM
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(st, cs)
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps
    acc = st["out"][0].cpu().numpy()
    dl = st["out"][2].cpu().numpy()

    # the same steps once more, each bracketed by a synchronize of its own: median and minimum
    per_step = []
    for _ in range(args.steps):
        t1 = time.perf_counter()
        one_step(st, cs)
        torch.cuda.synchronize()
        per_step.append(time.perf_counter() - t1)
    per_step.sort()

    # third pass of the same steps with HIP-event timing of the kernel classes
    classes = ["scan", "gemm", "attn", "attn_merge", "argmax", "lm_head"]
    cs.cs_profile_enable(classes)
    cs.cs_profile_reset()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(st, cs)
    torch.cuda.synchronize()
    t_step_prof = (time.perf_counter() - t0) / args.steps
    prof = {c: cs.cs_profile_read(c) for c in classes}
    cs.cs_profile_enable([])

    # the step takes the argmax inside the lm_head (no logits in memory, no argmax pass); the
    # stand-alone argmax kernel, which serves callers that ask for the logits, is timed on its own
    argmax_fused = prof["argmax"][1] == 0
    if argmax_fused:
        gen = torch.Generator(device="cuda:0")
        gen.manual_seed(5)
        logits = torch.randn((B, k + 1, st["shape"].vocab), generator=gen, device="cuda:0")
        draft0 = torch.zeros((B, max(k, 1)), dtype=torch.int32, device="cuda:0")
        dl0 = torch.zeros(B, dtype=torch.int32, device="cuda:0")
        for _ in range(3):
            cs.cs_op_argmax_accept(st["model"], logits, draft0, dl0)
        torch.cuda.synchronize()
        cs.cs_profile_enable(["argmax"])
        cs.cs_profile_reset()
        for _ in range(20):
            cs.cs_op_argmax_accept(st["model"], logits, draft0, dl0)
        torch.cuda.synchronize()
        prof["argmax"] = cs.cs_profile_read("argmax")
        cs.cs_profile_enable([])
        del logits

    ab = algorithmic_bytes(st)
    attn_ms, attn_n = prof["attn"]
    attn_s = attn_ms / attn_n * 1e-3
    gemm_ms, gemm_n = prof["gemm"]
    lm_ms, lm_n = prof["lm_head"]
    am_ms, am_n = prof["argmax"]
    kern = {
        "attention": {"bound": "hbm", "avg_us": attn_s * 1e6, "launches_per_step": attn_n // args.steps,
                      "achieved_GBps": ab["attn_launch"] / attn_s / 1e9,
                      "frac": ab["attn_launch"] / attn_s / 1e9 / HBM_PEAK_GBS},
        "gemm_all": {"bound": "hbm", "ms_per_step": gemm_ms / args.steps,
                     "achieved_GBps": ab["gemm_step"] / (gemm_ms / args.steps * 1e-3) / 1e9,
                     "frac": ab["gemm_step"] / (gemm_ms / args.steps * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "mfma_TFLOPs": ab["gemm_flops_step"] / (gemm_ms / args.steps * 1e-3) / 1e12,
                     "mfma_frac": ab["gemm_flops_step"] / (gemm_ms / args.steps * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "lm_head": {"bound": "hbm", "avg_us": lm_ms / lm_n * 1e3,
                    "achieved_GBps": ab["lm_head_launch"] / (lm_ms / lm_n * 1e-3) / 1e9,
                    "frac": ab["lm_head_launch"] / (lm_ms / lm_n * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "argmax": {"bound": "hbm", "in_step": "fused into the lm_head epilogue" if argmax_fused else "own kernel",
                   "avg_us": am_ms / am_n * 1e3,
                   "achieved_GBps": ab["argmax_launch"] / (am_ms / am_n * 1e-3) / 1e9,
                   "frac": ab["argmax_launch"] / (am_ms / am_n * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "attn_merge": {"avg_us": prof["attn_merge"][0] / max(prof["attn_merge"][1], 1) * 1e3},
        "scan_in_step": {"avg_us": prof["scan"][0] / max(prof["scan"][1], 1) * 1e3},
    }
    # more than 48 query rows per KV head go to the LDS-ring attention kernel
    g_rows = (k + 1) * (st["shape"].n_heads // st["shape"].n_kv_heads)
    attn_kernel = "k_attn_mfma" if g_rows <= 48 else "k_attn_lds"
    # the committed counter summary covers the default workload only
    default_workload = (args.shape, B, k, args.doc, args.hist, args.layers) == ("8b", 8, 10, 2048, 16384, 0)
    step_bytes = ab["gemm_step"] + ab["attn_step"] + ab["scan_launch"] + (0 if argmax_fused else ab["argmax_launch"])
    out = {
        "metric": f"verified tokens/sec/GPU ({args.shape.upper()} shape, k={k})",
        "value": B * k / t_step,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": t_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"llama-{args.shape} shape x{st['shape'].n_layers} layers, batch {B} streams, "
                               f"{args.doc}-token document + {args.hist}-token history with planted "
                               f"document spans (KV length {st['L']} + pending), gamma={st['gamma']}, k={k}, "
                               f"one whole cs_step per step",
                   "batch": B, "k": k, "gamma": st["gamma"], "kv_len": st["L"], "rows": B * (k + 1)},
        "roofline": {"bound": "hbm", "kernel": f"{attn_kernel} (block attention, one layer, all streams)",
                     "achieved": ab["attn_launch"] / attn_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": ab["attn_launch"] / attn_s / 1e9 / HBM_PEAK_GBS,
                     "traffic": measured_traffic("k_attn_mfma") if default_workload else None,
                     "algorithmic_bytes_per_launch": ab["attn_launch"], "avg_launch_us": attn_s * 1e6},
        "kernels": kern,
        "step": {"algorithmic_GB": step_bytes / 1e9,
                 "whole_step_hbm_frac": step_bytes / t_step / 1e9 / HBM_PEAK_GBS,
                 "ms_per_step_median": per_step[len(per_step) // 2] * 1e3, "ms_per_step_min": per_step[0] * 1e3,
                 "ms_per_step_with_event_timing": t_step_prof * 1e3,
                 "draft_len": dl.tolist(), "accepted_len": acc.tolist(),
                 "emitted_tokens_per_s": float((acc + 1).sum()) / t_step},
    }
    if not args.no_scan:
        out["match_scan"] = bench_scan(cs, torch, synth, log)
        out["metric"] += " + match-scan Gtokens/s"
    if not args.no_cpu:
        t0 = time.time()
        out["cpu_baseline"] = cpu_baseline(st, args)
        log(f"[bench] cpu baseline took {time.time() - t0:.1f}s")
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
