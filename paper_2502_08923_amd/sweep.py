"""Block-size, gamma and match-policy sweeps on one MI355X (the paper's Sec. 5.2 / Table 4 and
Sec. 5.1 questions, asked of this implementation on synthetic data).

    python -m paper_2502_08923_amd.sweep [--layers N] [--json out.json]

Two measurements are combined:

1. Step cost: one whole cs_step (scan + verify forward + accept + rollback) of the 8B-shape
   workload (batch 8, 18431 cached rows) timed for copy blocks k = 0 (plain decoding through
   the same kernels) .. 100.
2. Acceptance: a synthetic self-correction dialogue (three versions of a 1024-token answer,
   each the previous one with 5 % token edits) is replayed through the library's match
   search alone; the "target model" is the third version itself, so a draft token is accepted
   iff it equals the next token of that version.  This gives tokens emitted per step for
   every (gamma, k, policy) without any trained model.  The rightmost policy copies from the
   second version (one round of edits away), the first-match policy from the original (two);
   the context policy ranks the candidates by the length of their agreeing backward context.

emitted tokens/s = batch * (mean tokens per step) / (step time); the speed-up column is
relative to k = 0.  The acceptance side is a projection for that edit law, not a property of
a language model.

3. (--merged) Cost of the merge with draft-model speculative decoding (Sec. 3.3): one stream,
   8B-shape target, 1B-shape draft model (same vocabulary), 4096-token prompt with planted
   repeats, 64 new tokens through plain greedy decoding, CopySpec alone and the merged loop with
   delta = 3 and 5.  With random-init weights nothing is accepted, so the figures are the cost
   side only: time per target step, per draft-model forward pass, and the acceptance a merged
   step needs to break even with plain decoding.

4. (--index) The gamma-gram hash index of Sec. 3.1 against the linear scan on one long history.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def replay_acceptance(cs, synth, gamma: int, k: int, policy: str, streams=(0, 1, 2, 3),
                      workload: str = "multiturn"):
    """Mean tokens emitted per step and mean accepted drafts per attempt when the "truth" of a
    replay workload (synth.multiturn_replay or synth.zipf_replay) is decoded with CopySpec and
    the target always emits that truth."""
    import numpy as np
    tot_steps = tot_tokens = attempts = accepted = 0
    for s in streams:
        g = synth.multiturn_replay(s) if workload == "multiturn" else synth.zipf_replay(s)
        ctx, truth = g["context"].tolist(), g["truth"].tolist()
        seq = ctx + truth[:gamma]                 # the first gamma tokens are generated plainly
        pos = gamma
        while pos < len(truth):
            tot_steps += 1
            if k > 0:
                _, _, draft = cs.cs_find_match_ex(np.asarray(seq, dtype=np.int32), gamma, k, policy)
            else:
                draft = []
            draft = draft[:len(truth) - pos - 1]
            tau = 0
            while tau < len(draft) and draft[tau] == truth[pos + tau]:
                tau += 1
            if draft:
                attempts += 1
                accepted += tau
            emit = min(tau + 1, len(truth) - pos)
            seq.extend(truth[pos:pos + emit])
            pos += emit
            tot_tokens += emit
    return tot_tokens / tot_steps, (accepted / attempts if attempts else 0.0)


def merged_costs(cs, synth, model, torch):
    """Wall-clock cost of greedy / CopySpec / merged decoding of one stream (see the module text)."""
    draft_shape = synth.LLAMA_1B.with_vocab(model.shape.vocab)
    wd = synth.model_weights(draft_shape, synth.seed_for(3), threads=16)
    dmodel = cs.Model(wd, max_batch=1, max_k=31)
    prompt = synth.history_cfg4(0)["tokens"][:4096].tolist()
    new, cap = 64, 4096 + 64 + 128
    kv, dkv = cs.KV(model, 1, cap), cs.KV(dmodel, 1, cap)
    rows = []

    def timed(label, fn):
        fn()                                              # warm-up (includes the prompt pass)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = fn()
        torch.cuda.synchronize()
        return label, time.perf_counter() - t0, out

    t_prefill = timed("prefill", lambda: cs.cs_prefill(model, kv, 0, prompt))[1]
    label, t, out = timed("greedy", lambda: cs.cs_decode_greedy(model, kv, prompt, new))
    greedy = out
    t_plain_step = (t - t_prefill) / new
    rows.append({"mode": label, "total_ms": t * 1e3, "steps": new, "ms_per_target_step": t_plain_step * 1e3})
    label, t, (out, st) = timed("copyspec k=10", lambda: cs.cs_decode(model, kv, prompt, new, 3, 10))
    assert out == greedy
    rows.append({"mode": label, "total_ms": t * 1e3, "steps": st["steps"], "copy_attempts": st["attempts"],
                 "ms_per_target_step": (t - t_prefill) / st["steps"] * 1e3})
    for delta in (3, 5):
        label, t, (out, st) = timed(f"merged k=10 delta={delta}",
                                    lambda: cs.cs_decode_merged(model, kv, dmodel, dkv, prompt, new, 3, 10, delta))
        assert out == greedy
        # every step here is a rejected proposal: target block of delta+1 rows + delta draft forwards
        t_step = (t - t_prefill) / st["steps"]
        rows.append({"mode": label, "total_ms": t * 1e3, "steps": st["steps"], "copy_attempts": st["copy_attempts"],
                     "spec_attempts": st["spec_attempts"], "draft_forwards": st["draft_forwards"],
                     "ms_per_merged_step": t_step * 1e3,
                     "break_even_tokens_per_step": t_step / t_plain_step})
    for h in (dkv, kv, dmodel):
        h.destroy()
    return {"prefill_ms": t_prefill * 1e3, "prefill_tokens_per_s": (len(prompt) - 1) / t_prefill, "rows": rows}


def index_vs_scan(cs, torch):
    """Match search through the gamma-gram index (the paper's data structure, Sec. 3.1) against
    the linear scan, one stream, uniform tokens over a 128256-token vocabulary with the last
    gamma tokens planted once: time to build the index over n tokens, time of a call after the
    history grew by 11 tokens (insert + lookup + draft gather), time of a scan call."""
    import numpy as np
    rows = []
    for n in (32768, 1 << 20, 1 << 24, 1 << 26):
        g = torch.Generator(device="cuda:0")
        g.manual_seed(n)
        cap = n + 1024
        hist = torch.randint(0, 128256, (1, cap), generator=g, device="cuda:0", dtype=torch.int32)
        hist[0, n - 3:n] = hist[0, n // 3:n // 3 + 3]
        d_len = torch.tensor([n], dtype=torch.int32, device="cuda:0")
        ix = cs.Index(1, cap, 3)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        a = cs.cs_index_find_match_batch_dev(ix, hist, d_len, n, 10)
        torch.cuda.synchronize()
        t_build = time.perf_counter() - t0
        b = cs.cs_find_match_batch_dev(hist, d_len, 3, 10)
        torch.cuda.synchronize()
        assert all(torch.equal(x, y) for x, y in zip(a, b)) and int(a[0][0]) >= n // 3
        lens = [torch.tensor([n + 11 * (i + 1)], dtype=torch.int32, device="cuda:0") for i in range(50)]
        t0 = time.perf_counter()
        for dl in lens:
            a = cs.cs_index_find_match_batch_dev(ix, hist, dl, 11, 10)
        torch.cuda.synchronize()
        t_inc = (time.perf_counter() - t0) / len(lens)
        t0 = time.perf_counter()
        for dl in lens:
            b = cs.cs_find_match_batch_dev(hist, dl, 3, 10)
        torch.cuda.synchronize()
        t_scan = (time.perf_counter() - t0) / len(lens)
        assert all(torch.equal(x, y) for x, y in zip(a, b))
        rows.append({"tokens": n, "index_build_ms": t_build * 1e3, "index_call_us": t_inc * 1e6,
                     "scan_call_us": t_scan * 1e6})
        ix.destroy()
        del hist
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=0, help="depth override (0 = full 32 layers)")
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--ks", default="0,5,10,20,32,50,100")
    ap.add_argument("--json", default="")
    ap.add_argument("--merged", action="store_true", help="also time the merge with a draft model")
    ap.add_argument("--index", action="store_true", help="also time the gamma-gram index against the scan")
    args = ap.parse_args()

    import numpy as np
    import torch
    import synth
    from paper_2502_08923_amd import binding as cs
    from paper_2502_08923_amd import workload as wl

    cs.load_library()
    ks = [int(x) for x in args.ks.split(",")]
    kmax = max(ks)
    # the benchmark's workload, with room for the largest block
    shape, model = wl.build_model("8b", args.layers, 8, kmax)
    hists = [synth.history_cfg4(b, vocab=shape.vocab, k=kmax)["tokens"] for b in range(8)]
    st = wl.build_state(shape, model, 8, kmax, 3, hists)
    B = st["B"]

    rows = []
    for k in ks:
        for _ in range(2):
            wl.one_step(st, k=k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            wl.one_step(st, k=k)
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) / args.steps
        rows.append({"k": k, "ms_per_step": t * 1e3})
        print(f"[sweep] k={k:3d}: {t * 1e3:7.2f} ms/step", file=sys.stderr, flush=True)
    base = rows[0]["ms_per_step"] if ks[0] == 0 else None

    table = []
    for gamma in (2, 3, 5, 10):
        for policy in ("rightmost", "first", "context"):
            for r in rows:
                k = r["k"]
                tps, tau = replay_acceptance(cs, synth, gamma, k, policy)
                emitted = B * tps / (r["ms_per_step"] * 1e-3)
                table.append({"gamma": gamma, "policy": policy, "k": k, "ms_per_step": r["ms_per_step"],
                              "tokens_per_step": tps, "accepted_per_attempt": tau,
                              "emitted_tokens_per_s": emitted,
                              "speedup_vs_plain": (emitted / (B / (base * 1e-3))) if base else None})

    # second replay workload: Zipf-distributed tokens with 30 % copied spans, k = 10 only
    k10 = next((r for r in rows if r["k"] == 10), rows[-1])
    ztable = []
    for gamma in (2, 3, 5):
        for policy in ("rightmost", "first", "context"):
            tps, tau = replay_acceptance(cs, synth, gamma, k10["k"], policy, workload="zipf")
            ztable.append({"gamma": gamma, "policy": policy, "k": k10["k"], "tokens_per_step": tps,
                           "accepted_per_attempt": tau,
                           "speedup_vs_plain": (tps * base / k10["ms_per_step"]) if base else None})

    # match-scan cost by gamma and policy on the 64 x 32768 scan configuration
    hs = np.stack([synth.history_cfg2(s)["tokens"] for s in range(64)])
    d_hist = torch.from_numpy(hs).to("cuda:0")
    d_len = torch.full((64,), 32768, dtype=torch.int32, device="cuda:0")
    scan = []
    for gamma in (1, 2, 3, 5, 10, 16):
        for policy in ("rightmost", "first", "context"):
            cs.cs_find_match_batch_dev(d_hist, d_len, gamma, 10, policy)
            torch.cuda.synchronize()
            cs.cs_profile_enable(["scan"])
            cs.cs_profile_reset()
            for _ in range(50):
                cs.cs_find_match_batch_dev(d_hist, d_len, gamma, 10, policy)
            ms, n = cs.cs_profile_read("scan")
            cs.cs_profile_enable([])
            scan.append({"gamma": gamma, "policy": policy, "kernel_us": ms / n * 1e3})

    merged = merged_costs(cs, synth, st["model"], torch) if args.merged else None
    index = index_vs_scan(cs, torch) if args.index else None
    out = {"step_cost": rows, "projection": table, "projection_zipf": ztable, "scan": scan, "merged": merged, "index": index,
           "workload": f"llama-8b shape x{st['shape'].n_layers} layers, batch {B}, KV {st['L']}"}
    if args.json:
        with open(args.json, "w") as f:
            json.dump(out, f, indent=1)
    print("| gamma | policy | k | ms/step | tokens/step | accepted/attempt | emitted tok/s | vs k=0 |")
    print("|---|---|---|---|---|---|---|---|")
    for r in table:
        sp = f"{r['speedup_vs_plain']:.2f}x" if r["speedup_vs_plain"] else "-"
        print(f"| {r['gamma']} | {r['policy']} | {r['k']} | {r['ms_per_step']:.2f} | {r['tokens_per_step']:.2f} | "
              f"{r['accepted_per_attempt']:.2f} | {r['emitted_tokens_per_s']:.0f} | {sp} |")
    print()
    print("Zipf-law tokens (exponent 1.1) with 30 % of the answer copied from the context in spans of 8-64:")
    print("| gamma | policy | k | tokens/step | accepted/attempt | vs k=0 |")
    print("|---|---|---|---|---|---|")
    for r in ztable:
        sp = f"{r['speedup_vs_plain']:.2f}x" if r["speedup_vs_plain"] else "-"
        print(f"| {r['gamma']} | {r['policy']} | {r['k']} | {r['tokens_per_step']:.2f} | {r['accepted_per_attempt']:.2f} | {sp} |")
    print()
    print("| gamma | policy | scan kernel us (64 x 32768 tokens) |")
    print("|---|---|---|")
    for r in scan:
        print(f"| {r['gamma']} | {r['policy']} | {r['kernel_us']:.2f} |")
    if merged:
        print()
        print(f"One stream, 4096-token prompt (prompt pass {merged['prefill_ms']:.1f} ms = "
              f"{merged['prefill_tokens_per_s']:.0f} tokens/s, subtracted below), 64 new tokens:")
        print("| mode | steps | ms per step | break-even tokens per step |")
        print("|---|---|---|---|")
        for r in merged["rows"]:
            ms = r.get("ms_per_merged_step", r.get("ms_per_target_step"))
            be = f"{r['break_even_tokens_per_step']:.2f}" if "break_even_tokens_per_step" in r else "-"
            print(f"| {r['mode']} | {r['steps']} | {ms:.2f} | {be} |")
    if index:
        print()
        print("Match search, one stream, gamma=3, k=10 (whole calls, wall clock):")
        print("| history tokens | index build ms | index call us (11 new tokens) | scan call us |")
        print("|---|---|---|---|")
        for r in index:
            print(f"| {r['tokens']} | {r['index_build_ms']:.2f} | {r['index_call_us']:.1f} | {r['scan_call_us']:.1f} |")


if __name__ == "__main__":
    main()
