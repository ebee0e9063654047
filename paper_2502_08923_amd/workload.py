"""Device-resident benchmark workloads for the copy-and-verify step: a model, a filled KV cache
and token histories with planted repeats, plus the rewind-and-step helper the timing loops use.
Shared by bench.py and the sweep; it only draws inputs (synth) and calls the library (binding).
"""
from __future__ import annotations

import sys
import time

import numpy as np
import torch

import synth
from . import binding as cs

SHAPES = {"8b": synth.LLAMA_8B, "1b": synth.LLAMA_1B, "qwen7b": synth.QWEN_7B, "70b": synth.LLAMA_70B,
          "qwen72b": synth.QWEN_72B}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_model(shape_name: str, layers: int, max_batch: int, max_k: int, dev="cuda:0"):
    shape = SHAPES[shape_name]
    if layers:
        shape = shape.with_layers(layers)
    t0 = time.time()
    params = shape.n_layers * (shape.d_model * (shape.n_heads + 2 * shape.n_kv_heads) * shape.head_dim
                               + shape.n_heads * shape.head_dim * shape.d_model + 3 * shape.d_model * shape.d_ff) \
        + 2 * shape.vocab * shape.d_model
    if params > 20e9:
        # too large to hold next to the library's copy: drawn, uploaded and handed over layer by layer
        model = cs.Model(synth.model_weights_lazy(shape, synth.seed_for(4), threads=16), max_batch=max_batch,
                         max_k=max_k, device=dev)
        log(f"[workload] {params / 1e9:.1f} G weights generated and loaded in stages in {time.time() - t0:.1f}s")
        return shape, model
    w = synth.model_weights(shape, synth.seed_for(4), threads=16)
    log(f"[workload] weights generated in {time.time() - t0:.1f}s")
    t0 = time.time()
    model = cs.Model(w, max_batch=max_batch, max_k=max_k, device=dev)
    del w
    log(f"[workload] model uploaded in {time.time() - t0:.1f}s")
    return shape, model


def build_state(shape, model, B: int, k: int, gamma: int, hists, host_kv_streams=(), dev="cuda:0"):
    """KV cache of B streams filled with seeded random K/V (N(0,1) rounded to bf16; rotary
    embedding preserves norms, so post-rotary keys of a random-init model look the same), the
    histories uploaded, and the buffers one_step rewinds.  Streams listed in host_kv_streams get
    their rows from synth.random_kv (so that a CPU run can be given the same contents, returned
    in state["host_kv"]); the others from the device generator."""
    n = len(hists[0])
    assert all(len(h) == n for h in hists)
    L = n - 1
    cap = n + 64 * (k + 1) + 64
    kv = cs.KV(model, B, cap)
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.seed_for(4) + 17)
    host_kv = {b: [] for b in host_kv_streams}
    t0 = t_log = time.time()
    shp = (shape.n_kv_heads, L, shape.head_dim)
    for layer in range(shape.n_layers):
        if time.time() - t_log > 20.0:                     # slow under a profiler: show that it moves
            log(f"[workload] filling the KV cache: layer {layer} of {shape.n_layers}")
            t_log = time.time()
        for b in range(B):
            if b in host_kv:
                kr, vr = synth.random_kv(shape, L, synth.seed_for(4), layer, b)
                host_kv[b].append((kr, vr))
            else:
                kr = torch.randn(shp, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
                vr = torch.randn(shp, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
            kv.load(layer, b, 0, kr, vr)
    log(f"[workload] KV cache ({B} x {L} rows x {shape.n_layers} layers) filled in {time.time() - t0:.1f}s")
    stride = ((n + 64 * (k + 1) + 3) // 4) * 4
    hist = np.zeros((B, stride), dtype=np.int32)
    for b in range(B):
        hist[b, :n] = hists[b]
    st = {
        "shape": shape, "model": model, "kv": kv, "B": B, "k": k, "gamma": gamma, "n": n, "L": L,
        "hist": torch.from_numpy(hist).to(dev), "hist_host": hist,
        "hist_len0": torch.full((B,), n, dtype=torch.int32, device=dev),
        "kv_len0": torch.full((B,), L, dtype=torch.int32, device=dev),
        "room0": torch.full((B,), 1 << 20, dtype=torch.int32, device=dev),
        "host_kv": host_kv,
    }
    st["hist_len"] = st["hist_len0"].clone()
    st["room"] = st["room0"].clone()
    st["out"] = tuple(torch.empty(B, dtype=torch.int32, device=dev) for _ in range(3))
    return st


def one_step(st, k=None, policy="rightmost"):
    """Rewind the state (asynchronous, a few bytes) and run one whole copy-and-verify step."""
    st["hist_len"].copy_(st["hist_len0"])
    st["room"].copy_(st["room0"])
    st["kv"].set_len_dev(st["kv_len0"], st["L"])
    return cs.cs_step(st["model"], st["kv"], st["hist"], st["hist_len"], st["room"], st["gamma"],
                      st["k"] if k is None else k, policy, out=st["out"])


def plant_acceptance(st, taus):
    """Make the drafts of the timed step partly right, as a trained model's copies are (the paper
    reports 0.6 to 8.7 accepted tokens per attempt, Sec. 6.3): the random-init model's own greedy
    continuation from the benchmark state is computed with plain steps (k = 0), and its first
    taus[b] tokens are written behind the matched gamma-gram of stream b's history, followed by a
    token that is wrong.  Returns the accepted lengths one step then yields."""
    B, k, n = st["B"], st["k"], st["n"]
    _, src, _, dl = cs.cs_find_match_batch_dev(st["hist"][:, :n].contiguous(), st["hist_len0"], st["gamma"], k)
    src, dl = src.cpu().numpy(), dl.cpu().numpy()
    assert (dl == k).all(), "every benchmark history ends mid-span with k source tokens left"
    # greedy continuation: k + 1 plain steps on a scratch copy of the histories
    keep = st["hist"].clone()
    st["hist_len"].copy_(st["hist_len0"])
    st["room"].copy_(st["room0"])
    st["kv"].set_len_dev(st["kv_len0"], st["L"])
    for _ in range(k + 1):
        cs.cs_step(st["model"], st["kv"], st["hist"], st["hist_len"], st["room"], st["gamma"], 0, out=st["out"])
    torch.cuda.synchronize()
    greedy = st["hist"][:, n:n + k + 1].cpu().numpy()
    st["hist"].copy_(keep)
    h = st["hist_host"]
    V = st["shape"].vocab
    for b in range(B):
        t = int(taus[b])
        h[b, src[b]:src[b] + t] = greedy[b, :t]
        if t < k:
            h[b, src[b] + t] = (greedy[b, t] + 1) % V
    st["hist"].copy_(torch.from_numpy(h))
    acc, _, dl2 = one_step(st)
    torch.cuda.synchronize()
    assert (dl2.cpu().numpy() == k).all(), "planting the drafts must not move the match"
    return acc.cpu().numpy().copy()
