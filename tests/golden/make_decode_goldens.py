#!/usr/bin/env python3
"""Writes the stored greedy continuations that the GPU parity tests at the headline sizes
compare against.  Calls only the CPU oracle and the seeded input generators; nothing here
touches the HIP library.  Run from the repository root:

    python tests/golden/make_decode_goldens.py cfg3     # -> tests/golden/cfg3_greedy_256.json
    python tests/golden/make_decode_goldens.py cfg4     # -> tests/golden/cfg4_greedy_chain.json

cfg3: Llama-style 1B shape (seed of configuration 3), the 4096-token planted history as the
prompt, plain greedy decoding of 256 tokens (Sec. 3.2: CopySpec must emit exactly these), with
the top-2 logit margin of every decision.

cfg4: Llama-style 8B shape at full depth (seed of configuration 4), stream 0 of the batch-8
workload: the cache holds 18431 rows of seeded random K/V (synth.random_kv), the pending token is
the last token of the stream's history; eleven plain greedy steps from that state give the
tokens a fully accepted 10-token draft must consist of (App. B.2: a draft token is accepted iff
it is the target's argmax) plus the token that follows them, each with its margin.

Runtime on 8 host cores: about 25 minutes (cfg3) and 15 minutes (cfg4); cfg4 needs ~40 GB of RAM.
"""
from __future__ import annotations

import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth                                        # noqa: E402
from oracle import copyspec_oracle as orc           # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def top2_margin(row) -> float:
    top = np.partition(np.asarray(row), -2)[-2:]
    return float(top[1] - top[0])


def greedy_chain(w, okv, pending, steps, tag):
    """Plain greedy steps; per step the token, the runner-up (second largest logit) and the gap."""
    toks, runner_up, margins = [], [], []
    for i in range(steps):
        t0 = time.time()
        logits = orc.forward_block(w, okv, [int(pending)])[0]
        okv.truncate(okv.length + 1)
        pending = orc.argmax_first(logits)
        rest = logits.copy()
        rest[pending] = -np.inf
        toks.append(int(pending))
        runner_up.append(orc.argmax_first(rest))
        margins.append(top2_margin(logits))
        print(f"[{tag}] step {i}: token {pending}, margin {margins[-1]:.4f}, {time.time() - t0:.1f}s", flush=True)
    return toks, runner_up, margins


def cfg3():
    shape = synth.LLAMA_1B
    w = synth.model_weights(shape, synth.seed_for(3), threads=8)
    prompt = synth.history_cfg3()["tokens"].tolist()
    okv = orc.KVCache(shape, len(prompt) + 256 + 16)
    pending = orc.prefill(w, okv, prompt, chunk=512)
    toks, runner_up, margins = greedy_chain(w, okv, pending, 256, "cfg3")
    out = {"what": "oracle greedy continuation, configuration 3 (1B shape, 4096-token prompt, 256 new tokens)",
           "weights_seed": synth.seed_for(3), "prompt": "synth.history_cfg3()", "tokens": toks, "runner_up": runner_up, "margins": margins}
    json.dump(out, open(os.path.join(HERE, "cfg3_greedy_256.json"), "w"))


def cfg4():
    shape = synth.LLAMA_8B
    seed = synth.seed_for(4)
    L = 2048 + 16384 - 1
    w = synth.model_weights(shape, seed, threads=8)
    okv = orc.KVCache(shape, L + 16)
    for layer in range(shape.n_layers):
        kr, vr = synth.random_kv(shape, L, seed, layer, 0)
        okv.load(layer, kr, vr)
    okv.truncate(L)
    pending = int(synth.history_cfg4(0)["tokens"][-1])
    toks, runner_up, margins = greedy_chain(w, okv, pending, 11, "cfg4")
    out = {"what": "oracle greedy chain, configuration 4 stream 0 (8B shape, 32 layers, 18431 cached rows of "
                   "synth.random_kv(seed_for(4), layer, 0), pending = last token of synth.history_cfg4(0))",
           "weights_seed": seed, "kv_len": L, "pending": pending, "tokens": toks, "runner_up": runner_up, "margins": margins}
    json.dump(out, open(os.path.join(HERE, "cfg4_greedy_chain.json"), "w"))


if __name__ == "__main__":
    {"cfg3": cfg3, "cfg4": cfg4}[sys.argv[1]]()
