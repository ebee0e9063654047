"""Seeded sweep of cs_verify configurations against the oracle: batch sizes, block sizes
(both attention kernels), ragged draft lengths and cache lengths at and around the 32-token
block and 64-row capacity boundaries, caches with given random contents (Sec. 3.2, App. B.2)."""
import numpy as np
import pytest
import torch

import synth
from synth import ModelShape
from oracle import copyspec_oracle as orc

pytestmark = pytest.mark.gpu
cs = pytest.importorskip("paper_2502_08923_amd.binding")
DEV = "cuda:0"
MARGIN = 1e-2

MINI64 = ModelShape("mini-hd64", 2, 256, 4, 2, 64, 512, 1024, 10000.0, 1e-5, "bf16")
MINI128 = ModelShape("mini-hd128", 3, 512, 8, 2, 128, 1024, 2000, 500000.0, 1e-5, "bf16")
BOUNDARY_LENGTHS = [0, 1, 5, 30, 31, 32, 33, 63, 64, 65, 95, 96, 127, 128, 129, 255, 256, 257, 300, 511, 513]


def t32(a):
    return torch.tensor(np.asarray(a), dtype=torch.int32, device=DEV)


@pytest.mark.parametrize("case", range(12))
def test_verify_sweep(case):
    rng = np.random.default_rng(1000 + case)
    shape = (MINI64, MINI128)[case % 2]
    B = int(rng.integers(1, 5))
    k = int(rng.choice([0, 1, 3, 10, 12, 13, 24, 32]))          # 12/13 straddle the two attention kernels at G=4
    lens = [int(rng.choice(BOUNDARY_LENGTHS)) for _ in range(B)]
    cap = max(lens) + k + 1 + int(rng.integers(0, 70))
    w = synth.model_weights(shape, 3000 + case, threads=4)
    model = cs.Model(w, max_batch=B, max_k=k)
    kv = cs.KV(model, B, cap)
    okvs = []
    for b, n in enumerate(lens):
        okv = orc.KVCache(shape, cap + 64)
        for layer in range(shape.n_layers):
            kr, vr = synth.random_kv(shape, n, 50 + case, layer, b)
            if n:
                kv.load(layer, b, 0, kr, vr)
            okv.load(layer, kr, vr)
        okv.truncate(n)
        kv.set_len(b, n)
        okvs.append(okv)
    pending = rng.integers(0, shape.vocab, B)
    draft = rng.integers(0, shape.vocab, (B, max(k, 1)))
    dlen = rng.integers(0, k + 1, B)
    acc, nxt, logits = cs.cs_verify(model, kv, t32(pending), t32(draft[:, :k]) if k else t32(np.zeros((B, 0))),
                                    t32(dlen), k, want_logits=True)
    torch.cuda.synchronize()
    logits = logits.cpu().numpy()
    for b in range(B):
        d = draft[b, :dlen[b]].tolist()
        tau, nx, ol = orc.verify(w, okvs[b], int(pending[b]), d)
        err = np.abs(logits[b, :len(d) + 1] - ol).max()
        assert err <= 2e-2, (case, b, lens[b], k, len(d), err)
        rows = [np.partition(ol[i], -2)[-2:] for i in range(tau + 1)]
        if all(r[1] - r[0] > MARGIN for r in rows):
            assert (int(acc[b]), int(nxt[b])) == (tau, nx), (case, b)
            assert kv.len(b) == lens[b] + tau + 1 == okvs[b].length
    kv.destroy()
    model.destroy()
