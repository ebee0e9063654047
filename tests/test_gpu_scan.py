"""GPU parity of the match scan and draft gather against the CPU oracle: bit-exact."""
import json
import os

import numpy as np
import pytest
import torch

import synth
from oracle import copyspec_oracle as orc

pytestmark = pytest.mark.gpu
cs = pytest.importorskip("paper_2502_08923_amd.binding")
GOLD = os.path.join(os.path.dirname(__file__), "golden")
DEV = "cuda:0"


def _batch(histories, stride=None):
    B = len(histories)
    lens = [len(h) for h in histories]
    stride = stride or max(4, -(-max(lens + [1]) // 4) * 4)
    buf = np.full((B, stride), -7, dtype=np.int32)
    for b, h in enumerate(histories):
        buf[b, :len(h)] = h
    return (torch.from_numpy(buf).to(DEV), torch.tensor(lens, dtype=torch.int32, device=DEV))


def _check_batch(histories, gamma, k, policy, stride=None):
    d_hist, d_len = _batch(histories, stride)
    mp, sp, dr, dl = cs.cs_find_match_batch_dev(d_hist, d_len, gamma, k, policy)
    torch.cuda.synchronize()
    mp, sp, dr, dl = (t.cpu().numpy() for t in (mp, sp, dr, dl))
    for b, h in enumerate(histories):
        m, s, d = orc.find_match_np(h, gamma, k, policy) if len(h) else (-1, -1, [])
        assert (mp[b], sp[b], dl[b]) == (m, s, len(d)), (b, len(h), gamma, k, policy)
        assert dr[b, :len(d)].tolist() == d
        assert (dr[b, len(d):] == -1).all()


def test_hand_cases():
    for case in json.load(open(os.path.join(GOLD, "find_match_cases.json")))["cases"]:
        got = cs.cs_find_match_ex(case["h"], case["gamma"], 10, case["policy"])
        assert got == (case["match"], case["src"], case["draft"]), case["why"]
        if case["policy"] == "rightmost":
            assert cs.cs_find_match(case["h"], case["gamma"]) == case["src"]


@pytest.mark.parametrize("policy", ["rightmost", "first", "context"])
def test_cfg2_all_histories(policy):
    """Configuration 2 in full: 64 histories x 32768 tokens, gamma=3, k=10."""
    gens = [synth.history_cfg2(s) for s in range(64)]
    hs = [g["tokens"] for g in gens]
    _check_batch(hs, 3, 10, policy, stride=32768)
    d_hist, d_len = _batch(hs, 32768)
    mp = cs.cs_find_match_batch_dev(d_hist, d_len, 3, 10, policy)[0].cpu().numpy()
    if policy != "context":      # the generator records where the extreme candidates were planted
        key = "rightmost_match" if policy == "rightmost" else "first_match"
        assert mp.tolist() == [g[key] for g in gens]


@pytest.mark.parametrize("gamma", [1, 2, 3, 5, 16])
@pytest.mark.parametrize("k", [0, 1, 10, 32])
def test_ragged_lengths_small_vocab(gamma, k):
    """Ragged batch over a tiny vocabulary (many matches, overlap rule exercised), lengths
    from empty to several scan chunks with a ragged tail."""
    rng = np.random.default_rng(100 * gamma + k)
    lens = [0, 1, 2, 5, 6, 7, 63, 64, 65, 4095, 4096, 4097, 8191, 12289, 20000, 33]
    hs = [rng.integers(0, 2 + (i % 3), n).astype(np.int32) for i, n in enumerate(lens)]
    for policy in ("rightmost", "first", "context"):
        _check_batch(hs, gamma, k, policy, stride=20000)


def test_degenerate_histories():
    same = np.full(9000, 5, dtype=np.int32)
    period = np.tile(np.array([1, 2, 3], dtype=np.int32), 3000)
    nomatch = np.arange(10000, dtype=np.int32)
    late = np.concatenate([np.arange(5000), [7, 8, 9, 1, 2, 3], np.arange(100, 300), [7, 8, 9]]).astype(np.int32)
    for policy in ("rightmost", "first", "context"):
        _check_batch([same, period, nomatch, late], 3, 10, policy)
    # unaligned stride takes the scalar load path
    _check_batch([same[:777], period[:1001], late], 3, 10, "rightmost", stride=5211)


def test_other_configurations_and_long_history():
    for g in (synth.history_cfg1(), synth.history_cfg3(), synth.history_cfg4(0), synth.history_cfg5(1)):
        got = cs.cs_find_match_ex(g["tokens"], 3, g["k"], "rightmost")
        assert got == orc.find_match_np(g["tokens"], 3, g["k"], "rightmost")
        assert got[0] == g["rightmost_match"]
    rng = np.random.default_rng(7)
    big = rng.integers(0, 50000, 3_000_001).astype(np.int32)
    big[-3:] = big[1_234_567:1_234_570]
    got = cs.cs_find_match_ex(big, 3, 10, "rightmost")
    assert got == orc.find_match_np(big, 3, 10, "rightmost") and got[0] >= 1_234_567


def test_empty_batch_and_bad_arguments():
    d_hist = torch.zeros((0, 8), dtype=torch.int32, device=DEV)
    d_len = torch.zeros(0, dtype=torch.int32, device=DEV)
    cs.cs_find_match_batch_dev(d_hist, d_len, 3, 10)
    assert cs.cs_find_match([], 3) == -1
    assert cs.cs_find_match([1, 2, 3, 4, 5], 3) == -1
    for bad in (dict(gamma=0, k=10), dict(gamma=17, k=10), dict(gamma=3, k=-1), dict(gamma=3, k=257)):
        with pytest.raises(cs.CopySpecError) as e:
            cs.cs_find_match_ex([1, 2, 3, 1, 2, 3], bad["gamma"], bad["k"])
        assert e.value.code == -2
    with pytest.raises(cs.CopySpecError):
        cs.cs_find_match_ex([1, 2, 3], 3, 10, policy=7)


def test_deterministic_repeat():
    hs = [synth.history_cfg2(s)["tokens"] for s in range(8)]
    d_hist, d_len = _batch(hs, 32768)
    a = [t.clone() for t in cs.cs_find_match_batch_dev(d_hist, d_len, 3, 10)]
    b = cs.cs_find_match_batch_dev(d_hist, d_len, 3, 10)
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(a, b))


@pytest.mark.parametrize("policy", ["rightmost", "first", "context"])
def test_acceptance_replay_matches_oracle(policy):
    """The gamma/k/policy sweep replays a synthetic self-correction dialogue through the library's
    match search; the same replay through the oracle's search must emit the same number of
    tokens per step (Sec. 5.1, Sec. 5.2: the quantities those sweeps vary)."""
    from paper_2502_08923_amd import sweep

    class OracleSearch:
        @staticmethod
        def cs_find_match_ex(hist, gamma, k, pol):
            return orc.find_match_np(np.asarray(hist), gamma, k, pol)

    for gamma, k in [(2, 5), (3, 10), (5, 32)]:
        got = sweep.replay_acceptance(cs, synth, gamma, k, policy, streams=(0,))
        want = sweep.replay_acceptance(OracleSearch, synth, gamma, k, policy, streams=(0,))
        assert got == want, (gamma, k, policy, got, want)
    # Zipf-law tokens: many chance matches of frequent gamma-grams
    got = sweep.replay_acceptance(cs, synth, 2, 10, policy, streams=(1,), workload="zipf")
    want = sweep.replay_acceptance(OracleSearch, synth, 2, 10, policy, streams=(1,), workload="zipf")
    assert got == want
    # the newest version of the answer is the better copy source
    r = sweep.replay_acceptance(OracleSearch, synth, 3, 10, "rightmost", streams=(0,))
    f = sweep.replay_acceptance(OracleSearch, synth, 3, 10, "first", streams=(0,))
    assert r[0] > f[0]
