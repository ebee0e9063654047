"""Pins for the oracle's match search and acceptance rule (CPU only).

The oracle is checked against things other than itself: hand-worked cases,
Python's bytes.find / bytes.rfind as an independent substring search, the
paper's incremental gamma-gram dictionary written separately, and the
positions the input generator planted by construction.
"""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import copyspec_oracle as orc
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _cases(name):
    with open(os.path.join(GOLD, name)) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _cases("find_match_cases.json"))
@pytest.mark.parametrize("impl", ["loop", "np", "dict"])
def test_find_match_hand_cases(case, impl):
    fn = {"loop": orc.find_match, "np": orc.find_match_np, "dict": orc.find_match_dict}[impl]
    m, s, d = fn(case["h"], case["gamma"], 10, case["policy"])
    assert (m, s, list(d)) == (case["match"], case["src"], case["draft"]), case["why"]


def _bytes_search(h, gamma, policy):
    """Independent formulation with the standard library's substring search: the earlier
    occurrence must lie entirely inside h[0 : n-gamma]."""
    n = len(h)
    if n < 2 * gamma:
        return -1
    b = bytes(h)
    suffix = b[n - gamma:]
    return b.rfind(suffix, 0, n - gamma) if policy == "rightmost" else b.find(suffix, 0, n - gamma)


@pytest.mark.parametrize("vocab,nmax", [(2, 11), (3, 8)])
def test_find_match_exhaustive_tiny(vocab, nmax):
    """Every history over a tiny vocabulary, every gamma in 1..4, both policies."""
    k = 4
    for n in range(0, nmax + 1):
        for h in itertools.product(range(vocab), repeat=n):
            h = list(h)
            for gamma in (1, 2, 3, 4):
                for policy in ("rightmost", "first"):
                    want = _bytes_search(h, gamma, policy)
                    m, s, d = orc.find_match(h, gamma, k, policy)
                    assert m == want, (h, gamma, policy)
                    if want >= 0:
                        assert s == want + gamma
                        assert d == h[s:min(s + k, n)]
                    else:
                        assert (s, d) == (-1, [])
                    assert orc.find_match_dict(h, gamma, k, policy) == (m, s, d)
                    if n > 0:
                        assert orc.find_match_np(h, gamma, k, policy) == (m, s, d)


def test_find_match_random_medium_vs_bytes():
    rng = np.random.default_rng(5)
    for _ in range(300):
        n = int(rng.integers(1, 400))
        vocab = int(rng.integers(2, 6))
        h = rng.integers(0, vocab, n).tolist()
        gamma = int(rng.integers(1, 7))
        for policy in ("rightmost", "first"):
            want = _bytes_search(h, gamma, policy)
            for fn in (orc.find_match, orc.find_match_np, orc.find_match_dict):
                m, s, d = fn(h, gamma, 10, policy)
                assert m == want
                if m >= 0:
                    assert d == h[m + gamma:min(m + gamma + 10, n)]


def test_find_match_invariants():
    """Validity, non-overlap (App. B.3 step 1c) and extremality of the returned position."""
    rng = np.random.default_rng(11)
    for _ in range(200):
        n = int(rng.integers(6, 200))
        h = rng.integers(0, 3, n).tolist()
        gamma = int(rng.integers(1, 4))
        for policy in ("rightmost", "first"):
            m, s, d = orc.find_match(h, gamma, 10, policy)
            valid = [p for p in range(0, n - 2 * gamma + 1)
                     if h[p:p + gamma] == h[n - gamma:]]
            if not valid:
                assert m == -1
                continue
            assert h[m:m + gamma] == h[n - gamma:]
            assert m + gamma - 1 < n - gamma
            assert m == (max(valid) if policy == "rightmost" else min(valid))
            assert len(d) == min(10, n - s) and len(d) >= min(10, gamma)


def _bytes_search_context(h, gamma, cap):
    """Independent formulation of the "context" policy with the standard library's substring
    search: a candidate whose x preceding tokens agree with the x tokens before the suffix is
    an occurrence of the last gamma + x tokens that ends before the suffix starts.  The longest
    such x (at most cap) wins, and among its occurrences the rightmost."""
    n = len(h)
    if n < 2 * gamma:
        return -1
    b = bytes(h)
    for x in range(min(cap, n - 2 * gamma), -1, -1):
        q = b.rfind(b[n - gamma - x:], 0, n - gamma)
        if q >= 0:
            return q + x
    return -1


def test_context_policy_exhaustive_and_random(monkeypatch):
    k = 4
    for cap in (64, 2):                     # the cap itself is exercised with a small value
        monkeypatch.setattr(orc, "CONTEXT_CAP", cap)
        for n in range(0, 11):
            for h in itertools.product(range(2), repeat=n):
                h = list(h)
                for gamma in (1, 2, 3):
                    want = _bytes_search_context(h, gamma, cap)
                    m, s, d = orc.find_match(h, gamma, k, "context")
                    assert m == want, (h, gamma, cap)
                    assert orc.find_match_dict(h, gamma, k, "context") == (m, s, d)
                    if n > 0:
                        assert orc.find_match_np(h, gamma, k, "context") == (m, s, d)
                    if m >= 0:
                        assert (s, d) == (m + gamma, h[m + gamma:min(m + gamma + k, n)])
        rng = np.random.default_rng(23)
        for _ in range(200):
            n = int(rng.integers(1, 500))
            h = rng.integers(0, int(rng.integers(2, 5)), n).tolist()
            gamma = int(rng.integers(1, 6))
            want = _bytes_search_context(h, gamma, cap)
            for fn in (orc.find_match, orc.find_match_np, orc.find_match_dict):
                assert fn(h, gamma, 10, "context")[0] == want


def test_context_policy_hand_cases():
    # suffix (7, 8): candidates at 1 (preceded by 5) and 5 (preceded by 6); the suffix is preceded by 5
    h = [5, 7, 8, 1, 6, 7, 8, 2, 5, 7, 8]
    assert orc.find_match(h, 2, 3, "rightmost")[0] == 5
    assert orc.find_match(h, 2, 3, "first")[0] == 1
    assert orc.find_match(h, 2, 3, "context") == (1, 3, [1, 6, 7])
    # equal context lengths (both 0): the rightmost candidate
    h = [3, 7, 8, 1, 4, 7, 8, 2, 5, 7, 8]
    assert orc.find_match(h, 2, 3, "context")[0] == 5
    # a candidate at position 0 has no context
    h = [7, 8, 9, 7, 8]
    assert orc.find_match(h, 2, 3, "context") == (0, 2, [9, 7, 8])
    assert orc.context_length([1, 2, 3, 9, 1, 2, 3], 2, 1) == 2


def test_find_match_bad_args():
    with pytest.raises(ValueError):
        orc.find_match([1, 2, 3], 0, 10)
    with pytest.raises(ValueError):
        orc.find_match_np([1, 2, 3], 1, -1)


@pytest.mark.parametrize("stream", list(range(16)))
def test_planted_ground_truth_cfg2(stream):
    """The generator knows by construction where the final span was copied from; the
    vocabulary makes chance 3-gram collisions negligible (n / V^3 ~ 1e-9)."""
    g = synth.history_cfg2(stream)
    h = g["tokens"]
    assert h.shape == (32768,) and h.dtype == np.int32
    for policy, key in (("rightmost", "rightmost_match"), ("first", "first_match")):
        m, s, d = orc.find_match_np(h, 3, 10, policy)
        assert m == g[key]
        if m >= 0:
            assert d == h[m + 3:m + 13].tolist() and len(d) == 10
    if stream % 2 == 1:
        assert g["rightmost_match"] == -1
    if stream % 4 == 2:
        assert g["rightmost_match"] > g["first_match"] >= 0


def test_planted_ground_truth_other_cfgs():
    for g in (synth.history_cfg1(), synth.history_cfg3(), synth.history_cfg4(0),
              synth.history_cfg4(5), synth.history_cfg5(0), synth.history_cfg5(3)):
        h, k = g["tokens"], g["k"]
        m, s, d = orc.find_match_np(h, 3, k, "rightmost")
        assert m == g["rightmost_match"] >= 0
        assert len(d) == k
        assert orc.find_match_np(h, 3, k, "first")[0] == g["first_match"]


def test_cfg_shapes_and_density():
    g = synth.history_cfg1()
    assert len(g["tokens"]) == 512 and len(g["spans"]) == 4
    assert all(ln == 24 for _, _, ln in g["spans"])
    assert g["spans"][-1][0] + 24 == 512
    cov = sum(ln for _, _, ln in synth.history_cfg2(0)["spans"]) / 32768
    assert 0.04 < cov < 0.07
    g4 = synth.history_cfg4(1)
    assert len(g4["tokens"]) == 2048 + 16384
    assert all(src + ln <= 2048 and dst >= 2048 for dst, src, ln in g4["spans"])
    cov4 = sum(ln for _, _, ln in g4["spans"]) / 16384
    assert 0.18 < cov4 < 0.24
    g5 = synth.history_cfg5(2)
    assert len(g5["tokens"]) == 65536 and g5["edits"] > 0


def test_loop_and_np_agree_on_long_history():
    h = synth.history_cfg2(0, n=3000)["tokens"]
    for policy in ("rightmost", "first"):
        assert orc.find_match(h, 3, 10, policy) == orc.find_match_np(h, 3, 10, policy)


@pytest.mark.parametrize("case", _cases("accept_cases.json"))
def test_accept_hand_cases(case):
    tau, nxt = orc.accept_prefix(case["argmax"], case["draft"])
    assert (tau, nxt) == (case["tau"], case["next"]), case["why"]


def test_argmax_first_ties_and_loop():
    assert orc.argmax_first([1.0, 3.0, 3.0, 2.0]) == 1
    assert orc.argmax_first([-1.0]) == 0
    rng = np.random.default_rng(0)
    for _ in range(50):
        row = rng.integers(0, 5, 40).astype(np.float64)
        best, bi = None, -1
        for i, v in enumerate(row):
            if best is None or v > best:
                best, bi = v, i
        assert orc.argmax_first(row) == bi
