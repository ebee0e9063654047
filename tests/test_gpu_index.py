"""GPU parity of the gamma-gram hash index (the paper's own data structure, Sec. 3.1, App. B.1,
App. B.3 steps 1b / 2d) against the CPU oracle and against the scan: bit-exact."""
import numpy as np
import pytest
import torch

import synth
from oracle import copyspec_oracle as orc

pytestmark = pytest.mark.gpu
cs = pytest.importorskip("paper_2502_08923_amd.binding")
DEV = "cuda:0"


def _batch(histories, stride):
    buf = np.full((len(histories), stride), -7, dtype=np.int32)
    for b, h in enumerate(histories):
        buf[b, :len(h)] = h
    lens = torch.tensor([len(h) for h in histories], dtype=torch.int32, device=DEV)
    return torch.from_numpy(buf).to(DEV), lens


def _check(ix, d_hist, d_len, histories, gamma, k, policy, hint):
    mp, sp, dr, dl = cs.cs_index_find_match_batch_dev(ix, d_hist, d_len, hint, k, policy)
    torch.cuda.synchronize()
    mp, sp, dr, dl = (t.cpu().numpy() for t in (mp, sp, dr, dl))
    for b, h in enumerate(histories):
        m, s, d = orc.find_match_np(h, gamma, k, policy) if len(h) else (-1, -1, [])
        assert (mp[b], sp[b], dl[b]) == (m, s, len(d)), (b, len(h), gamma, k, policy)
        assert dr[b, :len(d)].tolist() == d
        assert (dr[b, len(d):] == -1).all()


@pytest.mark.parametrize("gamma", [1, 2, 3, 5, 16])
def test_full_build_ragged_small_vocab(gamma):
    """Ragged batch over a tiny vocabulary: many occurrences per gram (max / min folding) and
    many grams per slot neighbourhood; lengths from empty to 20000."""
    rng = np.random.default_rng(40 + gamma)
    lens = [0, 1, 2, 5, 6, 7, 63, 64, 65, 4095, 4096, 4097, 8191, 12289, 20000, 33]
    hs = [rng.integers(0, 2 + (i % 3), n).astype(np.int32) for i, n in enumerate(lens)]
    d_hist, d_len = _batch(hs, 20000)
    ix = cs.Index(len(hs), 20000, gamma)
    for policy in ("rightmost", "first"):
        _check(ix, d_hist, d_len, hs, gamma, 10, policy, 20000)    # second pass inserts nothing new
    ix.destroy()


def test_cfg2_equals_scan():
    hs = [synth.history_cfg2(s)["tokens"] for s in range(64)]
    d_hist, d_len = _batch(hs, 32768)
    ix = cs.Index(64, 32768, 3)
    for policy in ("rightmost", "first"):
        a = cs.cs_index_find_match_batch_dev(ix, d_hist, d_len, 32768, 10, policy)
        b = cs.cs_find_match_batch_dev(d_hist, d_len, 3, 10, policy)
        torch.cuda.synchronize()
        assert all(torch.equal(x, y) for x, y in zip(a, b))
    _check(ix, d_hist, d_len, hs, 3, 10, "rightmost", 0)
    ix.destroy()


def test_incremental_growth_follows_the_oracle():
    """Histories grow by a few tokens between lookups, as in decoding (App. B.3 step 2d); every
    intermediate answer equals the oracle's on the history so far.  Small hints exercise the
    launch sizing, a hint of 0 the loop that inserts whatever is missing."""
    rng = np.random.default_rng(9)
    B, gamma, k, cap = 6, 3, 8, 1200
    full = [rng.integers(0, 3 + b, cap).astype(np.int32) for b in range(B)]
    for b in range(B):                                   # planted repeats
        full[b][700:760] = full[b][100:160]
        full[b][900:930] = full[b][705:735]
    d_hist, _ = _batch(full, cap)
    lens = np.array([7, 40, 300, 650, 2, 0])
    ix = cs.Index(B, cap, gamma)
    step = 0
    while (lens < cap).any():
        d_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
        hs = [full[b][:lens[b]] for b in range(B)]
        grow_hint = [11, 0, 64][step % 3] if step else cap
        _check(ix, d_hist, d_len, hs, gamma, k, ("rightmost", "first")[step % 2], grow_hint)
        lens = np.minimum(lens + rng.integers(0, 12, B), cap)
        step += 1
    assert step > 100
    # after a reset the same index serves unrelated histories
    ix.reset()
    other = [rng.integers(0, 4, 500).astype(np.int32) for _ in range(B)]
    d_hist2, d_len2 = _batch(other, cap)
    _check(ix, d_hist2, d_len2, other, gamma, k, "rightmost", cap)
    ix.destroy()


def test_long_history_and_errors():
    rng = np.random.default_rng(7)
    big = rng.integers(0, 50000, 3_000_001).astype(np.int32)
    big[-3:] = big[1_234_567:1_234_570]
    d_hist, d_len = _batch([big], 3_000_004)
    ix = cs.Index(1, 3_000_004, 3)
    _check(ix, d_hist, d_len, [big], 3, 10, "rightmost", 3_000_004)
    with pytest.raises(cs.CopySpecError) as e:
        cs.cs_index_find_match_batch_dev(ix, d_hist, d_len, 0, 10, "context")
    assert e.value.code == -6
    ix.destroy()
    small = cs.Index(1, 100, 3)
    with pytest.raises(cs.CopySpecError):                # stride beyond the index's max_len
        cs.cs_index_find_match_batch_dev(small, d_hist, d_len, 0, 10)
    small.destroy()
    with pytest.raises(cs.CopySpecError):
        cs.Index(1, 100, 0)
