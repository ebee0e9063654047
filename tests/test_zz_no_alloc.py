"""The match-search entry point that allocates nothing (cs_find_match_batch_dev_noalloc) against
the allocating one (cs_find_match_batch_dev): bit-exact outputs on two calls in a row, the second
with a smaller input, so that keys left in the shared static array by the first call would show if
the second read them; then the size limit."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu
cs = pytest.importorskip("paper_2502_08923_amd.binding")
DEV = "cuda:0"


def _histories(B, n, vocab, seed):
    hs = np.zeros((B, n), dtype=np.int32)
    lens = np.zeros(B, dtype=np.int32)
    for b in range(B):
        ln = n if b % 3 else max(8, n - 97 * b)                   # ragged lengths
        g = synth.planted_history(seed + b, ln, vocab, (8, 40), density=0.1,
                                  end="span" if b % 2 == 0 else "fresh", twice=(b % 4 == 2))
        hs[b, :ln] = g["tokens"]
        lens[b] = ln
    return hs, lens


def _same(a, b):
    for x, y in zip(a, b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("policy", ["rightmost", "first", "context"])
def test_noalloc_equals_allocating_entry_point_twice_in_a_row(policy):
    # first call: 48 histories of 20000 tokens (5 chunks each: 240 keys in the static array)
    hs, lens = _histories(48, 20000, 500, 9100)
    d_hist, d_len = torch.from_numpy(hs).to(DEV), torch.from_numpy(lens).to(DEV)
    want = cs.cs_find_match_batch_dev(d_hist, d_len, 3, 10, policy)
    got = cs.cs_find_match_batch_dev_noalloc(d_hist, d_len, 3, 10, policy)
    torch.cuda.synchronize()
    _same(want, got)
    assert int((want[0] >= 0).sum()) >= 24                         # matches exist
    # second call, smaller in both dimensions (5 histories of 3000 tokens: one chunk each); the
    # keys of the first call are still in the array
    hs2, lens2 = _histories(5, 3000, 7, 9200)                      # tiny vocabulary: many candidates
    d_hist2, d_len2 = torch.from_numpy(hs2).to(DEV), torch.from_numpy(lens2).to(DEV)
    want2 = cs.cs_find_match_batch_dev(d_hist2, d_len2, 2, 16, policy)
    got2 = cs.cs_find_match_batch_dev_noalloc(d_hist2, d_len2, 2, 16, policy)
    torch.cuda.synchronize()
    _same(want2, got2)
    # and the first input again, into caller-provided outputs
    out = tuple(torch.full_like(t, -7) for t in want)
    cs.cs_find_match_batch_dev_noalloc(d_hist, d_len, 3, 10, policy, out=out)
    torch.cuda.synchronize()
    _same(want, out)


def test_noalloc_rejects_sizes_beyond_the_static_array():
    B, stride = 17, 4096 * 4096                                    # 17 * 4096 chunks > 65536
    d_len = torch.zeros(B, dtype=torch.int32, device=DEV)
    d_hist = torch.zeros((1, 8), dtype=torch.int32, device=DEV)    # never read: the call is refused first
    lib = cs.load_library()
    out = torch.zeros(B * 12, dtype=torch.int32, device=DEV)
    rc = lib.cs_find_match_batch_dev_noalloc(d_hist.data_ptr(), stride, d_len.data_ptr(), B, 3, 10, 0,
                                             None, None, out.data_ptr(), out.data_ptr(), None)
    assert rc == -3 and b"static scratch" in lib.cs_last_error()
    # the largest size that fits is accepted (zero-length histories: nothing to scan, no match)
    B = 16
    d_len = torch.zeros(B, dtype=torch.int32, device=DEV)
    big = torch.zeros((B, 4096 * 4096), dtype=torch.int32, device=DEV)        # 1 GiB
    mp, sp, dr, dl = cs.cs_find_match_batch_dev_noalloc(big, d_len, 3, 10)
    torch.cuda.synchronize()
    assert mp.tolist() == [-1] * B and dl.tolist() == [0] * B
