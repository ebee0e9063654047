"""CPU checks of the replay workloads and of the sweep's acceptance replay (host logic only;
the match search is the oracle's here)."""
import numpy as np

import synth
from oracle import copyspec_oracle as orc
from paper_2502_08923_amd import sweep


class OracleSearch:
    @staticmethod
    def cs_find_match_ex(hist, gamma, k, policy):
        return orc.find_match_np(np.asarray(hist), gamma, k, policy)


def test_multiturn_replay_structure():
    g = synth.multiturn_replay(3)
    h = synth.multiturn_replay(3)
    assert np.array_equal(g["context"], h["context"]) and np.array_equal(g["truth"], h["truth"])
    ctx, truth = g["context"], g["truth"]
    assert ctx.shape == (5 * 1024,) and truth.shape == (1024,) and ctx.dtype == np.int32
    v1, v2 = ctx[1024:2048], ctx[3072:4096]
    e12, e23, e13 = (v1 != v2).mean(), (v2 != truth).mean(), (v1 != truth).mean()
    assert 0.02 < e12 < 0.08 and 0.02 < e23 < 0.08          # 5 % edits per version
    assert e13 > max(e12, e23)                               # edits accumulate
    assert not np.array_equal(synth.multiturn_replay(4)["truth"], truth)


def test_zipf_replay_structure():
    g = synth.zipf_replay(0)
    ctx, truth = g["context"], g["truth"]
    assert ctx.shape == (6144,) and truth.shape == (2048,)
    assert ctx.min() >= 0 and ctx.max() < 128256
    # heavy head: the most frequent token covers several per cent of the context
    counts = np.bincount(ctx)
    assert counts.max() / ctx.size > 0.05
    # about 30 % of the answer is verbatim context: count answer 8-grams that occur in the context
    grams = {tuple(ctx[i:i + 8]) for i in range(ctx.size - 7)}
    hit = sum(tuple(truth[i:i + 8]) in grams for i in range(truth.size - 7)) / (truth.size - 7)
    assert 0.15 < hit < 0.45


def test_replay_host_logic():
    # k = 0 is plain decoding: one token per step, no attempts
    assert sweep.replay_acceptance(OracleSearch, synth, 3, 0, "rightmost", streams=(0,)) == (1.0, 0.0)
    tps = [sweep.replay_acceptance(OracleSearch, synth, 3, k, "rightmost", streams=(0,))[0] for k in (2, 5, 10)]
    assert 1.0 < tps[0] < tps[1] < tps[2]                   # larger blocks emit more per step
    r = sweep.replay_acceptance(OracleSearch, synth, 3, 10, "rightmost", streams=(0, 1))
    f = sweep.replay_acceptance(OracleSearch, synth, 3, 10, "first", streams=(0, 1))
    assert r[0] > f[0] and r[1] > f[1]                       # the newer version is the better source
    # accepted drafts per attempt can never exceed the block size
    for k in (2, 10):
        assert sweep.replay_acceptance(OracleSearch, synth, 2, k, "context", streams=(0,), workload="zipf")[1] <= k
