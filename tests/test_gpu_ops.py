"""Per-kernel GPU parity at the benchmark's full shapes (sampled outputs) and edge cases.

The oracle computes sampled outputs one by one (a GEMM column, an attention head, an argmax
row); every stream is independent, so a sampled stream is a complete check of that stream.
"""
import numpy as np
import pytest
import torch

import synth
from synth import ModelShape
from oracle import copyspec_oracle as orc

pytestmark = pytest.mark.gpu
cs = pytest.importorskip("paper_2502_08923_amd.binding")
DEV = "cuda:0"

HOST = ModelShape("host-8b-width", 1, 4096, 32, 8, 128, 14336, 2048, 500000.0, 1e-5, "bf16")


def t32(a):
    return torch.tensor(np.asarray(a), dtype=torch.int32, device=DEV)


def bf16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(DEV)


@pytest.fixture(scope="module")
def host_model():
    """A one-layer model at the 8B width: owns the workspace the op entry points use."""
    w = synth.model_weights(HOST, 99, threads=16)
    m = cs.Model(w, max_batch=16, max_k=32)
    yield m
    m.destroy()


# ----------------------------------------------------------------------------------------
# argmax + accept
# ----------------------------------------------------------------------------------------

@pytest.mark.parametrize("B,k,V", [(8, 10, 128256), (16, 32, 128256), (3, 4, 97), (1, 0, 1024)])
def test_argmax_accept_full_size(host_model, B, k, V):
    rng = np.random.default_rng(B * 1000 + k)
    logits = rng.standard_normal((B, k + 1, V)).astype(np.float32)
    # exact ties: duplicate the maximum at a later index in some rows (lowest index must win)
    for b in range(B):
        for i in range(0, k + 1, 3):
            j = int(np.argmax(logits[b, i]))
            if j + 5 < V:
                logits[b, i, j + 5] = logits[b, i, j]
    am = np.array([[orc.argmax_first(logits[b, i]) for i in range(k + 1)] for b in range(B)])
    draft = np.zeros((B, max(k, 1)), dtype=np.int32)
    dlen = np.zeros(B, dtype=np.int32)
    for b in range(B):
        m = int(rng.integers(0, k + 1))
        dlen[b] = m
        draft[b, :k] = rng.integers(0, V, k) if k else 0
        good = int(rng.integers(0, m + 1))                 # accept exactly `good`, unless luck
        draft[b, :good] = am[b, :good]
    acc, nxt, ram = cs.cs_op_argmax_accept(host_model, torch.from_numpy(logits).to(DEV),
                                           t32(draft[:, :k]) if k else t32(np.zeros((B, 0))),
                                           t32(dlen))
    torch.cuda.synchronize()
    assert np.array_equal(ram.cpu().numpy(), am)
    for b in range(B):
        tau, nx = orc.accept_prefix(am[b], draft[b, :dlen[b]].tolist())
        assert (int(acc[b]), int(nxt[b])) == (tau, nx)


# ----------------------------------------------------------------------------------------
# projections at the 8B shapes, R = 88 (benchmark) and 528 (batch 16, k = 32)
# ----------------------------------------------------------------------------------------

def _gemm_case(host_model, N, K, R):
    seed = N * 7 + K + R
    xb = synth.workloads._draw(seed, (R, K), "n", 1.0, "bf16")
    wb = synth.workloads._draw(seed + 1, (N, K), "u", (3.0 / K) ** 0.5, "bf16")
    Y = cs.cs_op_gemm(host_model, bf16_dev(xb), bf16_dev(wb)).cpu().numpy()
    rng = np.random.default_rng(seed)
    cols = np.unique(np.concatenate([rng.integers(0, N, 192), [0, 15, 16, N - 17, N - 1]]))
    x64 = synth.bf16_bits_to_f32(xb).astype(np.float64)
    w64 = synth.bf16_bits_to_f32(wb[cols]).astype(np.float64)
    ref = x64 @ w64.T
    err = np.abs(Y[:, cols] - ref).max()
    assert err < 2e-4 * max(1.0, np.abs(ref).max()), err      # fp32 accumulation of exact products


@pytest.mark.parametrize("N,K", [(6144, 4096), (4096, 4096), (28672, 4096), (4096, 14336),
                                 (128256, 4096)])
@pytest.mark.parametrize("R", [88, 528, 1])
def test_gemm_bf16_full_shapes(host_model, N, K, R):
    _gemm_case(host_model, N, K, R)


@pytest.mark.parametrize("R", [97, 120, 168, 200, 250, 264, 300, 408, 528])
@pytest.mark.parametrize("N,K", [(49168, 512), (49168, 128), (6144, 4096)])
def test_gemm_row_sweep(host_model, N, K, R):
    """Row counts between the two regimes.  The 193 W tiles of the 49168-row matrix send every
    row count above 96 to the many-row kernel (each of its row-tile counts, one and two row
    blocks, ragged last tiles in both dimensions, K of one and of four pipeline trips); the
    q/k/v shape switches kernels at 289 rows and is split along K."""
    _gemm_case(host_model, N, K, R)


def test_gemm_tiny_weights_are_not_flushed(host_model):
    """The tuned projections multiply in float16 (weights converted from bfloat16, exactly for
    |w| >= 2^-17).  Weights in float16's subnormal range must still contribute."""
    N, K, R = 64, 512, 16
    rng = np.random.default_rng(3)
    w = (rng.integers(1, 8, (N, K)) * 2.0 ** -17 * rng.choice([-1.0, 1.0], (N, K))).astype(np.float32)
    x = (rng.integers(1, 4, (R, K)) * 256.0).astype(np.float32)
    wb, xb = synth.f32_to_bf16_bits(w), synth.f32_to_bf16_bits(x)
    assert np.array_equal(synth.bf16_bits_to_f32(wb), w) and np.array_equal(synth.bf16_bits_to_f32(xb), x)
    Y = cs.cs_op_gemm(host_model, bf16_dev(xb), bf16_dev(wb)).cpu().numpy()
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.abs(ref).max() > 0.05
    assert np.abs(Y - ref).max() <= 1e-5 * np.abs(ref).max() + 1e-7


def test_gemm_f32_plain(host_model):
    rng = np.random.default_rng(5)
    X = rng.standard_normal((11, 256)).astype(np.float32)
    W = rng.standard_normal((777, 256)).astype(np.float32)
    Y = cs.cs_op_gemm(host_model, torch.from_numpy(X).to(DEV), torch.from_numpy(W).to(DEV))
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    assert np.abs(Y.cpu().numpy() - ref).max() < 1e-4


# ----------------------------------------------------------------------------------------
# block attention
# ----------------------------------------------------------------------------------------

def _attention_case(model, shape, lens, rows, sample, seed, poison=False, k_ramp=None, device_fill=False):
    """device_fill: streams the oracle does not look at get their cache rows from a device-side
    generator (cheap at long lengths); sampled streams always get the seeded host rows."""
    B = len(lens)
    cap = max(lens) + rows + 5
    kv = cs.KV(model, B, cap)
    ks, vs = {}, {}
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    for b, L in enumerate(lens):
        if device_fill and b not in {sb for sb, _ in sample}:
            shp = (shape.n_kv_heads, L + rows, shape.head_dim)
            kv.load(0, b, 0, torch.randn(shp, generator=gen, device=DEV).bfloat16(),
                    torch.randn(shp, generator=gen, device=DEV).bfloat16())
            kv.set_len(b, L)
            continue
        kr, vr = synth.random_kv(shape, L + rows, seed, 0, b)
        if k_ramp is not None:
            # keys scaled along the sequence: the scores, and with them the running maximum of
            # the online softmax, drift by many powers of two over the cache
            t = np.arange(L + rows, dtype=np.float32) / max(L + rows - 1, 1)
            scale = (k_ramp[0] + (k_ramp[1] - k_ramp[0]) * t)[None, :, None]
            kr = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(kr) * scale)
        kv.load(0, b, 0, kr, vr)
        if poison and L + rows + 3 <= cap:
            # rows past the block are dead: whatever they hold must not matter
            bad = np.full((shape.n_kv_heads, 3, shape.head_dim), 0x7FC0, dtype=np.uint16)  # bf16 NaN
            kv.load(0, b, L + rows, bad, bad)
        kv.set_len(b, L)
        ks[b], vs[b] = kr, vr
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, rows, shape.n_heads, shape.head_dim)).astype(np.float32)
    if k_ramp is not None:
        # with scores this large the rounding of the queries to bfloat16 (what the tuned kernels
        # take) moves the softmax weights by percents: give both sides the rounded queries
        q = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(q))
    out = cs.cs_op_attention(model, kv, 0, torch.from_numpy(q).to(DEV)).cpu().numpy()
    G = shape.n_heads // shape.n_kv_heads
    worst = 0.0
    for b, h in sample:
        L = lens[b]
        kc = synth.bf16_bits_to_f32(ks[b][h // G]).astype(np.float64)
        vc = synth.bf16_bits_to_f32(vs[b][h // G]).astype(np.float64)
        ref = orc.causal_attention(q[b, :, h].astype(np.float64), kc, vc, L + np.arange(rows))
        got = out[b, :, h * shape.head_dim:(h + 1) * shape.head_dim]
        err = np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-6)
        worst = max(worst, err)
    kv.destroy()
    return worst


def test_attention_benchmark_shape(host_model):
    """8 streams x 18431 cached rows, 11 block rows, 32 heads over 8 KV heads, hd 128."""
    worst = _attention_case(host_model, HOST, [18431] * 8, 11,
                            [(0, 0), (0, 31), (3, 13), (7, 5), (5, 22)], seed=11)
    assert worst < 1e-2, worst


def test_attention_ragged_and_degenerate_lengths(host_model):
    lens = [0, 1, 31, 32, 33, 1000, 4097, 129]
    sample = [(b, h) for b in range(8) for h in (0, 17, 31)]
    worst = _attention_case(host_model, HOST, lens, 11, sample, seed=12, poison=True)
    assert worst < 1e-2, worst
    worst = _attention_case(host_model, HOST, [5, 300], 1, [(0, 3), (1, 30)], seed=13, poison=True)
    assert worst < 1e-2, worst


def test_attention_k32_block(host_model):
    """k = 32: 132 query rows per KV head, three query groups per workgroup column."""
    worst = _attention_case(host_model, HOST, [3000, 2999, 64, 7], 33,
                            [(0, 0), (0, 3), (1, 12), (2, 31), (3, 8)], seed=14)
    assert worst < 1e-2, worst


def test_attention_k32_block_65535_rows_batch16(host_model):
    """The long multi-turn configuration's launch: 16 streams x 65535 cached rows, 33 block rows
    (132 query rows per KV head, the wide-block kernel), 128-token V blocks up to index 511.
    Five (stream, head) pairs are checked element by element against the oracle's attention."""
    worst = _attention_case(host_model, HOST, [65535] * 16, 33,
                            [(0, 0), (3, 31), (9, 14), (15, 7), (15, 24)], seed=17, device_fill=True)
    assert worst < 1e-2, worst


def test_attention_k32_block_long_ragged(host_model):
    """Wide-block kernel with ragged long caches (lengths around the 128-token V blocks and the
    32-token K blocks) next to an empty one; rows past the block poisoned."""
    worst = _attention_case(host_model, HOST, [40000, 0, 16383, 16385, 127, 32769], 33,
                            [(0, 5), (1, 0), (2, 31), (3, 16), (4, 9), (5, 20)], seed=18, poison=True)
    assert worst < 1e-2, worst


@pytest.mark.parametrize("rows", [11, 33])
@pytest.mark.parametrize("k_ramp", [(0.05, 6.0), (6.0, 0.05)])
def test_attention_drifting_maximum(host_model, rows, k_ramp):
    """Keys that grow (shrink) 120-fold along the cache: the row maxima rise by far more than
    the 2^8 slack of the lazily updated reference again and again (or sit at the start, with
    everything after it far below), in both tuned kernels."""
    worst = _attention_case(host_model, HOST, [2500, 777, 40], rows,
                            [(0, 0), (0, 21), (1, 6), (1, 31), (2, 15)], seed=16, k_ramp=k_ramp)
    assert worst < 1e-2, worst


@pytest.mark.parametrize("k_ramp", [None, (0.05, 6.0)])
def test_attention_prompt_block(k_ramp):
    """256 block rows per stream (1024 query rows per KV head): the kernel for prompt blocks, which
    walks the tokens unsplit and writes the normalised rows itself.  Empty, short and long caches
    under the block, rows past the block poisoned."""
    w = synth.model_weights(HOST, 99, threads=16)
    m = cs.Model(w, max_batch=3, max_k=255)
    sample = [(0, 0), (0, 31), (1, 13), (2, 5), (2, 22)]
    worst = _attention_case(m, HOST, [0, 700, 2049], 256, sample, seed=21, poison=True, k_ramp=k_ramp)
    m.destroy()
    assert worst < 1e-2, worst


@pytest.mark.parametrize("rows", [6, 21, 51, 101])
def test_attention_block_size_sweep(rows):
    """Block sizes of the paper's sweep (Sec. 5.3, Table 4: 5, 10, 50, 100 draft tokens; 20 added):
    6 rows fit one 48-row query group, 21 rows fill two groups of a three-group workgroup column
    partly, 51 and 101 rows need two and three columns with a ragged last one."""
    w = synth.model_weights(HOST, 99, threads=16)
    m = cs.Model(w, max_batch=5, max_k=100)
    sample = [(0, 0), (0, 31), (1, 13), (2, 5), (3, 22), (4, 9)]
    worst = _attention_case(m, HOST, [2500, 777, 40, 0, 4100], rows, sample, seed=30 + rows, poison=True)
    m.destroy()
    assert worst < 1e-2, worst


def test_attention_hd64():
    shape = ModelShape("w-hd64", 1, 2048, 32, 8, 64, 8192, 1024, 10000.0, 1e-5, "bf16")
    w = synth.model_weights(shape, 5, threads=16)
    m = cs.Model(w, max_batch=4, max_k=10)
    worst = _attention_case(m, shape, [4096, 100, 0, 2500], 11, [(0, 0), (1, 9), (2, 31), (3, 20)],
                            seed=15)
    m.destroy()
    assert worst < 1e-2, worst


# ----------------------------------------------------------------------------------------
# whole verify step at depth
# ----------------------------------------------------------------------------------------

def _deep_verify(shape, B, L, k, check_streams, seed):
    w = synth.model_weights(shape, seed, threads=16)
    model = cs.Model(w, max_batch=B, max_k=k)
    kv = cs.KV(model, B, L + k + 8)
    rng = np.random.default_rng(seed)
    pending = rng.integers(0, shape.vocab, B)
    draft = rng.integers(0, shape.vocab, (B, k))
    dlen = np.full(B, k)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    for b in range(B):
        for layer in range(shape.n_layers):
            if b in check_streams:
                kr, vr = synth.random_kv(shape, L, seed, layer, b)
            else:   # streams the oracle does not look at: cheap device-side fill
                kr = torch.randn((shape.n_kv_heads, L, shape.head_dim), generator=gen, device=DEV).bfloat16()
                vr = torch.randn((shape.n_kv_heads, L, shape.head_dim), generator=gen, device=DEV).bfloat16()
            kv.load(layer, b, 0, kr, vr)
        kv.set_len(b, L)
    acc, nxt, logits = cs.cs_verify(model, kv, t32(pending), t32(draft), t32(dlen), k, want_logits=True)
    torch.cuda.synchronize()
    # the same step without the logits: the lm_head then takes the argmax in its own epilogue and
    # writes no logits; every stream must come out identical (same accumulators, same tie rule)
    for b in range(B):
        kv.set_len(b, L)
    acc2, nxt2, _ = cs.cs_verify(model, kv, t32(pending), t32(draft), t32(dlen), k, want_logits=False)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc2) and torch.equal(nxt, nxt2)
    for b in range(B):
        row = logits[b, int(acc2[b])]
        assert float(row[int(nxt2[b])]) == float(row.max())
    logits = logits.cpu().numpy()
    worst = 0.0
    for b in check_streams:
        okv = orc.KVCache(shape, L + k + 8)
        for layer in range(shape.n_layers):
            kr, vr = synth.random_kv(shape, L, seed, layer, b)
            okv.load(layer, kr, vr)
        okv.truncate(L)
        tau, nx, ol = orc.verify(w, okv, int(pending[b]), draft[b].tolist())
        worst = max(worst, np.abs(logits[b] - ol).max())
        am = [orc.argmax_first(r) for r in ol]
        if all((np.partition(ol[i], -2)[-1] - np.partition(ol[i], -2)[-2]) > 1e-2 for i in range(tau + 1)):
            assert (int(acc[b]), int(nxt[b])) == (tau, nx)
        assert kv.len(b) == L + int(acc[b]) + 1
    kv.destroy()
    model.destroy()
    return worst


def test_verify_llama1b_full_depth():
    """Configuration 3 shape at full depth: 16 layers, 4096 cached rows, k = 10."""
    worst = _deep_verify(synth.LLAMA_1B, 1, 4096, 10, [0], seed=synth.seed_for(3))
    assert worst <= 2e-2, worst


def test_verify_llama8b_width_many_rows():
    """8B width, batch 8, k = 32: 264 block rows go through the many-row projection kernel
    (SwiGLU epilogue, K splits) and the wide-block attention kernel; 2 layers, short cache."""
    shape = synth.LLAMA_8B.with_layers(2)
    worst = _deep_verify(shape, 8, 700, 32, [0, 7], seed=synth.seed_for(5))
    assert worst <= 2e-2, worst


def test_verify_llama8b_width_528_rows():
    """8B width, batch 16, k = 32: with 528 block rows every projection runs the many-row kernel,
    so every GEMM input (both norms, the merged attention output, the SwiGLU output) is written in
    fragment order by its producer; 1 layer, short cache."""
    shape = synth.LLAMA_8B.with_layers(1)
    worst = _deep_verify(shape, 16, 300, 32, [3, 15], seed=synth.seed_for(5) + 1)
    assert worst <= 2e-2, worst


def test_verify_llama8b_width_batch8():
    """8B width, batch 8, 18431 cached rows, k = 10 (the benchmark's launch configuration),
    4 of the 32 layers; the oracle checks two sampled streams."""
    shape = synth.LLAMA_8B.with_layers(4)
    worst = _deep_verify(shape, 8, 18431, 10, [0, 5], seed=synth.seed_for(4))
    assert worst <= 2e-2, worst


@pytest.mark.parametrize("B,k", [(1, 50), (1, 100), (8, 100), (8, 20), (8, 5)])
def test_verify_llama8b_width_block_size_sweep(B, k):
    """Block sizes of the paper's sweep (Sec. 5.3, Table 4) at the 8B width, one layer, short cache:
    51 and 101 rows of a single stream (the paper's batch size) go through the weight-streaming
    projections with one and two row blocks and the wide-block attention; 808 rows (batch 8,
    k = 100) take three row blocks of the many-row projections; 168 and 48 rows sit between."""
    shape = synth.LLAMA_8B.with_layers(1)
    worst = _deep_verify(shape, B, 300, k, [B - 1], seed=synth.seed_for(5) + 10 * k + B)
    assert worst <= 2e-2, worst


@pytest.mark.parametrize("B,k", [(8, 10), (16, 32), (1, 50)])
def test_verify_llama8b_width_with_qkv_bias(B, k):
    """Biases on the q, k, v projections at the 8B width, one layer: 88 rows (added in the attention
    kernel's own rotary stage), 528 rows (the many-row rotary kernel), 51 rows of one stream (the
    small rotary kernel), against the oracle with the same biases."""
    shape = synth.LLAMA_8B.with_layers(1).with_qkv_bias()
    worst = _deep_verify(shape, B, 300, k, [B - 1], seed=synth.seed_for(5) + 100 + k)
    assert worst <= 2e-2, worst


QWEN_7B = ModelShape("qwen2.5-7b-width", 1, 3584, 28, 4, 128, 18944, 152064, 1000000.0, 1e-6, "bf16", True)


@pytest.mark.parametrize("B,k,L", [(8, 10, 300), (1, 10, 4000), (16, 32, 300)])
def test_verify_qwen7b_width(B, k, L):
    """The other model family of Sec. 4.1 at its 7B width, one layer: 28 query heads over 4 KV heads
    (seven per KV head, so 11 block rows already need two 48-row query groups), d_model 3584,
    d_ff 18944, 152064-token vocabulary, q/k/v biases; 88 and 528 block rows and one stream."""
    worst = _deep_verify(QWEN_7B, B, L, k, [B - 1], seed=synth.seed_for(5) + 300 + k + B)
    assert worst <= 2e-2, worst


LLAMA_70B_WIDTH = ModelShape("llama-70b-width", 1, 8192, 64, 8, 128, 28672, 128256, 500000.0, 1e-5, "bf16")


@pytest.mark.parametrize("B,k", [(8, 10), (1, 10)])
def test_verify_llama70b_width(B, k):
    """The largest width the paper runs (Sec. 4.1: 70B / 72B models), one layer: d_model 8192 (the
    widest row the norm kernel takes), 64 heads over 8 KV heads, d_ff 28672."""
    worst = _deep_verify(LLAMA_70B_WIDTH, B, 300, k, [B - 1], seed=synth.seed_for(5) + 700 + B)
    assert worst <= 2e-2, worst
