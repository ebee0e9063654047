"""Seeded generators for the synthetic CopySpec workloads.

The paper evaluates on summarisation, multi-turn chat and self-correction
data (Sec. 4.2, Sec. 4.4, Sec. 6.3): long contexts in which spans of the
output recur verbatim in the input.  Those datasets are not available here,
so the generators below draw token sequences with the same *structure*:
uniform random tokens with verbatim spans copied from earlier positions.

Every generator is a pure function of its integer seed (numpy PCG64).  For the
histories the generator also records, by construction, where the final planted
span came from, so a test knows the expected match position without running
any search.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
import math

import numpy as np

BASE_SEED = 250208923


def seed_for(cfg: int, stream: int = 0) -> int:
    return BASE_SEED + 1000 * cfg + stream


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


# ----------------------------------------------------------------------------
# bf16 <-> f32 bit helpers (storage format conversion only)
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# model shapes
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rope_theta: float
    rms_eps: float
    dtype: str  # "f32" or "bf16": storage type of weights and KV cache
    qkv_bias: bool = False  # additive biases on the q, k and v projections (the Qwen2.5 family)

    def with_layers(self, n_layers: int) -> "ModelShape":
        return replace(self, n_layers=n_layers)

    def with_vocab(self, vocab: int) -> "ModelShape":
        return replace(self, vocab=vocab)

    def with_qkv_bias(self, on: bool = True) -> "ModelShape":
        return replace(self, qkv_bias=on)


TINY = ModelShape("tiny", 2, 256, 4, 4, 64, 1024, 1024, 10000.0, 1e-5, "f32")
LLAMA_1B = ModelShape("llama-1b", 16, 2048, 32, 8, 64, 8192, 32000, 10000.0, 1e-5, "bf16")
LLAMA_8B = ModelShape("llama-8b", 32, 4096, 32, 8, 128, 14336, 128256, 500000.0, 1e-5, "bf16")
# the 7B member of the other family the paper runs (Sec. 4.1): seven query heads per KV head, q/k/v biases
QWEN_7B = ModelShape("qwen2.5-7b", 28, 3584, 28, 4, 128, 18944, 152064, 1000000.0, 1e-6, "bf16", True)
# the largest model of the paper's tables in the 8B shape's family: 141 GB of bfloat16 weights
LLAMA_70B = ModelShape("llama-70b", 80, 8192, 64, 8, 128, 28672, 128256, 500000.0, 1e-5, "bf16")
# the model of the paper's largest speed-up (Table 1, Sec. 5): 145 GB of bfloat16 weights
QWEN_72B = ModelShape("qwen2.5-72b", 80, 8192, 64, 8, 128, 29568, 152064, 1000000.0, 1e-6, "bf16", True)


# ----------------------------------------------------------------------------
# weights and KV caches
# ----------------------------------------------------------------------------

def _uniform_lut(a: float) -> np.ndarray:
    """bf16 bit patterns of a 65536-point uniform grid on (-a, a)."""
    grid = (np.arange(65536, dtype=np.float64) - 32767.5) / 32768.0 * a
    return f32_to_bf16_bits(grid.astype(np.float32))


def _normal_lut() -> np.ndarray:
    """bf16 bit patterns of a 65536-point grid of standard-normal quantiles."""
    from scipy.special import ndtri
    q = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    return f32_to_bf16_bits(q.astype(np.float32))


def _draw(seed: int, shape, kind: str, scale: float, dtype: str) -> np.ndarray:
    """kind 'u': U(-scale, scale); kind 'n': N(0, scale^2).
    dtype 'bf16' -> uint16 bit patterns, 'f32' -> float32 values."""
    rng = _rng(seed)
    n = int(np.prod(shape))
    if dtype == "bf16":
        lut = _uniform_lut(scale) if kind == "u" else _normal_lut()
        out = lut[rng.integers(0, 65536, n, dtype=np.uint16)]
        if kind == "n" and scale != 1.0:
            out = f32_to_bf16_bits(bf16_bits_to_f32(out) * np.float32(scale))
        return out.reshape(shape)
    if kind == "u":
        v = (rng.random(n, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)) * np.float32(scale)
    else:
        v = rng.standard_normal(n, dtype=np.float32) * np.float32(scale)
    return v.reshape(shape)


def _head_jobs(shape: ModelShape, seed: int) -> dict:
    d, V, dt = shape.d_model, shape.vocab, shape.dtype
    return {("embed",): (seed * 1000 + 1, (V, d), "n", 1.0, dt),
            ("lm_head",): (seed * 1000 + 2, (V, d), "u", math.sqrt(3.0 / d), dt),
            ("final_norm",): (seed * 1000 + 3, (d,), "g", 0.1, "f32")}


def _layer_jobs(shape: ModelShape, seed: int, l: int) -> dict:
    d, hd = shape.d_model, shape.head_dim
    H, KVH, F = shape.n_heads, shape.n_kv_heads, shape.d_ff
    dt = shape.dtype
    a_d = math.sqrt(3.0 / d)
    s = seed * 1000 + 100 + 16 * l
    jobs = {}
    jobs[("layers", l, "wq")] = (s + 0, (H * hd, d), "u", a_d, dt)
    jobs[("layers", l, "wk")] = (s + 1, (KVH * hd, d), "u", a_d, dt)
    jobs[("layers", l, "wv")] = (s + 2, (KVH * hd, d), "u", a_d, dt)
    jobs[("layers", l, "wo")] = (s + 3, (d, H * hd), "u", math.sqrt(3.0 / (H * hd)), dt)
    jobs[("layers", l, "wg")] = (s + 4, (F, d), "u", a_d, dt)
    jobs[("layers", l, "wu")] = (s + 5, (F, d), "u", a_d, dt)
    jobs[("layers", l, "wd")] = (s + 6, (d, F), "u", math.sqrt(3.0 / F), dt)
    jobs[("layers", l, "norm1")] = (s + 7, (d,), "g", 0.1, "f32")
    jobs[("layers", l, "norm2")] = (s + 8, (d,), "g", 0.1, "f32")
    if shape.qkv_bias:      # float32, N(0, 0.5): of the size of the projected values themselves
        jobs[("layers", l, "bq")] = (s + 9, (H * hd,), "n", 0.5, "f32")
        jobs[("layers", l, "bk")] = (s + 10, (KVH * hd,), "n", 0.5, "f32")
        jobs[("layers", l, "bv")] = (s + 11, (KVH * hd,), "n", 0.5, "f32")
    return jobs


def _run_jobs(jobs: dict, threads: int) -> dict:
    def run(job):
        sd, shp, kind, scale, dtype = job
        if kind == "g":
            return (np.float32(1.0) + _draw(sd, shp, "u", scale, "f32")).astype(np.float32)
        return _draw(sd, shp, kind, scale, dtype)

    keys = list(jobs)
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        vals = list(ex.map(run, [jobs[k] for k in keys]))
    return dict(zip(keys, vals))


def model_weights(shape: ModelShape, seed: int, threads: int = 8) -> dict:
    """Random-init decoder weights.

    Linear weights are U(-a, a) with a = sqrt(3 / fan_in) (unit-variance
    outputs for unit-variance inputs); embedding rows are N(0, 1); RMSNorm
    gains are 1 + 0.1 U(-1, 1) so that a dropped or mis-indexed gain shows.
    bf16 shapes return uint16 bit patterns for matrices; norm gains are always
    float32.  Linear weights are stored [out_features][in_features].  Shapes with qkv_bias also
    get float32 bias vectors bq, bk, bv per layer.
    """
    jobs = _head_jobs(shape, seed)
    for l in range(shape.n_layers):
        jobs.update(_layer_jobs(shape, seed, l))
    vals = _run_jobs(jobs, threads)
    out = {"shape": shape, "layers": [dict() for _ in range(shape.n_layers)]}
    for k, v in vals.items():
        if k[0] == "layers":
            out["layers"][k[1]][k[2]] = v
        else:
            out[k[0]] = v
    return out


def model_weights_lazy(shape: ModelShape, seed: int, threads: int = 8) -> dict:
    """The same weights as model_weights, drawn one part at a time: "layers" is a function of the
    layer index and "head" a function without arguments (embed, lm_head, final_norm), so that a
    model too large to hold twice can be handed over piece by piece."""
    def layer(l: int) -> dict:
        return {k[2]: v for k, v in _run_jobs(_layer_jobs(shape, seed, l), threads).items()}

    def head() -> dict:
        return {k[0]: v for k, v in _run_jobs(_head_jobs(shape, seed), threads).items()}

    return {"shape": shape, "layers": layer, "head": head}


def random_kv(shape: ModelShape, n_tokens: int, seed: int, layer: int, stream: int):
    """Random K and V rows for one (layer, stream): each [n_kv_heads][n_tokens][head_dim],
    N(0,1) entries in the cache storage type.  Rotary embedding preserves norms, so
    post-rotary keys of a random-init model have the same distribution."""
    shp = (shape.n_kv_heads, n_tokens, shape.head_dim)
    s = (seed * 1000 + 7) * 4096 + layer * 64 + stream
    k = _draw(2 * s, shp, "n", 1.0, shape.dtype)
    v = _draw(2 * s + 1, shp, "n", 1.0, shape.dtype)
    return k, v


# ----------------------------------------------------------------------------
# token histories with planted verbatim repeats
# ----------------------------------------------------------------------------

def planted_history(seed: int, n: int, vocab: int, span_len, *, density: float | None = None,
                    n_spans: int | None = None, gamma: int = 3, k: int = 10,
                    end: str = "span", twice: bool = False,
                    src_region=None, dst_region=None) -> dict:
    """A length-n int32 history of uniform tokens with verbatim spans copied from
    earlier positions.

    end="span":  the history ends in the middle of a planted span whose source
                 lies in a protected zone of fresh tokens, followed by at least
                 k more fresh tokens.  The generator therefore knows where the
                 last gamma tokens occur earlier: at `first_match` (the source)
                 and, with twice=True, also at a second planted copy further
                 right (`rightmost_match`).
    end="fresh": the last tokens are fresh random draws (no planted match).

    Returned dict: tokens, first_match, rightmost_match (start index of the
    earlier gamma-gram, -1 if none was planted), spans [(dst, src, len)].
    The expected positions hold exactly unless a chance gamma-gram collision
    occurs (probability about n / vocab**gamma).
    """
    rng = _rng(seed)
    lo, hi = span_len
    h = rng.integers(0, vocab, n, dtype=np.int64).astype(np.int32)
    W = hi + k + gamma + 8                      # protected zone width
    src_lo, src_hi = src_region if src_region else (0, n)
    dst_lo, dst_hi = dst_region if dst_region else (0, n)
    z1 = src_lo + max(gamma, (src_hi - src_lo) // 8)      # source zone of the final span
    z2 = dst_lo + (dst_hi - dst_lo) // 2                  # zone of its optional second copy
    if src_region is None and dst_region is None:
        z2 = n // 2
    final_len = int(rng.integers(lo, hi + 1)) if end == "span" else 0
    tail = max(final_len, gamma + 1)
    zones = [(z1, z1 + W), (z2, z2 + W), (n - tail - 1, n)]

    def clear(a, b):
        return all(b <= za or a >= zb for za, zb in zones)

    spans = []
    taken = []                                   # destination intervals already used
    covered = final_len
    target = density * n if density is not None else None
    want = (n_spans - (1 if end == "span" else 0)) if n_spans is not None else None
    tries = 0
    while tries < 100000:
        if want is not None and len(spans) >= want:
            break
        if target is not None and covered >= target:
            break
        tries += 1
        ln = int(rng.integers(lo, hi + 1))
        d0 = max(dst_lo, ln)
        d1 = min(dst_hi, n - tail - 1) - ln
        if d1 <= d0:
            continue
        dst = int(rng.integers(d0, d1))
        s1 = min(src_hi, dst) - ln
        if s1 <= src_lo:
            continue
        src = int(rng.integers(src_lo, s1 + 1))
        if not (clear(src, src + ln) and clear(dst, dst + ln)):
            continue
        if any(not (dst + ln <= a or dst >= b) for a, b in taken):
            continue
        h[dst:dst + ln] = h[src:src + ln]
        taken.append((dst, dst + ln))
        spans.append((dst, src, ln))
        covered += ln
    first = right = -1
    if end == "span":
        s = z1 + 2
        h[n - final_len:n] = h[s:s + final_len]
        spans.append((n - final_len, s, final_len))
        first = right = s + final_len - gamma
        if twice:
            h[z2:z2 + final_len] = h[s:s + final_len]
            spans.append((z2, s, final_len))
            right = z2 + final_len - gamma
    return {"tokens": h, "first_match": first, "rightmost_match": right, "spans": spans,
            "gamma": gamma, "k": k}


def history_cfg1(seed: int | None = None) -> dict:
    """512 tokens over a 1024-token vocabulary, 4 planted spans of 24 tokens, the last
    one ending exactly at position 512 (so the first decode step finds a match)."""
    return planted_history(seed_for(1) if seed is None else seed, 512, 1024, (24, 24),
                           n_spans=4, end="span")


def history_cfg2(stream: int, n: int = 32768, vocab: int = 32000) -> dict:
    """One of the 64 scan histories: spans of 16..128 tokens covering about 5 % of the
    positions.  Even streams end inside a span (every fourth stream has the source
    planted twice, so rightmost and first matches differ); odd streams end in fresh
    tokens (no match expected)."""
    even = stream % 2 == 0
    return planted_history(seed_for(2, stream), n, vocab, (16, 128), density=0.05,
                           end="span" if even else "fresh", twice=(stream % 4 == 2))


def history_cfg3(seed: int | None = None) -> dict:
    """4096 tokens, 64-token repeats at 10 % density, the last ending at 4096."""
    return planted_history(seed_for(3) if seed is None else seed, 4096, 32000, (64, 64),
                           density=0.10, end="span")


def history_cfg4(stream: int, vocab: int = 128256, doc: int = 2048, hist: int = 16384,
                 k: int = 10) -> dict:
    """A `doc`-token document followed by `hist` tokens of history that re-contains
    document spans of 32..256 tokens at 20 % density and ends mid-span with at least k
    source tokens left."""
    n = doc + hist
    return planted_history(seed_for(4, stream), n, vocab, (32, 256), density=0.20 * hist / n,
                           k=k, end="span", src_region=(0, doc), dst_region=(doc, n))


def history_cfg5(stream: int, n: int = 65536, vocab: int = 128256, answer: int = 1024,
                 edit_rate: float = 0.05, gamma: int = 3, k: int = 32) -> dict:
    """Multi-turn stand-in: filler, a first-turn answer A of `answer` tokens, filler, then
    the first j tokens of A' = A with i.i.d. token substitutions at `edit_rate`; the last
    gamma tokens are left unedited so the copy source is A[j:]."""
    rng = _rng(seed_for(5, stream))
    h = rng.integers(0, vocab, n, dtype=np.int64).astype(np.int32)
    a = n // 2
    j = answer // 2 + 7 * (stream % 16)
    assert j + k <= answer
    ap = h[a:a + j].copy()
    edit = rng.random(j) < edit_rate
    edit[j - gamma:] = False
    sub = rng.integers(0, vocab, j, dtype=np.int64).astype(np.int32)
    ap[edit] = sub[edit]
    h[n - j:n] = ap
    m = a + j - gamma
    return {"tokens": h, "first_match": m, "rightmost_match": m,
            "spans": [(n - j, a, j)], "gamma": gamma, "k": k, "edits": int(edit.sum())}


def multiturn_replay(stream: int, answer: int = 1024, filler: int = 1024, vocab: int = 128256,
                     edit_rate: float = 0.05, turns: int = 3) -> dict:
    """Self-correction stand-in for acceptance replays: `turns` versions of one answer, each the
    previous version with i.i.d. token substitutions at `edit_rate`, separated by random filler.
    "context" holds everything up to the start of the last version, "truth" is the last
    version (what a faithful target model would emit next)."""
    rng = _rng(seed_for(5, 100 + stream))
    draw = lambda m: rng.integers(0, vocab, m, dtype=np.int64).astype(np.int32)
    ver = draw(answer)
    parts = [draw(filler), ver]
    for _ in range(turns - 1):
        nxt = ver.copy()
        edit = rng.random(answer) < edit_rate
        nxt[edit] = draw(answer)[edit]
        parts += [draw(filler), nxt]
        ver = nxt
    return {"context": np.concatenate(parts[:-1]), "truth": parts[-1]}


def zipf_replay(stream: int, context: int = 6144, answer: int = 2048, vocab: int = 128256,
                exponent: float = 1.1, copy_density: float = 0.3, span=(8, 64)) -> dict:
    """Natural-text-like stand-in for acceptance replays: token ranks follow a Zipf law
    (p(rank r) ~ r^-exponent, truncated at `vocab`), so short gamma-grams of frequent tokens
    recur by chance and produce matches whose continuation is wrong; on top of that,
    `copy_density` of the answer consists of spans copied verbatim from the context (lengths
    uniform in `span`).  "context" is what the model has seen, "truth" what a faithful target
    model would emit next."""
    rng = _rng(seed_for(5, 200 + stream))
    ranks = np.arange(1, vocab + 1, dtype=np.float64)
    p = ranks ** -exponent
    p /= p.sum()
    perm = rng.permutation(vocab).astype(np.int32)          # which token id has which rank
    draw = lambda m: perm[rng.choice(vocab, size=m, p=p)]
    ctx = draw(context)
    truth = draw(answer)
    covered, lo, hi = 0, span[0], span[1]
    while covered < copy_density * answer:
        ln = int(rng.integers(lo, hi + 1))
        src = int(rng.integers(0, context - ln))
        dst = int(rng.integers(0, answer - ln))
        truth[dst:dst + ln] = ctx[src:src + ln]
        covered += ln
    return {"context": ctx, "truth": truth}

