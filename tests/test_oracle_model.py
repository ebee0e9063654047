"""Pins for the oracle's target-model forward, verify step and decode loops (CPU only).

Independent references: the Llama implementation of the `transformers` library
(same architecture, loaded with the same random weights), torch's attention and
bfloat16 conversion, closed-form properties of rotary embedding and RMSNorm,
and the paper's invariants (greedy CopySpec == plain greedy; rollback leaves no
trace of rejected tokens; one guaranteed token per step).
"""
import numpy as np
import pytest
import torch

from oracle import copyspec_oracle as orc
import synth
from synth import ModelShape

SMALL = ModelShape("small-gqa", 2, 64, 4, 2, 16, 96, 97, 10000.0, 1e-5, "f32")
SMALL_BF16 = ModelShape("small-gqa-bf16", 2, 64, 4, 2, 16, 96, 97, 10000.0, 1e-5, "bf16")


@pytest.fixture(scope="module")
def small_w():
    return synth.model_weights(SMALL, 1234, threads=1)


@pytest.fixture(scope="module")
def tiny_w():
    return synth.model_weights(synth.TINY, synth.seed_for(1), threads=4)


def _hf_model(w):
    from transformers import LlamaConfig, LlamaForCausalLM
    sh = w["shape"]
    cfg = LlamaConfig(vocab_size=sh.vocab, hidden_size=sh.d_model, intermediate_size=sh.d_ff,
                      num_hidden_layers=sh.n_layers, num_attention_heads=sh.n_heads,
                      num_key_value_heads=sh.n_kv_heads, head_dim=sh.head_dim,
                      rms_norm_eps=sh.rms_eps, rope_theta=sh.rope_theta,
                      tie_word_embeddings=False, attention_bias=False, mlp_bias=False,
                      max_position_embeddings=4096, hidden_act="silu")
    m = LlamaForCausalLM(cfg).double().eval()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    sd = {"model.embed_tokens.weight": t(w["embed"]), "model.norm.weight": t(w["final_norm"]),
          "lm_head.weight": t(w["lm_head"])}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "wg": "mlp.gate_proj", "wu": "mlp.up_proj",
             "wd": "mlp.down_proj", "norm1": "input_layernorm", "norm2": "post_attention_layernorm"}
    for l, lw in enumerate(w["layers"]):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}.weight"] = t(lw[k])
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not [k for k in missing if "rotary" not in k], missing
    assert not unexpected
    return m


def test_forward_matches_library_llama(small_w):
    """Whole-model pin: same weights in an independently written Llama implementation."""
    m = _hf_model(small_w)
    rng = np.random.default_rng(3)
    toks = rng.integers(0, SMALL.vocab, 37)
    with torch.no_grad():
        ref = m(torch.from_numpy(toks)[None]).logits[0].numpy()
    kv = orc.KVCache(SMALL, 64)
    got = orc.forward_block(small_w, kv, toks, store_dtype="f64")
    # the library builds its rotary cos/sin tables in float32, which limits agreement to
    # ~1e-6; any structural mistake (pairing, head mapping, norm, activation) gives O(1)
    assert np.abs(got - ref).max() < 5e-6
    # block over a non-empty cache: same logits for the tail rows
    kv2 = orc.KVCache(SMALL, 64)
    orc.forward_block(small_w, kv2, toks[:20], store_dtype="f64")
    kv2.truncate(20)
    tail = orc.forward_block(small_w, kv2, toks[20:], store_dtype="f64")
    assert np.abs(tail - ref[20:]).max() < 5e-6
    assert np.abs(tail - got[20:]).max() < 1e-11


def _llama3_inv_freq(hd, theta, factor, low, high, orig_len):
    """Rescaled rotary frequencies of the Llama-3.1 checkpoints, from their published recipe:
    wavelengths beyond orig_len/low are slowed down by `factor`, those below orig_len/high are kept,
    the band between is blended linearly in orig_len/wavelength."""
    inv = theta ** (-(np.arange(hd // 2, dtype=np.float64) * 2.0) / hd)
    out = []
    for f in inv:
        wavelen = 2.0 * np.pi / f
        if wavelen < orig_len / high:
            out.append(f)
        elif wavelen > orig_len / low:
            out.append(f / factor)
        else:
            smooth = (orig_len / wavelen - low) / (high - low)
            out.append((1.0 - smooth) * f / factor + smooth * f)
    return np.array(out)


def test_rescaled_rotary_frequencies_match_library_llama3():
    """Models that bring their own rotary frequencies (the Llama-3.1 checkpoints of Sec. 4.1 rescale
    theirs): the oracle rotates pair j at position p by p * inv_freq[j].  Pinned against the
    `transformers` Llama with rope_type llama3, on a table written out from the published recipe;
    the short original context (32) puts the three bands of the recipe inside this head size."""
    from transformers import LlamaConfig, LlamaForCausalLM
    sh = SMALL
    w = dict(synth.model_weights(sh, 2468, threads=1))
    scaling = {"rope_type": "llama3", "factor": 8.0, "low_freq_factor": 1.0, "high_freq_factor": 4.0,
               "original_max_position_embeddings": 32, "rope_theta": sh.rope_theta}
    inv = _llama3_inv_freq(sh.head_dim, sh.rope_theta, 8.0, 1.0, 4.0, 32)
    plain = sh.rope_theta ** (-(np.arange(sh.head_dim // 2) * 2.0) / sh.head_dim)
    kept, slowed = np.isclose(inv, plain), np.isclose(inv, plain / 8.0)
    assert kept.any() and slowed.any() and (~kept & ~slowed).any()       # all three bands occur
    try:
        cfg = LlamaConfig(vocab_size=sh.vocab, hidden_size=sh.d_model, intermediate_size=sh.d_ff,
                          num_hidden_layers=sh.n_layers, num_attention_heads=sh.n_heads,
                          num_key_value_heads=sh.n_kv_heads, head_dim=sh.head_dim,
                          rms_norm_eps=sh.rms_eps, rope_parameters=scaling,
                          tie_word_embeddings=False, attention_bias=False, mlp_bias=False,
                          max_position_embeddings=4096, hidden_act="silu")
    except TypeError:                                    # older releases of the library
        cfg = LlamaConfig(vocab_size=sh.vocab, hidden_size=sh.d_model, intermediate_size=sh.d_ff,
                          num_hidden_layers=sh.n_layers, num_attention_heads=sh.n_heads,
                          num_key_value_heads=sh.n_kv_heads, head_dim=sh.head_dim,
                          rms_norm_eps=sh.rms_eps, rope_theta=sh.rope_theta, rope_scaling=scaling,
                          tie_word_embeddings=False, attention_bias=False, mlp_bias=False,
                          max_position_embeddings=4096, hidden_act="silu")
    m = LlamaForCausalLM(cfg).double().eval()
    lib_inv = m.model.rotary_emb.inv_freq.double().numpy()
    assert np.abs(lib_inv - inv).max() < 1e-6 * inv.max()              # float32 table in the library
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    sd = {"model.embed_tokens.weight": t(w["embed"]), "model.norm.weight": t(w["final_norm"]),
          "lm_head.weight": t(w["lm_head"])}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "wg": "mlp.gate_proj", "wu": "mlp.up_proj",
             "wd": "mlp.down_proj", "norm1": "input_layernorm", "norm2": "post_attention_layernorm"}
    for l, lw in enumerate(w["layers"]):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}.weight"] = t(lw[k])
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not [k for k in missing if "rotary" not in k] and not unexpected
    rng = np.random.default_rng(9)
    toks = rng.integers(0, sh.vocab, 60)
    with torch.no_grad():
        ref = m(torch.from_numpy(toks)[None]).logits[0].numpy()
    w["rope_inv_freq"] = inv
    got = orc.forward_block(w, orc.KVCache(sh, 64), toks, store_dtype="f64")
    assert np.abs(got - ref).max() < 2e-5
    del w["rope_inv_freq"]
    unscaled = orc.forward_block(w, orc.KVCache(sh, 64), toks, store_dtype="f64")
    assert np.abs(unscaled - ref).max() > 1e-2           # the rescaling matters at these positions


def test_qkv_bias_matches_library_qwen2():
    """The q/k/v biases of the Qwen2.5 family (Sec. 4.1 runs both families): same weights and
    biases in the `transformers` Qwen2 implementation; a dropped, doubled or head-misplaced bias,
    or one added after the rotary embedding, changes the logits by O(1)."""
    from transformers import Qwen2Config, Qwen2ForCausalLM
    sh = SMALL.with_qkv_bias()
    w = synth.model_weights(sh, 4321, threads=1)
    cfg = Qwen2Config(vocab_size=sh.vocab, hidden_size=sh.d_model, intermediate_size=sh.d_ff,
                      num_hidden_layers=sh.n_layers, num_attention_heads=sh.n_heads,
                      num_key_value_heads=sh.n_kv_heads, rms_norm_eps=sh.rms_eps,
                      rope_theta=sh.rope_theta, tie_word_embeddings=False,
                      max_position_embeddings=4096, hidden_act="silu", use_sliding_window=False)
    m = Qwen2ForCausalLM(cfg).double().eval()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    sd = {"model.embed_tokens.weight": t(w["embed"]), "model.norm.weight": t(w["final_norm"]),
          "lm_head.weight": t(w["lm_head"])}
    names = {"wq": "self_attn.q_proj.weight", "wk": "self_attn.k_proj.weight", "wv": "self_attn.v_proj.weight",
             "bq": "self_attn.q_proj.bias", "bk": "self_attn.k_proj.bias", "bv": "self_attn.v_proj.bias",
             "wo": "self_attn.o_proj.weight", "wg": "mlp.gate_proj.weight", "wu": "mlp.up_proj.weight",
             "wd": "mlp.down_proj.weight", "norm1": "input_layernorm.weight",
             "norm2": "post_attention_layernorm.weight"}
    for l, lw in enumerate(w["layers"]):
        assert set(lw) == set(names)
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}"] = t(lw[k])
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not [k for k in missing if "rotary" not in k], missing
    assert not unexpected
    rng = np.random.default_rng(5)
    toks = rng.integers(0, sh.vocab, 33)
    with torch.no_grad():
        ref = m(torch.from_numpy(toks)[None]).logits[0].numpy()
    kv = orc.KVCache(sh, 64)
    got = orc.forward_block(w, kv, toks, store_dtype="f64")
    assert np.abs(got - ref).max() < 5e-6
    # the biases matter at this scale: without them the logits are far off
    w0 = dict(w, layers=[{k: v for k, v in lw.items() if k not in ("bq", "bk", "bv")} for lw in w["layers"]])
    plain = orc.forward_block(w0, orc.KVCache(sh, 64), toks, store_dtype="f64")
    assert np.abs(plain - ref).max() > 0.1
    # block over a non-empty cache and greedy == CopySpec with biases
    kv2 = orc.KVCache(sh, 64)
    orc.forward_block(w, kv2, toks[:20], store_dtype="f64")
    kv2.truncate(20)
    tail = orc.forward_block(w, kv2, toks[20:], store_dtype="f64")
    assert np.abs(tail - got[20:]).max() < 1e-11
    prompt = (list(toks[:12]) * 3)[:30]
    g = orc.greedy_decode(w, prompt, 12)
    c, _ = orc.copyspec_decode(w, prompt, 12, 3, 5)
    assert g == c


def test_act_clip_matches_library_llama_with_clamped_linear_inputs():
    """The optional input range of the projections (act_clip): the same weights in the library
    implementation, with a hook on every linear layer that clamps its input, give the same
    logits.  Gains are scaled so that every kind of projection input leaves the range; a clip
    that nothing reaches, and no clip, are the unclipped model."""
    w = synth.model_weights(SMALL, 4321, threads=1)
    w["layers"][0]["norm2"] = (w["layers"][0]["norm2"] * 3.0).astype(np.float32)    # gate/up input, SwiGLU output
    w["layers"][1]["norm1"] = (w["layers"][1]["norm1"] * 2.5).astype(np.float32)    # q/k/v input, attention output
    w["final_norm"] = (w["final_norm"] * 2.0).astype(np.float32)                    # lm_head input
    m = _hf_model(w)
    clip = 1.5
    seen = {}

    def clamp_input(name):
        def hook(mod, args):
            seen[name] = max(seen.get(name, 0.0), float(args[0].abs().max()))
            return (args[0].clamp(-clip, clip),)
        return hook

    hooks = [mod.register_forward_pre_hook(clamp_input(name.split(".")[-1]))
             for name, mod in m.named_modules() if isinstance(mod, torch.nn.Linear)]
    assert len(hooks) == 7 * SMALL.n_layers + 1
    rng = np.random.default_rng(6)
    toks = rng.integers(0, SMALL.vocab, 29)
    with torch.no_grad():
        ref = m(torch.from_numpy(toks)[None]).logits[0].numpy()
    for h in hooks:
        h.remove()
    # the clip bites at every kind of projection input
    for name in ("q_proj", "o_proj", "gate_proj", "down_proj", "lm_head"):
        assert seen[name] > clip, (name, seen[name])
    got = orc.forward_block(w, orc.KVCache(SMALL, 32), toks, store_dtype="f64", act_clip=clip)
    assert np.abs(got - ref).max() < 5e-6
    plain = orc.forward_block(w, orc.KVCache(SMALL, 32), toks, store_dtype="f64")
    assert np.abs(plain - got).max() > 1e-2                       # ... and changes the result
    loose = orc.forward_block(w, orc.KVCache(SMALL, 32), toks, store_dtype="f64", act_clip=1e30)
    assert np.array_equal(loose, plain)


def test_block_equals_sequential_rows(small_w):
    """Causality: an (m+1)-row block gives the logits of m+1 single-row steps."""
    rng = np.random.default_rng(4)
    toks = rng.integers(0, SMALL.vocab, 19)
    kv = orc.KVCache(SMALL, 32)
    block = orc.forward_block(small_w, kv, toks)
    kv1 = orc.KVCache(SMALL, 32)
    for i, t in enumerate(toks):
        row = orc.forward_block(small_w, kv1, [t])
        kv1.truncate(i + 1)
        assert np.abs(row[0] - block[i]).max() < 1e-9
    assert np.array_equal(kv.k[:, :, :19], kv1.k[:, :, :19])


def test_attention_vs_torch_sdpa():
    rng = np.random.default_rng(8)
    n, R, hd = 75, 6, 16
    L = n - R
    q, kc, vc = rng.standard_normal((R, hd)), rng.standard_normal((n, hd)), rng.standard_normal((n, hd))
    pos = L + np.arange(R)
    got = orc.causal_attention(q, kc, vc, pos)
    mask = torch.from_numpy(np.arange(n)[None, :] <= pos[:, None])
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None], torch.from_numpy(kc)[None, None],
        torch.from_numpy(vc)[None, None], attn_mask=mask[None, None])[0, 0].numpy()
    assert np.abs(got - ref).max() < 1e-12
    # brute force, one output element at a time
    for i in range(R):
        s = np.array([q[i] @ kc[j] / np.sqrt(hd) for j in range(L + i + 1)])
        p = np.exp(s - s.max())
        p /= p.sum()
        assert np.abs(sum(p[j] * vc[j] for j in range(L + i + 1)) - got[i]).max() < 1e-12


def test_rotary_properties():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((5, 3, 32))
    y = rng.standard_normal((5, 3, 32))
    zero = orc.rotary(x, np.zeros(5), 10000.0)
    assert np.array_equal(zero, x)                                    # position 0 = identity
    pos = np.array([0, 1, 7, 100, 4095])
    rx = orc.rotary(x, pos, 10000.0)
    assert np.allclose(np.linalg.norm(rx, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    # <rot(q,m), rot(k,n)> depends only on m - n
    a = np.sum(orc.rotary(x, pos, 1e4) * orc.rotary(y, pos - 3 + 10, 1e4), -1)
    b = np.sum(orc.rotary(x, pos + 50, 1e4) * orc.rotary(y, pos - 3 + 60, 1e4), -1)
    assert np.allclose(a, b, rtol=1e-9, atol=1e-9)
    # explicit 2x2 rotation of pair (j, j+hd/2) by pos * theta^(-2j/hd)
    hd, j, p, th = 32, 5, 7.0, 10000.0
    ang = p * th ** (-2 * j / hd)
    got = orc.rotary(x[:1, :1], np.array([p]), th)[0, 0]
    assert np.isclose(got[j], x[0, 0, j] * np.cos(ang) - x[0, 0, j + 16] * np.sin(ang))
    assert np.isclose(got[j + 16], x[0, 0, j + 16] * np.cos(ang) + x[0, 0, j] * np.sin(ang))


def test_rmsnorm_and_silu():
    rng = np.random.default_rng(10)
    x = rng.standard_normal((4, 64)) * 3
    y = orc.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, -1)), 1.0)
    g = rng.standard_normal(64)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), 1e-5).numpy()
    assert np.abs(orc.rmsnorm(x, g, 1e-5) - ref).max() < 1e-12
    assert np.abs(orc.silu(x) - torch.nn.functional.silu(torch.from_numpy(x)).numpy()).max() < 1e-12


def test_round_bf16_vs_torch():
    rng = np.random.default_rng(12)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000),
                        np.array([0.0, 1.0, 1.00390625, 1.01171875, -3.0e38, 1e-40])])
    ref = torch.from_numpy(x.astype(np.float32)).bfloat16().double().numpy()
    assert np.array_equal(orc.round_bf16(x), ref)
    bits = synth.f32_to_bf16_bits(x.astype(np.float32))
    assert np.array_equal(synth.bf16_bits_to_f32(bits).astype(np.float64), ref)


def test_bf16_bit_patterns_and_cache_load_vs_torch():
    """The oracle reads bf16 data (weights, cache rows) as uint16 bit patterns: every one of the
    65536 patterns must decode to the value torch's bfloat16 gives it, and KVCache.load must put
    rows [kv_head][n][hd] of one layer at cache[layer][kv_head][0..n) and nowhere else."""
    bits = np.arange(65536, dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    with np.errstate(invalid="ignore"):                     # signalling-NaN patterns
        got = orc._f64(bits)
    assert got.dtype == np.float64 and np.array_equal(got, ref, equal_nan=True)
    assert got[0x3F80] == 1.0 and got[0xC000] == -2.0 and got[0x3DCD] == 0.10009765625   # hand-decoded
    x = np.array([[1.5, -2.25], [3.0, 0.125]], dtype=np.float32)
    assert np.array_equal(orc._f64(x), x.astype(np.float64))
    shape = SMALL_BF16
    rng = np.random.default_rng(5)
    kb = rng.integers(0, 0x7F80, (shape.n_kv_heads, 7, shape.head_dim)).astype(np.uint16)   # finite, positive
    vb = (rng.integers(0, 0x7F80, kb.shape) | 0x8000).astype(np.uint16)                     # finite, negative
    kv = orc.KVCache(shape, 9)
    kv.load(1, kb, vb)
    tk = torch.from_numpy(kb.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    tv = torch.from_numpy(vb.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    assert np.array_equal(kv.k[1, :, :7], tk) and np.array_equal(kv.v[1, :, :7], tv)
    assert not kv.k[0].any() and not kv.k[1, :, 7:].any() and not kv.v[0].any() and not kv.v[1, :, 7:].any()
    assert kv.length == 0                                   # loading does not change the length
    kf = orc.KVCache(shape, 9)
    kf.load(1, tk.astype(np.float32), tv.astype(np.float32))   # the same values as floats
    assert np.array_equal(kf.k, kv.k) and np.array_equal(kf.v, kv.v)


def test_bf16_cache_rounding_is_the_only_rounding():
    w = synth.model_weights(SMALL_BF16, 77, threads=1)
    toks = np.arange(12) % SMALL_BF16.vocab
    kv = orc.KVCache(SMALL_BF16, 16)
    orc.forward_block(w, kv, toks)
    live = kv.k[:, :, :12]
    assert np.array_equal(orc.round_bf16(live), live) and np.abs(live).max() > 0
    assert np.array_equal(orc.round_bf16(kv.v[:, :, :12]), kv.v[:, :, :12])


def test_verify_rollback_leaves_no_trace(small_w):
    """App. B.2 / B.3 'Discussion of Truncation': rejected tokens affect neither the
    context nor the KV state.  Dead rows are poisoned with NaN to prove they are unread."""
    rng = np.random.default_rng(13)
    prompt = rng.integers(0, SMALL.vocab, 25).tolist()
    truth = orc.greedy_decode(small_w, prompt, 8)
    for j in range(0, 5):
        kv = orc.KVCache(SMALL, 64)
        pending = orc.prefill(small_w, kv, prompt)
        draft = truth[:j] + [(truth[j] + 1) % SMALL.vocab] + truth[j + 1:6]
        tau, nxt, _ = orc.verify(small_w, kv, pending, draft)
        assert tau == j and nxt == truth[j]                 # longest prefix, then the greedy token
        assert kv.length == len(prompt) - 1 + j + 1
        kv.k[:, :, kv.length:] = np.nan
        kv.v[:, :, kv.length:] = np.nan
        logits = orc.forward_block(small_w, kv, [nxt])
        fresh = orc.KVCache(SMALL, 64)
        p2 = orc.prefill(small_w, fresh, prompt + truth[:j + 1])
        assert p2 == nxt
        ref = orc.forward_block(small_w, fresh, [p2])
        assert np.abs(logits - ref).max() < 1e-9
        assert orc.argmax_first(logits[0]) == truth[j + 1]


def test_copyspec_equals_greedy_cfg1(tiny_w):
    """Output invariance (abstract; Sec. 3.2; App. B.2): on configuration 1 (tiny fp32
    decoder, 512-token context with planted spans, gamma=3, k=10, 64 new tokens) the
    CopySpec sequence is the plain greedy sequence."""
    prompt = synth.history_cfg1()["tokens"].tolist()
    ref = orc.greedy_decode(tiny_w, prompt, 64)
    for policy in ("rightmost", "first"):
        out, st = orc.copyspec_decode(tiny_w, prompt, 64, 3, 10, policy)
        assert out == ref
        assert st["attempts"] >= 1 and st["steps"] <= 64
    out0, st0 = orc.copyspec_decode(tiny_w, prompt, 64, 3, 0)     # k = 0: plain decoding
    assert out0 == ref and st0["steps"] == 64 and st0["attempts"] == 0


def test_draft_independence(small_w):
    """Whatever is drafted (noise, the true continuation, a true prefix with one edit),
    the emitted sequence is the greedy one; with the true continuation every attempt is
    fully accepted."""
    rng = np.random.default_rng(14)
    prompt = rng.integers(0, SMALL.vocab, 30).tolist()
    n_new = 24
    ref = orc.greedy_decode(small_w, prompt, n_new + 8)

    def true_cont(seq, room):
        done = len(seq) - len(prompt)
        return ref[done:done + min(5, room)]

    def noise(seq, room):
        return rng.integers(0, SMALL.vocab, min(5, room)).tolist()

    def edited(seq, room):
        d = true_cont(seq, room)
        if len(d) >= 3:
            d[2] = (d[2] + 1) % SMALL.vocab
        return d

    out, st = orc.copyspec_decode(small_w, prompt, n_new, 3, 5, draft_override=true_cont)
    assert out == ref[:n_new] and st["steps"] == 4 and st["accepted"] == 20
    out, st = orc.copyspec_decode(small_w, prompt, n_new, 3, 5, draft_override=noise)
    assert out == ref[:n_new]
    out, st = orc.copyspec_decode(small_w, prompt, n_new, 3, 5, draft_override=edited)
    assert out == ref[:n_new] and all(t == 2 for t in st["taus"][:-1])


def test_repeat_model_accepts_everything():
    """Closed form for the full-accept path: with attention and FFN outputs zeroed and
    lm_head = embedding, the greedy token repeats the current token, so the history
    becomes x,x,x,... and every attempt after the first gamma tokens accepts all k."""
    w = synth.model_weights(SMALL, 99, threads=1)
    for lw in w["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["wd"] = np.zeros_like(lw["wd"])
    w["lm_head"] = w["embed"].copy()
    w["final_norm"] = np.ones_like(w["final_norm"])
    prompt = [3, 1, 4, 1, 5, 9, 2, 6]
    assert orc.greedy_decode(w, prompt, 40) == [6] * 40
    # rightmost policy: the match is always at n - 2*gamma, its source runs into the end of
    # the history after gamma tokens, so every attempt drafts and accepts exactly gamma
    out, st = orc.copyspec_decode(w, prompt, 40, 3, 10, "rightmost")
    assert out == [6] * 40
    assert set(st["taus"][:-1]) == {3} and st["attempts"] == st["steps"] - 5
    # earliest policy: the source starts at the first run of 6s and grows with the history
    # until the full block of k = 10 is drafted and accepted
    out, st = orc.copyspec_decode(w, prompt, 60, 3, 10, "first")
    assert out == [6] * 60
    # by hand: 5 plain steps until six 6s exist (n = 13), then the source at index 10 offers
    # min(10, n - 10) tokens: 3 (n -> 17), 7 (n -> 25), then full blocks of 10
    assert st["taus"][:5] == [3, 7, 10, 10, 10] and st["steps"] - st["attempts"] == 5
    assert st["accepted"] == sum(st["taus"])


def test_one_guaranteed_token_per_step(small_w):
    rng = np.random.default_rng(15)
    prompt = rng.integers(0, SMALL.vocab, 20).tolist()
    kv = orc.KVCache(SMALL, 64)
    pending = orc.prefill(small_w, kv, prompt)
    L = kv.length
    tau, nxt, logits = orc.verify(small_w, kv, pending, [1, 2, 3])
    assert logits.shape == (4, SMALL.vocab)
    assert kv.length == L + tau + 1 and 0 <= nxt < SMALL.vocab
    with pytest.raises(ValueError):
        orc.forward_block(small_w, kv, list(range(64)))


# ----------------------------------------------------------------------------------------
# CopySpec merged with speculative decoding (Sec. 3.3, App. B.3 step 3)
# ----------------------------------------------------------------------------------------

def _looping_prompt(rng, n=36):
    """A prompt that already contains a repeated span, so the copy branch fires early."""
    p = rng.integers(0, SMALL.vocab, n).tolist()
    p[n - 9:n - 3] = p[4:10]
    return p


def test_merged_output_is_greedy_for_any_draft_model(small_w):
    """Whatever the draft model proposes, the emitted sequence is the target's greedy sequence
    (Sec. 3.3: the merge changes speed only).  Three draft models: unrelated weights, the
    target itself, and a model that always repeats its input token."""
    rng = np.random.default_rng(77)
    other = synth.model_weights(SMALL, 4321, threads=1)
    rep = synth.model_weights(SMALL, 99, threads=1)
    for lw in rep["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["wd"] = np.zeros_like(lw["wd"])
    rep["lm_head"] = rep["embed"].copy()
    rep["final_norm"] = np.ones_like(rep["final_norm"])
    for trial in range(3):
        prompt = _looping_prompt(rng)
        ref = orc.greedy_decode(small_w, prompt, 48)
        for wd in (other, small_w, rep):
            for gamma, k, delta in ((3, 10, 4), (2, 5, 3), (3, 0, 5)):
                out, st = orc.merged_decode(small_w, wd, prompt, 48, gamma, k, delta)
                assert out == ref, (trial, gamma, k, delta)
                assert st["copy_accepted"] <= st["copy_drafted"] and st["spec_accepted"] <= st["spec_drafted"]
                assert st["copy_attempts"] + st["spec_attempts"] <= st["steps"]
                if k == 0:
                    assert st["copy_attempts"] == 0
                if wd is small_w:              # a perfect draft model is never rejected
                    assert st["spec_accepted"] == st["spec_drafted"]


def test_merged_pure_speculative_closed_form(small_w):
    """No copying (k = 0) and draft == target: every step emits delta + 1 tokens until the
    budget clamps the last block."""
    rng = np.random.default_rng(78)
    prompt = rng.integers(0, SMALL.vocab, 17).tolist()
    out, st = orc.merged_decode(small_w, small_w, prompt, 23, 3, 0, 4)
    assert out == orc.greedy_decode(small_w, prompt, 23)
    # 5 + 5 + 5 + 5 + 3 tokens: drafts of 4, 4, 4, 4 and min(4, 23 - 20 - 1) = 2
    assert (st["steps"], st["spec_attempts"], st["spec_drafted"], st["spec_accepted"]) == (5, 5, 18, 18)


def test_merged_draft_cache_is_never_stale(small_w):
    """Catch-up and rollback of the draft model's cache: what it proposes at every attempt
    equals a fresh greedy continuation, by the draft model, of the sequence accepted so far."""
    rng = np.random.default_rng(79)
    other = synth.model_weights(SMALL, 555, threads=1)
    prompt = _looping_prompt(rng)
    out, st = orc.merged_decode(small_w, other, prompt, 40, 3, 6, 4)
    assert st["spec_attempts"] >= 3 and st["copy_attempts"] >= 1     # both branches ran
    seq = prompt + out
    for n, proposed in st["spec_trace"]:
        assert proposed == orc.greedy_decode(other, seq[:n], len(proposed)), n


def test_merged_without_draft_model_is_copyspec(small_w):
    rng = np.random.default_rng(80)
    prompt = _looping_prompt(rng)
    a, sa = orc.merged_decode(small_w, small_w, prompt, 40, 3, 8, 0)
    b, sb = orc.copyspec_decode(small_w, prompt, 40, 3, 8)
    assert a == b
    assert (sa["steps"], sa["copy_attempts"], sa["copy_accepted"], sa["spec_attempts"]) == \
           (sb["steps"], sb["attempts"], sb["accepted"], 0)

