"""CPU oracle for the CopySpec copy-and-verify step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct statement of what the hot path computes,
written from the paper in numpy float64.  It is imported only by the tests,
the smoke check and the benchmark's cpu_baseline leg; the product path never
calls it and shares no code with it.

What follows the paper, and where:
  * find_match / find_match_dict   Sec. 3.1 (dictionary of all gamma-token
        subsequences), Sec. 3.2 (copy the tokens after the match), App. B.1
        (match location p, chunk X_{p+gamma : p+gamma+m-1}), App. B.3 step 1
        (non-overlap condition p + gamma - 1 < t - gamma + 1).
  * accept_prefix                  Sec. 3.2 (tau accepted tokens plus one
        guaranteed token), App. B.2 (temperature 0: accept iff argmax; the
        first failure rejects everything after it).
  * verify / KV truncation         App. B.2, App. B.3 step 2 (truncate every
        layer's K, V to the accepted prefix).
  * copyspec_decode                Sec. 3.2 (re-match after every attempt),
        App. B.3 steps 1, 2, 4.
  * forward_block                  the target model.  The paper uses released
        Llama-3.1 / Qwen2.5 checkpoints (Sec. 4.1) and does not restate the
        architecture; this is the standard pre-norm Llama decoder block
        (RMSNorm, rotary with rotate-half pairing, grouped-query attention,
        SwiGLU), pinned in the tests against an independent library
        implementation of the same architecture.

Readings taken where the paper is silent (all listed again in the design
notes): indices are 0-based; among several matches the rightmost is the
default and the earliest selectable; a source that runs past the end of the
history truncates the draft; argmax ties go to the lowest index; a verify
block has draft_len + 1 rows (the pending token plus the drafts) so that full
acceptance still yields the guaranteed extra token.

Arithmetic: float64 everywhere.  The only rounding is the data contract's:
weights arrive already rounded to the storage type, and K/V rows are rounded
to the cache storage type ("f32" or "bf16") when they are stored.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------
# match search (Sec. 3.1, Sec. 3.2, App. B.1, App. B.3 step 1)
# ----------------------------------------------------------------------------

CONTEXT_CAP = 64    # longest backward agreement the "context" policy looks at


def context_length(h, p: int, gamma: int) -> int:
    """Number of tokens immediately before candidate p that equal the tokens immediately
    before the query suffix h[n-gamma:], counted backwards until the first difference,
    the start of the history or CONTEXT_CAP."""
    n = len(h)
    e = 0
    while e < CONTEXT_CAP and p - e - 1 >= 0 and int(h[p - e - 1]) == int(h[n - gamma - e - 1]):
        e += 1
    return e


def find_match(h, gamma: int, k: int, policy: str = "rightmost"):
    """Search history h[0..n) for an earlier, non-overlapping occurrence of its
    last gamma tokens and copy what follows.

    M = { p : 0 <= p <= n - 2*gamma, h[p+j] == h[n-gamma+j] for all j < gamma }.
    Returns (match_pos, src_pos, draft) with match_pos = max M ("rightmost"),
    min M ("first"), or ("context") the candidate whose preceding tokens agree longest
    with the tokens preceding the suffix (context_length; the rightmost among equals),
    src_pos = match_pos + gamma, draft = h[src_pos : src_pos+k] truncated at n.
    No match (or n < 2*gamma): (-1, -1, []).

    "context" is one concrete form of the structural ranking of candidates that the
    paper's Limitations section leaves to future work; like the other policies it only
    changes which draft is proposed, never the emitted tokens.
    """
    h = [int(t) for t in h]
    n = len(h)
    if gamma < 1 or k < 0:
        raise ValueError("gamma must be >= 1 and k >= 0")
    matches = []
    for p in range(0, n - 2 * gamma + 1):
        same = True
        for j in range(gamma):
            if h[p + j] != h[n - gamma + j]:
                same = False
                break
        if same:
            matches.append(p)
    if not matches:
        return -1, -1, []
    if policy == "rightmost":
        p = max(matches)
    elif policy == "first":
        p = min(matches)
    elif policy == "context":
        p = max(matches, key=lambda c: (context_length(h, c, gamma), c))
    else:
        raise ValueError(policy)
    src = p + gamma
    return p, src, h[src:min(src + k, n)]


def find_match_np(h, gamma: int, k: int, policy: str = "rightmost"):
    """Same definition as find_match with the inner position loop written as numpy
    array comparisons, for histories too long for the pure-Python loop."""
    h = np.asarray(h)
    n = h.shape[0]
    if gamma < 1 or k < 0:
        raise ValueError("gamma must be >= 1 and k >= 0")
    cnt = n - 2 * gamma + 1                     # candidate start positions 0..cnt-1
    if cnt <= 0:
        return -1, -1, []
    same = np.ones(cnt, dtype=bool)
    for j in range(gamma):
        same &= h[j:j + cnt] == h[n - gamma + j]
    pos = np.flatnonzero(same)
    if pos.size == 0:
        return -1, -1, []
    if policy == "rightmost":
        p = int(pos.max())
    elif policy == "first":
        p = int(pos.min())
    elif policy == "context":
        p = max((int(c) for c in pos), key=lambda c: (context_length(h, c, gamma), c))
    else:
        raise ValueError(policy)
    src = p + gamma
    return p, src, [int(t) for t in h[src:min(src + k, n)]]


class GammaGramDict:
    """The paper's own data structure (Sec. 3.1; the dictionary D of App. B.1): a hash map
    from every gamma-token subsequence to the positions where it starts, updated as
    tokens are appended (App. B.3 step 2d).  Used as a second, independently written
    formulation of the match search."""

    def __init__(self, gamma: int):
        self.gamma = gamma
        self.tokens: list[int] = []
        self.table: dict[tuple, list[int]] = {}

    def append(self, tok: int):
        self.tokens.append(int(tok))
        t = len(self.tokens)
        if t >= self.gamma:
            key = tuple(self.tokens[t - self.gamma:t])
            self.table.setdefault(key, []).append(t - self.gamma)

    def lookup(self, k: int, policy: str = "rightmost"):
        g, t = self.gamma, len(self.tokens)
        if t < g:
            return -1, -1, []
        occ = self.table.get(tuple(self.tokens[t - g:t]), [])
        # App. B.3 step 1c in 0-based form: last matched index p+g-1 must lie before the
        # first index t-g of the query suffix.
        occ = [p for p in occ if p + g - 1 < t - g]
        if not occ:
            return -1, -1, []
        if policy == "context":
            p = max(occ, key=lambda c: (context_length(self.tokens, c, g), c))
        else:
            p = occ[-1] if policy == "rightmost" else occ[0]
        return p, p + g, self.tokens[p + g:min(p + g + k, t)]


def find_match_dict(h, gamma: int, k: int, policy: str = "rightmost"):
    d = GammaGramDict(gamma)
    for t in h:
        d.append(t)
    return d.lookup(k, policy)


# ----------------------------------------------------------------------------
# acceptance (Sec. 3.2, App. B.2)
# ----------------------------------------------------------------------------

def argmax_first(row) -> int:
    """Index of the largest entry; the lowest index among equal maxima (numpy's argmax
    returns the first occurrence of the maximum)."""
    return int(np.argmax(np.asarray(row)))


def accept_prefix(argmax_rows, draft):
    """argmax_rows[i] is the target model's greedy token after row i of the verify
    block (row 0 = pending token, row i>0 = draft[i-1]).  Draft token i is accepted
    iff it equals argmax_rows[i] and all earlier draft tokens were accepted.
    Returns (tau, next_token): tau accepted drafts and the guaranteed extra token."""
    m = len(draft)
    assert len(argmax_rows) >= m + 1
    tau = 0
    while tau < m and int(argmax_rows[tau]) == int(draft[tau]):
        tau += 1
    return tau, int(argmax_rows[tau])


# ----------------------------------------------------------------------------
# target model (Llama-style decoder; Sec. 4.1 names the model families)
# ----------------------------------------------------------------------------

def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (ties to even), returned as float64."""
    f = x.astype(np.float32)          # double -> float rounding first, as storing a float would
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def _f64(w) -> np.ndarray:
    """Weights arrive as float arrays or as uint16 bfloat16 bit patterns."""
    w = np.asarray(w)
    if w.dtype == np.uint16:
        return (w.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return w.astype(np.float64)


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rotary(x: np.ndarray, pos: np.ndarray, theta: float, inv_freq=None) -> np.ndarray:
    """x: [rows][heads][hd]; pos: [rows].  Pairs (j, j + hd/2) are rotated by the angle
    pos * theta**(-2j/hd)  (rotate-half convention), or by pos * inv_freq[j] when the model
    brings its own frequencies (checkpoints with rescaled rotary frequencies, e.g. the
    Llama-3.1 models of Sec. 4.1)."""
    hd = x.shape[-1]
    half = hd // 2
    inv = theta ** (-(np.arange(half, dtype=np.float64) * 2.0) / hd)
    if inv_freq is not None:
        inv = np.asarray(inv_freq, dtype=np.float64)
        if inv.shape != (half,):
            raise ValueError("inv_freq must hold head_dim/2 frequencies")
    ang = pos.astype(np.float64)[:, None] * inv[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def causal_attention(q: np.ndarray, kc: np.ndarray, vc: np.ndarray, pos: np.ndarray) -> np.ndarray:
    """Softmax attention of query rows q [R][hd] over cache rows kc, vc [n][hd]; query row i
    sits at position pos[i] and sees cache rows j <= pos[i].  Scores are scaled by
    1/sqrt(hd)."""
    hd = q.shape[-1]
    visible = np.arange(kc.shape[0])[None, :] <= np.asarray(pos)[:, None]
    s = q @ kc.T / np.sqrt(hd)
    s = np.where(visible, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=1, keepdims=True)
    return p @ vc


class KVCache:
    """Per-layer K and V rows of one stream: [layer][kv_head][capacity][hd] float64 holding
    values representable in the cache storage type.  `length` is the number of valid rows;
    rows at and beyond it are dead."""

    def __init__(self, shape, capacity: int):
        self.shape = shape
        self.capacity = capacity
        z = (shape.n_layers, shape.n_kv_heads, capacity, shape.head_dim)
        self.k = np.zeros(z)
        self.v = np.zeros(z)
        self.length = 0

    def load(self, layer: int, k_rows, v_rows):
        """k_rows, v_rows: [kv_head][n][hd] (float or bf16 bits)."""
        n = k_rows.shape[1]
        self.k[layer, :, :n] = _f64(k_rows)
        self.v[layer, :, :n] = _f64(v_rows)

    def truncate(self, length: int):
        """App. B.2: keep only the first `length` positions."""
        assert 0 <= length <= self.capacity
        self.length = length


def forward_block(w: dict, kv: KVCache, tokens, store_dtype: str | None = None,
                  return_hidden: bool = False, act_clip: float | None = None) -> np.ndarray:
    """Run the decoder over `tokens` placed at positions kv.length, kv.length+1, ...;
    row i attends to cache rows 0 .. kv.length+i (its own included).  Writes the new K/V
    rows into the cache (it does not change kv.length) and returns logits [rows][vocab].

    act_clip (default None: no effect) models an implementation whose linear layers take inputs
    of limited range: the input of every projection (q/k/v, output, gate/up, down, lm_head) is
    clipped to [-act_clip, act_clip] before it is multiplied.  This is not part of the model or
    of the paper; it exists so that a library which documents such a range can be compared on
    inputs that leave it."""
    sh = w["shape"]
    store = store_dtype or sh.dtype
    H, KVH, hd, d = sh.n_heads, sh.n_kv_heads, sh.head_dim, sh.d_model
    G = H // KVH
    tokens = np.asarray(tokens, dtype=np.int64)
    R = tokens.shape[0]
    L = kv.length
    if L + R > kv.capacity:
        raise ValueError("KV capacity exceeded")
    pos = L + np.arange(R)
    clip = (lambda t: t) if act_clip is None else (lambda t: np.clip(t, -act_clip, act_clip))
    x = _f64(w["embed"][tokens])                                  # [R][d]
    for l, lw in enumerate(w["layers"]):
        a = clip(rmsnorm(x, _f64(lw["norm1"]), sh.rms_eps))
        q, kk, vv = a @ _f64(lw["wq"]).T, a @ _f64(lw["wk"]).T, a @ _f64(lw["wv"]).T
        if "bq" in lw:      # model families whose q, k, v projections carry a bias (Sec. 4.1: Qwen2.5)
            q, kk, vv = q + _f64(lw["bq"]), kk + _f64(lw["bk"]), vv + _f64(lw["bv"])
        q, kk, vv = q.reshape(R, H, hd), kk.reshape(R, KVH, hd), vv.reshape(R, KVH, hd)
        q = rotary(q, pos, sh.rope_theta, w.get("rope_inv_freq"))
        kk = rotary(kk, pos, sh.rope_theta, w.get("rope_inv_freq"))
        if store == "bf16":
            kk, vv = round_bf16(kk), round_bf16(vv)
        elif store == "f32":
            kk, vv = kk.astype(np.float32).astype(np.float64), vv.astype(np.float32).astype(np.float64)
        kv.k[l, :, L:L + R] = kk.transpose(1, 0, 2)
        kv.v[l, :, L:L + R] = vv.transpose(1, 0, 2)
        o = np.zeros((R, H, hd))
        for hq in range(H):
            g = hq // G                                               # grouped-query mapping
            o[:, hq] = causal_attention(q[:, hq], kv.k[l, g, :L + R], kv.v[l, g, :L + R], pos)
        x = x + clip(o.reshape(R, H * hd)) @ _f64(lw["wo"]).T
        b = clip(rmsnorm(x, _f64(lw["norm2"]), sh.rms_eps))
        gate = b @ _f64(lw["wg"]).T
        up = b @ _f64(lw["wu"]).T
        x = x + clip(silu(gate) * up) @ _f64(lw["wd"]).T
    hidden = clip(rmsnorm(x, _f64(w["final_norm"]), sh.rms_eps))
    if return_hidden:
        return hidden
    return hidden @ _f64(w["lm_head"]).T


# ----------------------------------------------------------------------------
# verify, greedy and CopySpec decoding (Sec. 3.2, App. B.2, App. B.3)
# ----------------------------------------------------------------------------

def verify(w: dict, kv: KVCache, pending: int, draft):
    """One copy-and-verify step.  The block [pending, draft...] is evaluated in one
    forward pass; the longest draft prefix that matches the greedy tokens is accepted,
    one more token comes for free, and the cache is truncated past the accepted rows.
    Returns (tau, next_token, logits).  Afterwards kv.length = L + tau + 1: the cache
    holds `pending` and the accepted drafts; next_token is not yet in it."""
    draft = [int(t) for t in draft]
    L = kv.length
    logits = forward_block(w, kv, [int(pending)] + draft)
    am = [argmax_first(row) for row in logits]
    tau, nxt = accept_prefix(am, draft)
    kv.truncate(L + tau + 1)
    return tau, nxt, logits


def prefill(w: dict, kv: KVCache, prompt, chunk: int = 64):
    """Fill the cache with prompt[0 .. n-1) and return the pending token prompt[n-1]."""
    prompt = [int(t) for t in prompt]
    body = prompt[:-1]
    for c in range(0, len(body), chunk):
        part = body[c:c + chunk]
        forward_block(w, kv, part, return_hidden=True)
        kv.truncate(kv.length + len(part))
    return prompt[-1]


def greedy_decode(w: dict, prompt, max_new: int, capacity: int | None = None):
    """Plain greedy decoding: one row per step."""
    sh = w["shape"]
    kv = KVCache(sh, capacity or (len(prompt) + max_new + 1))
    pending = prefill(w, kv, prompt)
    out = []
    for _ in range(max_new):
        logits = forward_block(w, kv, [pending])
        kv.truncate(kv.length + 1)
        pending = argmax_first(logits[0])
        out.append(pending)
    return out


def copyspec_decode(w: dict, prompt, max_new: int, gamma: int, k: int,
                    policy: str = "rightmost", capacity: int | None = None,
                    draft_override=None):
    """CopySpec decoding (App. B.3 without the draft-model branch): search the whole
    sequence so far for the last gamma tokens, draft the next k tokens, verify, accept,
    truncate, append, repeat.  Without a match the step is an ordinary decode step.
    `draft_override(seq, m)` lets a test substitute arbitrary drafts.
    Returns (tokens, stats) with stats = dict(steps, attempts, accepted)."""
    sh = w["shape"]
    kv = KVCache(sh, capacity or (len(prompt) + max_new + k + 2))
    seq = [int(t) for t in prompt]
    pending = prefill(w, kv, seq)
    out = []
    stats = {"steps": 0, "attempts": 0, "accepted": 0, "taus": []}
    while len(out) < max_new:
        _, _, draft = find_match_np(seq, gamma, k, policy) if len(seq) > 64 else \
            find_match(seq, gamma, k, policy)
        m = min(len(draft), max_new - len(out) - 1)     # never emit more than max_new
        draft = draft[:m]
        if draft_override is not None:
            draft = list(draft_override(seq, max_new - len(out) - 1))
        tau, nxt, _ = verify(w, kv, pending, draft)
        new = draft[:tau] + [nxt]
        seq.extend(new)
        out.extend(new)
        pending = nxt
        stats["steps"] += 1
        if draft:
            stats["attempts"] += 1
            stats["accepted"] += tau
            stats["taus"].append(tau)
    return out, stats


def _top2_margin(row) -> float:
    top = np.partition(np.asarray(row), -2)[-2:]
    return float(top[1] - top[0])


def merged_decode(w_target: dict, w_draft: dict, prompt, max_new: int, gamma: int, k: int,
                  delta: int, policy: str = "rightmost"):
    """CopySpec merged with vanilla speculative decoding (Sec. 3.3, App. B.3 steps 1-4).

    Every step first looks for a copy opportunity (step 1).  With a match the copied block
    is verified by the target model exactly as in copyspec_decode (step 2).  Without one the
    draft model proposes delta tokens greedily, one at a time, continuing the accepted
    sequence (step 3a); the target verifies them in one block with the same acceptance rule
    (step 3b); both caches are truncated to the accepted prefix (step 3c).  The draft model
    is only run when it is needed, so before drafting it first reads the tokens accepted
    since it last ran.

    Returns (tokens, stats); stats counts steps and, per branch, attempts / drafted /
    accepted tokens, records the smallest top-2 logit margin of every target and of every
    draft-model decision (how close the run came to a tie), and lists (history length,
    proposed tokens) of every draft-model attempt in "spec_trace".
    """
    assert w_target["shape"].vocab == w_draft["shape"].vocab
    cap = len(prompt) + max_new + max(k, delta) + 2
    kv_t = KVCache(w_target["shape"], cap)
    kv_d = KVCache(w_draft["shape"], cap)
    seq = [int(t) for t in prompt]
    pending = prefill(w_target, kv_t, seq)
    out = []
    st = {"steps": 0, "copy_attempts": 0, "copy_drafted": 0, "copy_accepted": 0,
          "spec_attempts": 0, "spec_drafted": 0, "spec_accepted": 0,
          "target_margin": np.inf, "draft_margin": np.inf, "spec_trace": []}
    while len(out) < max_new:
        room = max_new - len(out) - 1                      # drafts that can still be emitted
        n = len(seq)
        _, _, draft = find_match_np(seq, gamma, k, policy) if n > 64 else find_match(seq, gamma, k, policy)
        draft = draft[:room]
        copied = len(draft) > 0
        if not copied and delta > 0 and room > 0:
            # draft model: catch up on seq[kv_d.length : n-1], then generate from the pending token
            while kv_d.length < n - 1:
                part = seq[kv_d.length:min(n - 1, kv_d.length + 64)]
                forward_block(w_draft, kv_d, part, return_hidden=True)
                kv_d.truncate(kv_d.length + len(part))
            tok = pending
            for _ in range(min(delta, room)):
                lg = forward_block(w_draft, kv_d, [tok])
                kv_d.truncate(kv_d.length + 1)
                st["draft_margin"] = min(st["draft_margin"], _top2_margin(lg[0]))
                tok = argmax_first(lg[0])
                draft.append(tok)
            st["spec_trace"].append((n, list(draft)))
        L = kv_t.length
        logits = forward_block(w_target, kv_t, [pending] + draft)
        am = [argmax_first(r) for r in logits]
        tau, nxt = accept_prefix(am, draft)
        kv_t.truncate(L + tau + 1)
        for i in range(tau + 1):
            st["target_margin"] = min(st["target_margin"], _top2_margin(logits[i]))
        if draft and not copied:
            # the draft cache holds seq[0:n] and the drafts it was fed (all but the last one)
            kv_d.truncate(n + min(tau, len(draft) - 1))
        new = draft[:tau] + [nxt]
        seq.extend(new)
        out.extend(new)
        pending = nxt
        st["steps"] += 1
        if draft:
            key = "copy" if copied else "spec"
            st[key + "_attempts"] += 1
            st[key + "_drafted"] += len(draft)
            st[key + "_accepted"] += tau
    return out, st

