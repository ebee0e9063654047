"""ctypes binding of libcopyspec.so: same names as the C ABI, argument marshalling only.

Every step of the copy-and-verify path runs in the library's HIP kernels; this file
allocates output tensors with torch, passes raw pointers and turns status codes into
exceptions.  There is no fallback: if the shared library is missing, importing the
binding's functions fails with an explicit error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcopyspec.so")

CS_POLICY_RIGHTMOST, CS_POLICY_FIRST, CS_POLICY_CONTEXT = 0, 1, 2
CS_F32, CS_BF16 = 0, 1
CS_RANGE_NORM, CS_RANGE_ATTN, CS_RANGE_FFN, CS_RANGE_WEIGHT = 1, 2, 4, 8
CS_E_RANGE = -7
POLICIES = {"rightmost": CS_POLICY_RIGHTMOST, "first": CS_POLICY_FIRST, "context": CS_POLICY_CONTEXT}

EXPORTS = [
    "cs_last_error", "cs_version", "cs_find_match", "cs_find_match_ex", "cs_find_match_batch_dev", "cs_find_match_batch_dev_noalloc",
    "cs_model_create", "cs_model_create_staged", "cs_model_load_head", "cs_model_load_layer", "cs_model_destroy",
    "cs_model_range_status", "cs_model_set_rope_inv_freq", "cs_kv_create", "cs_kv_destroy", "cs_kv_set_len",
    "cs_kv_len", "cs_kv_load", "cs_kv_read", "cs_verify", "cs_step", "cs_decode",
    "cs_decode_greedy", "cs_decode_merged", "cs_prefill", "cs_prefill_batch", "cs_decode_batch", "cs_index_create", "cs_index_destroy",
    "cs_index_reset", "cs_index_find_match_batch_dev", "cs_op_gemm", "cs_op_attention", "cs_op_argmax_accept",
    "cs_set_plain_kernels", "cs_set_prompt_block_rows", "cs_kv_set_len_dev", "cs_profile_enable", "cs_profile_reset",
    "cs_profile_read",
]

CS_PROF = {"scan": 1, "gemm": 2, "attn": 4, "attn_merge": 8, "argmax": 16, "lm_head": 32}


class CopySpecError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libcopyspec error {code}: {msg}")
        self.code = code


class cs_model_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim",
                                         "d_ff", "vocab", "dtype")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float),
                ("max_batch", C.c_int32), ("max_k", C.c_int32)]


class cs_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "norm1", "norm2",
                                          "bq", "bk", "bv")]


class cs_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("layers", C.POINTER(cs_layer_weights))]


class cs_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("steps", "attempts", "drafted", "accepted")]


class cs_merged_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("steps", "copy_attempts", "copy_drafted", "copy_accepted",
                                         "spec_attempts", "spec_drafted", "spec_accepted",
                                         "draft_forwards")]


_lib = None


def load_library(path: Optional[str] = None) -> C.CDLL:
    """Load libcopyspec.so and declare its prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise ImportError(f"{p} not found: build it with `python -m paper_2502_08923_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(p)
    i32, i64, vp, f32p = C.c_int32, C.c_int64, C.c_void_p, C.c_void_p
    lib.cs_last_error.restype = C.c_char_p
    lib.cs_version.restype = C.c_char_p
    lib.cs_find_match.restype = i64
    lib.cs_find_match.argtypes = [vp, i64, i32]
    lib.cs_find_match_ex.argtypes = [vp, i64, i32, i32, i32, C.POINTER(i64), C.POINTER(i64), vp,
                                     C.POINTER(i32)]
    lib.cs_find_match_batch_dev.argtypes = [vp, i64, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.cs_find_match_batch_dev_noalloc.argtypes = [vp, i64, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.cs_index_create.argtypes = [i32, i64, i32, C.POINTER(vp)]
    lib.cs_index_destroy.argtypes = [vp]
    lib.cs_index_destroy.restype = None
    lib.cs_index_reset.argtypes = [vp, vp]
    lib.cs_index_find_match_batch_dev.argtypes = [vp, vp, i64, vp, i64, i32, i32, vp, vp, vp, vp, vp]
    lib.cs_model_create.argtypes = [C.POINTER(cs_model_cfg), C.POINTER(cs_weights), C.POINTER(vp)]
    lib.cs_model_create_staged.argtypes = [C.POINTER(cs_model_cfg), C.POINTER(vp)]
    lib.cs_model_load_head.argtypes = [vp, vp, vp, vp]
    lib.cs_model_load_layer.argtypes = [vp, i32, C.POINTER(cs_layer_weights)]
    lib.cs_model_destroy.argtypes = [vp]
    lib.cs_model_destroy.restype = None
    lib.cs_model_range_status.argtypes = [vp, C.POINTER(i32), i32]
    lib.cs_model_set_rope_inv_freq.argtypes = [vp, C.POINTER(C.c_double)]
    lib.cs_kv_create.argtypes = [vp, i32, i64, C.POINTER(vp)]
    lib.cs_kv_destroy.argtypes = [vp]
    lib.cs_kv_destroy.restype = None
    lib.cs_kv_set_len.argtypes = [vp, i32, i64]
    lib.cs_kv_len.argtypes = [vp, i32]
    lib.cs_kv_len.restype = i64
    lib.cs_kv_load.argtypes = [vp, i32, i32, i64, i64, vp, vp]
    lib.cs_kv_read.argtypes = [vp, i32, i32, i64, i64, vp, vp]
    lib.cs_verify.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, f32p, vp]
    lib.cs_step.argtypes = [vp, vp, vp, i64, vp, vp, i32, i32, i32, vp, vp, vp, vp]
    lib.cs_decode.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, i32, vp, C.POINTER(i64),
                              C.POINTER(cs_stats)]
    lib.cs_decode_greedy.argtypes = [vp, vp, vp, i64, i64, i32, vp, C.POINTER(i64)]
    lib.cs_decode_merged.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, i32, i32, i32, vp,
                                     C.POINTER(i64), C.POINTER(cs_merged_stats)]
    lib.cs_prefill.argtypes = [vp, vp, i32, vp, i64]
    lib.cs_prefill_batch.argtypes = [vp, vp, vp, i64, vp]
    lib.cs_decode_batch.argtypes = [vp, vp, vp, i64, vp, i64, i32, i32, i32, i32, vp, vp, vp]
    lib.cs_op_gemm.argtypes = [vp, i32, vp, vp, vp, i32, i32, i32, vp]
    lib.cs_op_attention.argtypes = [vp, vp, i32, vp, i32, vp, vp]
    lib.cs_op_argmax_accept.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.cs_kv_set_len_dev.argtypes = [vp, vp, i64, vp]
    lib.cs_profile_enable.argtypes = [i32]
    lib.cs_profile_enable.restype = None
    lib.cs_profile_reset.restype = None
    lib.cs_profile_read.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.cs_set_plain_kernels.argtypes = [i32]
    lib.cs_set_plain_kernels.restype = None
    lib.cs_set_prompt_block_rows.argtypes = [i32]
    lib.cs_set_prompt_block_rows.restype = None
    for name in EXPORTS:
        getattr(lib, name)
    if path is None:
        _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise CopySpecError(int(rc), load_library().cs_last_error().decode())


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dev_i32(t: torch.Tensor, name: str) -> torch.Tensor:
    if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous int32 CUDA tensor")
    return t


def _policy(p) -> int:
    return POLICIES[p] if isinstance(p, str) else int(p)


# ----------------------------------------------------------------------------------------
# match search
# ----------------------------------------------------------------------------------------

def cs_find_match(history, gamma: int) -> int:
    h = np.ascontiguousarray(history, dtype=np.int32)
    r = load_library().cs_find_match(h.ctypes.data, h.shape[0], gamma)
    if r <= -2:
        _check(int(r))
    return int(r)


def cs_find_match_ex(history, gamma: int, k: int, policy="rightmost"):
    """Returns (match_pos, src_pos, draft list of draft_len tokens)."""
    h = np.ascontiguousarray(history, dtype=np.int32)
    mp, sp, dl = C.c_int64(), C.c_int64(), C.c_int32()
    draft = np.full(max(k, 1), -1, dtype=np.int32)
    _check(load_library().cs_find_match_ex(h.ctypes.data, h.shape[0], gamma, k, _policy(policy),
                                           C.byref(mp), C.byref(sp), draft.ctypes.data, C.byref(dl)))
    return int(mp.value), int(sp.value), draft[:dl.value].tolist()


def cs_find_match_batch_dev(d_hist: torch.Tensor, d_len: torch.Tensor, gamma: int, k: int,
                            policy="rightmost", stream=None):
    """d_hist: int32 [B][stride] on the GPU, d_len: int32 [B].
    Returns (match_pos[B], src_pos[B], draft[B][k], draft_len[B]) device tensors."""
    _dev_i32(d_hist, "d_hist"), _dev_i32(d_len, "d_len")
    B, stride = d_hist.shape
    dev = d_hist.device
    mp = torch.empty(B, dtype=torch.int32, device=dev)
    sp = torch.empty(B, dtype=torch.int32, device=dev)
    dr = torch.empty((B, k), dtype=torch.int32, device=dev)
    dl = torch.empty(B, dtype=torch.int32, device=dev)
    _check(load_library().cs_find_match_batch_dev(d_hist.data_ptr(), stride, d_len.data_ptr(), B,
                                                  gamma, k, _policy(policy), mp.data_ptr(),
                                                  sp.data_ptr(), dr.data_ptr(), dl.data_ptr(),
                                                  _stream(stream)))
    return mp, sp, dr, dl


def cs_find_match_batch_dev_noalloc(d_hist: torch.Tensor, d_len: torch.Tensor, gamma: int, k: int,
                                    policy="rightmost", stream=None, out=None):
    """Same as cs_find_match_batch_dev through the entry point that allocates nothing; `out` =
    (match_pos, src_pos, draft, draft_len) lets the caller bring the outputs too."""
    _dev_i32(d_hist, "d_hist"), _dev_i32(d_len, "d_len")
    B, stride = d_hist.shape
    dev = d_hist.device
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, k), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev))
    mp, sp, dr, dl = out
    _check(load_library().cs_find_match_batch_dev_noalloc(d_hist.data_ptr(), stride, d_len.data_ptr(), B,
                                                          gamma, k, _policy(policy), mp.data_ptr(),
                                                          sp.data_ptr(), dr.data_ptr(), dl.data_ptr(),
                                                          _stream(stream)))
    return mp, sp, dr, dl


class Index:
    """cs_index handle: the gamma-gram hash index of B device-resident histories."""

    def __init__(self, B: int, max_len: int, gamma: int):
        self.B, self.max_len, self.gamma = B, max_len, gamma
        h = C.c_void_p()
        _check(load_library().cs_index_create(B, max_len, gamma, C.byref(h)))
        self.handle = h

    def reset(self, stream=None):
        _check(load_library().cs_index_reset(self.handle, _stream(stream)))

    def destroy(self):
        if self.handle:
            load_library().cs_index_destroy(self.handle)
            self.handle = None


def cs_index_find_match_batch_dev(index: Index, d_hist: torch.Tensor, d_len: torch.Tensor,
                                  max_new_positions: int, k: int, policy="rightmost", stream=None):
    """Same outputs as cs_find_match_batch_dev, answered from the index (which is first brought
    up to date with the histories)."""
    _dev_i32(d_hist, "d_hist"), _dev_i32(d_len, "d_len")
    B, stride = d_hist.shape
    if B != index.B:
        raise ValueError(f"index was created for {index.B} streams, got {B}")
    dev = d_hist.device
    mp = torch.empty(B, dtype=torch.int32, device=dev)
    sp = torch.empty(B, dtype=torch.int32, device=dev)
    dr = torch.empty((B, k), dtype=torch.int32, device=dev)
    dl = torch.empty(B, dtype=torch.int32, device=dev)
    _check(load_library().cs_index_find_match_batch_dev(index.handle, d_hist.data_ptr(), stride,
                                                        d_len.data_ptr(), max_new_positions, k,
                                                        _policy(policy), mp.data_ptr(), sp.data_ptr(),
                                                        dr.data_ptr(), dl.data_ptr(), _stream(stream)))
    return mp, sp, dr, dl


# ----------------------------------------------------------------------------------------
# handles
# ----------------------------------------------------------------------------------------

def _to_dev(a, bf16: bool, device) -> torch.Tensor:
    """numpy / torch array -> device tensor; uint16 arrays are bfloat16 bit patterns."""
    if isinstance(a, torch.Tensor):
        t = a
    else:
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            t = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
        else:
            t = torch.from_numpy(a)
    want = torch.bfloat16 if bf16 else torch.float32
    if t.dtype != want:
        t = t.to(want)
    return t.to(device).contiguous()


class Model:
    """cs_model handle.  `weights` is a dict like synth.model_weights returns (numpy or torch
    arrays; uint16 = bfloat16 bits); they are uploaded, handed to cs_model_create (which copies
    them into library-owned memory) and released.  If weights["layers"] is a function of the
    layer index (and weights["head"] a function returning embed, lm_head, final_norm), as
    synth.model_weights_lazy returns, the model is created in stages: one part at a time is
    drawn, uploaded, handed to cs_model_load_layer / cs_model_load_head and released, so the
    caller-side copy never exceeds one layer."""

    def __init__(self, weights: dict, max_batch: int, max_k: int, plain: bool = False,
                 device="cuda:0", prompt_block_rows: int = 0):
        lib = load_library()
        sh = weights["shape"]
        self.shape = sh
        bf16 = sh.dtype == "bf16"
        self.dtype = CS_BF16 if bf16 else CS_F32
        self.max_batch, self.max_k = max_batch, max_k
        dev = torch.device(device)
        cfg = cs_model_cfg(sh.n_layers, sh.d_model, sh.n_heads, sh.n_kv_heads, sh.head_dim, sh.d_ff,
                           sh.vocab, self.dtype, sh.rope_theta, sh.rms_eps, max_batch, max_k)
        keep = []

        def up(a, as_bf16):
            t = _to_dev(a, as_bf16, dev)
            keep.append(t)
            return t.data_ptr()

        def fill_layer(dst, lw):
            for name in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
                setattr(dst, name, up(lw[name], bf16))
            dst.norm1 = up(lw["norm1"], False)
            dst.norm2 = up(lw["norm2"], False)
            for name in ("bq", "bk", "bv"):           # optional float32 projection biases
                if name in lw:
                    setattr(dst, name, up(lw[name], False))

        staged = callable(weights["layers"])
        h = C.c_void_p()
        lib.cs_set_plain_kernels(1 if plain else 0)
        lib.cs_set_prompt_block_rows(prompt_block_rows)
        try:
            torch.cuda.synchronize(dev)
            if staged:
                _check(lib.cs_model_create_staged(C.byref(cfg), C.byref(h)))
            else:
                layers = (cs_layer_weights * sh.n_layers)()
                for l, lw in enumerate(weights["layers"]):
                    fill_layer(layers[l], lw)
                w = cs_weights(up(weights["embed"], bf16), up(weights["lm_head"], bf16),
                               up(weights["final_norm"], False), layers)
                _check(lib.cs_model_create(C.byref(cfg), C.byref(w), C.byref(h)))
        finally:
            lib.cs_set_plain_kernels(0)
            lib.cs_set_prompt_block_rows(0)
        self.handle = h
        self.device = dev
        del keep[:]
        if staged:
            try:
                head = weights["head"]()
                _check(lib.cs_model_load_head(h, up(head["embed"], bf16), up(head["lm_head"], bf16),
                                              up(head["final_norm"], False)))
                del head, keep[:]
                for l in range(sh.n_layers):
                    one = cs_layer_weights()
                    lw = weights["layers"](l)
                    fill_layer(one, lw)
                    torch.cuda.synchronize(dev)
                    _check(lib.cs_model_load_layer(h, l, C.byref(one)))
                    del lw, keep[:]
            except Exception:
                self.destroy()
                raise
        if weights.get("rope_inv_freq") is not None:      # the model brings its own rotary frequencies
            self.set_rope_inv_freq(weights["rope_inv_freq"])

    def load_layer(self, layer: int, lw: dict):
        """New weights for one layer (cs_model_load_layer): the dict of one entry of weights["layers"]."""
        bf16 = self.dtype == CS_BF16
        keep = []
        one = cs_layer_weights()
        for name in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
            keep.append(_to_dev(lw[name], bf16, self.device))
            setattr(one, name, keep[-1].data_ptr())
        for name in ("norm1", "norm2", "bq", "bk", "bv"):
            if name in lw:
                keep.append(_to_dev(lw[name], False, self.device))
                setattr(one, name, keep[-1].data_ptr())
        torch.cuda.synchronize(self.device)
        _check(load_library().cs_model_load_layer(self.handle, layer, C.byref(one)))

    def set_rope_inv_freq(self, inv_freq):
        """head_dim/2 rotary frequencies (angle of pair j at position p = p * inv_freq[j]); None
        goes back to rope_theta."""
        if inv_freq is None:
            _check(load_library().cs_model_set_rope_inv_freq(self.handle, None))
            return
        a = np.ascontiguousarray(np.asarray(inv_freq, dtype=np.float64))
        if a.shape != (self.shape.head_dim // 2,):
            raise ValueError("inv_freq must hold head_dim/2 values")
        _check(load_library().cs_model_set_rope_inv_freq(self.handle, a.ctypes.data_as(C.POINTER(C.c_double))))

    def range_status(self, clear: bool = True) -> int:
        """CS_RANGE_* bits raised since the last clear (waits for the device)."""
        f = C.c_int32()
        _check(load_library().cs_model_range_status(self.handle, C.byref(f), 1 if clear else 0))
        return int(f.value)

    def destroy(self):
        if getattr(self, "handle", None):
            load_library().cs_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class KV:
    """cs_kv handle."""

    def __init__(self, model: Model, batch: int, capacity: int):
        h = C.c_void_p()
        _check(load_library().cs_kv_create(model.handle, batch, capacity, C.byref(h)))
        self.handle, self.model, self.batch, self.capacity = h, model, batch, capacity

    def set_len(self, stream_idx: int, length: int):
        _check(load_library().cs_kv_set_len(self.handle, stream_idx, length))

    def len(self, stream_idx: int) -> int:
        r = load_library().cs_kv_len(self.handle, stream_idx)
        if r < 0:
            _check(int(r))
        return int(r)

    def set_len_dev(self, d_len: torch.Tensor, upper_bound: int, stream=None):
        _dev_i32(d_len, "d_len")
        _check(load_library().cs_kv_set_len_dev(self.handle, d_len.data_ptr(), upper_bound,
                                                _stream(stream)))

    def load(self, layer: int, stream_idx: int, pos0: int, k_rows, v_rows):
        bf16 = self.model.dtype == CS_BF16
        k = _to_dev(k_rows, bf16, self.model.device)
        v = _to_dev(v_rows, bf16, self.model.device)
        assert k.shape == v.shape and k.dim() == 3
        _check(load_library().cs_kv_load(self.handle, layer, stream_idx, pos0, k.shape[1],
                                         k.data_ptr(), v.data_ptr()))

    def read(self, layer: int, stream_idx: int, pos0: int, n: int):
        sh = self.model.shape
        dt = torch.bfloat16 if self.model.dtype == CS_BF16 else torch.float32
        k = torch.empty((sh.n_kv_heads, n, sh.head_dim), dtype=dt, device=self.model.device)
        v = torch.empty_like(k)
        _check(load_library().cs_kv_read(self.handle, layer, stream_idx, pos0, n, k.data_ptr(),
                                         v.data_ptr()))
        return k, v

    def destroy(self):
        if getattr(self, "handle", None):
            load_library().cs_kv_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


# ----------------------------------------------------------------------------------------
# verify, step, decode
# ----------------------------------------------------------------------------------------

def cs_verify(model: Model, kv: KV, pending: torch.Tensor, draft: torch.Tensor,
              draft_len: torch.Tensor, k: int, want_logits: bool = False, stream=None):
    """Returns (accepted_len[B], next_token[B], logits[B][k+1][V] or None), device tensors."""
    B = kv.batch
    dev = model.device
    _dev_i32(pending, "pending"), _dev_i32(draft_len, "draft_len")
    if k > 0:
        _dev_i32(draft, "draft")
        assert tuple(draft.shape) == (B, k)
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    logits = torch.empty((B, k + 1, model.shape.vocab), dtype=torch.float32, device=dev) \
        if want_logits else None
    _check(load_library().cs_verify(model.handle, kv.handle, pending.data_ptr(),
                                    draft.data_ptr() if k > 0 else None, draft_len.data_ptr(), k,
                                    acc.data_ptr(), nxt.data_ptr(), _ptr(logits), _stream(stream)))
    return acc, nxt, logits


def cs_step(model: Model, kv: KV, hist: torch.Tensor, hist_len: torch.Tensor,
            room: Optional[torch.Tensor], gamma: int, k: int, policy="rightmost", stream=None,
            out=None):
    """One whole copy-and-verify step on device-resident histories [B][stride].
    Returns (accepted_len, next_token, draft_len) device tensors (reused if `out` is given)."""
    _dev_i32(hist, "hist"), _dev_i32(hist_len, "hist_len")
    B, stride = hist.shape
    dev = model.device
    if out is None:
        out = tuple(torch.empty(B, dtype=torch.int32, device=dev) for _ in range(3))
    acc, nxt, dl = out
    _check(load_library().cs_step(model.handle, kv.handle, hist.data_ptr(), stride,
                                  hist_len.data_ptr(), _ptr(room), gamma, k, _policy(policy),
                                  acc.data_ptr(), nxt.data_ptr(), dl.data_ptr(), _stream(stream)))
    return acc, nxt, dl


def cs_decode(model: Model, kv: KV, prompt: Sequence[int], max_new: int, gamma: int, k: int,
              policy="rightmost", eos_id: int = -1):
    """Returns (tokens list, stats dict)."""
    p = np.ascontiguousarray(prompt, dtype=np.int32)
    out = np.zeros(max(max_new, 1), dtype=np.int32)
    n_out, st = C.c_int64(), cs_stats()
    _check(load_library().cs_decode(model.handle, kv.handle, p.ctypes.data, p.shape[0], max_new,
                                    gamma, k, _policy(policy), eos_id, out.ctypes.data,
                                    C.byref(n_out), C.byref(st)))
    return out[:n_out.value].tolist(), {"steps": st.steps, "attempts": st.attempts,
                                        "drafted": st.drafted, "accepted": st.accepted}


def cs_decode_greedy(model: Model, kv: KV, prompt: Sequence[int], max_new: int, eos_id: int = -1):
    p = np.ascontiguousarray(prompt, dtype=np.int32)
    out = np.zeros(max(max_new, 1), dtype=np.int32)
    n_out = C.c_int64()
    _check(load_library().cs_decode_greedy(model.handle, kv.handle, p.ctypes.data, p.shape[0],
                                           max_new, eos_id, out.ctypes.data, C.byref(n_out)))
    return out[:n_out.value].tolist()


def cs_decode_merged(model: Model, kv: KV, draft_model: Model, draft_kv: KV, prompt: Sequence[int],
                     max_new: int, gamma: int, k: int, delta: int, policy="rightmost", eos_id: int = -1):
    """Returns (tokens list, stats dict)."""
    p = np.ascontiguousarray(prompt, dtype=np.int32)
    out = np.zeros(max(max_new, 1), dtype=np.int32)
    n_out, st = C.c_int64(), cs_merged_stats()
    _check(load_library().cs_decode_merged(model.handle, kv.handle, draft_model.handle, draft_kv.handle,
                                           p.ctypes.data, p.shape[0], max_new, gamma, k, _policy(policy),
                                           delta, eos_id, out.ctypes.data, C.byref(n_out), C.byref(st)))
    return out[:n_out.value].tolist(), {n: getattr(st, n) for n, _ in cs_merged_stats._fields_}


def cs_prefill(model: Model, kv: KV, stream_idx: int, prompt: Sequence[int]):
    p = np.ascontiguousarray(prompt, dtype=np.int32)
    _check(load_library().cs_prefill(model.handle, kv.handle, stream_idx, p.ctypes.data, p.shape[0]))


def _pack_prompts(kv: KV, prompts: Sequence[Sequence[int]]):
    assert len(prompts) == kv.batch, "one prompt per stream of the cache"
    lens = np.array([len(p) for p in prompts], dtype=np.int64)
    flat = np.zeros((kv.batch, max(int(lens.max()), 1)), dtype=np.int32)
    for b, p in enumerate(prompts):
        flat[b, :len(p)] = np.asarray(p, dtype=np.int32)
    return flat, lens


def cs_prefill_batch(model: Model, kv: KV, prompts: Sequence[Sequence[int]]):
    flat, lens = _pack_prompts(kv, prompts)
    _check(load_library().cs_prefill_batch(model.handle, kv.handle, flat.ctypes.data, flat.shape[1],
                                           lens.ctypes.data))


def cs_decode_batch(model: Model, kv: KV, prompts: Sequence[Sequence[int]], max_new: int, gamma: int,
                    k: int, policy="rightmost", eos_id: int = -1):
    """Returns (one token list per stream, one stats dict per stream)."""
    flat, lens = _pack_prompts(kv, prompts)
    B = kv.batch
    out = np.zeros((B, max(max_new, 1)), dtype=np.int32)
    n_out = np.zeros(B, dtype=np.int64)
    st = (cs_stats * B)()
    _check(load_library().cs_decode_batch(model.handle, kv.handle, flat.ctypes.data, flat.shape[1],
                                          lens.ctypes.data, max_new, gamma, k, _policy(policy), eos_id,
                                          out.ctypes.data, n_out.ctypes.data, C.cast(st, C.c_void_p)))
    toks = [out[b, :int(n_out[b])].tolist() for b in range(B)]
    stats = [{n: getattr(st[b], n) for n, _ in cs_stats._fields_} for b in range(B)]
    return toks, stats


# ----------------------------------------------------------------------------------------
# single operations
# ----------------------------------------------------------------------------------------

def cs_op_gemm(model: Model, X: torch.Tensor, W: torch.Tensor, stream=None) -> torch.Tensor:
    """Y[R][N] float32 = X[R][K] * W[N][K]^T; X and W both bfloat16 or both float32."""
    assert X.is_cuda and W.is_cuda and X.is_contiguous() and W.is_contiguous()
    assert X.dtype == W.dtype and X.shape[1] == W.shape[1]
    dt = CS_BF16 if X.dtype == torch.bfloat16 else CS_F32
    R, K = X.shape
    N = W.shape[0]
    Y = torch.empty((R, N), dtype=torch.float32, device=X.device)
    _check(load_library().cs_op_gemm(model.handle, dt, X.data_ptr(), W.data_ptr(), Y.data_ptr(), R, N,
                                     K, _stream(stream)))
    return Y


def cs_op_attention(model: Model, kv: KV, layer: int, q: torch.Tensor, stream=None) -> torch.Tensor:
    """q: float32 [B][rows][H][hd] (rotated).  Returns float32 [B][rows][H*hd]."""
    assert q.is_cuda and q.dtype == torch.float32 and q.is_contiguous()
    B, rows, H, hd = q.shape
    assert B == kv.batch
    out = torch.empty((B, rows, H * hd), dtype=torch.float32, device=q.device)
    _check(load_library().cs_op_attention(model.handle, kv.handle, layer, q.data_ptr(), rows,
                                          out.data_ptr(), _stream(stream)))
    return out


def cs_op_argmax_accept(model: Model, logits: torch.Tensor, draft: torch.Tensor,
                        draft_len: torch.Tensor, stream=None):
    """logits: float32 [B][k+1][V].  Returns (accepted_len[B], next_token[B], row_argmax[B][k+1])."""
    assert logits.is_cuda and logits.dtype == torch.float32 and logits.is_contiguous()
    B, rows, V = logits.shape
    k = rows - 1
    dev = logits.device
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    am = torch.empty((B, rows), dtype=torch.int32, device=dev)
    _check(load_library().cs_op_argmax_accept(model.handle, logits.data_ptr(), B, k, V,
                                              draft.data_ptr() if k > 0 else None,
                                              draft_len.data_ptr(), acc.data_ptr(), nxt.data_ptr(),
                                              am.data_ptr(), _stream(stream)))
    return acc, nxt, am


# ----------------------------------------------------------------------------------------
# instrumentation
# ----------------------------------------------------------------------------------------

def cs_profile_enable(classes: Sequence[str] = ()):
    mask = 0
    for c in classes:
        mask |= CS_PROF[c]
    load_library().cs_profile_enable(mask)


def cs_profile_reset():
    load_library().cs_profile_reset()


def cs_profile_read(cls: str):
    """Returns (total_ms, launches) of one kernel class since the last reset."""
    ms, n = C.c_double(), C.c_int64()
    _check(load_library().cs_profile_read(CS_PROF[cls], C.byref(ms), C.byref(n)))
    return ms.value, n.value
