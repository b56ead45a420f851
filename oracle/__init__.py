"""CPU oracle for Speculative Jacobi Decoding -- TEST INFRASTRUCTURE ONLY.

Builds `sjd_oracle.c` with gcc and exposes it through ctypes.  Only the tests, the smoke
check and the CPU-baseline leg of the benchmark may import this package; the product path
(the HIP library and its binding) never does.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sjd_oracle.c")
_LIB = os.path.join(_HERE, "libsjd_oracle.so")

_CFLAGS = ["-O2", "-fopenmp", "-shared", "-fPIC", "-std=gnu11", "-ffp-contract=off", "-mavx2", "-mfma",
           "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle (the checker is built like any other artefact; building it is not using it)."""
    stale = (not os.path.exists(_LIB)) or any(
        os.path.getmtime(os.path.join(_HERE, f)) > os.path.getmtime(_LIB) for f in ("sjd_oracle.c", "sjd_oracle.h"))
    if force or stale:
        subprocess.check_call(["gcc", *_CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Sampler(C.Structure):
    _fields_ = [("top_k", C.c_int32), ("temperature", C.c_float)]


class Init(C.Structure):
    _fields_ = [("mode", C.c_int32), ("row_stride", C.c_int32), ("eol_id", C.c_int32), ("flags", C.c_int32)]


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "d_ffn", "vocab_total", "samp_lo",
                                          "samp_hi", "max_seq", "dtype")] + [("rope_theta", C.c_float),
                                                                             ("rms_eps", C.c_float)]


class Stats(C.Structure):
    _fields_ = [("steps", C.c_int32), ("accept_hist", C.c_int32 * 65)]


class TfCtx(C.Structure):
    _fields_ = [("m", C.c_void_p), ("kv", C.c_void_p)]


FORWARD_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_float))

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, i32, u32, u64, i64, f32 = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64, C.c_int64, C.c_float
        P = C.POINTER
        sig = {
            "orc_num_threads": (i32, []),
            "orc_philox4x32_10": (None, [vp, vp, vp]),
            "orc_draw": (None, [u64, u64, u32, vp]),
            "orc_u_acc": (f32, [u32]),
            "orc_exp": (f32, [f32]),
            "orc_guide": (None, [vp, vp, f32, i64, vp]),
            "orc_dist": (None, [vp, i32, i32, f32, i32, vp]),
            "orc_sample": (i32, [vp, i32, u32]),
            "orc_verify_probs": (i32, [vp, vp, vp, i32, i32, i32, P(Init), i32, vp, u64, u64, vp, vp, vp]),
            "orc_verify": (i32, [vp, vp, vp, i32, i32, i32, P(Sampler), P(Init), i32, vp, u64, u64, vp, vp, vp]),
            "orc_first_window": (None, [vp, i32, i32, i32, P(Init), u64, vp, vp]),
            "orc_model_create": (vp, [P(Config), vp]),
            "orc_model_free": (None, [vp]),
            "orc_kv_create": (vp, [vp]),
            "orc_kv_free": (None, [vp]),
            "orc_kv_set_len": (None, [vp, i32]),
            "orc_kv_len": (i32, [vp]),
            "orc_forward_full": (None, [vp, vp, i32, vp]),
            "orc_forward_window": (None, [vp, vp, vp, i32, vp]),
            "orc_embed": (None, [vp, vp, i32, vp]),
            "orc_generate_sjd": (None, [vp, vp, i32, vp, i32, i32, i32, i32, P(Sampler), P(Init), u64, vp, P(Stats)]),
            "orc_generate_ar": (None, [vp, vp, i32, vp, i32, i32, i32, P(Sampler), P(Init), u64, vp]),
            "orc_tf_forward": (None, [vp, i32, vp, i32, vp]),
            "orc_tf_prefill": (None, [P(TfCtx), vp, i32, vp, i32, vp]),
            "orc_toy_forward": (None, [vp, i32, vp, i32, vp]),
            "orc_toy_histogram": (None, [vp, i32, i32, i32, P(Sampler), P(Init), u64, i64, i32, vp, vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ---- thin numpy wrappers -------------------------------------------------------------------
def philox(key, ctr):
    k = np.asarray(key, dtype=np.uint32); c = np.asarray(ctr, dtype=np.uint32); o = np.zeros(4, np.uint32)
    lib().orc_philox4x32_10(_p(k), _p(c), _p(o))
    return o


def draw(seed, c, i):
    o = np.zeros(4, np.uint32)
    lib().orc_draw(seed, c, i, _p(o))
    return o


def u_acc(word):
    return float(lib().orc_u_acc(int(word)))


def exp(x):
    return float(lib().orc_exp(float(np.float32(x))))


def guide(z_cond, z_uncond, w):
    zc = _f32(z_cond); zu = _f32(z_uncond); out = np.empty_like(zc)
    assert zc.shape == zu.shape
    lib().orc_guide(_p(zc), _p(zu), float(w), zc.size, _p(out))
    return out


def dist(z, top_k, temperature, forced=-1):
    z = _f32(z); q = np.empty_like(z)
    lib().orc_dist(_p(z), z.size, top_k, temperature, forced, _p(q))
    return q


def sample(w, k32):
    w = _f32(w)
    return int(lib().orc_sample(_p(w), w.size, int(k32)))


def _ring_arg(init, ring, V):
    """sample-above keeps [row_stride x V] recorded distributions in a caller-owned array, updated in place"""
    if init.mode != 4:
        return None
    assert ring is not None and ring.dtype == np.float32 and ring.flags.c_contiguous
    assert ring.shape == (init.row_stride, V)
    return _p(ring)


def verify_probs(q, p_old, draft, lo, init, img_pos0, hist, seed, counter, ring=None):
    q = _f32(q); p_old = _f32(p_old); draft = _i32(draft)
    L, V = p_old.shape
    assert q.shape == (L + 1, V)
    hist = _i32(hist if hist is not None else np.zeros(0))
    nd = np.empty(L, np.int32); pn = np.empty((L, V), np.float32)
    a = lib().orc_verify_probs(_p(q), _p(p_old), _p(draft), L, V, lo, C.byref(init), img_pos0, _p(hist), seed,
                               counter, _ring_arg(init, ring, V), _p(nd), _p(pn))
    return a, nd, pn


def verify(logits, p_old, draft, lo, sampler, init, img_pos0, hist, seed, counter, ring=None):
    logits = _f32(logits); p_old = _f32(p_old); draft = _i32(draft)
    L, V = p_old.shape
    assert logits.shape == (L, V)
    hist = _i32(hist if hist is not None else np.zeros(0))
    nd = np.empty(L, np.int32); pn = np.empty((L, V), np.float32)
    a = lib().orc_verify(_p(logits), _p(p_old), _p(draft), L, V, lo, C.byref(sampler), C.byref(init), img_pos0,
                         _p(hist), seed, counter, _ring_arg(init, ring, V), _p(nd), _p(pn))
    return a, nd, pn


def first_window(q_first, L, lo, init, seed):
    q_first = _f32(q_first); V = q_first.size
    d = np.empty(L, np.int32); p = np.empty((L, V), np.float32)
    lib().orc_first_window(_p(q_first), L, V, lo, C.byref(init), seed, _p(d), _p(p))
    return d, p


def config_from_shape(s) -> Config:
    return Config(s.n_layers, s.d_model, s.n_heads, s.d_ffn, s.vocab_total, s.samp_lo, s.samp_hi, s.max_seq,
                  s.dtype, s.rope_theta, s.rms_eps)


class Model:
    """Transformer oracle bound to a weight blob (kept alive here)."""

    def __init__(self, shape, blob: np.ndarray):
        self.shape = shape
        self.blob = np.ascontiguousarray(blob)
        self.cfg = config_from_shape(shape)
        self.h = lib().orc_model_create(C.byref(self.cfg), _p(self.blob))
        self.kv = lib().orc_kv_create(self.h)
        self.ctx = TfCtx(self.h, self.kv)

    def close(self):
        if self.h:
            lib().orc_kv_free(self.kv); lib().orc_model_free(self.h); self.h = None

    def __del__(self):
        self.close()

    def embed(self, ids):
        ids = _i32(ids); x = np.empty((ids.size, self.shape.d_model), np.float64)
        lib().orc_embed(self.h, _p(ids), ids.size, _p(x))
        return x

    def forward_full(self, x):
        x = np.ascontiguousarray(x, dtype=np.float64); T = x.shape[0]
        out = np.empty((T, self.shape.v_s), np.float32)
        lib().orc_forward_full(self.h, _p(x), T, _p(out))
        return out

    def kv_set_len(self, n):
        lib().orc_kv_set_len(self.kv, n)

    def forward_window(self, x):
        """rows at positions len..len+L-1; does not advance the length"""
        x = np.ascontiguousarray(x, dtype=np.float64); T = x.shape[0]
        out = np.empty((T, self.shape.v_s), np.float32)
        lib().orc_forward_window(self.h, self.kv, _p(x), T, _p(out))
        return out

    def forward_tokens(self, n_fixed, tokens):
        tokens = _i32(tokens); out = np.empty((tokens.size, self.shape.v_s), np.float32)
        lib().orc_tf_forward(C.byref(self.ctx), n_fixed, _p(tokens), tokens.size, _p(out))
        return out

    def prefill(self, ids, embeds=None):
        ids = _i32(ids)
        emb = _f32(embeds) if embeds is not None and len(embeds) else np.zeros((0, self.shape.d_model), np.float32)
        out = np.empty(self.shape.v_s, np.float32)
        lib().orc_tf_prefill(C.byref(self.ctx), _p(ids), ids.size, _p(emb), emb.shape[0], _p(out))
        return out

    def generate_sjd(self, n_prompt, logits_prompt, N, L, sampler, init, seed):
        lp = _f32(logits_prompt); out = np.empty(N, np.int32); st = Stats()
        fwd = C.cast(lib().orc_tf_forward, C.c_void_p)
        lib().orc_generate_sjd(fwd, C.byref(self.ctx), n_prompt, _p(lp), self.shape.v_s, self.shape.samp_lo, N, L,
                               C.byref(sampler), C.byref(init), seed, _p(out), C.byref(st))
        return out, st

    def generate_ar(self, n_prompt, logits_prompt, N, sampler, init, seed):
        lp = _f32(logits_prompt); out = np.empty(N, np.int32)
        fwd = C.cast(lib().orc_tf_forward, C.c_void_p)
        lib().orc_generate_ar(fwd, C.byref(self.ctx), n_prompt, _p(lp), self.shape.v_s, self.shape.samp_lo, N,
                              C.byref(sampler), C.byref(init), seed, _p(out))
        return out


def toy_histogram(table, V, depth, L, sampler, init, seed0, runs, use_ar=False):
    table = _f32(table)
    hist = np.zeros(V ** depth, np.int64); steps = C.c_int64(0)
    lib().orc_toy_histogram(_p(table), V, depth, L, C.byref(sampler), C.byref(init), seed0, runs, int(use_ar),
                            _p(hist), C.byref(steps))
    return hist, steps.value


def generate_sjd_callback(py_forward, n_prompt, logits_prompt, V, lo, N, L, sampler, init, seed):
    """SJD loop with a Python model callback py_forward(n_fixed, tokens[L]) -> logits [L, V]."""
    def _cb(_ctx, n_fixed, tok_p, Lc, out_p):
        toks = np.ctypeslib.as_array(tok_p, shape=(Lc,)).copy()
        lg = _f32(py_forward(n_fixed, toks))
        C.memmove(out_p, lg.ctypes.data, lg.nbytes)
    cb = FORWARD_FN(_cb)
    lp = _f32(logits_prompt); out = np.empty(N, np.int32); st = Stats()
    lib().orc_generate_sjd(C.cast(cb, C.c_void_p), None, n_prompt, _p(lp), V, lo, N, L, C.byref(sampler),
                           C.byref(init), seed, _p(out), C.byref(st))
    return out, st
