"""ctypes binding of the SJD HIP library: same names as include/sjd.h, argument marshalling only.

Device buffers are torch tensors (torch is used for device memory and streams, nothing else);
host buffers are numpy arrays.  Every step of the path runs inside the library's kernels.
Importing this module raises if the library has not been built: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsjd_hip.so")

SJD_OK, SJD_EINVAL, SJD_ENOMEM, SJD_ESEQ, SJD_EHIP, SJD_ELIMIT = 0, -1, -2, -3, -4, -5
SJD_STATIC_VERIFY_FLOATS = 17 * 16384
SJD_MAX_WINDOW = 64
SJD_MAX_ROWS = 128          # rows one forward computes (window x contexts x images)
SJD_MAX_SAMP_VOCAB = 32768

EXPORTS = ["sjd_init_model", "sjd_free_model", "sjd_kv_create", "sjd_kv_free", "sjd_kv_reset", "sjd_kv_len",
           "sjd_kv_set_len", "sjd_prefill", "sjd_first_window", "sjd_step", "sjd_generate", "sjd_forward_logits",
           "sjd_verify", "sjd_verify_probs", "sjd_dist", "sjd_gemm_test", "sjd_strerror", "sjd_decode_begin",
           "sjd_decode_steps", "sjd_decode_status", "sjd_decode_result", "sjd_kv_use_graph", "sjd_profile_steps", "sjd_gemm_bench",
           "sjd_prefill_uncond", "sjd_generate_cfg", "sjd_decode_steps_batch", "sjd_forward_logits_batch",
           "sjd_generate_batch", "sjd_profile_steps_batch", "sjd_verify_static"]

PROF_KINDS = ("gemm", "attention", "elementwise", "verify")


class sjd_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "d_ffn", "vocab_total", "samp_lo",
                                          "samp_hi", "max_seq", "dtype")] + [("rope_theta", C.c_float),
                                                                             ("rms_eps", C.c_float)]


class sjd_sampler(C.Structure):
    _fields_ = [("top_k", C.c_int32), ("temperature", C.c_float)]


class sjd_init(C.Structure):
    _fields_ = [("mode", C.c_int32), ("row_stride", C.c_int32), ("eol_id", C.c_int32), ("flags", C.c_int32)]


class sjd_stats(C.Structure):
    _fields_ = [("steps", C.c_int32), ("accept_hist", C.c_int32 * 65), ("ms_prefill", C.c_float),
                ("ms_decode", C.c_float)]


class sjd_profile(C.Structure):
    _fields_ = [("ms", C.c_double * 4), ("bytes", C.c_double * 4), ("launches", C.c_int64 * 4), ("steps", C.c_int32),
                ("ms_gemm_back_to_back", C.c_double)]


class SjdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"sjd error {code}: {msg}")
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2410_01699_amd.build` "
                      "(there is no CPU fallback)")
_lib = C.CDLL(LIB_PATH)

_vp, _i32, _u64, _sz = C.c_void_p, C.c_int32, C.c_uint64, C.c_size_t
_P = C.POINTER
_SIG = {
    "sjd_init_model": (C.c_int, [_P(sjd_config), _vp, _sz, _P(_vp)]),
    "sjd_free_model": (None, [_vp]),
    "sjd_kv_create": (C.c_int, [_vp, _P(_vp)]),
    "sjd_kv_free": (None, [_vp]),
    "sjd_kv_reset": (C.c_int, [_vp]),
    "sjd_kv_len": (C.c_int, [_vp, _P(_i32)]),
    "sjd_kv_set_len": (C.c_int, [_vp, _i32]),
    "sjd_prefill": (C.c_int, [_vp, _vp, _vp, _i32, _vp, _i32, _P(sjd_sampler), _P(sjd_init), _vp, _vp]),
    "sjd_prefill_uncond": (C.c_int, [_vp, _vp, _vp, _i32, _vp, _i32, C.c_float, _P(sjd_sampler), _P(sjd_init), _vp, _vp]),
    "sjd_generate_cfg": (C.c_int, [_vp, _vp, _vp, _i32, _vp, _i32, _vp, _i32, _vp, _i32, C.c_float, _i32, _i32,
                                   _P(sjd_sampler), _P(sjd_init), _u64, _vp, _P(sjd_stats)]),
    "sjd_first_window": (C.c_int, [_vp, _vp, _i32, _P(sjd_init), _u64, _vp, _vp, _vp]),
    "sjd_step": (C.c_int, [_vp, _vp, _vp, _vp, _i32, _P(sjd_sampler), _P(sjd_init), _i32, _u64, _u64, _vp, _vp, _vp,
                           _vp]),
    "sjd_generate": (C.c_int, [_vp, _vp, _vp, _i32, _vp, _i32, _i32, _i32, _P(sjd_sampler), _P(sjd_init), _u64, _vp,
                               _P(sjd_stats)]),
    "sjd_forward_logits": (C.c_int, [_vp, _vp, _vp, _i32, _vp, _vp]),
    "sjd_forward_logits_batch": (C.c_int, [_vp, _vp, _i32, _vp, _i32, _vp, _vp]),
    "sjd_decode_steps_batch": (C.c_int, [_vp, _vp, _i32, _i32, _vp]),
    "sjd_profile_steps_batch": (C.c_int, [_vp, _vp, _i32, _i32, _P(sjd_profile), _vp]),
    "sjd_generate_batch": (C.c_int, [_vp, _vp, _i32, _vp, _vp, _vp, _vp, _i32, _i32, _P(sjd_sampler), _P(sjd_init), _vp,
                                     _vp, _vp]),
    "sjd_verify": (C.c_int, [_vp, _vp, _vp, _i32, _i32, _i32, _P(sjd_sampler), _P(sjd_init), _i32, _vp, _vp, _u64, _u64,
                             _vp, _vp, _vp, _vp]),
    "sjd_verify_static": (C.c_int, [_vp, _vp, _vp, _i32, _i32, _i32, _P(sjd_sampler), _P(sjd_init), _i32, _vp, _vp, _u64, _u64,
                                    _vp, _vp, _vp, _vp]),
    "sjd_verify_probs": (C.c_int, [_vp, _vp, _vp, _i32, _i32, _i32, _P(sjd_init), _i32, _vp, _vp, _u64, _u64, _vp, _vp,
                                   _vp, _vp]),
    "sjd_dist": (C.c_int, [_vp, _i32, _i32, _P(sjd_sampler), _vp, _vp, _vp]),
    "sjd_gemm_test": (C.c_int, [_i32, _vp, _vp, _i32, _i32, _i32, _vp, _vp]),
    "sjd_strerror": (C.c_char_p, [C.c_int]),
    "sjd_decode_begin": (C.c_int, [_vp, _vp, _vp, _i32, _i32, _P(sjd_sampler), _P(sjd_init), _u64, _vp]),
    "sjd_decode_steps": (C.c_int, [_vp, _vp, _i32, _vp]),
    "sjd_decode_status": (C.c_int, [_vp, _P(_i32), _P(_i32), _P(_i32)]),
    "sjd_decode_result": (C.c_int, [_vp, _vp, _P(sjd_stats)]),
    "sjd_kv_use_graph": (C.c_int, [_vp, _i32]),
    "sjd_profile_steps": (C.c_int, [_vp, _vp, _i32, _P(sjd_profile), _vp]),
    "sjd_gemm_bench": (C.c_int, [_i32, _i32, _i32, _i32, _i32, _i32, _i32, _P(C.c_float)]),
}
for _name, (_res, _args) in _SIG.items():
    _fn = getattr(_lib, _name)
    _fn.restype, _fn.argtypes = _res, _args


def sjd_strerror(code: int) -> str:
    return _lib.sjd_strerror(code).decode()


def _check(rc):
    if rc != SJD_OK:
        raise SjdError(rc, sjd_strerror(rc))


def _dev(t):
    """device address of a torch tensor (None -> NULL)"""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device buffers must be contiguous GPU tensors"
    return C.c_void_p(t.data_ptr())


def _host(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _stream(stream):
    if stream is None:
        return None
    return C.c_void_p(stream.cuda_stream)


def config_from_shape(s) -> sjd_config:
    return sjd_config(s.n_layers, s.d_model, s.n_heads, s.d_ffn, s.vocab_total, s.samp_lo, s.samp_hi, s.max_seq,
                      s.dtype, s.rope_theta, s.rms_eps)


def sjd_init_model(cfg: sjd_config, host_weights: np.ndarray):
    host_weights = np.ascontiguousarray(host_weights)
    out = _vp()
    _check(_lib.sjd_init_model(C.byref(cfg), _host(host_weights), host_weights.nbytes, C.byref(out)))
    return out


def sjd_free_model(m):
    _lib.sjd_free_model(m)


def sjd_kv_create(m):
    out = _vp()
    _check(_lib.sjd_kv_create(m, C.byref(out)))
    return out


def sjd_kv_free(kv):
    _lib.sjd_kv_free(kv)


def sjd_kv_reset(kv):
    _check(_lib.sjd_kv_reset(kv))


def sjd_kv_len(kv) -> int:
    n = _i32(0)
    _check(_lib.sjd_kv_len(kv, C.byref(n)))
    return n.value


def sjd_kv_set_len(kv, n: int):
    _check(_lib.sjd_kv_set_len(kv, n))


def _ids_embeds(ids, embeds):
    ids = None if ids is None or len(ids) == 0 else np.ascontiguousarray(ids, dtype=np.int32)
    embeds = None if embeds is None or len(embeds) == 0 else np.ascontiguousarray(embeds, dtype=np.float32)
    return ids, (0 if ids is None else ids.size), embeds, (0 if embeds is None else embeds.shape[0])


def sjd_prefill(m, kv, ids, embeds, smp: sjd_sampler, init: sjd_init, q_last, stream=None):
    ids, n_ids, embeds, n_emb = _ids_embeds(ids, embeds)
    _check(_lib.sjd_prefill(m, kv, _host(ids), n_ids, _host(embeds), n_emb, C.byref(smp), C.byref(init), _dev(q_last),
                            _stream(stream)))


def sjd_prefill_uncond(m, kv, ids, embeds, guidance: float, smp: sjd_sampler, init: sjd_init, q_last, stream=None):
    ids, n_ids, embeds, n_emb = _ids_embeds(ids, embeds)
    _check(_lib.sjd_prefill_uncond(m, kv, _host(ids), n_ids, _host(embeds), n_emb, guidance, C.byref(smp), C.byref(init),
                                   _dev(q_last), _stream(stream)))


def sjd_generate_cfg(m, kv, ids, embeds, uncond_ids, uncond_embeds, guidance, N, L, smp, init, seed):
    ids, n_ids, embeds, n_emb = _ids_embeds(ids, embeds)
    u_ids, n_u_ids, u_embeds, n_u_emb = _ids_embeds(uncond_ids, uncond_embeds)
    out = np.empty(N, np.int32)
    st = sjd_stats()
    _check(_lib.sjd_generate_cfg(m, kv, _host(ids), n_ids, _host(embeds), n_emb, _host(u_ids), n_u_ids, _host(u_embeds),
                                 n_u_emb, guidance, N, L, C.byref(smp), C.byref(init), seed, _host(out), C.byref(st)))
    return out, st


def sjd_first_window(m, q_first, L, init: sjd_init, seed, draft, p_old, stream=None):
    _check(_lib.sjd_first_window(m, _dev(q_first), L, C.byref(init), seed, _dev(draft), _dev(p_old), _stream(stream)))


def sjd_step(m, kv, draft, p_old, L, smp, init, img_pos0, seed, counter, n_accepted, new_draft, p_new, stream=None):
    _check(_lib.sjd_step(m, kv, _dev(draft), _dev(p_old), L, C.byref(smp), C.byref(init), img_pos0, seed, counter,
                         _dev(n_accepted), _dev(new_draft), _dev(p_new), _stream(stream)))


def sjd_generate(m, kv, ids, embeds, N, L, smp, init, seed):
    ids, n_ids, embeds, n_emb = _ids_embeds(ids, embeds)
    out = np.empty(N, np.int32)
    st = sjd_stats()
    _check(_lib.sjd_generate(m, kv, _host(ids), n_ids, _host(embeds), n_emb, N, L, C.byref(smp), C.byref(init), seed,
                             _host(out), C.byref(st)))
    return out, st


def _handles(kvs):
    """host array of cache handles"""
    return (C.c_void_p * len(kvs))(*[kv.value for kv in kvs])


def sjd_decode_steps_batch(m, kvs, n_steps, stream=None):
    _check(_lib.sjd_decode_steps_batch(m, _handles(kvs), len(kvs), n_steps, _stream(stream)))


def sjd_forward_logits_batch(m, kvs, tokens, L, logits, stream=None):
    """tokens: device int32 [B, L]; logits: device fp32 [B, L, V_s]"""
    _check(_lib.sjd_forward_logits_batch(m, _handles(kvs), len(kvs), _dev(tokens), L, _dev(logits), _stream(stream)))


def sjd_generate_batch(m, kvs, ids_list, embeds_list, N, L, smp, init, seeds):
    """ids_list / embeds_list: one prompt per handle (embeds_list may be None); returns tokens [B, N], stats list"""
    B = len(kvs)
    prm = [_ids_embeds(ids_list[b], None if embeds_list is None else embeds_list[b]) for b in range(B)]
    idp = (C.c_void_p * B)(*[None if p[0] is None else p[0].ctypes.data for p in prm])
    nid = (C.c_int32 * B)(*[p[1] for p in prm])
    emp = (C.c_void_p * B)(*[None if p[2] is None else p[2].ctypes.data for p in prm])
    nem = (C.c_int32 * B)(*[p[3] for p in prm])
    sd = (C.c_uint64 * B)(*[int(x) for x in seeds])
    out = np.empty((B, N), np.int32)
    st = (sjd_stats * B)()
    _check(_lib.sjd_generate_batch(m, _handles(kvs), B, idp, nid, emp, nem, N, L, C.byref(smp), C.byref(init), sd,
                                   _host(out), st))
    return out, list(st)


def sjd_forward_logits(m, kv, tokens, L, logits, stream=None):
    _check(_lib.sjd_forward_logits(m, kv, _dev(tokens), L, _dev(logits), _stream(stream)))


def sjd_verify(logits, p_old, draft, L, V_s, samp_lo, smp, init, img_pos0, hist, seed, counter, n_accepted, new_draft,
               p_new, stream=None, ring=None):
    _check(_lib.sjd_verify(_dev(logits), _dev(p_old), _dev(draft), L, V_s, samp_lo, C.byref(smp), C.byref(init),
                           img_pos0, _dev(hist), _dev(ring), seed, counter, _dev(n_accepted), _dev(new_draft),
                           _dev(p_new), _stream(stream)))


def sjd_verify_static(logits, p_old, draft, L, V_s, samp_lo, smp, init, img_pos0, hist, seed, counter, n_accepted,
                      new_draft, p_new, stream=None, ring=None):
    _check(_lib.sjd_verify_static(_dev(logits), _dev(p_old), _dev(draft), L, V_s, samp_lo, C.byref(smp), C.byref(init),
                                  img_pos0, _dev(hist), _dev(ring), seed, counter, _dev(n_accepted), _dev(new_draft),
                                  _dev(p_new), _stream(stream)))


def sjd_verify_probs(q, p_old, draft, L, V_s, samp_lo, init, img_pos0, hist, seed, counter, n_accepted, new_draft,
                     p_new, stream=None, ring=None):
    _check(_lib.sjd_verify_probs(_dev(q), _dev(p_old), _dev(draft), L, V_s, samp_lo, C.byref(init), img_pos0,
                                 _dev(hist), _dev(ring), seed, counter, _dev(n_accepted), _dev(new_draft), _dev(p_new),
                                 _stream(stream)))


def sjd_dist(logits, rows, V_s, smp, forced, q, stream=None):
    _check(_lib.sjd_dist(_dev(logits), rows, V_s, C.byref(smp), _dev(forced), _dev(q), _stream(stream)))


def sjd_gemm_test(dtype, A, W, M, N, K, Cout, stream=None):
    _check(_lib.sjd_gemm_test(dtype, _dev(A), _dev(W), M, N, K, _dev(Cout), _stream(stream)))


def sjd_decode_begin(m, kv, q_first, N, L, smp, init, seed, stream=None):
    _check(_lib.sjd_decode_begin(m, kv, _dev(q_first), N, L, C.byref(smp), C.byref(init), seed, _stream(stream)))


def sjd_decode_steps(m, kv, n_steps, stream=None):
    _check(_lib.sjd_decode_steps(m, kv, n_steps, _stream(stream)))


def sjd_decode_status(kv):
    """-> (image tokens fixed, iterations run, done)"""
    a, b, c = _i32(0), _i32(0), _i32(0)
    _check(_lib.sjd_decode_status(kv, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, bool(c.value)


def sjd_decode_result(kv, N):
    out = np.empty(N, np.int32)
    st = sjd_stats()
    _check(_lib.sjd_decode_result(kv, _host(out), C.byref(st)))
    return out, st


def sjd_kv_use_graph(kv, on: bool):
    _check(_lib.sjd_kv_use_graph(kv, int(on)))


def sjd_profile_steps(m, kv, n_steps, stream=None) -> sjd_profile:
    p = sjd_profile()
    _check(_lib.sjd_profile_steps(m, kv, n_steps, C.byref(p), _stream(stream)))
    return p


def sjd_profile_steps_batch(m, kvs, n_steps, stream=None) -> sjd_profile:
    p = sjd_profile()
    _check(_lib.sjd_profile_steps_batch(m, _handles(kvs), len(kvs), n_steps, C.byref(p), _stream(stream)))
    return p


def sjd_gemm_bench(M, N, K, tn, wk, u, iters=50) -> float:
    """microseconds per launch of the bf16 projection kernel at this shape and tiling"""
    us = C.c_float(0)
    _check(_lib.sjd_gemm_bench(M, N, K, tn, wk, u, iters, C.byref(us)))
    return us.value
