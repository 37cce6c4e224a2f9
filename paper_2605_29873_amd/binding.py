"""ctypes binding over the C ABI of include/mkv.h.

Argument marshalling only: every step of the decode path runs in the HIP kernels of libmkv.so.
There is no fallback: if the library has not been built, load() raises.
Device pointers are passed as integers (e.g. torch.Tensor.data_ptr()).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_LIB = None
LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmkv.so")

MKV_F32, MKV_BF16 = 0, 1
MKV_SCORE_LAYER_MEAN, MKV_SCORE_PER_KV_HEAD = 0, 1
MKV_OK, MKV_ERR_ARG, MKV_ERR_STATE, MKV_ERR_FROZEN = 0, -1, -2, -3
MKV_ERR_CAPACITY, MKV_ERR_NOMEM, MKV_ERR_HIP = -4, -5, -6
MKV_NEVER_EVICT = 2**31 - 1

EXPORTS = ["mkv_required_bytes", "mkv_create", "mkv_destroy", "mkv_prefill_append", "mkv_prefill_compress", "mkv_project_append",
           "mkv_decode_step", "mkv_decode_step_static", "mkv_decode_step_multi", "mkv_evict", "mkv_read_scores", "mkv_write_scores",
           "mkv_load_decode", "mkv_read_kv", "mkv_read_probs", "mkv_read_slots", "mkv_set_score_view", "mkv_get_lens", "mkv_set_profiling",
           "mkv_read_profile", "mkv_last_error"]


class mkv_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("dtype", C.c_int32),
                ("max_prefill", C.c_int32), ("decode_budget", C.c_int32),
                ("evict_trigger", C.c_int32), ("decode_capacity", C.c_int32),
                ("recent_window", C.c_int32), ("alpha", C.c_float), ("softmax_scale", C.c_float),
                ("score_mode", C.c_int32), ("split_keys", C.c_int32), ("attn_variant", C.c_int32),
                ("groups_per_cu", C.c_int32), ("max_q_len", C.c_int32),
                ("stream", C.c_void_p),
                ("arena", C.c_void_p), ("arena_bytes", C.c_size_t)]


class MkvError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"mkv error {code}: {message}")
        self.code = code


def load() -> C.CDLL:
    """Loads libmkv.so (built by __graft_entry__.build()); raises if it is missing."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; "
                           "g.build()'` first; there is no fallback path")
    # torch first: the process must end up with ONE HIP runtime, the one torch brings, because the
    # device memory and streams handed to the library come from torch
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    lib.mkv_required_bytes.restype = C.c_size_t
    lib.mkv_required_bytes.argtypes = [C.POINTER(mkv_config)]
    lib.mkv_create.argtypes = [C.POINTER(mkv_config), C.POINTER(vp)]
    lib.mkv_destroy.argtypes = [vp]
    lib.mkv_prefill_append.argtypes = [vp, i32, i32, vp, vp, i32]
    lib.mkv_prefill_compress.argtypes = [vp, i32, i32, vp, i32]
    lib.mkv_project_append.argtypes = [vp, i32, vp, vp, vp, i32, vp, C.c_float, vp]
    lib.mkv_decode_step.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.mkv_decode_step_static.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.mkv_decode_step_multi.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
    lib.mkv_evict.argtypes = [vp, i32, i32]
    lib.mkv_read_scores.argtypes = [vp, i32, i32, vp, vp, i32, C.POINTER(i32)]
    lib.mkv_write_scores.argtypes = [vp, i32, i32, vp, i32]
    lib.mkv_load_decode.argtypes = [vp, i32, i32, vp, vp, vp, vp, i32, i64]
    lib.mkv_read_kv.argtypes = [vp, i32, i32, i32, i32, vp, vp, i32, C.POINTER(i32)]
    lib.mkv_read_probs.argtypes = [vp, i32, i32, vp, vp, i32, C.POINTER(i32)]
    lib.mkv_read_slots.argtypes = [vp, i32, i32, vp, vp, vp, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.mkv_set_score_view.argtypes = [vp, i32]
    lib.mkv_get_lens.argtypes = [vp, i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i64)]
    lib.mkv_set_profiling.argtypes = [vp, i32]
    lib.mkv_read_profile.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.mkv_last_error.restype = C.c_char_p
    lib.mkv_last_error.argtypes = [vp]
    for name in EXPORTS:
        if name not in ("mkv_required_bytes", "mkv_last_error"):
            getattr(lib, name).restype = C.c_int
    _LIB = lib
    return lib


def _check(ctx, rc: int) -> None:
    if rc != MKV_OK:
        raise MkvError(rc, (load().mkv_last_error(ctx) or b"").decode())


def make_config(**kw) -> mkv_config:
    cfg = mkv_config()
    for k, v in kw.items():
        if not hasattr(cfg, k):
            raise TypeError(f"unknown mkv_config field {k}")
        setattr(cfg, k, v)
    return cfg


def mkv_required_bytes(cfg: mkv_config) -> int:
    return int(load().mkv_required_bytes(C.byref(cfg)))


def mkv_create(cfg: mkv_config) -> int:
    out = C.c_void_p()
    _check(None, load().mkv_create(C.byref(cfg), C.byref(out)))
    return out.value


def mkv_destroy(ctx: int) -> None:
    _check(None, load().mkv_destroy(ctx))


def mkv_prefill_append(ctx, layer, seq, k_ptr, v_ptr, n_tokens) -> None:
    _check(ctx, load().mkv_prefill_append(ctx, layer, seq, k_ptr, v_ptr, n_tokens))


def mkv_prefill_compress(ctx, layer, seq, scores_ptr, keep) -> None:
    _check(ctx, load().mkv_prefill_compress(ctx, layer, seq, scores_ptr, keep))


def mkv_project_append(ctx, layer, x_ptr, wk_ptr, wv_ptr, hidden, rope_pos_ptr, rope_theta, seq_mask=None) -> None:
    mp = None
    if seq_mask is not None:
        seq_mask = np.ascontiguousarray(seq_mask, dtype=np.uint8)
        mp = seq_mask.ctypes.data
    _check(ctx, load().mkv_project_append(ctx, layer, x_ptr, wk_ptr, wv_ptr, hidden, rope_pos_ptr,
                                          rope_theta, mp))


def mkv_decode_step(ctx, layer, q_ptr, k_ptr, v_ptr, out_ptr, seq_mask=None) -> None:
    mp = None
    if seq_mask is not None:
        seq_mask = np.ascontiguousarray(seq_mask, dtype=np.uint8)
        mp = seq_mask.ctypes.data
    _check(ctx, load().mkv_decode_step(ctx, layer, q_ptr, k_ptr, v_ptr, out_ptr, mp))


def mkv_decode_step_static(ctx, layer, q_ptr, k_ptr, v_ptr, out_ptr, seq_mask=None) -> None:
    mp = None
    if seq_mask is not None:
        seq_mask = np.ascontiguousarray(seq_mask, dtype=np.uint8)
        mp = seq_mask.ctypes.data
    _check(ctx, load().mkv_decode_step_static(ctx, layer, q_ptr, k_ptr, v_ptr, out_ptr, mp))


def mkv_decode_step_multi(ctx, layer, q_len, q_ptr, k_ptr, v_ptr, out_ptr, seq_mask=None) -> None:
    mp = None
    if seq_mask is not None:
        seq_mask = np.ascontiguousarray(seq_mask, dtype=np.uint8)
        mp = seq_mask.ctypes.data
    _check(ctx, load().mkv_decode_step_multi(ctx, layer, q_len, q_ptr, k_ptr, v_ptr, out_ptr, mp))


def mkv_evict(ctx, layer, seq=-1) -> None:
    _check(ctx, load().mkv_evict(ctx, layer, seq))


def mkv_get_lens(ctx, layer, seq):
    m, n, t = C.c_int(), C.c_int(), C.c_int64()
    _check(ctx, load().mkv_get_lens(ctx, layer, seq, C.byref(m), C.byref(n), C.byref(t)))
    return m.value, n.value, t.value


def mkv_read_scores(ctx, layer, seq):
    """Returns (scores float32[n], positions int32[n])."""
    _, cap, _ = mkv_get_lens(ctx, layer, seq)
    s = np.empty(max(cap, 1), dtype=np.float32)
    p = np.empty(max(cap, 1), dtype=np.int32)
    n = C.c_int()
    _check(ctx, load().mkv_read_scores(ctx, layer, seq, s.ctypes.data, p.ctypes.data, s.size, C.byref(n)))
    return s[:n.value].copy(), p[:n.value].copy()


def mkv_write_scores(ctx, layer, seq, scores) -> None:
    s = np.ascontiguousarray(scores, dtype=np.float32)
    _check(ctx, load().mkv_write_scores(ctx, layer, seq, s.ctypes.data, s.size))


def mkv_load_decode(ctx, layer, seq, k_ptr, v_ptr, scores, positions, next_step) -> None:
    s = np.ascontiguousarray(scores, dtype=np.float32)
    p = np.ascontiguousarray(positions, dtype=np.int32)
    assert s.size == p.size
    _check(ctx, load().mkv_load_decode(ctx, layer, seq, k_ptr, v_ptr, s.ctypes.data, p.ctypes.data,
                                       s.size, next_step))


def mkv_read_kv(ctx, layer, seq, pool, kv_head, head_dim, dtype):
    """Returns (K, V) of one KV head as arrays [n, head_dim]: float32, or uint16 bf16 patterns."""
    m, n_d, _ = mkv_get_lens(ctx, layer, seq)
    n = m if pool else n_d
    np_dtype = np.uint16 if dtype == MKV_BF16 else np.float32
    k = np.empty((max(n, 1), head_dim), dtype=np_dtype)
    v = np.empty((max(n, 1), head_dim), dtype=np_dtype)
    got = C.c_int()
    _check(ctx, load().mkv_read_kv(ctx, layer, seq, pool, kv_head, k.ctypes.data, v.ctypes.data,
                                   k.shape[0], C.byref(got)))
    return k[:got.value].copy(), v[:got.value].copy()


def mkv_read_probs(ctx, layer, seq, n_q_heads, capacity):
    """Returns (abar float32[n], lse float32[H]) of the last decode step of `layer`."""
    a = np.empty(max(capacity, 1), dtype=np.float32)
    lse = np.empty(n_q_heads, dtype=np.float32)
    n = C.c_int()
    _check(ctx, load().mkv_read_probs(ctx, layer, seq, a.ctypes.data, lse.ctypes.data, a.size, C.byref(n)))
    return a[:n.value].copy(), lse


def mkv_read_slots(ctx, layer, seq, capacity):
    """Returns (scores float32[n], positions int32[n], live bool[n], pending slot or -1) slot by slot."""
    s = np.empty(max(capacity, 1), dtype=np.float32)
    p = np.empty(max(capacity, 1), dtype=np.int32)
    lv = np.empty(max(capacity, 1), dtype=np.uint8)
    n, pend = C.c_int(), C.c_int()
    _check(ctx, load().mkv_read_slots(ctx, layer, seq, s.ctypes.data, p.ctypes.data, lv.ctypes.data, s.size,
                                      C.byref(n), C.byref(pend)))
    return s[:n.value].copy(), p[:n.value].copy(), lv[:n.value].astype(bool), pend.value


def mkv_set_score_view(ctx, kv_head: int) -> None:
    _check(ctx, load().mkv_set_score_view(ctx, kv_head))


def mkv_set_profiling(ctx, enable: bool) -> None:
    _check(ctx, load().mkv_set_profiling(ctx, int(bool(enable))))


def mkv_read_profile(ctx):
    """Returns ({'attn_us','finish_us','evict_us'} sums, steps, steps_that_evicted)."""
    us = (C.c_double * 3)()
    cnt = (C.c_int64 * 2)()
    _check(ctx, load().mkv_read_profile(ctx, us, cnt))
    return {"attn_us": us[0], "finish_us": us[1], "evict_us": us[2]}, cnt[0], cnt[1]


def mkv_last_error(ctx=None) -> str:
    return (load().mkv_last_error(ctx) or b"").decode()
