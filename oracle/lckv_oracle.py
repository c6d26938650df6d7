"""ctypes front end of ``lckv_oracle.c`` (the plain double-precision CPU oracle).

TEST INFRASTRUCTURE, not product code: only tests, the smoke check and the
benchmark's CPU-baseline leg may import it.  Argument marshalling only; every
number is computed by the C file, which follows Section 2.1 of the paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lckv_oracle.c")
_LIB = os.path.join(_HERE, "liblckv_oracle.so")

PAIR_TOP_OF_CONDENSED = 0  # rule 1 (default)
PAIR_LAST_LAYER = 1        # rule 2

_lib = None
_lib_path = None


def compile_c(src: str, out: str) -> str:
    """gcc line used for the oracle: plain -O2, OpenMP only over independent items."""
    subprocess.check_call(
        ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", out, src, "-lm"])
    return out


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_c(_SRC, _LIB)
    return _LIB


def use_library(path=None) -> None:
    """Point this module at another build of the oracle (the tests use this to check that planted
    mistakes are caught); ``None`` goes back to the real one."""
    global _lib, _lib_path
    _lib = None
    _lib_path = path


def _load():
    global _lib
    if _lib is None:
        if _lib_path is None:
            build()
        lib = ctypes.CDLL(_lib_path or _LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        i64p = ctypes.POINTER(ctypes.c_int64)
        lib.lckv_oracle_pairing.argtypes = [ctypes.c_int, u8p, ctypes.c_int, i32p, i32p, i32p, i32p]
        lib.lckv_oracle_pairing.restype = ctypes.c_int
        lib.lckv_oracle_attend.argtypes = [f32p, f32p, f32p, ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_int, ctypes.c_double, f64p, f64p]
        lib.lckv_oracle_attend.restype = None
        lib.lckv_oracle_attend_many.argtypes = [ctypes.c_int64, f32p, f32p, f32p, i64p, ctypes.c_int64,
                                                ctypes.c_int, ctypes.c_double, f64p, ctypes.c_int]
        lib.lckv_oracle_attend_many.restype = ctypes.c_int
        lib.lckv_oracle_step.argtypes = [ctypes.c_int] * 5 + [ctypes.c_int64, u8p, ctypes.c_int,
                                                              ctypes.c_double, f32p, f32p, i32p, f32p, f32p,
                                                              f32p, f64p, ctypes.c_int]
        lib.lckv_oracle_step.restype = ctypes.c_int
        lib.lckv_oracle_step_streaming.argtypes = [ctypes.c_int] * 5 + [
            ctypes.c_int64, u8p, ctypes.c_int, ctypes.c_double, f32p, f32p, i32p, f32p, f32p, f32p, f64p,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
        lib.lckv_oracle_step_streaming.restype = ctypes.c_int
        lib.lckv_oracle_prefill_attention.argtypes = [ctypes.c_int] * 4 + [
            ctypes.c_int64, ctypes.c_int64, f32p, f32p, i32p, ctypes.c_int, ctypes.c_double, f32p, f64p, ctypes.c_int]
        lib.lckv_oracle_prefill_attention.restype = ctypes.c_int
        lib.lckv_oracle_project.argtypes = [ctypes.c_int] * 4 + [f32p, f32p, i64p, ctypes.c_double, f64p]
        lib.lckv_oracle_project.restype = ctypes.c_int
        lib.lckv_oracle_footprint.argtypes = [ctypes.c_int, u8p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                              ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.lckv_oracle_footprint.restype = ctypes.c_int64
        lib.lckv_oracle_max_batch.argtypes = [ctypes.c_int, u8p, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                              ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64]
        lib.lckv_oracle_max_batch.restype = ctypes.c_int64
        lib.lckv_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def max_threads() -> int:
    return int(_load().lckv_oracle_max_threads())


def pairing(warm, rule: int = PAIR_TOP_OF_CONDENSED):
    """Return (kv_slot[L], self_visible[L], producer[n_slots]) as int32 arrays."""
    warm = np.ascontiguousarray(np.asarray(warm, dtype=np.uint8))
    L = warm.shape[0]
    kv_slot = np.zeros(L, np.int32)
    vis = np.zeros(L, np.int32)
    prod = np.zeros(L, np.int32)
    ns = ctypes.c_int32(0)
    rc = _load().lckv_oracle_pairing(L, _p(warm, ctypes.c_uint8), rule, _p(kv_slot, ctypes.c_int32),
                                     _p(vis, ctypes.c_int32), _p(prod, ctypes.c_int32), ctypes.byref(ns))
    if rc != 0:
        raise ValueError("lckv_oracle_pairing: bad argument")
    return kv_slot, vis, prod[: ns.value].copy()


def attend(q, K, V, scale: float, want_probs: bool = False):
    """One query [D] over keys K[n][D], values V[n][D]; returns out[D] (float64)."""
    q = _f32(q)
    D = q.shape[0]
    K = _f32(K).reshape(-1, D)
    V = _f32(V).reshape(-1, D)
    n = K.shape[0]
    assert V.shape[0] == n
    out = np.zeros(D, np.float64)
    probs = np.zeros(max(n, 1), np.float64) if want_probs else None
    _load().lckv_oracle_attend(_p(q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float), n, D, D,
                               float(scale), _p(out, ctypes.c_double),
                               _p(probs, ctypes.c_double) if want_probs else None)
    if want_probs:
        return out, probs[:n]
    return out


def attend_many(q, K, V, n_keys, scale: float, threads: int = 0):
    """Items i: q[i][D], K[i][T][D], V[i][T][D], n_keys[i] visible keys -> (out[i][D], threads used)."""
    q = _f32(q)
    N, D = q.shape
    K = _f32(K)
    V = _f32(V)
    T = K.shape[1]
    assert K.shape == (N, T, D) and V.shape == (N, T, D)
    n_keys = np.ascontiguousarray(n_keys, dtype=np.int64)
    assert n_keys.shape == (N,) and (n_keys <= T).all() and (n_keys >= 0).all()
    out = np.zeros((N, D), np.float64)
    used = _load().lckv_oracle_attend_many(N, _p(q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float),
                                           _p(n_keys, ctypes.c_int64), T, D, float(scale),
                                           _p(out, ctypes.c_double), threads)
    return out, int(used)


def step(warm, Kc, Vc, lens, q, k_new, v_new, scale: float, rule: int = PAIR_TOP_OF_CONDENSED,
         threads: int = 0, sink: int = 0, window: int = 0):
    """One decode step.

    Kc, Vc: float32 [n_slots][B][T_cap][Hkv][D], C-contiguous, UPDATED IN PLACE (the new token is
    appended); lens: int32 [B], UPDATED IN PLACE (+1); q: [L][B][Hq][D]; k_new, v_new:
    [n_slots][B][Hkv][D] in slot order.  Returns (out float64 [L][B][Hq][D], threads used).
    window > 0: sink + window policy (Section 3.3): only the first `sink` and the last `window` of a query's
    candidate positions are attended to; Kc, Vc still hold the whole history.
    """
    warm = np.ascontiguousarray(np.asarray(warm, dtype=np.uint8))
    L = warm.shape[0]
    for a in (Kc, Vc):
        assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"] and a.ndim == 5
    assert lens.dtype == np.int32 and lens.flags["C_CONTIGUOUS"]
    n_slots, B, T_cap, Hkv, D = Kc.shape
    assert Vc.shape == Kc.shape and lens.shape == (B,)
    q = _f32(q)
    Hq = q.shape[2]
    assert q.shape == (L, B, Hq, D)
    k_new = _f32(k_new, (n_slots, B, Hkv, D))
    v_new = _f32(v_new, (n_slots, B, Hkv, D))
    _, _, prod = pairing(warm, rule)
    assert len(prod) == n_slots, "cache has %d slots, pairing needs %d" % (n_slots, len(prod))
    out = np.zeros((L, B, Hq, D), np.float64)
    args = (L, Hq, Hkv, D, B, T_cap, _p(warm, ctypes.c_uint8), rule, float(scale),
            _p(Kc, ctypes.c_float), _p(Vc, ctypes.c_float), _p(lens, ctypes.c_int32),
            _p(q, ctypes.c_float), _p(k_new, ctypes.c_float), _p(v_new, ctypes.c_float), _p(out, ctypes.c_double))
    if window > 0 or sink > 0:
        rc = _load().lckv_oracle_step_streaming(*args, int(sink), int(window), threads)
    else:
        rc = _load().lckv_oracle_step(*args, threads)
    if rc < 0:
        raise ValueError("lckv_oracle_step failed with code %d" % rc)
    return out, int(rc)


def prefill_attention(Kc, Vc, lens, q, self_visible: bool, scale: float, threads: int = 0):
    """All prompt tokens of one layer at once (Sections 2.2 and 2.3): token i attends to positions j < i of the
    slot (condensed layer) or j <= i (warmup layer).  Kc, Vc: one slot, float32 [B][T_cap][Hkv][D];
    lens: int32 [B] prompt lengths; q: [B][S][Hq][D].  Returns (out float64 [B][S][Hq][D], threads used)."""
    Kc, Vc = _f32(Kc), _f32(Vc)
    B, T_cap, Hkv, D = Kc.shape
    assert Vc.shape == Kc.shape
    q = _f32(q)
    S, Hq = q.shape[1], q.shape[2]
    assert q.shape == (B, S, Hq, D)
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    out = np.zeros((B, S, Hq, D), np.float64)
    rc = _load().lckv_oracle_prefill_attention(Hq, Hkv, D, B, S, T_cap, _p(Kc, ctypes.c_float), _p(Vc, ctypes.c_float),
                                               _p(lens, ctypes.c_int32), int(bool(self_visible)), float(scale),
                                               _p(q, ctypes.c_float), _p(out, ctypes.c_double), threads)
    if rc < 0:
        raise ValueError("lckv_oracle_prefill_attention: bad argument")
    return out, int(rc)


def project(x, W, n_heads: int, pos=None, rope_base: float = 10000.0):
    """One projection either side of the attention (Section 2.1): y = x W^T with W [n_heads*D][hidden], then, when
    `pos` (int [B]) is given, the rotary position embedding per head (queries and keys; never values).
    Returns float64 [B][n_heads][D]."""
    x, W = _f32(x), _f32(W)
    B, hidden = x.shape
    N = W.shape[0]
    assert W.shape == (N, hidden) and N % n_heads == 0
    D = N // n_heads
    out = np.zeros((B, N), np.float64)
    if pos is not None:
        pos = np.ascontiguousarray(pos, dtype=np.int64)
        assert pos.shape == (B,)
    rc = _load().lckv_oracle_project(B, hidden, n_heads, D, _p(x, ctypes.c_float), _p(W, ctypes.c_float),
                                     _p(pos, ctypes.c_int64) if pos is not None else None, float(rope_base),
                                     _p(out, ctypes.c_double))
    if rc < 0:
        raise ValueError("lckv_oracle_project: bad argument")
    return out.reshape(B, n_heads, D)


def footprint(warm, B: int, T: int, Hkv: int, D: int, elem_bytes: int, rule: int = PAIR_TOP_OF_CONDENSED) -> int:
    """Bytes of KV cache for B sequences of T positions: every cache the pairing table names keeps K and V of
    Hkv heads of D elements per position (Sections 1, 2.1)."""
    warm = np.ascontiguousarray(np.asarray(warm, dtype=np.uint8))
    n = _load().lckv_oracle_footprint(warm.shape[0], _p(warm, ctypes.c_uint8), rule, B, T, Hkv, D, elem_bytes)
    if n < 0:
        raise ValueError("lckv_oracle_footprint: bad argument")
    return int(n)


def max_batch(warm, T: int, Hkv: int, D: int, elem_bytes: int, budget: int, limit: int = 65535,
              rule: int = PAIR_TOP_OF_CONDENSED) -> int:
    """Largest batch (at most `limit`) whose caches fit in `budget` bytes (Section 3.1)."""
    warm = np.ascontiguousarray(np.asarray(warm, dtype=np.uint8))
    n = _load().lckv_oracle_max_batch(warm.shape[0], _p(warm, ctypes.c_uint8), rule, T, Hkv, D, elem_bytes, budget,
                                      limit)
    if n < 0:
        raise ValueError("lckv_oracle_max_batch: bad argument")
    return int(n)
