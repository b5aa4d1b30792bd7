"""ctypes loader for the C oracle (TEST INFRASTRUCTURE ONLY; see nats_oracle_c.c).

`build()` compiles oracle/nats_oracle_c.c with gcc; `fwd()` / `decode()` marshal
numpy arrays.  No arithmetic of the method lives here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nats_oracle_c.c")
_LIB = os.path.join(_HERE, "libnats_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.nats_oracle_threads.restype = ctypes.c_int
        _lib.nats_oracle_fwd.restype = ctypes.c_int
        _lib.nats_oracle_decode.restype = ctypes.c_int
        _lib.nats_oracle_fwd_chunk.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().nats_oracle_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def fwd(Q, K, V, alpha, beta, mask, softmax_scale=None, la_scale=1.0, mode=0, w_nla=None, w_la=None,
        eps=1e-6, S0=None, chunk_routing=0, want=("O", "O_la", "O_nla", "lse", "S", "cnt", "idx", "n_s"),
        linear_op=0, freeze_on_softmax=0):
    """Inputs [B,H,L,d] / [B,H,L]; returns a dict of fp64 / int32 arrays shaped like the inputs.

    chunk_routing = C > 0: mask is [B,H,L/C], one routing decision per chunk (nats_oracle_fwd_chunk).
    linear_op, freeze_on_softmax: the variants of nats_oracle_set_variant."""
    Q, K, V, alpha, beta = (_f32(a) for a in (Q, K, V, alpha, beta))
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    B, H, L, d = Q.shape
    BH = B * H
    scale = (1.0 / np.sqrt(d)) if softmax_scale is None else float(softmax_scale)
    w_nla, w_la = _f32(w_nla), _f32(w_la)
    S0 = None if S0 is None else np.ascontiguousarray(S0, dtype=np.float64)
    out = {"O": np.empty((B, H, L, d))}
    if "O_la" in want: out["O_la"] = np.empty((B, H, L, d))
    if "O_nla" in want: out["O_nla"] = np.empty((B, H, L, d))
    if "lse" in want: out["lse"] = np.empty((B, H, L))
    if "S" in want: out["S"] = np.empty((B, H, d, d))
    if "cnt" in want: out["cnt"] = np.empty((B, H, L), dtype=np.int32)
    if "idx" in want: out["idx"] = np.full((B, H, L), -1, dtype=np.int32)
    if "n_s" in want: out["n_s"] = np.empty((B, H), dtype=np.int32)
    lib = _load()
    if chunk_routing:
        assert mask.shape == (B, H, L // chunk_routing)
        call = lambda *a: lib.nats_oracle_fwd_chunk(a[0], a[1], a[2], ctypes.c_int(chunk_routing), *a[3:])
    else:
        assert mask.shape == (B, H, L)
        call = lib.nats_oracle_fwd
    lib.nats_oracle_set_variant(ctypes.c_int(linear_op), ctypes.c_int(freeze_on_softmax))
    try:
        rc = call(
            ctypes.c_int(BH), ctypes.c_int(L), ctypes.c_int(d), _p(Q), _p(K), _p(V), _p(alpha), _p(beta),
            _p(mask), ctypes.c_double(scale), ctypes.c_double(la_scale), ctypes.c_int(mode), _p(w_nla),
            _p(w_la), ctypes.c_double(eps), _p(S0), _p(out["O"]), _p(out.get("O_la")), _p(out.get("O_nla")),
            _p(out.get("lse")), _p(out.get("S")), _p(out.get("cnt")), _p(out.get("idx")), _p(out.get("n_s")))
    finally:
        lib.nats_oracle_set_variant(ctypes.c_int(0), ctypes.c_int(0))
    if rc != 0:
        raise RuntimeError(f"nats_oracle_fwd returned {rc}")
    return out


def decode(state, k_cache, v_cache, cache_len, q, k, v, alpha, beta, mask, softmax_scale=None,
           la_scale=1.0, mode=0, w_nla=None, w_la=None, eps=1e-6, linear_op=0, freeze_on_softmax=0):
    """In place on state (fp64 [B,H,d,d]), k_cache/v_cache (f32 [B,H,cap,d]), cache_len (i32 [B,H]).

    Returns (o fp64 [B,H,d], overflow i32 [B,H]).
    """
    for a, dt in ((state, np.float64), (k_cache, np.float32), (v_cache, np.float32), (cache_len, np.int32)):
        assert a.dtype == dt and a.flags["C_CONTIGUOUS"]
    B, H, cap, d = k_cache.shape
    q, k, v, alpha, beta = (_f32(a) for a in (q, k, v, alpha, beta))
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    scale = (1.0 / np.sqrt(d)) if softmax_scale is None else float(softmax_scale)
    o = np.empty((B, H, d))
    overflow = np.zeros((B, H), dtype=np.int32)
    lib = _load()
    lib.nats_oracle_set_variant(ctypes.c_int(linear_op), ctypes.c_int(freeze_on_softmax))
    try:
        rc = lib.nats_oracle_decode(
            ctypes.c_int(B * H), ctypes.c_int(d), ctypes.c_int(cap), _p(state), _p(k_cache), _p(v_cache),
            _p(cache_len), _p(q), _p(k), _p(v), _p(alpha), _p(beta), _p(mask), ctypes.c_double(scale),
            ctypes.c_double(la_scale), ctypes.c_int(mode), _p(_f32(w_nla)), _p(_f32(w_la)),
            ctypes.c_double(eps), _p(o), _p(overflow))
    finally:
        lib.nats_oracle_set_variant(ctypes.c_int(0), ctypes.c_int(0))
    if rc != 0:
        raise RuntimeError(f"nats_oracle_decode returned {rc}")
    return o, overflow
