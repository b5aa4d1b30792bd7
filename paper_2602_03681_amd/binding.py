"""ctypes binding of the C ABI declared in include/nats.h.

Argument marshalling only: tensors must already live on the GPU; this module
passes their device pointers and torch's current HIP stream to libnats.so, and
allocates outputs / workspace with torch.  No step of the operator is computed
here, and there is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libnats.so")
_lib = None

NATS_F32, NATS_BF16 = 0, 1
NATS_MATH_AUTO, NATS_MATH_FP32 = 0, 1
NATS_ROUTE_TOKEN, NATS_ROUTE_CHUNK = 0, 1
NATS_LINEAR_GDN, NATS_LINEAR_GATED = 0, 1
NATS_WEIGHTS_SOFTMAX, NATS_WEIGHTS_SIGMOID, NATS_WEIGHTS_LINEAR = 0, 1, 2


class NatsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"nats status {status}: {message}")
        self.status = status


class FwdParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32), ("d", ctypes.c_int32),
                ("C", ctypes.c_int32), ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("la_scale", ctypes.c_float), ("combine_mode", ctypes.c_int32), ("rms_eps", ctypes.c_float),
                ("math", ctypes.c_int32), ("routing", ctypes.c_int32), ("linear_op", ctypes.c_int32),
                ("freeze_on_softmax", ctypes.c_int32), ("weight_act", ctypes.c_int32),
                ("gdn_segments", ctypes.c_int32), ("group", ctypes.c_int32), ("inner_chunk", ctypes.c_int32)]


class FwdExtra(ctypes.Structure):
    _fields_ = [("w_nla", ctypes.c_void_p), ("w_la", ctypes.c_void_p), ("initial_state", ctypes.c_void_p),
                ("final_state", ctypes.c_void_p), ("Kc", ctypes.c_void_p), ("Vc", ctypes.c_void_p),
                ("cap", ctypes.c_int32), ("n_s", ctypes.c_void_p), ("idx", ctypes.c_void_p),
                ("cnt", ctypes.c_void_p), ("O_la", ctypes.c_void_p), ("O_nla", ctypes.c_void_p),
                ("lse", ctypes.c_void_p), ("W_out", ctypes.c_void_p), ("Q_nla", ctypes.c_void_p),
                ("K_nla", ctypes.c_void_p)]


class BwdExtra(ctypes.Structure):
    _fields_ = [("initial_state", ctypes.c_void_p), ("d_initial_state", ctypes.c_void_p), ("g_nla", ctypes.c_void_p),
                ("g_la", ctypes.c_void_p), ("dscore_nla", ctypes.c_void_p), ("dscore_la", ctypes.c_void_p),
                ("Q_nla", ctypes.c_void_p), ("K_nla", ctypes.c_void_p), ("dQ_nla", ctypes.c_void_p),
                ("dK_nla", ctypes.c_void_p), ("w_nla", ctypes.c_void_p), ("w_la", ctypes.c_void_p),
                ("dw_nla", ctypes.c_void_p), ("dw_la", ctypes.c_void_p)]


class DecChunkState(ctypes.Structure):
    _fields_ = [("state", ctypes.c_void_p), ("state_start", ctypes.c_void_p), ("chunk_decay", ctypes.c_void_p),
                ("chunk_pos", ctypes.c_void_p), ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
                ("cache_len", ctypes.c_void_p)]


class DecParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d", ctypes.c_int32), ("cap", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float), ("la_scale", ctypes.c_float),
                ("combine_mode", ctypes.c_int32), ("rms_eps", ctypes.c_float), ("linear_op", ctypes.c_int32),
                ("freeze_on_softmax", ctypes.c_int32), ("q_nla", ctypes.c_void_p), ("k_nla", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


EXPORTS = ("nats_hybrid_attn_fwd_workspace_bytes", "nats_hybrid_attn_fwd", "nats_hybrid_attn_fwd_ex",
           "nats_hybrid_attn_decode", "nats_last_error", "nats_abi_version", "nats_profile_begin",
           "nats_profile_end", "nats_probe_mfma", "nats_hybrid_attn_decode_chunk",
           "nats_hybrid_attn_decode_commit", "nats_merge_weights", "nats_route_chunks",
           "nats_hybrid_attn_bwd_workspace_bytes", "nats_hybrid_attn_bwd", "nats_hybrid_attn_fwd_noalloc",
           "nats_hybrid_attn_decode_workspace_bytes", "nats_merge_weights_from_x")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libnats.so (built in-tree by paper_2602_03681_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2602_03681_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp = ctypes.c_void_p
    lib.nats_hybrid_attn_fwd_workspace_bytes.restype = ctypes.c_size_t
    lib.nats_hybrid_attn_fwd_workspace_bytes.argtypes = [ctypes.POINTER(FwdParams)]
    lib.nats_hybrid_attn_fwd.restype = ctypes.c_int
    lib.nats_hybrid_attn_fwd.argtypes = [ctypes.POINTER(FwdParams)] + [vp] * 7 + [vp, ctypes.c_size_t, vp]
    lib.nats_hybrid_attn_fwd_noalloc.restype = ctypes.c_int
    lib.nats_hybrid_attn_fwd_noalloc.argtypes = [ctypes.POINTER(FwdParams)] + [vp] * 7 + [vp]
    lib.nats_hybrid_attn_fwd_ex.restype = ctypes.c_int
    lib.nats_hybrid_attn_fwd_ex.argtypes = ([ctypes.POINTER(FwdParams)] + [vp] * 7
                                            + [ctypes.POINTER(FwdExtra), vp, ctypes.c_size_t, vp])
    lib.nats_hybrid_attn_decode.restype = ctypes.c_int
    lib.nats_hybrid_attn_decode.argtypes = [ctypes.POINTER(DecParams)] + [vp] * 15
    lib.nats_hybrid_attn_decode_chunk.restype = ctypes.c_int
    lib.nats_hybrid_attn_decode_chunk.argtypes = [ctypes.POINTER(DecParams), ctypes.POINTER(DecChunkState)] + [vp] * 10
    lib.nats_hybrid_attn_decode_commit.restype = ctypes.c_int
    lib.nats_hybrid_attn_decode_commit.argtypes = [ctypes.POINTER(DecParams), ctypes.POINTER(DecChunkState)] + [vp] * 3
    lib.nats_merge_weights.restype = ctypes.c_int
    lib.nats_merge_weights.argtypes = [ctypes.POINTER(FwdParams)] + [vp] * 5
    lib.nats_route_chunks.restype = ctypes.c_int
    lib.nats_route_chunks.argtypes = [ctypes.c_int32] * 6 + [vp] * 5
    lib.nats_merge_weights_from_x.restype = ctypes.c_int
    lib.nats_merge_weights_from_x.argtypes = [ctypes.c_int32] * 5 + [vp, vp, ctypes.c_int32, vp, vp, vp]
    lib.nats_hybrid_attn_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.nats_hybrid_attn_decode_workspace_bytes.argtypes = [ctypes.POINTER(DecParams)]
    lib.nats_hybrid_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.nats_hybrid_attn_bwd_workspace_bytes.argtypes = [ctypes.POINTER(FwdParams)]
    lib.nats_hybrid_attn_bwd.restype = ctypes.c_int
    lib.nats_hybrid_attn_bwd.argtypes = ([ctypes.POINTER(FwdParams)] + [vp] * 12 + [ctypes.POINTER(BwdExtra), vp,
                                          ctypes.c_size_t, vp])
    lib.nats_last_error.restype = ctypes.c_char_p
    lib.nats_abi_version.restype = ctypes.c_int
    lib.nats_probe_mfma.restype = ctypes.c_double
    lib.nats_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.nats_profile_begin.restype = ctypes.c_int
    lib.nats_profile_begin.argtypes = [ctypes.c_int]
    lib.nats_profile_end.restype = ctypes.c_int
    lib.nats_profile_end.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_float),
                                     ctypes.POINTER(ctypes.c_int32), ctypes.c_int]
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise NatsError(status, load_library().nats_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return NATS_F32
    if t.dtype == torch.bfloat16:
        return NATS_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _require(t: Optional[torch.Tensor], name: str, shape: Sequence[int], dtype: torch.dtype):
    if t is None:
        return
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous {dtype} of shape {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")


def _stream_ptr() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_fwd_params(B, H, L, d, C, dtype_code, softmax_scale=0.0, la_scale=0.0, combine_mode=0, rms_eps=0.0,
                    math=NATS_MATH_AUTO, routing=NATS_ROUTE_TOKEN, linear_op=NATS_LINEAR_GDN,
                    freeze_on_softmax=0, weight_act=0, gdn_segments=0, group=1, inner_chunk=0) -> FwdParams:
    return FwdParams(B, H, L, d, C, dtype_code, softmax_scale, la_scale, combine_mode, rms_eps, math, routing,
                     linear_op, int(freeze_on_softmax), weight_act, gdn_segments, group, inner_chunk)


def fwd_workspace_bytes(params: FwdParams) -> int:
    return int(load_library().nats_hybrid_attn_fwd_workspace_bytes(ctypes.byref(params)))


_EX_OUTPUTS = ("final_state", "Kc", "Vc", "n_s", "idx", "cnt", "O_la", "O_nla", "lse")


def hybrid_attn_fwd_ex(Q, K, V, alpha, beta, mask, C: int = 64, *, softmax_scale: float = 0.0,
                       la_scale: float = 0.0, combine_mode: int = 0, rms_eps: float = 0.0,
                       math: int = NATS_MATH_AUTO, routing: int = NATS_ROUTE_TOKEN, linear_op: int = NATS_LINEAR_GDN,
                       freeze_on_softmax: bool = False, w_nla=None, w_la=None,
                       W_out=None, weight_act: int = NATS_WEIGHTS_SOFTMAX, initial_state=None, Q_nla=None, K_nla=None,
                       want: Sequence[str] = (), cap: Optional[int] = None, out=None,
                       workspace=None, gdn_segments: int = 0, group: int = 1,
                       inner_chunk: int = 0) -> Dict[str, torch.Tensor]:
    """nats_hybrid_attn_fwd_ex.  `want` lists optional outputs to allocate and return
    (any of final_state, Kc, Vc, n_s, idx, cnt, O_la, O_nla, lse); the result dict always holds "O".
    group = G > 1 (head grouping): Q, K, alpha, beta, mask have H heads, everything else H * G."""
    lib = load_library()
    B, H, L, d = Q.shape
    HG = H * group
    dt = Q.dtype
    for name, t in (("Q", Q), ("K", K)):
        _require(t, name, (B, H, L, d), dt)
    _require(V, "V", (B, HG, L, d), dt)
    _require(alpha, "alpha", (B, H, L), torch.float32)
    _require(beta, "beta", (B, H, L), torch.float32)
    _require(mask, "mask", (B, H, L // C if routing == NATS_ROUTE_CHUNK else L), torch.uint8)
    _require(w_nla, "w_nla", (B, HG, L), torch.float32)
    _require(w_la, "w_la", (B, HG, L), torch.float32)
    _require(initial_state, "initial_state", (B, HG, d, d), torch.float32)
    _require(Q_nla, "Q_nla", (B, HG, L, d), dt)
    _require(K_nla, "K_nla", (B, HG, L, d), dt)
    _require(W_out, "W_out", (HG, 2, d), torch.float32)
    params = make_fwd_params(B, H, L, d, C, _dtype_code(Q), softmax_scale, la_scale, combine_mode, rms_eps, math,
                             routing, linear_op, freeze_on_softmax, weight_act, gdn_segments, group, inner_chunk)
    need = lib.nats_hybrid_attn_fwd_workspace_bytes(ctypes.byref(params))
    if need == 0:
        _check(lib.nats_hybrid_attn_fwd_ex(ctypes.byref(params), *([None] * 7), None, None, 0, None))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    dev = Q.device
    O = torch.empty_like(V) if out is None else out
    _require(O, "out", (B, HG, L, d), dt)
    want = set(want)
    unknown = want - set(_EX_OUTPUTS)
    if unknown:
        raise ValueError(f"unknown outputs {sorted(unknown)}")
    if ("Kc" in want) != ("Vc" in want):
        raise ValueError("Kc and Vc come together")
    cap = L if cap is None else cap
    res: Dict[str, torch.Tensor] = {"O": O}
    if "final_state" in want: res["final_state"] = torch.empty((B, HG, d, d), dtype=torch.float32, device=dev)
    if "Kc" in want:
        res["Kc"] = torch.zeros((B, HG, cap, d), dtype=dt, device=dev)
        res["Vc"] = torch.zeros((B, HG, cap, d), dtype=dt, device=dev)
    if "n_s" in want: res["n_s"] = torch.empty((B, H), dtype=torch.int32, device=dev)
    if "idx" in want: res["idx"] = torch.full((B, H, L), -1, dtype=torch.int32, device=dev)
    if "cnt" in want: res["cnt"] = torch.empty((B, H, L), dtype=torch.int32, device=dev)
    if "O_la" in want: res["O_la"] = torch.empty((B, HG, L, d), dtype=torch.float32, device=dev)
    if "O_nla" in want: res["O_nla"] = torch.empty((B, HG, L, d), dtype=torch.float32, device=dev)
    if "lse" in want: res["lse"] = torch.empty((B, HG, L), dtype=torch.float32, device=dev)
    g = lambda k: res[k].data_ptr() if k in res else None
    extra = FwdExtra(w_nla.data_ptr() if w_nla is not None else None,
                     w_la.data_ptr() if w_la is not None else None,
                     initial_state.data_ptr() if initial_state is not None else None,
                     g("final_state"), g("Kc"), g("Vc"), cap if "Kc" in want else 0, g("n_s"), g("idx"),
                     g("cnt"), g("O_la"), g("O_nla"), g("lse"), W_out.data_ptr() if W_out is not None else None,
                     Q_nla.data_ptr() if Q_nla is not None else None, K_nla.data_ptr() if K_nla is not None else None)
    _check(lib.nats_hybrid_attn_fwd_ex(ctypes.byref(params), _ptr(Q), _ptr(K), _ptr(V), _ptr(alpha), _ptr(beta),
                                       _ptr(mask), _ptr(O), ctypes.byref(extra), _ptr(workspace),
                                       workspace.numel(), _stream_ptr()))
    return res


def hybrid_attn_fwd(Q, K, V, alpha, beta, mask, C: int = 64, *, softmax_scale: float = 0.0,
                    la_scale: float = 0.0, combine_mode: int = 0, rms_eps: float = 0.0,
                    math: int = NATS_MATH_AUTO, routing: int = NATS_ROUTE_TOKEN, linear_op: int = NATS_LINEAR_GDN,
                    freeze_on_softmax: bool = False, out=None,
                    workspace=None, gdn_segments: int = 0) -> torch.Tensor:
    """nats_hybrid_attn_fwd(Q, K, V, alpha, beta, mask, C) -> O."""
    lib = load_library()
    B, H, L, d = Q.shape
    dt = Q.dtype
    for name, t in (("Q", Q), ("K", K), ("V", V)):
        _require(t, name, (B, H, L, d), dt)
    _require(alpha, "alpha", (B, H, L), torch.float32)
    _require(beta, "beta", (B, H, L), torch.float32)
    _require(mask, "mask", (B, H, L // C if routing == NATS_ROUTE_CHUNK else L), torch.uint8)
    params = make_fwd_params(B, H, L, d, C, _dtype_code(Q), softmax_scale, la_scale, combine_mode, rms_eps, math,
                             routing, linear_op, freeze_on_softmax, 0, gdn_segments)
    if workspace is None:
        workspace = torch.empty(max(fwd_workspace_bytes(params), 16), dtype=torch.uint8, device=Q.device)
    O = torch.empty_like(Q) if out is None else out
    _require(O, "out", (B, H, L, d), dt)
    _check(lib.nats_hybrid_attn_fwd(ctypes.byref(params), _ptr(Q), _ptr(K), _ptr(V), _ptr(alpha), _ptr(beta),
                                    _ptr(mask), _ptr(O), _ptr(workspace), workspace.numel(), _stream_ptr()))
    return O


NOALLOC_SCRATCH_BYTES = 32 << 20   # NATS_NOALLOC_SCRATCH_BYTES of nats.h


def hybrid_attn_fwd_noalloc(Q, K, V, alpha, beta, mask, out, C: int = 64, *, softmax_scale: float = 0.0,
                            la_scale: float = 0.0, combine_mode: int = 0, rms_eps: float = 0.0,
                            math: int = NATS_MATH_AUTO, routing: int = NATS_ROUTE_TOKEN,
                            linear_op: int = NATS_LINEAR_GDN, freeze_on_softmax: bool = False) -> torch.Tensor:
    """nats_hybrid_attn_fwd_noalloc: the forward on the library's built-in scratch buffer; the caller passes the
    output tensor, nothing is allocated here or in the library."""
    lib = load_library()
    B, H, L, d = Q.shape
    dt = Q.dtype
    for name, t in (("Q", Q), ("K", K), ("V", V), ("out", out)):
        _require(t, name, (B, H, L, d), dt)
    _require(alpha, "alpha", (B, H, L), torch.float32)
    _require(beta, "beta", (B, H, L), torch.float32)
    _require(mask, "mask", (B, H, L // C if routing == NATS_ROUTE_CHUNK else L), torch.uint8)
    params = make_fwd_params(B, H, L, d, C, _dtype_code(Q), softmax_scale, la_scale, combine_mode, rms_eps, math,
                             routing, linear_op, freeze_on_softmax)
    _check(lib.nats_hybrid_attn_fwd_noalloc(ctypes.byref(params), _ptr(Q), _ptr(K), _ptr(V), _ptr(alpha), _ptr(beta),
                                            _ptr(mask), _ptr(out), _stream_ptr()))
    return out


def hybrid_attn_bwd(Q, K, V, alpha, beta, mask, dO, C: int = 64, *, softmax_scale: float = 0.0, la_scale: float = 0.0,
                    linear_op: int = NATS_LINEAR_GDN, freeze_on_softmax: bool = False, initial_state=None,
                    want=(), workspace=None, routing: int = NATS_ROUTE_TOKEN,
                    math: int = NATS_MATH_AUTO, group: int = 1, Q_nla=None, K_nla=None, combine_mode: int = 0,
                    rms_eps: float = 0.0, w_nla=None, w_la=None) -> Dict[str, torch.Tensor]:
    """nats_hybrid_attn_bwd: gradients of O = O_la + O_nla given dO.  Returns dQ, dK, dV [B,H,L,d] f32, dalpha,
    dbeta [B,H,L] f32 and, if named in `want`, d_initial_state [B,H,d,d], g_nla, g_la [B,H,L] (routing per token),
    dscore_nla, dscore_la [B,H,L/C] (Eq. 16, Eq. 17).  math = NATS_MATH_FP32: the linear branch's adjoint token by
    token instead of by chunks.  group = G > 1 (head grouping): V, dO, dV [B,H*G,L,d], the states [B,H*G,d,d].
    Q_nla, K_nla [B,H*G,L,d] (both or neither): the softmax branch's own queries and keys; their gradients come back
    as dQ_nla, dK_nla, and dQ, dK are then the linear branch's alone.  combine_mode 1, 2 (Eq. 21 and its ablation
    with one normalisation) with the weights w_nla, w_la [B,H*G,L] f32 (or None): also returns dw_nla, dw_la."""
    lib = load_library()
    B, H, L, d = Q.shape
    dt = Q.dtype
    G = max(int(group), 1)
    for name, t in (("Q", Q), ("K", K)):
        _require(t, name, (B, H, L, d), dt)
    for name, t in (("V", V), ("dO", dO)):
        _require(t, name, (B, H * G, L, d), dt)
    _require(alpha, "alpha", (B, H, L), torch.float32)
    _require(beta, "beta", (B, H, L), torch.float32)
    _require(mask, "mask", (B, H, L // C if routing == NATS_ROUTE_CHUNK else L), torch.uint8)
    _require(initial_state, "initial_state", (B, H * G, d, d), torch.float32)
    if (Q_nla is None) != (K_nla is None):
        raise ValueError("Q_nla and K_nla: both or neither")
    _require(Q_nla, "Q_nla", (B, H * G, L, d), dt)
    _require(K_nla, "K_nla", (B, H * G, L, d), dt)
    _require(w_nla, "w_nla", (B, H * G, L), torch.float32)
    _require(w_la, "w_la", (B, H * G, L), torch.float32)
    unknown = set(want) - {"d_initial_state", "g_nla", "g_la", "dscore_nla", "dscore_la"}
    if unknown:
        raise ValueError(f"unknown outputs {sorted(unknown)}")
    params = make_fwd_params(B, H, L, d, C, _dtype_code(Q), softmax_scale, la_scale, combine_mode, rms_eps, math,
                             routing, linear_op, freeze_on_softmax, group=G)
    need = int(lib.nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(params)))
    if need == 0:   # let the library say what is wrong with the parameters
        _check(lib.nats_hybrid_attn_bwd(ctypes.byref(params), *([None] * 12), None, None, 0, None))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    dev = Q.device
    res = {k: torch.empty((B, H, L, d), dtype=torch.float32, device=dev) for k in ("dQ", "dK")}
    res["dV"] = torch.empty((B, H * G, L, d), dtype=torch.float32, device=dev)
    res["dalpha"] = torch.empty((B, H, L), dtype=torch.float32, device=dev)
    res["dbeta"] = torch.empty((B, H, L), dtype=torch.float32, device=dev)
    if "d_initial_state" in want: res["d_initial_state"] = torch.empty((B, H * G, d, d), dtype=torch.float32, device=dev)
    for key in ("g_nla", "g_la"):
        if key in want: res[key] = torch.empty((B, H, L), dtype=torch.float32, device=dev)
    for key in ("dscore_nla", "dscore_la"):
        if key in want: res[key] = torch.empty((B, H, L // C), dtype=torch.float32, device=dev)
    if Q_nla is not None:
        res["dQ_nla"] = torch.empty((B, H * G, L, d), dtype=torch.float32, device=dev)
        res["dK_nla"] = torch.empty((B, H * G, L, d), dtype=torch.float32, device=dev)
    if combine_mode != 0:
        res["dw_nla"] = torch.empty((B, H * G, L), dtype=torch.float32, device=dev)
        res["dw_la"] = torch.empty((B, H * G, L), dtype=torch.float32, device=dev)
    g = lambda k: res[k].data_ptr() if k in res else None
    extra = BwdExtra(initial_state.data_ptr() if initial_state is not None else None, g("d_initial_state"), g("g_nla"),
                     g("g_la"), g("dscore_nla"), g("dscore_la"), Q_nla.data_ptr() if Q_nla is not None else None,
                     K_nla.data_ptr() if K_nla is not None else None, g("dQ_nla"), g("dK_nla"),
                     w_nla.data_ptr() if w_nla is not None else None, w_la.data_ptr() if w_la is not None else None,
                     g("dw_nla"), g("dw_la"))
    _check(lib.nats_hybrid_attn_bwd(ctypes.byref(params), _ptr(Q), _ptr(K), _ptr(V), _ptr(alpha), _ptr(beta), _ptr(mask),
                                    _ptr(dO), _ptr(res["dQ"]), _ptr(res["dK"]), _ptr(res["dV"]), _ptr(res["dalpha"]),
                                    _ptr(res["dbeta"]), ctypes.byref(extra), _ptr(workspace), workspace.numel(),
                                    _stream_ptr()))
    return res


def hybrid_attn_decode(state, k_cache, v_cache, cache_len, q, k, v, alpha, beta, mask, *,
                       softmax_scale: float = 0.0, la_scale: float = 0.0, combine_mode: int = 0,
                       rms_eps: float = 0.0, linear_op: int = NATS_LINEAR_GDN, freeze_on_softmax: bool = False,
                       q_nla=None, k_nla=None, w_nla=None, w_la=None, out=None, err_flags=None,
                       workspace=None) -> torch.Tensor:
    """nats_hybrid_attn_decode: one token per (b,h); state, caches and cache_len are updated in place.
    workspace: uint8 device tensor of decode_workspace_bytes(...) bytes -> the step runs as many equal blocks."""
    lib = load_library()
    B, H, cap, d = k_cache.shape
    dt = k_cache.dtype
    _require(state, "state", (B, H, d, d), torch.float32)
    _require(k_cache, "k_cache", (B, H, cap, d), dt)
    _require(v_cache, "v_cache", (B, H, cap, d), dt)
    _require(cache_len, "cache_len", (B, H), torch.int32)
    for name, t in (("q", q), ("k", k), ("v", v)):
        _require(t, name, (B, H, d), dt)
    for name, t in (("alpha", alpha), ("beta", beta), ("w_nla", w_nla), ("w_la", w_la)):
        _require(t, name, (B, H), torch.float32)
    _require(mask, "mask", (B, H), torch.uint8)
    _require(err_flags, "err_flags", (B, H), torch.int32)
    o = torch.empty_like(q) if out is None else out
    _require(o, "out", (B, H, d), dt)
    _require(q_nla, "q_nla", (B, H, d), dt)
    _require(k_nla, "k_nla", (B, H, d), dt)
    params = DecParams(B, H, d, cap, _dtype_code(k_cache), softmax_scale, la_scale, combine_mode, rms_eps, linear_op,
                       int(freeze_on_softmax), q_nla.data_ptr() if q_nla is not None else None,
                       k_nla.data_ptr() if k_nla is not None else None,
                       workspace.data_ptr() if workspace is not None else None,
                       workspace.numel() if workspace is not None else 0)
    _check(lib.nats_hybrid_attn_decode(ctypes.byref(params), _ptr(state), _ptr(k_cache), _ptr(v_cache),
                                       _ptr(cache_len), _ptr(q), _ptr(k), _ptr(v), _ptr(alpha), _ptr(beta),
                                       _ptr(mask), _ptr(w_nla), _ptr(w_la), _ptr(o), _ptr(err_flags),
                                       _stream_ptr()))
    return o


def decode_workspace_bytes(B, H, d, cap, dtype_code) -> int:
    """nats_hybrid_attn_decode_workspace_bytes for a cache of `cap` rows per (b,h)."""
    params = DecParams(B, H, d, cap, dtype_code, 0.0, 0.0, 0, 0.0, 0, 0, None, None, None, 0)
    return int(load_library().nats_hybrid_attn_decode_workspace_bytes(ctypes.byref(params)))


def route_chunks(X, W_s, C: int = 64, want_scores: bool = True):
    """nats_route_chunks (Eq. 8-9): X [B,L,d_model], W_s [H,2,d_model] f32 -> (mask_c [B,H,L/C] u8, scores
    [B,L/C,H,2] f32 or None)."""
    lib = load_library()
    B, L, dm = X.shape
    H = W_s.shape[0]
    _require(X, "X", (B, L, dm), X.dtype)
    _require(W_s, "W_s", (H, 2, dm), torch.float32)
    mask_c = torch.empty((B, H, L // C), dtype=torch.uint8, device=X.device)
    scores = torch.empty((B, L // C, H, 2), dtype=torch.float32, device=X.device) if want_scores else None
    _check(lib.nats_route_chunks(B, L, C, dm, H, _dtype_code(X), _ptr(X), _ptr(W_s), _ptr(scores), _ptr(mask_c),
                                 _stream_ptr()))
    return mask_c, scores


def merge_weights_from_x(X, W_x, weight_act: int = NATS_WEIGHTS_SOFTMAX):
    """nats_merge_weights_from_x: X [B,L,d_model], W_x [H,2,d_model] f32 -> (w_nla, w_la) [B,H,L] f32."""
    lib = load_library()
    B, L, dm = X.shape
    H = W_x.shape[0]
    _require(X, "X", (B, L, dm), X.dtype)
    _require(W_x, "W_x", (H, 2, dm), torch.float32)
    w_nla = torch.empty((B, H, L), dtype=torch.float32, device=X.device)
    w_la = torch.empty_like(w_nla)
    _check(lib.nats_merge_weights_from_x(B, L, dm, H, _dtype_code(X), _ptr(X), _ptr(W_x), weight_act, _ptr(w_nla),
                                         _ptr(w_la), _stream_ptr()))
    return w_nla, w_la


def merge_weights(Q, W_out, weight_act: int = NATS_WEIGHTS_SOFTMAX):
    """nats_merge_weights (Eq. 22): Q [B,H,L,d], W_out [H,2,d] f32 -> (w_nla, w_la) [B,H,L] f32."""
    lib = load_library()
    B, H, L, d = Q.shape
    _require(Q, "Q", (B, H, L, d), Q.dtype)
    _require(W_out, "W_out", (H, 2, d), torch.float32)
    w_nla = torch.empty((B, H, L), dtype=torch.float32, device=Q.device)
    w_la = torch.empty_like(w_nla)
    params = make_fwd_params(B, H, L, d, 64, _dtype_code(Q), weight_act=weight_act)
    _check(lib.nats_merge_weights(ctypes.byref(params), _ptr(Q), _ptr(W_out), _ptr(w_nla), _ptr(w_la), _stream_ptr()))
    return w_nla, w_la


def _chunk_state(st: Dict[str, torch.Tensor]):
    """st: dict of tensors state, state_start [B,H,d,d] f32; chunk_decay [B,H] f32; chunk_pos, cache_len [B,H]
    i32; k_cache, v_cache [B,H,cap,d]."""
    B, H, cap, d = st["k_cache"].shape
    dt = st["k_cache"].dtype
    _require(st["state"], "state", (B, H, d, d), torch.float32)
    _require(st["state_start"], "state_start", (B, H, d, d), torch.float32)
    _require(st["chunk_decay"], "chunk_decay", (B, H), torch.float32)
    _require(st["chunk_pos"], "chunk_pos", (B, H), torch.int32)
    _require(st["k_cache"], "k_cache", (B, H, cap, d), dt)
    _require(st["v_cache"], "v_cache", (B, H, cap, d), dt)
    _require(st["cache_len"], "cache_len", (B, H), torch.int32)
    cs = DecChunkState(*(st[k].data_ptr() for k in ("state", "state_start", "chunk_decay", "chunk_pos", "k_cache",
                                                    "v_cache", "cache_len")))
    return cs, (B, H, cap, d, dt)


def hybrid_attn_decode_chunk(st, q, k, v, alpha, beta, *, softmax_scale: float = 0.0, la_scale: float = 0.0,
                             combine_mode: int = 0, rms_eps: float = 0.0, linear_op: int = NATS_LINEAR_GDN,
                             w_nla=None, w_la=None, out=None, err_flags=None) -> torch.Tensor:
    """nats_hybrid_attn_decode_chunk: one token per (b,h) under routing per chunk; `st` (see _chunk_state) is
    updated in place."""
    lib = load_library()
    cs, (B, H, cap, d, dt) = _chunk_state(st)
    for name, t in (("q", q), ("k", k), ("v", v)):
        _require(t, name, (B, H, d), dt)
    for name, t in (("alpha", alpha), ("beta", beta), ("w_nla", w_nla), ("w_la", w_la)):
        _require(t, name, (B, H), torch.float32)
    _require(err_flags, "err_flags", (B, H), torch.int32)
    o = torch.empty_like(q) if out is None else out
    _require(o, "out", (B, H, d), dt)
    params = DecParams(B, H, d, cap, _dtype_code(st["k_cache"]), softmax_scale, la_scale, combine_mode, rms_eps,
                       linear_op, 0)
    _check(lib.nats_hybrid_attn_decode_chunk(ctypes.byref(params), ctypes.byref(cs), _ptr(q), _ptr(k), _ptr(v),
                                             _ptr(alpha), _ptr(beta), _ptr(w_nla), _ptr(w_la), _ptr(o),
                                             _ptr(err_flags), _stream_ptr()))
    return o


def hybrid_attn_decode_commit(st, mask_c, *, freeze_on_softmax: bool = False, err_flags=None) -> None:
    """nats_hybrid_attn_decode_commit: settle the open chunk of every (b,h) with its routing decision."""
    lib = load_library()
    cs, (B, H, cap, d, dt) = _chunk_state(st)
    _require(mask_c, "mask_c", (B, H), torch.uint8)
    _require(err_flags, "err_flags", (B, H), torch.int32)
    params = DecParams(B, H, d, cap, _dtype_code(st["k_cache"]), 0.0, 0.0, 0, 0.0, 0, int(freeze_on_softmax))
    _check(lib.nats_hybrid_attn_decode_commit(ctypes.byref(params), ctypes.byref(cs), _ptr(mask_c), _ptr(err_flags),
                                              _stream_ptr()))


def profile_begin(max_records: int = 4096) -> None:
    """nats_profile_begin: bracket every kernel of the following calls with HIP events."""
    _check(load_library().nats_profile_begin(max_records))


def profile_end(max_kernels: int = 16) -> Dict[str, Dict[str, float]]:
    """nats_profile_end: {kernel name: {"total_ms", "launches", "avg_ms"}}."""
    names = ctypes.create_string_buffer(32 * max_kernels)
    ms = (ctypes.c_float * max_kernels)()
    cnt = (ctypes.c_int32 * max_kernels)()
    n = load_library().nats_profile_end(names, ms, cnt, max_kernels)
    if n < 0:
        _check(n)
    out = {}
    for i in range(n):
        name = names.raw[32 * i:32 * i + 32].split(b"\0", 1)[0].decode()
        out[name] = {"total_ms": float(ms[i]), "launches": int(cnt[i]), "avg_ms": float(ms[i]) / max(int(cnt[i]), 1)}
    return out


def probe_mfma(iters: int, out) -> float:
    """nats_probe_mfma: launch the MFMA-issue probe; `out` is a float32 device tensor of >= 2048 elements.
    Returns the FLOP of the launch (time it on torch's current stream)."""
    flop = load_library().nats_probe_mfma(int(iters), out.data_ptr(), out.numel(), _stream_ptr())
    if flop < 0:
        raise RuntimeError(load_library().nats_last_error().decode())
    return float(flop)


decode = hybrid_attn_decode
