"""Seeded synthetic inputs for the NAtS-L hybrid-attention operator.

This module only *draws numbers*: it holds none of the operator's arithmetic
(no prefix sums over the mask, no attention, no state updates).  Both the CPU
oracle's tests and the HIP path's tests / benchmark take their inputs from
here, so that the two sides see bit-identical tensors.

Workload recipe (stands in for the text workloads of the paper's Section 5,
which need trained weights and corpora):
  * q, k, v ~ N(0,1) i.i.d.; q and k are L2-normalised per token and head
    (the linear branch's q/k normalisation, Section 4.3);
  * alpha = sigmoid(N(2, 0.5^2)), beta = sigmoid(N(0, 1)) per (batch, head, token)
    (the sigmoid-gated decay / write strength of Gated DeltaNet, Eq. 19);
  * hard routing mask ~ Bernoulli(p) per (batch, head, token), 1 = softmax token,
    token 0 forced to softmax; optional runs of consecutive softmax tokens;
  * for bf16 workloads q, k, v are rounded to bf16 (round-to-nearest-even) after
    normalisation and handed out as float32 arrays holding exactly those values.
Draw order is fixed: Q, K, V, alpha, beta, mask, (run positions).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class FwdConfig:
    name: str
    B: int
    H: int
    L: int
    d: int
    C: int
    dtype: str  # "f32" | "bf16"
    p_softmax: float
    seed: int
    n_runs: int = 0  # contiguous softmax runs inserted per (b, h)
    run_len: int = 0


@dataclass(frozen=True)
class DecodeConfig:
    name: str
    B: int
    H: int
    d: int
    dtype: str
    p_softmax: float
    seed: int
    len_lo: int = 64
    len_hi: int = 2048
    steps: int = 256
    state_std: float = 0.02


# The five workloads the build is measured on.
CONFIGS: Dict[str, object] = {
    "cfg0_tiny_f32": FwdConfig("cfg0_tiny_f32", 1, 2, 256, 64, 64, "f32", 0.10, 20260200),
    "cfg1_bf16": FwdConfig("cfg1_bf16", 4, 8, 2048, 64, 64, "bf16", 0.10, 20260201),
    "cfg2_headline_bf16": FwdConfig("cfg2_headline_bf16", 2, 16, 8192, 128, 64, "bf16", 0.05, 20260202),
    "cfg3_long_bf16": FwdConfig("cfg3_long_bf16", 1, 16, 32768, 128, 64, "bf16", 0.02, 20260203,
                                n_runs=8, run_len=16),
    "cfg4_decode_bf16": DecodeConfig("cfg4_decode_bf16", 64, 16, 128, "bf16", 0.05, 20260204),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def _sigmoid(x: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-x))


def _unit_rows(x: np.ndarray) -> np.ndarray:
    x /= np.sqrt(np.einsum("...i,...i->...", x, x))[..., None]
    return x


def _normal32(rng: np.random.Generator, shape) -> np.ndarray:
    """N(0,1) float32 by Box-Muller on float32 uniforms, in fixed-size blocks (numpy's own
    float32 normal sampler is ~20x slower per element, which matters at 10^8 elements)."""
    n = int(np.prod(shape))
    out = np.empty(n + (n & 1), dtype=np.float32)
    block = 1 << 22
    for lo in range(0, out.size, block):
        m = min(block, out.size - lo) // 2
        u1 = 1.0 - rng.random(m, dtype=np.float32)          # (0, 1]
        u2 = rng.random(m, dtype=np.float32)
        r = np.sqrt(-2.0 * np.log(u1))
        ang = np.float32(2.0 * np.pi) * u2
        out[lo:lo + m] = r * np.cos(ang)
        out[lo + m:lo + 2 * m] = r * np.sin(ang)
    return out[:n].reshape(shape)


def _qkv_gates(rng: np.random.Generator, lead: tuple, d: int, dtype: str):
    q = _unit_rows(_normal32(rng, lead + (d,)))
    k = _unit_rows(_normal32(rng, lead + (d,)))
    v = _normal32(rng, lead + (d,))
    alpha = _sigmoid(2.0 + 0.5 * rng.standard_normal(lead))
    beta = _sigmoid(rng.standard_normal(lead))
    if dtype == "bf16":
        q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
    return q, k, v, alpha.astype(np.float32), beta.astype(np.float32)


def make_fwd_inputs(B: int, H: int, L: int, d: int, dtype: str, p_softmax: float, seed: int,
                    n_runs: int = 0, run_len: int = 0, force_first: bool = True,
                    mask_kind: str = "bernoulli") -> Dict[str, np.ndarray]:
    """Q, K, V [B,H,L,d] float32; alpha, beta [B,H,L] float32; mask [B,H,L] uint8.

    mask_kind: "bernoulli" (default), "all_softmax", "all_linear",
    "head_skew" (even heads p=0, odd heads p=0.5), "ramp" (p grows linearly
    with position from 0 to 2*p_softmax).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    q, k, v, alpha, beta = _qkv_gates(rng, (B, H, L), d, dtype)
    u = rng.random((B, H, L))
    if mask_kind == "bernoulli":
        mask = u < p_softmax
    elif mask_kind == "all_softmax":
        mask = np.ones((B, H, L), dtype=bool)
    elif mask_kind == "all_linear":
        mask = np.zeros((B, H, L), dtype=bool)
    elif mask_kind == "head_skew":
        p_head = np.where(np.arange(H) % 2 == 0, 0.0, 0.5)[None, :, None]
        mask = u < p_head
    elif mask_kind == "ramp":
        p_pos = (2.0 * p_softmax * np.arange(L) / max(L - 1, 1))[None, None, :]
        mask = u < p_pos
    else:
        raise ValueError(f"unknown mask_kind {mask_kind!r}")
    mask = mask.astype(np.uint8)
    if n_runs > 0:
        starts = rng.integers(1, L - run_len + 1, size=(B, H, n_runs))
        for b in range(B):
            for h in range(H):
                for s in starts[b, h]:
                    mask[b, h, s:s + run_len] = 1
    if force_first and mask_kind not in ("all_linear", "head_skew"):
        mask[:, :, 0] = 1
    return {"Q": q, "K": k, "V": v, "alpha": alpha, "beta": beta, "mask": mask}


def make_chunk_mask(B: int, H: int, n_chunks: int, p_softmax: float, seed: int,
                    mask_kind: str = "bernoulli") -> np.ndarray:
    """Routing mask with one decision per chunk, [B,H,n_chunks] uint8 (1 = softmax chunk).

    mask_kind: "bernoulli", "all_softmax", "all_linear", "head_skew" (even heads none, odd heads half),
    "alternate" (every other chunk).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    u = rng.random((B, H, n_chunks))
    if mask_kind == "bernoulli":
        mask = u < p_softmax
    elif mask_kind == "all_softmax":
        mask = np.ones((B, H, n_chunks), dtype=bool)
    elif mask_kind == "all_linear":
        mask = np.zeros((B, H, n_chunks), dtype=bool)
    elif mask_kind == "head_skew":
        mask = u < np.where(np.arange(H) % 2 == 0, 0.0, 0.5)[None, :, None]
    elif mask_kind == "alternate":
        mask = np.broadcast_to((np.arange(n_chunks) % 2 == 1)[None, None, :], (B, H, n_chunks))
    else:
        raise ValueError(f"unknown mask_kind {mask_kind!r}")
    return np.ascontiguousarray(mask, dtype=np.uint8)


def make_score_inputs(B: int, L: int, d_model: int, H: int, dtype: str, seed: int) -> Dict[str, np.ndarray]:
    """Inputs of the score layer: hidden states X [B,L,d_model] (unit variance, as after a normalisation
    layer; representable in `dtype`) and the layer's weights W_s [H,2,d_model] float32 (variance 1/d_model)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    X = _normal32(rng, (B, L, d_model))
    if dtype == "bf16":
        X = round_to_bf16(X)
    W_s = _normal32(rng, (H, 2, d_model)) / np.float32(np.sqrt(d_model))
    return {"X": X, "W_s": np.ascontiguousarray(W_s, dtype=np.float32)}


def make_grad_output(B: int, H: int, L: int, d: int, dtype: str, seed: int) -> np.ndarray:
    """dO [B,H,L,d] for the backward pass: N(0,1), representable in `dtype`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    dO = _normal32(rng, (B, H, L, d))
    return round_to_bf16(dO) if dtype == "bf16" else dO


def make_config_inputs(cfg: FwdConfig) -> Dict[str, np.ndarray]:
    return make_fwd_inputs(cfg.B, cfg.H, cfg.L, cfg.d, cfg.dtype, cfg.p_softmax, cfg.seed,
                           n_runs=cfg.n_runs, run_len=cfg.run_len)


def make_decode_inputs(cfg: DecodeConfig, steps: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Initial decode state and the per-step token streams.

    state [B,H,d,d] f32 ~ N(0, state_std^2); k_cache (unit rows), v_cache
    [B,H,cap,d] with cap = len_hi + steps, filled up to cache_len[b,h]
    (one length per sequence, shared by its heads at step 0); q, k, v
    [steps,B,H,d]; alpha, beta [steps,B,H]; mask [steps,B,H] uint8.
    """
    steps = cfg.steps if steps is None else steps
    B, H, d = cfg.B, cfg.H, cfg.d
    cap = cfg.len_hi + steps
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    state = (cfg.state_std * rng.standard_normal((B, H, d, d))).astype(np.float32)
    lens = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=(B,))
    cache_len = np.repeat(lens[:, None], H, axis=1).astype(np.int32)
    k_cache = np.zeros((B, H, cap, d), dtype=np.float32)
    v_cache = np.zeros((B, H, cap, d), dtype=np.float32)
    for b in range(B):                      # only the live rows are drawn; the rest stay zero
        n = int(lens[b])
        k_cache[b, :, :n] = _unit_rows(_normal32(rng, (H, n, d)))
        v_cache[b, :, :n] = _normal32(rng, (H, n, d))
    if cfg.dtype == "bf16":
        k_cache, v_cache = round_to_bf16(k_cache), round_to_bf16(v_cache)
    q, k, v, alpha, beta = _qkv_gates(rng, (steps, B, H), d, cfg.dtype)
    mask = (rng.random((steps, B, H)) < cfg.p_softmax).astype(np.uint8)
    return {"state": state, "k_cache": k_cache, "v_cache": v_cache, "cache_len": cache_len,
            "q": q, "k": k, "v": v, "alpha": alpha, "beta": beta, "mask": mask, "cap": cap}
