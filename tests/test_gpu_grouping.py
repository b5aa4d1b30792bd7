"""GPU parity of head grouping (Section 4.3: G softmax heads share the mask of one linear head) against the
grouped oracle: both routings, both arithmetic paths, both merges, with and without softmax-branch queries and
keys of their own, initial and final state, the compacted cache, and a generation step after a grouped prefill."""
import numpy as np
import pytest
import torch

import paper_2602_03681_amd as nats
from gpu_util import TOL, host, rel_err, stored, to_dev
from nats_inputs import make_chunk_mask, make_fwd_inputs, round_to_bf16
from oracle import c_oracle
from oracle import nats_oracle as npo
from paper_2602_03681_amd import binding as nb

pytestmark = pytest.mark.gpu

ALL_OUT = ("final_state", "Kc", "Vc", "n_s", "idx", "cnt", "O_la", "O_nla", "lse")


def grouped_inputs(B, H, G, L, d, dtype, p, seed, own_qk, chunk):
    x = make_fwd_inputs(B, H, L, d, dtype, p, seed=seed)
    rng = np.random.default_rng(seed + 1000)
    rnd = (lambda a: round_to_bf16(a)) if dtype == "bf16" else (lambda a: a)
    x["V"] = rnd(rng.standard_normal((B, H * G, L, d)).astype(np.float32))
    if own_qk:
        x["Q_nla"] = rnd(rng.standard_normal((B, H * G, L, d)).astype(np.float32))
        x["K_nla"] = rnd(rng.standard_normal((B, H * G, L, d)).astype(np.float32))
    if chunk:
        x["mask"] = make_chunk_mask(B, H, L // 64, 0.4, seed + 1, "bernoulli")
    x["S0"] = (0.1 * rng.standard_normal((B, H * G, d, d))).astype(np.float32)
    x["w_nla"] = rng.random((B, H * G, L)).astype(np.float32)
    x["w_la"] = rng.random((B, H * G, L)).astype(np.float32)
    return x


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(torch.float32 if dtype == "f32" else torch.bfloat16)
    return t.cuda()


def run_gpu(x, G, dtype, chunk, mode, own_qk, math=nb.NATS_MATH_AUTO, want=ALL_OUT):
    g = to_dev({k: x[k] for k in ("Q", "K", "V", "alpha", "beta", "mask")}, dtype)
    kw = {}
    if own_qk:
        kw.update(Q_nla=dev(x["Q_nla"], dtype), K_nla=dev(x["K_nla"], dtype))
    if mode:
        kw.update(w_nla=dev(x["w_nla"]), w_la=dev(x["w_la"]))
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, want=want,
                                routing=nb.NATS_ROUTE_CHUNK if chunk else nb.NATS_ROUTE_TOKEN, combine_mode=mode,
                                initial_state=dev(x["S0"]), group=G, math=math, **kw)
    torch.cuda.synchronize()
    return r


def run_oracle(x, G, chunk, mode, own_qk):
    return npo.hybrid_fwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], G, C=64 if chunk else None,
                                  mode=mode, w_nla=x["w_nla"] if mode else None, w_la=x["w_la"] if mode else None,
                                  S0=x["S0"], Q_nla=x.get("Q_nla") if own_qk else None,
                                  K_nla=x.get("K_nla") if own_qk else None)


def check(r, ref, x, G, dtype, own_qk):
    for key, rk, st in (("O", "O", stored(dtype)), ("O_la", "O_la", None), ("O_nla", "O_nla", None),
                        ("final_state", "S", None)):
        e = rel_err(host(r[key]), ref[rk], st)
        assert e <= TOL[dtype], (key, e)
    np.testing.assert_array_equal(host(r["cnt"]), ref["cnt"])
    np.testing.assert_array_equal(host(r["n_s"]), ref["n_s"])
    lse, lse_ref = host(r["lse"]), ref["lse"]
    fin = np.isfinite(lse_ref)
    np.testing.assert_array_equal(np.isfinite(lse), fin)
    assert np.max(np.abs(lse[fin] - lse_ref[fin]), initial=0.0) <= (1e-4 if dtype == "f32" else 2e-2)
    Kc, Vc, idx = host(r["Kc"]), host(r["Vc"]), host(r["idx"])
    B, H = ref["n_s"].shape
    for b in range(B):
        for h in range(H):
            n = int(ref["n_s"][b, h])
            want_idx = np.asarray(ref["idx"][b][h][:n], dtype=np.int64)
            np.testing.assert_array_equal(idx[b, h, :n], want_idx)
            for g in range(G):   # every output head's cache rows: its own values, its own or the linear head's keys
                ksrc = x["K_nla"][b, h * G + g] if own_qk else x["K"][b, h]
                np.testing.assert_array_equal(Kc[b, h * G + g, :n], ksrc[want_idx])
                np.testing.assert_array_equal(Vc[b, h * G + g, :n], x["V"][b, h * G + g][want_idx])


@pytest.mark.parametrize("own_qk", [False, True])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("chunk", [False, True])
@pytest.mark.parametrize("G,dtype,d,L", [(2, "f32", 64, 256), (3, "bf16", 128, 512), (2, "bf16", 64, 320),
                                          (3, "f32", 128, 128)])
def test_grouped_forward(G, dtype, d, L, chunk, mode, own_qk):
    B, H = 1, 2
    x = grouped_inputs(B, H, G, L, d, dtype, 0.15, 300 + 7 * G + d + L, own_qk, chunk)
    r = run_gpu(x, G, dtype, chunk, mode, own_qk)
    check(r, run_oracle(x, G, chunk, mode, own_qk), x, G, dtype, own_qk)


def test_grouped_bf16_tensors_in_fp32_arithmetic():
    B, H, G, L, d = 1, 2, 2, 256, 64
    x = grouped_inputs(B, H, G, L, d, "bf16", 0.15, 411, True, False)
    r = run_gpu(x, G, "bf16", False, 0, True, math=nb.NATS_MATH_FP32)
    check(r, run_oracle(x, G, False, 0, True), x, G, "bf16", True)


@pytest.mark.parametrize("G", [2, 3])
def test_grouped_equals_repeated_heads_at_size(G):
    """Several segments, several query tiles, odd head counts: the grouped call against the C oracle on H G heads
    with the linear head's inputs repeated (what the grouping is defined to equal)."""
    B, H, L, d = 2, 3, 2048, 128
    x = grouped_inputs(B, H, G, L, d, "bf16", 0.06, 500 + G, False, False)
    g = to_dev({k: x[k] for k in ("Q", "K", "V", "alpha", "beta", "mask")}, "bf16")
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, group=G,
                                want=("O_la", "O_nla", "final_state"))
    torch.cuda.synchronize()
    rep = lambda a: np.repeat(a, G, axis=1)
    ref = c_oracle.fwd(rep(x["Q"]), rep(x["K"]), x["V"], rep(x["alpha"]), rep(x["beta"]), rep(x["mask"]),
                       want=("O_la", "O_nla", "S"))
    for key, rk, st in (("O", "O", "bf16"), ("O_la", "O_la", None), ("O_nla", "O_nla", None), ("final_state", "S", None)):
        e = rel_err(host(r[key]), ref[rk], st)
        assert e <= TOL["bf16"], (key, e)


def test_weights_by_eq22_per_output_head():
    B, H, G, L, d = 1, 2, 2, 256, 128
    x = grouped_inputs(B, H, G, L, d, "bf16", 0.15, 611, False, False)
    rng = np.random.default_rng(612)
    W = rng.standard_normal((H * G, 2, d)).astype(np.float32)
    g = to_dev({k: x[k] for k in ("Q", "K", "V", "alpha", "beta", "mask")}, "bf16")
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, group=G, combine_mode=1,
                                W_out=dev(W))
    torch.cuda.synchronize()
    wn = np.zeros((B, H * G, L))
    wl = np.zeros((B, H * G, L))
    for h in range(H):
        for gg in range(G):   # Eq. 22 on the linear head's query, one weight pair per output head
            a, b = npo.eq22_weights(x["Q"][:, h:h + 1], W[h * G + gg:h * G + gg + 1])
            wn[:, h * G + gg], wl[:, h * G + gg] = a[:, 0], b[:, 0]
    ref = npo.hybrid_fwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], G, mode=1, w_nla=wn, w_la=wl)
    e = rel_err(host(r["O"]), ref["O"], "bf16")
    assert e <= TOL["bf16"], e


def test_generation_step_after_a_grouped_prefill():
    """Prefill of L tokens with grouping, then one decode call on H G heads with the linear head's q, k, alpha,
    beta, mask repeated: equals token L of a grouped prefill of L + 1 tokens."""
    B, H, G, L, d = 1, 2, 2, 192, 64
    x = grouped_inputs(B, H, G, L + 64, d, "f32", 0.2, 711, False, False)
    cut = lambda a, n: np.ascontiguousarray(a[:, :, :n])
    xs = {k: cut(x[k], L) for k in ("Q", "K", "V", "alpha", "beta", "mask")}
    g = to_dev(xs, "f32")
    cap = L + 8
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, group=G,
                                want=("final_state", "Kc", "Vc", "n_s"), cap=cap)
    rep = lambda a: np.ascontiguousarray(np.repeat(a, G, axis=1))
    clen = torch.from_numpy(rep(host(r["n_s"]))).cuda()
    ref = npo.hybrid_fwd_grouped(*(cut(x[k], L + 1) for k in ("Q", "K", "V", "alpha", "beta", "mask")), G)
    o = nats.hybrid_attn_decode(r["final_state"], r["Kc"], r["Vc"], clen, dev(rep(x["Q"][:, :, L])),
                                dev(rep(x["K"][:, :, L])), dev(np.ascontiguousarray(x["V"][:, :, L])),
                                dev(rep(x["alpha"][:, :, L])), dev(rep(x["beta"][:, :, L])), dev(rep(x["mask"][:, :, L])))
    torch.cuda.synchronize()
    e = rel_err(host(o), ref["O"][:, :, L], None)
    assert e <= TOL["f32"], e
