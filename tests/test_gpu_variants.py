"""GPU parity for the variants of the linear branch: Mamba2-style gated linear attention (appendix
"Mixture of SoftmaxAttention and Mamba2 architecture") and the ablation without decay on softmax tokens /
chunks (Section 5, Ablation Study (ii)), through the C ABI against the CPU oracle, same bars as the method
itself: forward with routing per token and per chunk on both arithmetic paths, and generation."""
import numpy as np
import pytest
import torch

import paper_2602_03681_amd as nats
from paper_2602_03681_amd import binding as nb
from nats_inputs import DecodeConfig, make_chunk_mask, make_decode_inputs, make_fwd_inputs
from oracle import c_oracle
from oracle import nats_oracle as npo

from gpu_util import TOL, host, rel_err, stored, to_dev
from test_gpu_parity import ALL_OUT, check_all

pytestmark = pytest.mark.gpu
VARIANTS = [(nb.NATS_LINEAR_GATED, 0), (nb.NATS_LINEAR_GDN, 1), (nb.NATS_LINEAR_GATED, 1)]


def fwd_both(x, dtype, op, freeze, chunk=False, **kw):
    g = to_dev(x, dtype)
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, want=ALL_OUT,
                                routing=nb.NATS_ROUTE_CHUNK if chunk else nb.NATS_ROUTE_TOKEN, linear_op=op,
                                freeze_on_softmax=bool(freeze), **kw)
    torch.cuda.synchronize()
    ref = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], chunk_routing=64 if chunk else 0,
                       linear_op=op, freeze_on_softmax=freeze)
    return r, ref


@pytest.mark.parametrize("op,freeze", VARIANTS)
@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f32", 128), ("bf16", 64), ("bf16", 128)])
def test_variants_routing_per_token(dtype, d, op, freeze):
    x = make_fwd_inputs(2, 3, 1088 if dtype == "bf16" else 320, d, dtype, 0.15, seed=41 + d + op)
    r, ref = fwd_both(x, dtype, op, freeze)
    check_all(x, dtype, r, ref)
    # the variant is not a no-op on these inputs
    base = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], want=())
    assert rel_err(base["O"], ref["O"]) > 10 * TOL[dtype]


@pytest.mark.parametrize("op,freeze", VARIANTS)
@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128), ("bf16", 64)])
def test_variants_routing_per_chunk(dtype, d, op, freeze):
    L = 1024 if dtype == "bf16" else 320
    x = make_fwd_inputs(2, 2, L, d, dtype, 0.1, seed=51 + d + op)
    x["mask"] = make_chunk_mask(2, 2, L // 64, 0.4, 60 + d, "bernoulli")
    r, ref = fwd_both(x, dtype, op, freeze, chunk=True)
    check_all(x, dtype, r, ref)


def test_variants_fp32_arithmetic_on_bf16_tensors_and_eq21():
    x = make_fwd_inputs(1, 2, 256, 64, "bf16", 0.2, seed=71)
    rng = np.random.default_rng(7)
    w = rng.random((2, 1, 2, 256)).astype(np.float32)
    g = to_dev(x, "bf16")
    for math in (nb.NATS_MATH_AUTO, nb.NATS_MATH_FP32):
        r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, want=(), math=math,
                                    combine_mode=1, w_nla=torch.from_numpy(w[0]).cuda(), w_la=torch.from_numpy(w[1]).cuda(),
                                    linear_op=nb.NATS_LINEAR_GATED, freeze_on_softmax=True)
        torch.cuda.synchronize()
        ref = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], mode=1, w_nla=w[0], w_la=w[1],
                           linear_op=1, freeze_on_softmax=1, want=())
        assert rel_err(host(r["O"]), ref["O"], "bf16") <= TOL["bf16"]


@pytest.mark.parametrize("op,freeze", VARIANTS)
@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_variants_decode_steps(dtype, d, op, freeze):
    cfg = DecodeConfig("small", 3, 2, d, dtype, 0.3, seed=81 + d + op, len_lo=1, len_hi=70, steps=24)
    x = make_decode_inputs(cfg, steps=cfg.steps)
    g = to_dev(x, dtype)
    state, kc, vc, clen = g["state"].clone(), g["k_cache"].clone(), g["v_cache"].clone(), g["cache_len"].clone()
    S_ref = x["state"].astype(np.float64)
    kc_ref, vc_ref, clen_ref = x["k_cache"].copy(), x["v_cache"].copy(), x["cache_len"].copy()
    for s in range(cfg.steps):
        o = nats.hybrid_attn_decode(state, kc, vc, clen, g["q"][s], g["k"][s], g["v"][s], g["alpha"][s], g["beta"][s],
                                    g["mask"][s], linear_op=op, freeze_on_softmax=bool(freeze))
        o_ref, _ = c_oracle.decode(S_ref, kc_ref, vc_ref, clen_ref, x["q"][s], x["k"][s], x["v"][s], x["alpha"][s],
                                   x["beta"][s], x["mask"][s], linear_op=op, freeze_on_softmax=freeze)
        assert rel_err(host(o), o_ref, stored(dtype)) <= TOL[dtype], f"step {s}"
    torch.cuda.synchronize()
    assert rel_err(host(state), S_ref) <= TOL[dtype]
    np.testing.assert_array_equal(host(clen), clen_ref)


@pytest.mark.parametrize("op,freeze", [(nb.NATS_LINEAR_GATED, 1), (nb.NATS_LINEAR_GDN, 1)])
def test_variants_generation_per_chunk_with_commits(op, freeze):
    """Two chunks generated token by token under routing per chunk (one softmax, one linear), every token and
    the state after each commit against the numpy oracle's generation functions."""
    B, H, d, cap, C = 1, 2, 64, 192, 64
    x = make_fwd_inputs(B, H, 2 * C, d, "f32", 0.0, seed=93)
    g = to_dev(x, "f32")
    st = {"state": torch.zeros((B, H, d, d), device="cuda"), "state_start": torch.zeros((B, H, d, d), device="cuda"),
          "chunk_decay": torch.ones((B, H), device="cuda"), "chunk_pos": torch.zeros((B, H), dtype=torch.int32, device="cuda"),
          "k_cache": torch.zeros((B, H, cap, d), device="cuda"), "v_cache": torch.zeros((B, H, cap, d), device="cuda"),
          "cache_len": torch.zeros((B, H), dtype=torch.int32, device="cuda")}
    ref = [[npo.decode_chunk_state(np.zeros((d, d)), np.zeros((cap, d)), np.zeros((cap, d)), 0) for _ in range(H)]
           for _ in range(B)]
    decisions = [np.array([[1, 0]], dtype=np.uint8), np.array([[0, 1]], dtype=np.uint8)]
    for c in range(2):
        for t in range(c * C, (c + 1) * C):
            o = nats.hybrid_attn_decode_chunk(st, g["Q"][:, :, t].contiguous(), g["K"][:, :, t].contiguous(),
                                              g["V"][:, :, t].contiguous(), g["alpha"][:, :, t].contiguous(),
                                              g["beta"][:, :, t].contiguous(), linear_op=op)
            for b in range(B):
                for h in range(H):
                    o_ref, _ = npo.decode_step_chunk_routed(ref[b][h], x["Q"][b, h, t], x["K"][b, h, t], x["V"][b, h, t],
                                                            x["alpha"][b, h, t], x["beta"][b, h, t], linear_op=op)
                    assert rel_err(host(o)[b, h], o_ref) <= TOL["f32"], (c, t, b, h)
        nats.hybrid_attn_decode_commit(st, torch.from_numpy(decisions[c]).cuda(), freeze_on_softmax=bool(freeze))
        torch.cuda.synchronize()
        for b in range(B):
            for h in range(H):
                npo.decode_commit_chunk(ref[b][h], int(decisions[c][b, h]), decay_on_softmax=not freeze)
                assert rel_err(host(st["state"])[b, h], ref[b][h]["S"]) <= TOL["f32"]
                assert int(host(st["cache_len"])[b, h]) == ref[b][h]["cache_len"]


# ---- queries and keys of the softmax branch given apart (Section 4.3: L2-normalised q, k for the linear
#      operation, RMS-normalised / rotated ones for softmax attention; V shared) ---------------------------

def nla_inputs(shape, dtype, seed):
    from nats_inputs import round_to_bf16
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(shape).astype(np.float32)
    b = rng.standard_normal(shape).astype(np.float32)
    return (round_to_bf16(a), round_to_bf16(b)) if dtype == "bf16" else (a, b)


@pytest.mark.parametrize("chunk", [False, True])
@pytest.mark.parametrize("dtype,d,L", [("f32", 64, 256), ("bf16", 128, 512), ("bf16", 64, 320)])
def test_separate_softmax_queries_and_keys_forward(dtype, d, L, chunk):
    B, H = 1, 2
    x = make_fwd_inputs(B, H, L, d, dtype, 0.15, seed=111 + d)
    if chunk:
        x["mask"] = make_chunk_mask(B, H, L // 64, 0.4, 112, "bernoulli")
    Qn, Kn = nla_inputs((B, H, L, d), dtype, 113)
    g = to_dev(x, dtype)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, want=ALL_OUT,
                                routing=nb.NATS_ROUTE_CHUNK if chunk else nb.NATS_ROUTE_TOKEN,
                                Q_nla=torch.from_numpy(Qn).to(tdt).cuda(), K_nla=torch.from_numpy(Kn).to(tdt).cuda())
    torch.cuda.synchronize()
    if chunk:
        ref = npo.hybrid_fwd_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], 64, Q_nla=Qn, K_nla=Kn)
    else:
        ref = npo.hybrid_fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], Q_nla=Qn, K_nla=Kn)
    for key, rk, st in (("O", "O", stored(dtype)), ("O_la", "O_la", None), ("O_nla", "O_nla", None), ("final_state", "S", None)):
        assert rel_err(host(r[key]), ref[rk], st) <= TOL[dtype], key
    np.testing.assert_array_equal(host(r["n_s"]), ref["n_s"])
    Kc = host(r["Kc"])
    for h in range(H):   # the compacted cache holds the softmax branch's keys
        n = int(ref["n_s"][0, h])
        np.testing.assert_array_equal(Kc[0, h, :n], Kn[0, h, np.asarray(ref["idx"][0][h][:n], dtype=np.int64)])


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_separate_softmax_queries_and_keys_decode(dtype, d):
    cfg = DecodeConfig("small", 2, 2, d, dtype, 0.4, seed=121 + d, len_lo=1, len_hi=40, steps=12)
    x = make_decode_inputs(cfg, steps=cfg.steps)
    g = to_dev(x, dtype)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    qn, kn = nla_inputs((cfg.steps, cfg.B, cfg.H, d), dtype, 122)
    gq, gk = torch.from_numpy(qn).to(tdt).cuda(), torch.from_numpy(kn).to(tdt).cuda()
    state, kc, vc, clen = g["state"].clone(), g["k_cache"].clone(), g["v_cache"].clone(), g["cache_len"].clone()
    ref = [[dict(S=x["state"][b, h].astype(np.float64), kc=x["k_cache"][b, h].astype(np.float64),
                 vc=x["v_cache"][b, h].astype(np.float64), n=int(x["cache_len"][b, h])) for h in range(cfg.H)]
           for b in range(cfg.B)]
    for s in range(cfg.steps):
        o = nats.hybrid_attn_decode(state, kc, vc, clen, g["q"][s], g["k"][s], g["v"][s], g["alpha"][s], g["beta"][s],
                                    g["mask"][s], q_nla=gq[s].contiguous(), k_nla=gk[s].contiguous())
        oh = host(o)
        for b in range(cfg.B):
            for h in range(cfg.H):
                st = ref[b][h]
                o_ref, st["S"], st["kc"], st["vc"], st["n"], _ = npo.decode_step(
                    st["S"], st["kc"], st["vc"], st["n"], x["q"][s, b, h], x["k"][s, b, h], x["v"][s, b, h],
                    x["alpha"][s, b, h], x["beta"][s, b, h], x["mask"][s, b, h], q_nla=qn[s, b, h], k_nla=kn[s, b, h])
                rms = max(float(np.sqrt(np.mean(o_ref ** 2))), 1e-6)
                diff = np.abs(oh[b, h] - o_ref)
                if dtype == "bf16":
                    from gpu_util import bf16_half_ulp
                    diff = np.maximum(diff - bf16_half_ulp(o_ref), 0.0)
                assert diff.max() / rms <= TOL[dtype], (s, b, h)
    torch.cuda.synchronize()
    for b in range(cfg.B):
        for h in range(cfg.H):
            assert int(host(clen)[b, h]) == ref[b][h]["n"]


@pytest.mark.parametrize("dtype,d,math", [("f32", 64, 0), ("bf16", 128, 0), ("bf16", 64, 1)])
def test_single_normalisation_merge(dtype, d, math):
    """combine_mode 2 (Section 5, ablation (iii)): RMSNorm of the weighted sum, forward and decode."""
    B, H, L = 1, 2, 320
    x = make_fwd_inputs(B, H, L, d, dtype, 0.15, seed=131 + d)
    w = (np.random.default_rng(132).random((2, B, H, L)) + 0.5).astype(np.float32)
    g = to_dev(x, dtype)
    for given in (True, False):
        kw = dict(w_nla=torch.from_numpy(w[0]).cuda(), w_la=torch.from_numpy(w[1]).cuda()) if given else {}
        r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, want=(), combine_mode=2,
                                    math=nb.NATS_MATH_FP32 if math else nb.NATS_MATH_AUTO, **kw)
        torch.cuda.synchronize()
        ref = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], mode=2,
                           w_nla=w[0] if given else None, w_la=w[1] if given else None, want=())
        assert rel_err(host(r["O"]), ref["O"], stored(dtype)) <= TOL[dtype], given
    # decode
    cfg = DecodeConfig("small", 2, 2, d, dtype, 0.4, seed=133, len_lo=1, len_hi=30, steps=6)
    xd = make_decode_inputs(cfg, steps=cfg.steps)
    gd = to_dev(xd, dtype)
    state, kc, vc, clen = gd["state"].clone(), gd["k_cache"].clone(), gd["v_cache"].clone(), gd["cache_len"].clone()
    S_ref, kc_ref, vc_ref, cl_ref = xd["state"].astype(np.float64), xd["k_cache"].copy(), xd["v_cache"].copy(), xd["cache_len"].copy()
    wd = (np.random.default_rng(134).random((2, cfg.steps, cfg.B, cfg.H)) + 0.5).astype(np.float32)
    for s in range(cfg.steps):
        o = nats.hybrid_attn_decode(state, kc, vc, clen, gd["q"][s], gd["k"][s], gd["v"][s], gd["alpha"][s], gd["beta"][s],
                                    gd["mask"][s], combine_mode=2, w_nla=torch.from_numpy(wd[0, s]).cuda(),
                                    w_la=torch.from_numpy(wd[1, s]).cuda())
        o_ref, _ = c_oracle.decode(S_ref, kc_ref, vc_ref, cl_ref, xd["q"][s], xd["k"][s], xd["v"][s], xd["alpha"][s],
                                   xd["beta"][s], xd["mask"][s], mode=2, w_nla=wd[0, s], w_la=wd[1, s])
        assert rel_err(host(o), o_ref, stored(dtype)) <= TOL[dtype], s


# ---- Section 5, ablation (i): the inner part of a chunk by one operation only; (v): weights from the features ----
@pytest.mark.parametrize("inner", [1, 2])
@pytest.mark.parametrize("dtype,d,L,math", [("f32", 64, 256, 0), ("bf16", 128, 512, 0), ("bf16", 64, 320, 0),
                                            ("bf16", 64, 256, 1)])
def test_inner_part_of_a_chunk_by_one_operation(dtype, d, L, math, inner):
    B, H = 1, 2
    x = make_fwd_inputs(B, H, L, d, dtype, 0.15, seed=900 + d + L)
    x["mask"] = make_chunk_mask(B, H, L // 64, 0.4, 901 + inner, "bernoulli")
    S0 = (0.1 * np.random.default_rng(902).standard_normal((B, H, d, d))).astype(np.float32)
    g = to_dev(x, dtype)
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, want=ALL_OUT,
                                routing=nb.NATS_ROUTE_CHUNK, inner_chunk=inner, math=math,
                                initial_state=torch.from_numpy(S0).cuda())
    torch.cuda.synchronize()
    ref = npo.hybrid_fwd_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], 64, S0=S0, inner=inner)
    for key, rk, st in (("O", "O", stored(dtype)), ("O_la", "O_la", None), ("O_nla", "O_nla", None), ("final_state", "S", None)):
        e = rel_err(host(r[key]), ref[rk], st)
        assert e <= TOL[dtype], (key, e)
    lse, lse_ref = host(r["lse"]), ref["lse"]
    fin = np.isfinite(lse_ref)
    np.testing.assert_array_equal(np.isfinite(lse), fin)     # inner = 2: queries before the first softmax chunk see nothing
    assert np.max(np.abs(lse[fin] - lse_ref[fin]), initial=0.0) <= (1e-4 if dtype == "f32" else 2e-2)
    np.testing.assert_array_equal(host(r["cnt"]), ref["cnt"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("act", [nb.NATS_WEIGHTS_SOFTMAX, nb.NATS_WEIGHTS_SIGMOID, nb.NATS_WEIGHTS_LINEAR])
def test_merge_weights_from_the_input_features(dtype, act):
    from nats_inputs import round_to_bf16
    B, L, dm, H = 2, 192, 1032, 6
    rng = np.random.default_rng(910 + act)
    X = rng.standard_normal((B, L, dm)).astype(np.float32)
    if dtype == "bf16":
        X = round_to_bf16(X)
    W = (rng.standard_normal((H, 2, dm)) / np.sqrt(dm)).astype(np.float32)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    wn, wl = nb.merge_weights_from_x(torch.from_numpy(X).to(tdt).cuda(), torch.from_numpy(W).cuda(), act)
    torch.cuda.synchronize()
    rn, rl = npo.weights_from_x(X, W, act)
    assert np.max(np.abs(host(wn) - rn)) <= 1e-5 and np.max(np.abs(host(wl) - rl)) <= 1e-5
