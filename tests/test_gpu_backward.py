"""GPU parity of the backward pass (Section 4.2; fp32-accurate gradients, routing per token, plain-sum merge) against
the backward oracle, through the C ABI.  Every gradient tensor is held to max|err| / RMS(oracle) <= 1e-4 (the
outputs are fp32 whatever the input dtype).  The linear branch's adjoint runs by chunks of 64
tokens on fp32 matrix instructions (the default) or token by token (math = NATS_MATH_FP32), with either routing: both
are held to the same bar."""
import numpy as np
import pytest
import torch

import paper_2602_03681_amd as nats
from paper_2602_03681_amd import binding as nb
from nats_inputs import make_chunk_mask, make_fwd_inputs, make_grad_output
from oracle import nats_oracle_bwd as nbw

from gpu_util import host, rel_err, to_dev

pytestmark = pytest.mark.gpu
TOL_BWD = 1e-4
KEYS = (("dQ", "dQ"), ("dK", "dK"), ("dV", "dV"), ("dalpha", "dalpha"), ("dbeta", "dbeta"))


def run_bwd(x, dO, dtype, want=("d_initial_state", "g_nla"), S0=None, **kw):
    g = to_dev(x, dtype)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    r = nats.hybrid_attn_bwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"],
                             torch.from_numpy(dO).to(tdt).cuda(), want=want,
                             initial_state=None if S0 is None else torch.from_numpy(S0.astype(np.float32)).cuda(), **kw)
    torch.cuda.synchronize()
    return r


def check(r, ref, extra=()):
    errs = {}
    for got, want in KEYS + tuple(extra):
        a, b = host(r[got]), ref[want]
        if np.all(b == 0):
            assert np.all(a == 0), got          # e.g. dbeta when nothing is ever written
            continue
        errs[got] = rel_err(a, b)
    for k, e in errs.items():
        assert e <= TOL_BWD, f"{k}: {e:.3e} (all: {errs})"
    return errs


@pytest.mark.parametrize("dtype,B,H,L,d,p", [("f32", 1, 2, 320, 64, 0.15), ("f32", 2, 2, 256, 128, 0.1),
                                             ("bf16", 1, 3, 1088, 64, 0.08), ("bf16", 1, 2, 448, 128, 0.2),
                                             ("f32", 1, 1, 64, 64, 0.5),
                                             # many key tiles, several query tiles per block share (MFMA dK / dV kernel)
                                             ("bf16", 1, 1, 2048, 128, 0.3), ("bf16", 2, 2, 1024, 64, 0.5)])
@pytest.mark.parametrize("math", [nb.NATS_MATH_AUTO, nb.NATS_MATH_FP32], ids=["by_chunks", "by_tokens"])
def test_backward_matches_the_oracle(dtype, B, H, L, d, p, math):
    x = make_fwd_inputs(B, H, L, d, dtype, p, seed=200 + L + d)
    dO = make_grad_output(B, H, L, d, dtype, seed=300 + L)
    S0 = (0.05 * np.random.default_rng(L).standard_normal((B, H, d, d))).astype(np.float32)
    r = run_bwd(x, dO, dtype, S0=S0, math=math)
    ref = nbw.hybrid_bwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, S0=S0)
    errs = check(r, ref, extra=(("d_initial_state", "dS0"), ("g_nla", "g_nla")))
    print(dtype, L, d, errs)
    # Section 4.2: nothing for the operation a token is inactive for
    soft = x["mask"] != 0
    assert np.all(host(r["dbeta"])[soft] == 0)
    assert np.all(host(r["g_nla"])[~soft] == 0)


@pytest.mark.parametrize("dtype,B,H,L,d,p", [("f32", 1, 2, 320, 64, 0.15), ("bf16", 1, 2, 448, 128, 0.2)])
@pytest.mark.parametrize("ask", ["all", "chunk sums only"])
def test_score_gradients_per_token_and_per_chunk(dtype, B, H, L, d, p, ask):
    """Eq. 16 and Eq. 17: the column sums of the softmax mask gradient, the linear operation's sum of dS . (written),
    and their sums per chunk of 64 tokens (asked for alone, the per-token sums live in the workspace)."""
    x = make_fwd_inputs(B, H, L, d, dtype, p, seed=700 + L)
    dO = make_grad_output(B, H, L, d, dtype, seed=701)
    want = ("g_nla", "g_la", "dscore_nla", "dscore_la") if ask == "all" else ("dscore_nla", "dscore_la")
    r = run_bwd(x, dO, dtype, want=want)
    ref = nbw.hybrid_bwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO)
    ref["dscore_nla"], ref["dscore_la"] = nbw.score_gradients(ref["g_nla"], ref["g_la"], 64)
    for key in want:
        e = rel_err(host(r[key]), ref[key])
        assert e <= TOL_BWD, (key, e)
    if ask == "all":
        assert np.all(host(r["g_la"])[x["mask"] != 0] == 0)


@pytest.mark.parametrize("linear_op,freeze", [(nb.NATS_LINEAR_GATED, False), (nb.NATS_LINEAR_GDN, True),
                                              (nb.NATS_LINEAR_GATED, True)])
@pytest.mark.parametrize("math", [nb.NATS_MATH_AUTO, nb.NATS_MATH_FP32], ids=["by_chunks", "by_tokens"])
def test_backward_variants_and_scales(linear_op, freeze, math):
    B, H, L, d = 1, 2, 256, 64
    x = make_fwd_inputs(B, H, L, d, "f32", 0.2, seed=410 + linear_op)
    dO = make_grad_output(B, H, L, d, "f32", seed=411)
    r = run_bwd(x, dO, "f32", softmax_scale=0.3, la_scale=1.7, linear_op=linear_op, freeze_on_softmax=freeze, math=math)
    ref = nbw.hybrid_bwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, softmax_scale=0.3, la_scale=1.7,
                         linear_op=linear_op, decay_on_softmax=not freeze)
    check(r, ref, extra=(("d_initial_state", "dS0"), ("g_nla", "g_nla")))
    if freeze:   # no decay on softmax tokens: their alpha has no effect at all
        assert np.all(host(r["dalpha"])[x["mask"] != 0] == 0)


@pytest.mark.parametrize("kind", ["all_softmax", "all_linear"])
@pytest.mark.parametrize("math", [nb.NATS_MATH_AUTO, nb.NATS_MATH_FP32], ids=["by_chunks", "by_tokens"])
def test_backward_degenerate_masks(kind, math):
    B, H, L, d = 1, 2, 192, 64
    x = make_fwd_inputs(B, H, L, d, "f32", 0.1, seed=420)
    x["mask"][:] = 1 if kind == "all_softmax" else 0
    dO = make_grad_output(B, H, L, d, "f32", seed=421)
    r = run_bwd(x, dO, "f32", math=math)
    ref = nbw.hybrid_bwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO)
    check(r, ref, extra=(("g_nla", "g_nla"),) if kind == "all_softmax" else ())
    if kind == "all_linear":
        assert np.all(host(r["g_nla"]) == 0)


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_backward_by_chunks_with_gates_at_their_ends(dtype, d):
    """Write strengths of exactly 0 and 1 on linear tokens, strong and no decay inside one chunk: the chunkwise form
    divides by no gate but alpha itself (dalpha comes through ln gamma)."""
    B, H, L = 1, 2, 256
    x = make_fwd_inputs(B, H, L, d, dtype, 0.2, seed=440)
    rng = np.random.default_rng(441)
    x["beta"][..., ::7] = 0.0
    x["beta"][..., 3::7] = 1.0
    x["alpha"][..., ::5] = 1.0
    x["alpha"][..., 2::11] = rng.uniform(0.01, 0.2, x["alpha"][..., 2::11].shape).astype(np.float32)
    dO = make_grad_output(B, H, L, d, dtype, seed=442)
    r = run_bwd(x, dO, dtype)
    ref = nbw.hybrid_bwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO)
    check(r, ref, extra=(("d_initial_state", "dS0"), ("g_nla", "g_nla")))
    lin0 = (x["mask"] == 0) & (x["beta"] == 0)
    assert lin0.any() and np.any(host(r["dbeta"])[lin0] != 0)   # a linear token with beta = 0 still has a gradient for it


def test_backward_at_the_headline_size_on_sampled_heads():
    """The shapes and launch configuration bench.py --backward times (B=2, H=16, L=8192, d=128, bf16): the oracle
    recomputes the first and the last (batch, head) in full; 128 chunks of state and state gradient in a row."""
    from nats_inputs import CONFIGS, make_config_inputs
    cfg = CONFIGS["cfg2_headline_bf16"]
    x = make_config_inputs(cfg)
    dO = make_grad_output(cfg.B, cfg.H, cfg.L, cfg.d, "bf16", seed=cfg.seed + 1)
    r = run_bwd(x, dO, "bf16", want=("d_initial_state", "g_nla", "g_la"))
    for b, h in ((0, 0), (cfg.B - 1, cfg.H - 1)):
        ref = nbw.hybrid_head_bwd(x["Q"][b, h], x["K"][b, h], x["V"][b, h], x["alpha"][b, h], x["beta"][b, h],
                                  x["mask"][b, h], dO[b, h])
        errs = {}
        for got, want in KEYS + (("d_initial_state", "dS0"), ("g_nla", "g_nla"), ("g_la", "g_la")):
            errs[got] = rel_err(host(r[got][b, h]), ref[want])
        print((b, h), errs)
        for k, e in errs.items():
            assert e <= TOL_BWD, f"{(b, h)} {k}: {e:.3e} (all: {errs})"


@pytest.mark.parametrize("routing", [nb.NATS_ROUTE_TOKEN, nb.NATS_ROUTE_CHUNK], ids=["per_token", "per_chunk"])
def test_backward_long_sequence_both_forms_agree(routing):
    """L = 32768 (512 chunks in a row), beyond what the oracle recomputes in seconds: the two forms of the linear
    branch's adjoint, which share no kernel of that branch (fp32 vector arithmetic token by token; fp32 matrix
    instructions by chunks), must give the same gradients; each is held to the oracle at the shorter lengths above."""
    B, H, L, d = 1, 3, 32768, 128
    x = make_fwd_inputs(B, H, L, d, "bf16", 0.05, seed=450)
    if routing == nb.NATS_ROUTE_CHUNK:
        x["mask"] = make_chunk_mask(B, H, L // 64, 0.05, 451, "bernoulli")
    dO = make_grad_output(B, H, L, d, "bf16", seed=452)
    want = ("d_initial_state",)
    a = run_bwd(x, dO, "bf16", want=want, routing=routing, math=nb.NATS_MATH_AUTO)
    b = run_bwd(x, dO, "bf16", want=want, routing=routing, math=nb.NATS_MATH_FP32)
    for k in ("dQ", "dK", "dV", "dalpha", "dbeta", "d_initial_state"):
        ya, yb = host(a[k]), host(b[k])
        assert np.all(np.isfinite(ya)) and np.all(np.isfinite(yb)), k
        e = rel_err(ya, yb)
        assert e <= TOL_BWD, f"{k}: {e:.3e}"


def test_backward_is_deterministic_and_reuses_a_poisoned_workspace():
    B, H, L, d = 1, 2, 256, 128
    x = make_fwd_inputs(B, H, L, d, "bf16", 0.1, seed=430)
    dO = make_grad_output(B, H, L, d, "bf16", seed=431)
    prm = nb.make_fwd_params(B, H, L, d, 64, nb.NATS_BF16)
    n = int(nb.load_library().nats_hybrid_attn_bwd_workspace_bytes(__import__("ctypes").byref(prm)))
    ws = torch.full((n,), 0xFF, dtype=torch.uint8, device="cuda")
    r1 = run_bwd(x, dO, "bf16", workspace=ws)
    r2 = run_bwd(x, dO, "bf16")
    for k in ("dQ", "dK", "dV", "dalpha", "dbeta", "g_nla", "d_initial_state"):
        assert torch.equal(r1[k], r2[k]), k


# ---- routing per chunk (Section 4.1 as stated): both operations compute every chunk's inner part, the masks act
#      between chunks; score gradients per chunk (Eq. 16, Eq. 17) ---------------------------------------------------
CHUNK_KEYS = (("d_initial_state", "dS0"), ("dscore_nla", "dscore_nla"), ("dscore_la", "dscore_la"))


@pytest.mark.parametrize("dtype,B,H,L,d,p", [("f32", 1, 2, 256, 64, 0.4), ("f32", 1, 1, 192, 128, 0.3),
                                             ("bf16", 2, 2, 512, 64, 0.3), ("bf16", 1, 2, 448, 128, 0.25),
                                             ("bf16", 1, 1, 1024, 128, 0.5)])
@pytest.mark.parametrize("math", [nb.NATS_MATH_AUTO, nb.NATS_MATH_FP32], ids=["by_chunks", "by_tokens"])
def test_backward_with_routing_per_chunk(dtype, B, H, L, d, p, math):
    x = make_fwd_inputs(B, H, L, d, dtype, 0.1, seed=800 + L + d)
    x["mask"] = make_chunk_mask(B, H, L // 64, p, 801 + L, "bernoulli")
    dO = make_grad_output(B, H, L, d, dtype, seed=802 + L)
    S0 = (0.05 * np.random.default_rng(L + 1).standard_normal((B, H, d, d))).astype(np.float32)
    r = run_bwd(x, dO, dtype, S0=S0, routing=nb.NATS_ROUTE_CHUNK, want=("d_initial_state", "dscore_nla", "dscore_la"),
                math=math)
    ref = nbw.hybrid_bwd_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], 64, dO, S0=S0)
    errs = check(r, ref, extra=CHUNK_KEYS)
    print(dtype, L, d, errs)
    # Section 4.2: no score gradient for the operation a chunk is inactive for
    soft = x["mask"] != 0
    assert np.all(host(r["dscore_la"])[soft] == 0) and np.all(host(r["dscore_nla"])[~soft] == 0)


@pytest.mark.parametrize("linear_op,freeze", [(nb.NATS_LINEAR_GATED, False), (nb.NATS_LINEAR_GDN, True)])
@pytest.mark.parametrize("math", [nb.NATS_MATH_AUTO, nb.NATS_MATH_FP32], ids=["by_chunks", "by_tokens"])
def test_backward_with_routing_per_chunk_variants(linear_op, freeze, math):
    B, H, L, d = 1, 2, 256, 64
    x = make_fwd_inputs(B, H, L, d, "f32", 0.1, seed=810 + linear_op)
    x["mask"] = make_chunk_mask(B, H, L // 64, 0.5, 811, "bernoulli")
    dO = make_grad_output(B, H, L, d, "f32", seed=812)
    r = run_bwd(x, dO, "f32", routing=nb.NATS_ROUTE_CHUNK, softmax_scale=0.3, la_scale=1.7, linear_op=linear_op,
                freeze_on_softmax=freeze, want=("d_initial_state", "dscore_nla", "dscore_la"), math=math)
    ref = nbw.hybrid_bwd_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], 64, dO, softmax_scale=0.3,
                                      la_scale=1.7, linear_op=linear_op, decay_on_softmax=not freeze)
    check(r, ref, extra=CHUNK_KEYS)


@pytest.mark.parametrize("kind", ["all_softmax", "all_linear"])
@pytest.mark.parametrize("math", [nb.NATS_MATH_AUTO, nb.NATS_MATH_FP32], ids=["by_chunks", "by_tokens"])
def test_backward_with_routing_per_chunk_degenerate_masks(kind, math):
    B, H, L, d = 1, 2, 192, 64
    x = make_fwd_inputs(B, H, L, d, "f32", 0.1, seed=820)
    x["mask"] = np.full((B, H, L // 64), 1 if kind == "all_softmax" else 0, dtype=np.uint8)
    dO = make_grad_output(B, H, L, d, "f32", seed=821)
    r = run_bwd(x, dO, "f32", routing=nb.NATS_ROUTE_CHUNK, want=("dscore_nla", "dscore_la"), math=math)
    ref = nbw.hybrid_bwd_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], 64, dO)
    check(r, ref, extra=CHUNK_KEYS[1:])


# ---- head grouping (Section 4.3): G output heads share the Q, K, alpha, beta and mask of a linear head ----------------
@pytest.mark.parametrize("dtype,B,H,G,L,d", [("f32", 1, 2, 2, 256, 64), ("bf16", 2, 1, 3, 320, 128),
                                             ("bf16", 1, 2, 2, 512, 64)])
@pytest.mark.parametrize("routing", ["token", "chunk"])
def test_backward_with_head_grouping(dtype, B, H, G, L, d, routing):
    """V, dO, dV and the states have H G heads; the gradients of the shared inputs (and the score gradients) are sums
    over the heads of a group."""
    x = make_fwd_inputs(B, H, L, d, dtype, 0.15, seed=900 + L + G)
    xv = make_fwd_inputs(B, H * G, L, d, dtype, 0.15, seed=901 + L + G)
    x["V"] = xv["V"]
    dO = make_grad_output(B, H * G, L, d, dtype, seed=902 + L)
    S0 = (0.05 * np.random.default_rng(L + G).standard_normal((B, H * G, d, d))).astype(np.float32)
    if routing == "chunk":
        x["mask"] = make_chunk_mask(B, H, L // 64, 0.35, 903 + L, "bernoulli")
        want = ("d_initial_state", "dscore_nla", "dscore_la")
        r = run_bwd(x, dO, dtype, S0=S0, routing=nb.NATS_ROUTE_CHUNK, want=want, group=G)
        ref = nbw.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, C=64, S0=S0)
        extra = CHUNK_KEYS
    else:
        want = ("d_initial_state", "g_nla", "g_la", "dscore_nla", "dscore_la")
        r = run_bwd(x, dO, dtype, S0=S0, want=want, group=G)
        ref = nbw.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, S0=S0)
        ref["dscore_nla"], ref["dscore_la"] = nbw.score_gradients(ref["g_nla"], ref["g_la"], 64)
        extra = (("d_initial_state", "dS0"), ("g_nla", "g_nla"), ("g_la", "g_la"), ("dscore_nla", "dscore_nla"),
                 ("dscore_la", "dscore_la"))
    assert tuple(r["dV"].shape) == (B, H * G, L, d) and tuple(r["dQ"].shape) == (B, H, L, d)
    errs = check(r, ref, extra=extra)
    print(dtype, G, routing, errs)


def test_head_grouping_of_one_is_the_plain_backward():
    B, H, L, d = 1, 2, 256, 64
    x = make_fwd_inputs(B, H, L, d, "bf16", 0.2, seed=950)
    dO = make_grad_output(B, H, L, d, "bf16", seed=951)
    r1 = run_bwd(x, dO, "bf16")
    r2 = run_bwd(x, dO, "bf16", group=1)
    for k in ("dQ", "dK", "dV", "dalpha", "dbeta"):
        assert torch.equal(r1[k], r2[k]), k


# ---- softmax heads with queries and keys of their own (Section 4.3: shared projections, different normalisation) ------
@pytest.mark.parametrize("dtype,B,H,G,L,d", [("f32", 1, 2, 1, 320, 64), ("bf16", 1, 2, 1, 448, 128),
                                             ("bf16", 1, 2, 2, 512, 64), ("f32", 1, 1, 3, 256, 128)])
@pytest.mark.parametrize("routing", ["token", "chunk"])
@pytest.mark.parametrize("math", [nb.NATS_MATH_AUTO, nb.NATS_MATH_FP32], ids=["by_chunks", "by_tokens"])
def test_backward_with_own_softmax_queries_and_keys(dtype, B, H, G, L, d, routing, math):
    """dQ_nla, dK_nla [B,H G,L,d] are the softmax branch's gradients; dQ, dK then hold the linear branch's alone."""
    x = make_fwd_inputs(B, H, L, d, dtype, 0.15, seed=960 + L + G)
    xs = make_fwd_inputs(B, H * G, L, d, dtype, 0.15, seed=961 + L + G)
    x["V"] = xs["V"]
    Qn, Kn = xs["Q"], xs["K"]
    dO = make_grad_output(B, H * G, L, d, dtype, seed=962 + L)
    S0 = (0.05 * np.random.default_rng(L + G).standard_normal((B, H * G, d, d))).astype(np.float32)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    kw = dict(S0=S0, group=G, math=math, Q_nla=torch.from_numpy(Qn).to(tdt).cuda(),
              K_nla=torch.from_numpy(Kn).to(tdt).cuda())
    own = (("dQ_nla", "dQ_nla"), ("dK_nla", "dK_nla"))
    if routing == "chunk":
        x["mask"] = make_chunk_mask(B, H, L // 64, 0.35, 963 + L, "bernoulli")
        r = run_bwd(x, dO, dtype, routing=nb.NATS_ROUTE_CHUNK, want=("d_initial_state", "dscore_nla", "dscore_la"), **kw)
        ref = nbw.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, C=64, S0=S0,
                                     Q_nla=Qn, K_nla=Kn)
        extra = CHUNK_KEYS + own
    else:
        r = run_bwd(x, dO, dtype, want=("d_initial_state", "g_nla", "g_la"), **kw)
        ref = nbw.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, S0=S0,
                                     Q_nla=Qn, K_nla=Kn)
        extra = (("d_initial_state", "dS0"), ("g_nla", "g_nla"), ("g_la", "g_la")) + own
    assert tuple(r["dQ_nla"].shape) == (B, H * G, L, d) and tuple(r["dQ"].shape) == (B, H, L, d)
    errs = check(r, ref, extra=extra)
    print(dtype, G, routing, errs)


# ---- the normalised, weighted merges (Eq. 21; Section 5, ablation (iii)) ------------------------------------------------
@pytest.mark.parametrize("dtype,B,H,G,L,d,own_qk,weights", [
    ("f32", 1, 2, 1, 320, 64, False, True), ("bf16", 1, 2, 1, 448, 128, False, True),
    ("bf16", 1, 2, 2, 256, 64, True, True), ("f32", 2, 1, 3, 256, 128, False, False)])
@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("routing", ["token", "chunk"])
def test_backward_through_the_normalised_merges(dtype, B, H, G, L, d, own_qk, weights, mode, routing):
    """combine_mode 1 (Eq. 21) and 2 (one normalisation): every gradient, those of the two weights included, against
    the oracle's adjoint of the same merge; bf16 tensors are widened and the pass runs in fp32."""
    x = make_fwd_inputs(B, H, L, d, dtype, 0.15, seed=980 + L + G)
    xs = make_fwd_inputs(B, H * G, L, d, dtype, 0.15, seed=981 + L + G)
    x["V"] = xs["V"]
    dO = make_grad_output(B, H * G, L, d, dtype, seed=982 + L)
    rng = np.random.default_rng(983 + L + mode)
    S0 = (0.05 * rng.standard_normal((B, H * G, d, d))).astype(np.float32)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    kw, okw = dict(S0=S0, group=G, combine_mode=mode, rms_eps=1e-5), dict(S0=S0, mode=mode, eps=1e-5)
    if own_qk:
        kw.update(Q_nla=torch.from_numpy(xs["Q"]).to(tdt).cuda(), K_nla=torch.from_numpy(xs["K"]).to(tdt).cuda())
        okw.update(Q_nla=xs["Q"], K_nla=xs["K"])
    if weights:
        wn = (rng.random((B, H * G, L)) + 0.1).astype(np.float32)
        wl = (rng.random((B, H * G, L)) + 0.1).astype(np.float32)
        kw.update(w_nla=torch.from_numpy(wn).cuda(), w_la=torch.from_numpy(wl).cuda())
        okw.update(w_nla=wn, w_la=wl)
    extra = (("dw_nla", "dw_nla"), ("dw_la", "dw_la")) + ((("dQ_nla", "dQ_nla"), ("dK_nla", "dK_nla")) if own_qk else ())
    if routing == "chunk":
        x["mask"] = make_chunk_mask(B, H, L // 64, 0.35, 984 + L, "bernoulli")
        r = run_bwd(x, dO, dtype, routing=nb.NATS_ROUTE_CHUNK, want=("d_initial_state", "dscore_nla", "dscore_la"), **kw)
        ref = nbw.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, C=64, **okw)
        extra = CHUNK_KEYS + extra
    else:
        r = run_bwd(x, dO, dtype, want=("d_initial_state", "g_nla", "g_la"), **kw)
        ref = nbw.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, **okw)
        extra = (("d_initial_state", "dS0"), ("g_nla", "g_nla"), ("g_la", "g_la")) + extra
    assert tuple(r["dw_nla"].shape) == (B, H * G, L)
    errs = check(r, ref, extra=extra)
    print(dtype, G, mode, routing, errs)


def test_backward_through_the_merge_token_by_token_adjoint():
    """The same with the linear branch's adjoint token by token (math = NATS_MATH_FP32)."""
    B, H, L, d = 1, 2, 256, 64
    x = make_fwd_inputs(B, H, L, d, "bf16", 0.2, seed=990)
    dO = make_grad_output(B, H, L, d, "bf16", seed=991)
    r = run_bwd(x, dO, "bf16", want=("d_initial_state",), combine_mode=1, math=nb.NATS_MATH_FP32)
    ref = nbw.hybrid_bwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, mode=1)
    check(r, ref, extra=(("d_initial_state", "dS0"), ("dw_nla", "dw_nla"), ("dw_la", "dw_la")))


@pytest.mark.parametrize("kind", ["all_softmax", "all_linear"])
@pytest.mark.parametrize("mode", [1, 2])
def test_backward_through_the_merges_degenerate_masks(kind, mode):
    """A branch whose rows are all zero (no softmax token at all; no linear token and no initial state): its
    normalised rows are zero and so is its weight's gradient; the normalisation's derivative at zero is 1/sqrt(eps)."""
    B, H, L, d = 1, 2, 192, 64
    x = make_fwd_inputs(B, H, L, d, "f32", 0.1, seed=995)
    x["mask"] = np.full((B, H, L), 1 if kind == "all_softmax" else 0, dtype=np.uint8)
    dO = make_grad_output(B, H, L, d, "f32", seed=996)
    r = run_bwd(x, dO, "f32", want=(), combine_mode=mode)
    ref = nbw.hybrid_bwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, mode=mode)
    if mode == 1:
        check(r, ref, extra=(("dw_nla", "dw_nla"), ("dw_la", "dw_la")))
        return
    # One normalisation of the weighted sum, one branch zero: the output does not depend on the scale of the other
    # branch's weight, whose gradient is the difference of two equal terms (exactly eps / (mean square + eps) of
    # one of them).  It is held to 1e-4 of those terms' size (|dO row| x |normalised row| = |dO row| sqrt(d)),
    # not of its own.
    check(r, ref)
    scale = float(np.sqrt(np.mean(np.sum(dO.astype(np.float64) ** 2, axis=-1)) * d))
    for key in ("dw_nla", "dw_la"):
        assert np.max(np.abs(host(r[key]) - ref[key])) <= TOL_BWD * scale, key
