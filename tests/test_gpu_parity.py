"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element
on the same seeded inputs.  Integer outputs must be bit-exact; floating-point outputs must
satisfy max|err| / RMS(oracle) <= 1e-4 (fp32 tensors) or 2e-2 (bf16 tensors)."""
import numpy as np
import pytest
import torch

import paper_2602_03681_amd as nats
from paper_2602_03681_amd import binding as nb
from nats_inputs import CONFIGS, make_config_inputs, make_fwd_inputs

from gpu_util import TOL, host, oracle_fwd, rel_err, stored, to_dev

pytestmark = pytest.mark.gpu

ALL_OUT = ("final_state", "Kc", "Vc", "n_s", "idx", "cnt", "O_la", "O_nla", "lse")


def run_ex(x, dtype, want=ALL_OUT, **kw):
    g = to_dev(x, dtype)
    extra_in = {k: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).cuda()
                for k, v in kw.items() if k in ("w_nla", "w_la", "initial_state") and v is not None}
    kw = {k: v for k, v in kw.items() if k not in ("w_nla", "w_la", "initial_state")}
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64,
                                want=want, **extra_in, **kw)
    torch.cuda.synchronize()
    return r


def check_all(x, dtype, r, ref, tol=None, n_cap=None):
    tol = TOL[dtype] if tol is None else tol
    B, H, L = x["Q"].shape[:3]
    # integers: exactly one correct answer
    np.testing.assert_array_equal(host(r["cnt"]), ref["cnt"])
    np.testing.assert_array_equal(host(r["n_s"]), ref["n_s"])
    idx = host(r["idx"])
    Kc, Vc = host(r["Kc"]), host(r["Vc"])
    cap = Kc.shape[2]
    for b in range(B):
        for h in range(H):
            n = int(ref["n_s"][b, h])
            np.testing.assert_array_equal(idx[b, h, :n], ref["idx"][b, h, :n])
            assert np.all(idx[b, h, n:] == -1)          # entries past n_s are left untouched
            m = min(n, cap)
            sel = ref["idx"][b, h, :m]
            np.testing.assert_array_equal(Kc[b, h, :m], x["K"][b, h, sel])   # a copy: bit-exact
            np.testing.assert_array_equal(Vc[b, h, :m], x["V"][b, h, sel])
            assert np.all(Kc[b, h, m:] == 0)
    # floating point
    errs = {"O": rel_err(host(r["O"]), ref["O"], stored(dtype)), "O_la": rel_err(host(r["O_la"]), ref["O_la"]),
            "O_nla": rel_err(host(r["O_nla"]), ref["O_nla"]), "S": rel_err(host(r["final_state"]), ref["S"])}
    lse, lse_ref = host(r["lse"]), ref["lse"]
    empty = np.isneginf(lse_ref)
    np.testing.assert_array_equal(np.isneginf(lse), empty)
    if (~empty).any():
        errs["lse"] = float(np.max(np.abs(lse[~empty] - lse_ref[~empty])))
    for k, e in errs.items():
        assert e <= tol, f"{k}: {e:.3e} > {tol:.1e} (all: {errs})"
    return errs


# ---------------------------------------------------------------------------------------------
# the measured workloads
# ---------------------------------------------------------------------------------------------
def test_cfg0_tiny_f32():
    cfg = CONFIGS["cfg0_tiny_f32"]
    x = make_config_inputs(cfg)
    r = run_ex(x, "f32")
    errs = check_all(x, "f32", r, oracle_fwd(x))
    print("cfg0", errs)


@pytest.mark.parametrize("math", [nb.NATS_MATH_AUTO, nb.NATS_MATH_FP32])
def test_cfg1_bf16(math):
    cfg = CONFIGS["cfg1_bf16"]
    x = make_config_inputs(cfg)
    r = run_ex(x, "bf16", math=math)
    errs = check_all(x, "bf16", r, oracle_fwd(x))
    print("cfg1", math, errs)


def report(tag, got, ref):
    """Raw and storage-adjusted max|err| / RMS of a tensor stored in bf16, side by side."""
    raw, adj = rel_err(got, ref), rel_err(got, ref, "bf16")
    print(f"{tag}: max|err|/RMS raw {raw:.3e}, less half a bf16 ulp of the reference {adj:.3e}")
    return raw, adj


def check_full_size(cfg_name):
    """A measured workload at full size: every element of every head.  O (stored in bf16) under the storage-adjusted
    reading of the bar; the fp32 per-branch outputs and the final state, which no storage rounding touches, under
    the raw bar; integers bit-exactly."""
    cfg = CONFIGS[cfg_name]
    x = make_config_inputs(cfg)
    want = ("cnt", "n_s", "idx", "O_la", "O_nla", "final_state", "lse")
    r = run_ex(x, "bf16", want=want)
    ref = oracle_fwd(x)
    np.testing.assert_array_equal(host(r["cnt"]), ref["cnt"])
    np.testing.assert_array_equal(host(r["n_s"]), ref["n_s"])
    idx = host(r["idx"])
    B, H = ref["n_s"].shape
    for b in range(B):
        for h in range(H):
            n = int(ref["n_s"][b, h])
            np.testing.assert_array_equal(idx[b, h, :n], ref["idx"][b, h, :n])
    raw, adj = report(f"{cfg_name} O", host(r["O"]), ref["O"])
    assert adj <= TOL["bf16"]
    errs = {"O_la": rel_err(host(r["O_la"]), ref["O_la"]), "O_nla": rel_err(host(r["O_nla"]), ref["O_nla"]),
            "S": rel_err(host(r["final_state"]), ref["S"])}
    lse, lse_ref = host(r["lse"]), ref["lse"]
    assert not np.isneginf(lse_ref).any() and not np.isneginf(lse).any()    # token 0 is a softmax token
    errs["lse"] = float(np.max(np.abs(lse - lse_ref)))
    print(f"{cfg_name} fp32 outputs, raw max|err|/RMS: {errs}")
    # per head as well: no head may hide behind the others' RMS
    O, Oref = host(r["O"]), ref["O"]
    per_head = [rel_err(O[b, h], Oref[b, h], "bf16") for b in range(B) for h in range(H)]
    print(f"{cfg_name} O per (batch, head), adjusted: max {max(per_head):.3e}")
    for k, e in errs.items():
        assert e <= TOL["bf16"], f"{k}: {e:.3e}"
    assert max(per_head) <= TOL["bf16"]
    return x, r


def test_cfg2_headline_bf16_full_tensor():
    """Full size, every output element, in the launch configuration the benchmark times."""
    cfg = CONFIGS["cfg2_headline_bf16"]
    x, r = check_full_size("cfg2_headline_bf16")
    g = to_dev(x, "bf16")
    # the plain entry point (what the benchmark calls) gives the same bits, twice
    O = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], cfg.C)
    O2 = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], cfg.C)
    torch.cuda.synchronize()
    assert torch.equal(O.view(torch.int16), O2.view(torch.int16))
    assert torch.equal(O.view(torch.int16), r["O"].view(torch.int16))


def test_cfg3_long_bf16_all_heads():
    """L = 32768, all 16 heads, every element (the oracle recomputes each head in full)."""
    check_full_size("cfg3_long_bf16")


# ---------------------------------------------------------------------------------------------
# edge cases and variants
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("mask_kind", ["all_softmax", "all_linear", "head_skew", "ramp", "bernoulli"])
def test_mask_patterns(dtype, d, mask_kind):
    """Degenerate routings: everything softmax (pure causal attention), everything linear (pure GDN,
    empty softmax set -> O_nla = 0, lse = -inf), heads that are 0% / 50% softmax, position ramp."""
    runs = 3 if mask_kind in ("bernoulli", "ramp") else 0
    x = make_fwd_inputs(2, 4, 320, d, dtype, 0.2, seed=7 + d, mask_kind=mask_kind, n_runs=runs, run_len=9)
    r = run_ex(x, dtype)
    check_all(x, dtype, r, oracle_fwd(x))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_softmax_scale_sqrt_d_and_large_logits(dtype):
    """softmax_scale = sqrt(d) (what RMS-normed q,k would give) exercises the running-max rescale;
    scale = 300 gives near one-hot rows."""
    d = 64
    x = make_fwd_inputs(1, 3, 512, d, dtype, 0.3, seed=11)
    for scale in (float(np.sqrt(d)), 300.0):
        r = run_ex(x, dtype, softmax_scale=scale, la_scale=0.5)
        check_all(x, dtype, r, oracle_fwd(x, softmax_scale=scale, la_scale=0.5))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_eq21_merge_and_initial_state(dtype):
    d = 128
    x = make_fwd_inputs(2, 2, 256, d, dtype, 0.1, seed=12)
    rng = np.random.default_rng(120)
    wn = rng.random((2, 2, 256)).astype(np.float32)
    wl = (1 - wn).astype(np.float32)
    S0 = (0.05 * rng.standard_normal((2, 2, d, d))).astype(np.float32)
    r = run_ex(x, dtype, combine_mode=1, w_nla=wn, w_la=wl, initial_state=S0, rms_eps=1e-5)
    check_all(x, dtype, r, oracle_fwd(x, mode=1, w_nla=wn, w_la=wl, S0=S0, eps=1e-5))
    r = run_ex(x, dtype, combine_mode=1)      # default weights 0.5 / 0.5
    check_all(x, dtype, r, oracle_fwd(x, mode=1))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_odd_batch_head_count_and_ragged_tiles(dtype):
    """B*H = 9 (not a multiple of the 8-way block interleave), L = 448 = 3.5 query tiles of 128,
    softmax counts that are not multiples of the 64-row key tile."""
    x = make_fwd_inputs(3, 3, 448, 128, dtype, 0.23, seed=16, n_runs=2, run_len=37)
    r = run_ex(x, dtype)
    check_all(x, dtype, r, oracle_fwd(x))
    # plain entry point (no optional outputs) gives the same O
    g = to_dev(x, dtype)
    O = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64)
    torch.cuda.synchronize()
    assert torch.equal(O.view(torch.int16 if dtype == "bf16" else torch.int32),
                       r["O"].view(torch.int16 if dtype == "bf16" else torch.int32))


def test_single_chunk_and_small_cache_capacity():
    x = make_fwd_inputs(1, 2, 64, 64, "f32", 0.5, seed=13)
    r = run_ex(x, "f32", cap=5)                # cap < n_s: only the first 5 rows are handed out
    assert host(r["n_s"]).min() > 5
    check_all(x, "f32", r, oracle_fwd(x))


def test_workspace_is_reusable_and_poison_safe():
    """A caller-owned workspace filled with garbage must not change the result."""
    x = make_fwd_inputs(1, 2, 256, 64, "bf16", 0.1, seed=14)
    g = to_dev(x, "bf16")
    p = nb.make_fwd_params(1, 2, 256, 64, 64, nb.NATS_BF16)
    ws = torch.full((nb.fwd_workspace_bytes(p),), 0xFF, dtype=torch.uint8, device="cuda")
    O1 = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, workspace=ws)
    O2 = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64)
    torch.cuda.synchronize()
    assert torch.equal(O1.view(torch.int16), O2.view(torch.int16))


def test_runs_on_a_side_stream():
    x = make_fwd_inputs(1, 2, 256, 64, "f32", 0.1, seed=15)
    g = to_dev(x, "f32")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        O = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64)
    s.synchronize()
    assert rel_err(host(O), oracle_fwd(x, want=())["O"]) <= TOL["f32"]


def test_bf16_path_on_a_side_stream_twice():
    """Every kernel of the bf16 path runs on the caller's stream: on a side stream the result must be
    complete when that stream is, call after call through one workspace."""
    x = make_fwd_inputs(1, 3, 1024, 128, "bf16", 0.08, seed=16)
    g = to_dev(x, "bf16")
    ref = oracle_fwd(x, want=())["O"]
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        O1 = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64)
        O2 = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64)
    s.synchronize()
    assert rel_err(host(O1), ref, stored="bf16") <= TOL["bf16"]
    assert torch.equal(O1, O2)


def test_forward_in_a_hip_graph_replays():
    """Capture one forward (caller-provided output and workspace, nothing allocated inside) into a
    graph; every replay, with eager work and synchronisation in between and new inputs written in
    place, must reproduce the eager result of the same inputs bit for bit."""
    from paper_2602_03681_amd import binding as nb
    B, H, L, d = 1, 2, 512, 128
    xs = [make_fwd_inputs(B, H, L, d, "bf16", 0.1, seed=30 + i) for i in range(3)]
    gs = [to_dev(x, "bf16") for x in xs]
    cur = {k: v.clone() for k, v in gs[0].items()}
    params = nb.make_fwd_params(B, H, L, d, 64, nb.NATS_BF16)
    ws = torch.empty(nb.fwd_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    O = torch.empty_like(cur["Q"])

    def run():
        nats.hybrid_attn_fwd(cur["Q"], cur["K"], cur["V"], cur["alpha"], cur["beta"], cur["mask"], 64,
                             out=O, workspace=ws)

    eager = []
    for g in gs:                       # eager results
        for k in cur:
            cur[k].copy_(g[k])
        run()
        torch.cuda.synchronize()
        eager.append(O.clone())
    graph = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        with torch.cuda.graph(graph, stream=s):
            run()
    torch.cuda.synchronize()
    for i in (1, 2, 0, 1):
        for k in cur:
            cur[k].copy_(gs[i][k])
        O.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, eager[i]), f"replay with input set {i} differs from the eager result"
    assert rel_err(host(eager[0]), oracle_fwd(xs[0], want=())["O"], stored="bf16") <= TOL["bf16"]


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_eq22_merge_weights_kernel_and_forward(dtype, d):
    """Eq. 22 on the device: the weights as a call of their own, and the forward given W_out against the
    oracle's Eq. 21 with the oracle's Eq. 22 weights."""
    from oracle import nats_oracle as no
    B, H, L = 2, 3, 320
    x = make_fwd_inputs(B, H, L, d, dtype, 0.1, seed=80 + d)
    rng = np.random.default_rng(81)
    W = (rng.standard_normal((H, 2, d)) * 2.0).astype(np.float32)
    w_ref = no.eq22_weights(x["Q"], W)
    g = to_dev(x, dtype)
    Wd = torch.from_numpy(W).cuda()
    w_nla, w_la = nats.merge_weights(g["Q"], Wd)
    torch.cuda.synchronize()
    assert np.abs(host(w_nla) - w_ref[0]).max() <= 2e-6 and np.abs(host(w_la) - w_ref[1]).max() <= 2e-6
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, combine_mode=1,
                                W_out=Wd)
    torch.cuda.synchronize()
    ref = oracle_fwd(x, mode=1, w_nla=w_ref[0], w_la=w_ref[1], want=())
    assert rel_err(host(r["O"]), ref["O"], stored(dtype)) <= TOL[dtype]
    with pytest.raises(nb.NatsError):   # given weights and W_out exclude each other
        nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, combine_mode=1,
                                W_out=Wd, w_nla=w_nla)


@pytest.mark.parametrize("act", [nb.NATS_WEIGHTS_SIGMOID, nb.NATS_WEIGHTS_LINEAR])
def test_merge_weight_activations(act):
    """Section 5, ablation (iv): sigmoid or no activation instead of the softmax of Eq. 22, as a call of its own
    and inside the forward."""
    from oracle import nats_oracle as no
    B, H, L, d = 1, 3, 256, 64
    x = make_fwd_inputs(B, H, L, d, "bf16", 0.1, seed=85)
    W = (np.random.default_rng(86).standard_normal((H, 2, d)) * 1.5).astype(np.float32)
    w_ref = no.eq22_weights(x["Q"], W, act=act)
    g = to_dev(x, "bf16")
    Wd = torch.from_numpy(W).cuda()
    w_nla, w_la = nats.merge_weights(g["Q"], Wd, weight_act=act)
    torch.cuda.synchronize()
    scale = max(1.0, float(np.abs(w_ref[0]).max()))
    assert np.abs(host(w_nla) - w_ref[0]).max() <= 4e-6 * scale and np.abs(host(w_la) - w_ref[1]).max() <= 4e-6 * scale
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, combine_mode=1, W_out=Wd,
                                weight_act=act)
    torch.cuda.synchronize()
    ref = oracle_fwd(x, mode=1, w_nla=w_ref[0], w_la=w_ref[1], want=())
    assert rel_err(host(r["O"]), ref["O"], "bf16") <= TOL["bf16"]


@pytest.mark.parametrize("d", [64, 128])
def test_more_pairs_than_the_chip_has_cus(d):
    """B*H = 80: the recurrence kernel's grid (320 blocks) exceeds the CU count, so it runs without its prefetch
    helper blocks and in more than one wave of blocks; the padded pair count of the one-dimensional grids
    (80 is a multiple of 8, 75 below is not) changes nothing."""
    for B, H in ((5, 16), (5, 15)):
        x = make_fwd_inputs(B, H, 256, d, "bf16", 0.1, seed=95 + H)
        r = run_ex(x, "bf16", want=("final_state", "n_s"))
        ref = oracle_fwd(x, want=("S", "n_s"))
        assert rel_err(host(r["O"]), ref["O"], "bf16") <= TOL["bf16"]
        assert rel_err(host(r["final_state"]), ref["S"]) <= TOL["bf16"]
        np.testing.assert_array_equal(host(r["n_s"]), ref["n_s"])


def test_one_chunk_and_long_thin_shapes_bf16():
    """L = 64 (a single chunk, a single query tile) and a long single head."""
    for B, H, L, d in ((2, 2, 64, 128), (1, 1, 16384, 64)):
        x = make_fwd_inputs(B, H, L, d, "bf16", 0.05, seed=97 + d)
        r = run_ex(x, "bf16", want=("final_state",))
        ref = oracle_fwd(x, want=("S",))
        assert rel_err(host(r["O"]), ref["O"], "bf16") <= TOL["bf16"], (L, d)
        assert rel_err(host(r["final_state"]), ref["S"]) <= TOL["bf16"], (L, d)


@pytest.mark.parametrize("d", [64, 128])
def test_every_chunk_count_up_to_nine_bf16(d):
    """1..9 chunks: the scan's staging wavefronts walk a segment's chunks two to a loop trip with an odd one behind,
    one chunk ahead of the state wavefronts and with a clamped index at the end; with the automatic segment count
    these lengths give segments of one to nine chunks (1 .. 7 chunks: one segment; 8, 9: two), with a given
    initial state."""
    for n_chunks in range(1, 10):
        L = 64 * n_chunks
        x = make_fwd_inputs(1, 3, L, d, "bf16", 0.1, seed=500 + 10 * n_chunks + d)
        S0 = (0.1 * np.random.default_rng(n_chunks).standard_normal((1, 3, d, d))).astype(np.float32)
        r = run_ex(x, "bf16", want=("final_state",), initial_state=S0)
        ref = oracle_fwd(x, S0=S0, want=("S",))
        assert rel_err(host(r["O"]), ref["O"], "bf16") <= TOL["bf16"], (L, d)
        assert rel_err(host(r["final_state"]), ref["S"]) <= TOL["bf16"], (L, d)


def test_pair_counts_between_powers_of_two_bf16():
    """B*H = 40, 48, 56 at 16 chunks: pair counts between the powers of two, four segments each (the automatic
    count, about 256 / (B*H), is capped at a quarter of the chunks): 200 to 280 blocks in the first pass."""
    for B, H in ((5, 8), (6, 8), (7, 8)):
        x = make_fwd_inputs(B, H, 1024, 128, "bf16", 0.05, seed=600 + B)
        r = run_ex(x, "bf16", want=("final_state",))
        ref = oracle_fwd(x, want=("S",))
        assert rel_err(host(r["O"]), ref["O"], "bf16") <= TOL["bf16"], (B, H)
        assert rel_err(host(r["final_state"]), ref["S"]) <= TOL["bf16"], (B, H)


# ---------------------------------------------------------------------------------------------
# value ranges of the bf16 path (its intermediates are fp16: accepted range stated in nats.h)
# ---------------------------------------------------------------------------------------------
def test_large_values_and_large_initial_state_bf16():
    """|V| up to about 1000 and an initial state of the same size: inside the stated range of the bf16 path
    (every intermediate below 65504), the bar holds as for unit-size values; both branches are linear in V."""
    d = 128
    x = make_fwd_inputs(1, 3, 1024, d, "bf16", 0.1, seed=701)
    x["V"] = (x["V"] * 256.0).astype(np.float32)            # still bf16 values: a power of two
    S0 = (200.0 * np.random.default_rng(702).standard_normal((1, 3, d, d))).astype(np.float32)
    r = run_ex(x, "bf16", want=("final_state", "O_la", "O_nla"), initial_state=S0)
    ref = oracle_fwd(x, S0=S0)
    report("large V, large S0: O", host(r["O"]), ref["O"])
    assert rel_err(host(r["O"]), ref["O"], "bf16") <= TOL["bf16"]
    assert rel_err(host(r["O_la"]), ref["O_la"]) <= TOL["bf16"]
    assert rel_err(host(r["O_nla"]), ref["O_nla"]) <= TOL["bf16"]
    assert rel_err(host(r["final_state"]), ref["S"]) <= TOL["bf16"]


@pytest.mark.parametrize("d", [64, 128])
def test_no_decay_over_a_long_sequence_bf16(d):
    """alpha = 1 everywhere (the delta rule of Eq. 18) over 8192 tokens: no decay damps the rounding of the
    carried state."""
    x = make_fwd_inputs(1, 2, 8192, d, "bf16", 0.05, seed=710 + d)
    x["alpha"] = np.ones_like(x["alpha"])
    r = run_ex(x, "bf16", want=("final_state", "O_la"))
    ref = oracle_fwd(x)
    report(f"alpha = 1, L = 8192, d = {d}: O", host(r["O"]), ref["O"])
    assert rel_err(host(r["O"]), ref["O"], "bf16") <= TOL["bf16"]
    assert rel_err(host(r["O_la"]), ref["O_la"]) <= TOL["bf16"]
    assert rel_err(host(r["final_state"]), ref["S"]) <= TOL["bf16"]


def test_decay_near_zero_bf16():
    """alpha between 1e-4 and 1e-2 at a third of the tokens: the cumulative decay inside a chunk underflows, the
    state forgets within a few tokens; nothing may turn into inf or NaN."""
    d = 128
    x = make_fwd_inputs(1, 2, 512, d, "bf16", 0.1, seed=720)
    rng = np.random.default_rng(721)
    tiny = rng.random(x["alpha"].shape) < 0.33
    x["alpha"] = np.where(tiny, 10.0 ** rng.uniform(-4, -2, x["alpha"].shape), x["alpha"]).astype(np.float32)
    r = run_ex(x, "bf16", want=("final_state", "O_la"))
    ref = oracle_fwd(x)
    assert np.isfinite(host(r["O"])).all() and np.isfinite(host(r["final_state"])).all()
    assert rel_err(host(r["O"]), ref["O"], "bf16") <= TOL["bf16"]
    assert rel_err(host(r["O_la"]), ref["O_la"]) <= TOL["bf16"]
    assert rel_err(host(r["final_state"]), ref["S"]) <= TOL["bf16"]


# ---------------------------------------------------------------------------------------------
# the segmented recurrence of the bf16 path
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d", [64, 128])
def test_every_segment_count_bf16(d):
    """The chunk recurrence cut into 1..8 segments (start states composed from the segments' affine maps): 22
    chunks, so that the last segment is ragged (and 7 segments collapse to 6), with an initial state; alpha near 1
    in half of the cases so that the carried state matters across many segments."""
    L = 64 * 22
    for slow_decay in (False, True):
        x = make_fwd_inputs(1, 3, L, d, "bf16", 0.1, seed=800 + d)
        if slow_decay:
            x["alpha"] = (1.0 - 0.002 * (1.0 - x["alpha"])).astype(np.float32)
        S0 = (0.3 * np.random.default_rng(801).standard_normal((1, 3, d, d))).astype(np.float32)
        ref = oracle_fwd(x, S0=S0, want=("S", "O_la"))
        for n_seg in (1, 2, 3, 4, 5, 7, 8):
            r = run_ex(x, "bf16", want=("final_state", "O_la"), initial_state=S0, gdn_segments=n_seg)
            e = {"O": rel_err(host(r["O"]), ref["O"], "bf16"), "O_la": rel_err(host(r["O_la"]), ref["O_la"]),
                 "S": rel_err(host(r["final_state"]), ref["S"])}
            assert max(e.values()) <= TOL["bf16"], (d, slow_decay, n_seg, e)


def test_segment_count_does_not_change_the_result_beyond_rounding_bf16():
    x = make_fwd_inputs(2, 2, 2048, 128, "bf16", 0.05, seed=810)
    base = run_ex(x, "bf16", want=("O_la",), gdn_segments=1)
    for n_seg in (2, 8):
        r = run_ex(x, "bf16", want=("O_la",), gdn_segments=n_seg)
        a, b = host(r["O_la"]), host(base["O_la"])
        assert np.abs(a - b).max() <= 2e-3 * np.sqrt(np.mean(b * b)), n_seg


def test_values_beyond_the_fp16_range_saturate_bf16():
    """|V| around 2^20: the linear branch's fp16 intermediates leave the stated range.  They saturate (the result
    is then inaccurate, as nats.h says) but nothing turns into inf or NaN."""
    x = make_fwd_inputs(1, 2, 512, 128, "bf16", 0.1, seed=730)
    x["V"] = (x["V"] * 2.0 ** 20).astype(np.float32)
    r = run_ex(x, "bf16", want=("final_state", "O_la"))
    assert np.isfinite(host(r["O"])).all() and np.isfinite(host(r["O_la"])).all()
    assert np.isfinite(host(r["final_state"])).all()
