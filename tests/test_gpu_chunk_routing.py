"""GPU parity for routing per chunk (Section 4.1 as stated: one decision per chunk, the intra-chunk part
computed by both operations, the unchosen state rolled back): the HIP path through the C ABI against
the chunk-routed CPU oracle, same bars as the per-token tests."""
import numpy as np
import pytest
import torch

import paper_2602_03681_amd as nats
from paper_2602_03681_amd import binding as nb
from nats_inputs import make_chunk_mask, make_fwd_inputs

from gpu_util import TOL, host, rel_err, stored, to_dev
from oracle import c_oracle
from test_gpu_parity import ALL_OUT, check_all

pytestmark = pytest.mark.gpu
C = 64


def inputs(B, H, L, d, dtype, p, seed, kind="bernoulli"):
    x = make_fwd_inputs(B, H, L, d, dtype, 0.1, seed=seed)
    x["mask"] = make_chunk_mask(B, H, L // C, p, seed + 7, kind)
    return x


def oracle(x, **kw):
    return c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], chunk_routing=C, **kw)


def run_ex(x, dtype, want=ALL_OUT, **kw):
    g = to_dev(x, dtype)
    extra_in = {k: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).cuda()
                for k, v in kw.items() if k in ("w_nla", "w_la", "initial_state") and v is not None}
    kw = {k: v for k, v in kw.items() if k not in ("w_nla", "w_la", "initial_state")}
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], C,
                                routing=nb.NATS_ROUTE_CHUNK, want=want, **extra_in, **kw)
    torch.cuda.synchronize()
    return r


@pytest.mark.parametrize("kind", ["bernoulli", "all_softmax", "all_linear", "head_skew", "alternate"])
@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f32", 128), ("bf16", 64), ("bf16", 128)])
def test_chunk_routing_mask_patterns(dtype, d, kind):
    x = inputs(2, 3, 512, d, dtype, 0.3, seed=40 + d, kind=kind)
    check_all(x, dtype, run_ex(x, dtype), oracle(x))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chunk_routing_eq21_initial_state_and_scales(dtype):
    x = inputs(1, 4, 384, 128, dtype, 0.35, seed=51)
    rng = np.random.default_rng(52)
    w = rng.random((2, 1, 4, 384)).astype(np.float32)
    S0 = (rng.standard_normal((1, 4, 128, 128)) * 0.05).astype(np.float32)
    kw = dict(combine_mode=1, softmax_scale=float(np.sqrt(128.0)), la_scale=0.5)
    r = run_ex(x, dtype, w_nla=w[0], w_la=w[1], initial_state=S0, **kw)
    ref = oracle(x, mode=1, softmax_scale=kw["softmax_scale"], la_scale=0.5, w_nla=w[0], w_la=w[1],
                 S0=S0.astype(np.float64))
    check_all(x, dtype, r, ref)


@pytest.mark.parametrize("kind", ["bernoulli", "alternate", "all_softmax"])
@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f32", 128), ("bf16", 128)])
def test_routing_chunks_of_128_tokens(dtype, d, kind):
    """One routing decision per 128 tokens (the chunk-size ablation of Section 5): the mask holds L / 128 bytes, a
    softmax chunk's provisional state lives for 128 tokens, its queries see all 128 of its own keys causally.  Runs on
    the token-by-token kernels (for bf16 tensors as well)."""
    B, H, L = 2, 2, 640
    x = make_fwd_inputs(B, H, L, d, dtype, 0.1, seed=60 + d)
    x["mask"] = make_chunk_mask(B, H, L // 128, 0.4, 67 + d, kind)
    g = to_dev(x, dtype)
    S0 = (np.random.default_rng(61).standard_normal((B, H, d, d)) * 0.05).astype(np.float32)
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 128, routing=nb.NATS_ROUTE_CHUNK,
                                want=ALL_OUT, initial_state=torch.from_numpy(S0).cuda())
    torch.cuda.synchronize()
    ref = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], chunk_routing=128, S0=S0.astype(np.float64))
    check_all(x, dtype, r, ref)


def test_routing_chunks_of_128_tokens_inner_part_by_one_operation():
    x = make_fwd_inputs(1, 2, 512, 64, "f32", 0.1, seed=62)
    x["mask"] = make_chunk_mask(1, 2, 4, 0.5, 63, "bernoulli")
    g = to_dev(x, "f32")
    from oracle import nats_oracle as no
    for inner in (1, 2):
        O = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 128,
                                    routing=nb.NATS_ROUTE_CHUNK, inner_chunk=inner, want=())["O"]
        torch.cuda.synchronize()
        ref = no.hybrid_fwd_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], 128, inner=inner)["O"]
        assert rel_err(host(O), ref, stored("f32")) <= TOL["f32"], inner


def test_chunk_routing_fp32_math_on_bf16_tensors():
    x = inputs(1, 2, 256, 64, "bf16", 0.4, seed=53)
    check_all(x, "bf16", run_ex(x, "bf16", math=nb.NATS_MATH_FP32), oracle(x))


def test_chunk_routing_long_sequence_ragged_query_tile_bf16():
    """L = 64 * 21: the last block of the softmax kernel holds one chunk only; many compacted tiles."""
    x = inputs(1, 5, 64 * 21, 128, "bf16", 0.5, seed=54)
    g = to_dev(x, "bf16")
    O = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], C,
                             routing=nb.NATS_ROUTE_CHUNK)
    torch.cuda.synchronize()
    assert rel_err(host(O), oracle(x, want=())["O"], stored("bf16")) <= TOL["bf16"]


# ---------------------------------------------------------------------------------------------
# generation: provisional updates inside the open chunk, commit per chunk
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_generation_with_commits_continues_the_forward(dtype, d):
    """Prefill L0 tokens with the forward (routing per chunk), then generate 3 chunks token by token with
    nats_hybrid_attn_decode_chunk and a commit per chunk: every output row must match the chunk-routed
    oracle's forward over the whole sequence, the final state and the settled cache likewise."""
    B, H, L0, n_new = 2, 2, 256, 192
    L = L0 + n_new
    x = inputs(B, H, L, d, dtype, 0.4, seed=60 + d)
    ref = oracle(x)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    pre = {k: v[:, :, :L0] for k, v in x.items() if k != "mask"}
    pre["mask"] = x["mask"][:, :, :L0 // C]
    g = to_dev({k: np.ascontiguousarray(v) for k, v in pre.items()}, dtype)
    cap = L
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], C,
                                routing=nb.NATS_ROUTE_CHUNK, want=("final_state", "Kc", "Vc", "n_s"), cap=cap)
    st = {"state": r["final_state"], "state_start": torch.zeros_like(r["final_state"]),
          "chunk_decay": torch.ones((B, H), dtype=torch.float32, device="cuda"),
          "chunk_pos": torch.zeros((B, H), dtype=torch.int32, device="cuda"),
          "k_cache": r["Kc"], "v_cache": r["Vc"], "cache_len": r["n_s"].clone()}
    full = to_dev(x, dtype)
    err = torch.zeros((B, H), dtype=torch.int32, device="cuda")
    worst = 0.0
    rms = np.sqrt(np.mean(ref["O"] ** 2))
    for t in range(L0, L):
        o = nats.hybrid_attn_decode_chunk(st, full["Q"][:, :, t].contiguous(), full["K"][:, :, t].contiguous(),
                                          full["V"][:, :, t].contiguous(), full["alpha"][:, :, t].contiguous(),
                                          full["beta"][:, :, t].contiguous(), err_flags=err)
        assert int(err.sum()) == 0
        diff = np.abs(host(o).astype(np.float64) - ref["O"][:, :, t])
        if dtype == "bf16":
            from gpu_util import bf16_half_ulp
            diff = np.maximum(diff - bf16_half_ulp(ref["O"][:, :, t]), 0.0)
        worst = max(worst, float(diff.max() / rms))
        if (t + 1) % C == 0:
            nats.hybrid_attn_decode_commit(st, full["mask"][:, :, t // C].contiguous(), err_flags=err)
            assert int(err.sum()) == 0
    torch.cuda.synchronize()
    assert worst <= TOL[dtype], f"worst output error {worst:.3e}"
    assert rel_err(host(st["state"]), ref["S"]) <= TOL[dtype]
    np.testing.assert_array_equal(host(st["cache_len"]), ref["n_s"])
    np.testing.assert_array_equal(host(st["chunk_pos"]), 0)
    kc = host(st["k_cache"])
    for b in range(B):
        for h in range(H):
            n = int(ref["n_s"][b, h])
            np.testing.assert_array_equal(kc[b, h, :n], x["K"][b, h, ref["idx"][b, h, :n]])


def test_generation_cache_overflow_is_flagged():
    """A cache of 70 rows and 128 tokens of softmax chunks: token 70 is the first without a row.  Every output,
    also those after the cache is full (they cover the 70 rows that exist), follows the oracle; the rows behind
    the cache of the last (batch, head) pair are never touched (canary rows stay as they were)."""
    from oracle import nats_oracle as npo
    B, H, d = 1, 2, 64
    cap = 70
    x = inputs(B, H, 128, d, "f32", 1.0, seed=70, kind="all_softmax")
    full = to_dev(x, "f32")
    # the caches are views of larger buffers whose tails hold a canary value
    kbuf = torch.full((B * H * cap + 64, d), 777.0, device="cuda")
    vbuf = torch.full((B * H * cap + 64, d), 777.0, device="cuda")
    kbuf[:B * H * cap] = 0
    vbuf[:B * H * cap] = 0
    st = {"state": torch.zeros((B, H, d, d), device="cuda"), "state_start": torch.zeros((B, H, d, d), device="cuda"),
          "chunk_decay": torch.ones((B, H), device="cuda"), "chunk_pos": torch.zeros((B, H), dtype=torch.int32, device="cuda"),
          "k_cache": kbuf[:B * H * cap].view(B, H, cap, d), "v_cache": vbuf[:B * H * cap].view(B, H, cap, d),
          "cache_len": torch.zeros((B, H), dtype=torch.int32, device="cuda")}
    ref = [[npo.decode_chunk_state(np.zeros((d, d)), np.zeros((cap, d)), np.zeros((cap, d)), 0) for _ in range(H)]
           for _ in range(B)]
    err = torch.zeros((B, H), dtype=torch.int32, device="cuda")
    flagged_at = None
    for t in range(128):
        o = nats.hybrid_attn_decode_chunk(st, *(full[k][:, :, t].contiguous() for k in ("Q", "K", "V", "alpha", "beta")),
                                          err_flags=err)
        o = host(o)
        for b in range(B):
            for h in range(H):
                o_ref, ovf = npo.decode_step_chunk_routed(ref[b][h], x["Q"][b, h, t], x["K"][b, h, t], x["V"][b, h, t],
                                                          x["alpha"][b, h, t], x["beta"][b, h, t])
                assert int(err[b, h]) == int(ovf), (t, b, h)
                e = np.abs(o[b, h] - o_ref).max() / max(np.sqrt(np.mean(o_ref ** 2)), 1e-3)
                assert e <= TOL["f32"], (t, b, h, e)
        if int(err.sum()) and flagged_at is None:
            flagged_at = t
        if (t + 1) % C == 0:
            cerr = torch.zeros_like(err)
            nats.hybrid_attn_decode_commit(st, full["mask"][:, :, t // C].contiguous(), err_flags=cerr)
            for b in range(B):
                for h in range(H):
                    npo.decode_commit_chunk(ref[b][h], int(x["mask"][b, h, t // C]))
            if t + 1 == 128:
                assert int(cerr.sum()) == B * H          # 128 rows do not fit into 70
    assert flagged_at == cap                             # token index 70 is the first one without a row
    np.testing.assert_array_equal(host(st["cache_len"]), cap)
    assert bool((kbuf[B * H * cap:] == 777.0).all()) and bool((vbuf[B * H * cap:] == 777.0).all())


def test_plain_decode_with_cache_len_beyond_cap_reads_only_the_cache():
    """nats_hybrid_attn_decode given a cache_len larger than cap (as n_s of a prefill whose softmax tokens did not
    all fit): the rows that exist are [0, cap), the output covers those, a softmax token is flagged."""
    B, H, d, cap = 1, 2, 64, 6
    rng = np.random.default_rng(9)
    f = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32)).cuda()
    state = f(B, H, d, d) * 0.1
    kc, vc = f(B, H, cap, d), f(B, H, cap, d)
    clen = torch.tensor([[cap + 5, cap + 1]], dtype=torch.int32, device="cuda")
    q, k, v = f(B, H, d), f(B, H, d), f(B, H, d)
    alpha = torch.full((B, H), 0.9, device="cuda"); beta = torch.full((B, H), 0.5, device="cuda")
    mask = torch.tensor([[0, 1]], dtype=torch.uint8, device="cuda")
    err = torch.zeros((B, H), dtype=torch.int32, device="cuda")
    S_ref = host(state).astype(np.float64)
    kc_ref, vc_ref = host(kc).copy(), host(vc).copy()
    o = nats.hybrid_attn_decode(state, kc, vc, clen, q, k, v, alpha, beta, mask, err_flags=err)
    o_ref, ovf = c_oracle.decode(S_ref, kc_ref, vc_ref, np.full((B, H), cap, dtype=np.int32), host(q), host(k), host(v),
                                 host(alpha), host(beta), host(mask))
    assert rel_err(host(o), o_ref) <= TOL["f32"]
    np.testing.assert_array_equal(host(err), [[0, 1]])
    np.testing.assert_array_equal(host(kc), kc_ref)


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_generation_with_the_single_normalisation_merge(dtype, d):
    """nats_hybrid_attn_decode_chunk with combine_mode 2 (Section 5, ablation (iii)) and given weights: two chunks
    generated from an empty state, every row against the oracle's chunk-routed generation step."""
    from oracle import nats_oracle as npo
    from gpu_util import bf16_half_ulp
    B, H, n_new = 2, 2, 2 * C
    cap = n_new
    x = inputs(B, H, n_new, d, dtype, 0.5, seed=90 + d)
    w = np.random.default_rng(91).random((2, B, H, n_new)).astype(np.float32)
    full = to_dev(x, dtype)
    wd = torch.from_numpy(w).cuda()
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    st = {"state": torch.zeros((B, H, d, d), device="cuda"), "state_start": torch.zeros((B, H, d, d), device="cuda"),
          "chunk_decay": torch.ones((B, H), device="cuda"), "chunk_pos": torch.zeros((B, H), dtype=torch.int32, device="cuda"),
          "k_cache": torch.zeros((B, H, cap, d), dtype=tdt, device="cuda"),
          "v_cache": torch.zeros((B, H, cap, d), dtype=tdt, device="cuda"),
          "cache_len": torch.zeros((B, H), dtype=torch.int32, device="cuda")}
    ref = [[npo.decode_chunk_state(np.zeros((d, d)), np.zeros((cap, d)), np.zeros((cap, d)), 0) for _ in range(H)]
           for _ in range(B)]
    worst = 0.0
    for t in range(n_new):
        o = nats.hybrid_attn_decode_chunk(st, *(full[k][:, :, t].contiguous() for k in ("Q", "K", "V", "alpha", "beta")),
                                          combine_mode=2, w_nla=wd[0, :, :, t].contiguous(), w_la=wd[1, :, :, t].contiguous())
        o = host(o).astype(np.float64)
        for b in range(B):
            for h in range(H):
                o_ref, _ = npo.decode_step_chunk_routed(ref[b][h], x["Q"][b, h, t], x["K"][b, h, t], x["V"][b, h, t],
                                                        x["alpha"][b, h, t], x["beta"][b, h, t], mode=2,
                                                        w_nla=float(w[0, b, h, t]), w_la=float(w[1, b, h, t]))
                diff = np.abs(o[b, h] - o_ref)
                if dtype == "bf16":
                    diff = np.maximum(diff - bf16_half_ulp(o_ref), 0.0)
                worst = max(worst, float(diff.max() / np.sqrt(np.mean(o_ref ** 2))))
        if (t + 1) % C == 0:
            nats.hybrid_attn_decode_commit(st, full["mask"][:, :, t // C].contiguous())
            for b in range(B):
                for h in range(H):
                    npo.decode_commit_chunk(ref[b][h], int(x["mask"][b, h, t // C]))
    assert worst <= TOL[dtype], worst


# ---- the score layer on the device (Eq. 8-9) ------------------------------------------------------------

def run_route(x, dtype):
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    X = torch.from_numpy(x["X"]).to(tdt).cuda()
    W = torch.from_numpy(x["W_s"]).cuda()
    mask_c, scores = nats.route_chunks(X, W, C)
    torch.cuda.synchronize()
    return mask_c, scores


@pytest.mark.parametrize("B,L,dm,H", [(2, 512, 1536, 6), (1, 64, 8, 1), (3, 1024, 2048, 16), (1, 192, 4088, 32), (1, 128, 8200, 3), (4, 32960, 64, 5)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_route_chunks_scores_and_mask(dtype, B, L, dm, H):
    from nats_inputs import make_score_inputs
    from oracle import nats_oracle
    x = make_score_inputs(B, L, dm, H, dtype, seed=31 + dm)
    mask_c, scores = run_route(x, dtype)
    ref_mask, ref_scores = nats_oracle.route_chunks(x["X"], x["W_s"], C)
    s = host(scores)
    assert s.shape == ref_scores.shape and tuple(mask_c.shape) == ref_mask.shape
    assert rel_err(s, ref_scores) <= TOL["f32"]       # fp32 sums of exact inputs, whatever X is stored in
    m = host(mask_c)
    # the decision is taken in fp32 on the device: it is exactly the argmax of the device's own scores ...
    own = (s[..., 0] >= s[..., 1]).astype(np.uint8).transpose(0, 2, 1)
    assert np.array_equal(m, own)
    # ... and equals the oracle's wherever the two scores are further apart than the fp32 error could bridge
    margin = np.abs(ref_scores[..., 0] - ref_scores[..., 1]).transpose(0, 2, 1)
    rms = np.sqrt(np.mean(ref_scores ** 2))
    clear = margin > 2 * TOL["f32"] * rms
    assert clear.mean() > 0.99
    assert np.array_equal(m[clear], ref_mask[clear])


def test_route_chunks_tie_goes_to_softmax_and_scores_are_optional():
    from nats_inputs import make_score_inputs
    x = make_score_inputs(2, 256, 512, 4, "bf16", seed=5)
    x["W_s"][1] = 0.0                      # head 1: both scores are exactly zero
    x["W_s"][2, 1] = x["W_s"][2, 0]        # head 2: both scores are the same sum
    mask_c, scores = run_route(x, "bf16")
    assert host(mask_c)[:, 1].all() and host(mask_c)[:, 2].all()
    X = torch.from_numpy(x["X"]).to(torch.bfloat16).cuda()
    m2, none = nats.route_chunks(X, torch.from_numpy(x["W_s"]).cuda(), C, want_scores=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(m2, mask_c)


def test_route_chunks_feeds_the_forward():
    """Mask produced on the device goes straight into the chunk-routed forward, no host round trip."""
    from nats_inputs import make_score_inputs
    from oracle import nats_oracle
    B, H, L, d = 2, 4, 512, 64
    x = make_fwd_inputs(B, H, L, d, "bf16", 0.1, seed=77)
    sx = make_score_inputs(B, L, H * d, H, "bf16", seed=78)
    mask_c, _ = run_route(sx, "bf16")
    ref_mask, _ = nats_oracle.route_chunks(sx["X"], sx["W_s"], C)
    assert np.array_equal(host(mask_c), ref_mask)   # seed chosen with every margin clear of rounding
    g = to_dev(x, "bf16")
    r = nats.hybrid_attn_fwd_ex(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], mask_c, C,
                                routing=nb.NATS_ROUTE_CHUNK, want=())
    torch.cuda.synchronize()
    x["mask"] = ref_mask
    ref = oracle(x, want=("O",))
    assert rel_err(host(r["O"]), ref["O"], stored("bf16")) <= TOL["bf16"]
