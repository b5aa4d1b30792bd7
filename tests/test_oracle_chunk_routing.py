"""Pins for the chunk-routed form of the oracle (Section 4.1: one routing decision per chunk,
both operations compute the intra-chunk part, the unchosen one is rolled back).

It is pinned to things other than itself:
  * a library attention routine with explicit boolean masks (softmax branch);
  * the per-token functions of the oracle, which have their own pins in test_oracle_pins.py:
    the outputs of chunk c equal those of a per-token run over tokens 0 .. end of chunk c in which
    the tokens of earlier softmax chunks are softmax tokens and the tokens of chunk c itself are
    linear tokens (linear branch), respectively softmax tokens (softmax branch);
  * special cases: all chunks linear (plain Gated DeltaNet + block-diagonal causal attention), all
    chunks softmax (full causal attention + per-chunk DeltaNet from a decayed-away state).
"""
import numpy as np
import pytest
import torch

from nats_inputs import make_fwd_inputs
from oracle import c_oracle, nats_oracle as no


def _inputs(L, d, seed, C, p=0.4):
    x = make_fwd_inputs(1, 1, L, d, "f32", 0.1, seed=seed)
    rng = np.random.default_rng(seed + 1000)
    mc = (rng.random(L // C) < p).astype(np.uint8)
    return {k: v[0, 0].astype(np.float64) for k, v in x.items() if k != "mask"}, mc


def _sdpa(q, k, v, allowed, scale):
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None], torch.from_numpy(k)[None, None], torch.from_numpy(v)[None, None],
        attn_mask=torch.from_numpy(allowed)[None, None], scale=scale)
    return out[0, 0].numpy()


@pytest.mark.parametrize("C", [4, 16])
def test_softmax_branch_equals_library_attention_with_the_chunk_mask(C):
    L, d = 64, 8
    x, mc = _inputs(L, d, 3, C)
    r = no.hybrid_head_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C, softmax_scale=0.7)
    i, j = np.arange(L)[:, None], np.arange(L)[None, :]
    allowed = ((mc[j // C] != 0) & (j // C < i // C)) | ((j // C == i // C) & (j <= i))
    np.testing.assert_allclose(r["O_nla"], _sdpa(x["Q"], x["K"], x["V"], allowed, 0.7), rtol=0, atol=1e-12)


@pytest.mark.parametrize("C", [4, 16])
def test_chunk_outputs_equal_per_token_runs_with_the_own_chunk_retyped(C):
    L, d = 48, 8
    x, mc = _inputs(L, d, 5, C)
    r = no.hybrid_head_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C, softmax_scale=1.3,
                                    la_scale=0.5)
    tok = np.repeat(mc, C)
    for c in range(L // C):
        end = (c + 1) * C
        m_lin = tok[:end].copy(); m_lin[c * C:] = 0      # own chunk written into the state
        m_sm = tok[:end].copy(); m_sm[c * C:] = 1        # own chunk visible to the softmax branch
        o_la, _ = no.gdn_recurrent(x["Q"][:end], x["K"][:end], x["V"][:end], x["alpha"][:end], x["beta"][:end],
                                   m_lin, la_scale=0.5)
        o_nla, lse = no.softmax_branch(x["Q"][:end], x["K"][:end], x["V"][:end], m_sm, 1.3)
        np.testing.assert_allclose(r["O_la"][c * C:end], o_la[c * C:], rtol=0, atol=1e-12)
        np.testing.assert_allclose(r["O_nla"][c * C:end], o_nla[c * C:], rtol=0, atol=1e-12)
        np.testing.assert_allclose(r["lse"][c * C:end], lse[c * C:], rtol=0, atol=1e-12)
    # the carried state is the per-token state with the chunk mask expanded to tokens
    _, S = no.gdn_recurrent(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], tok)
    np.testing.assert_allclose(r["S"], S, rtol=0, atol=1e-12)
    cnt, idx, n_s = no.compaction(tok)
    assert np.array_equal(r["cnt"], cnt) and np.array_equal(r["idx"], idx) and r["n_s"] == n_s


def test_all_linear_chunks_is_plain_deltanet_plus_block_diagonal_attention():
    L, d, C = 32, 8, 8
    x, _ = _inputs(L, d, 7, C)
    mc = np.zeros(L // C, dtype=np.uint8)
    r = no.hybrid_head_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C)
    o_la, S = no.gdn_recurrent(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], np.zeros(L, dtype=np.uint8))
    np.testing.assert_allclose(r["O_la"], o_la, rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["S"], S, rtol=0, atol=1e-12)
    i, j = np.arange(L)[:, None], np.arange(L)[None, :]
    allowed = (j // C == i // C) & (j <= i)
    np.testing.assert_allclose(r["O_nla"], _sdpa(x["Q"], x["K"], x["V"], allowed, 1.0 / np.sqrt(d)), rtol=0, atol=1e-12)
    assert r["n_s"] == 0


def test_all_softmax_chunks_is_full_causal_attention_plus_per_chunk_deltanet():
    L, d, C = 32, 8, 8
    x, _ = _inputs(L, d, 9, C)
    mc = np.ones(L // C, dtype=np.uint8)
    r = no.hybrid_head_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C)
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(x["Q"])[None, None], torch.from_numpy(x["K"])[None, None],
        torch.from_numpy(x["V"])[None, None], is_causal=True)[0, 0].numpy()
    np.testing.assert_allclose(r["O_nla"], out, rtol=0, atol=1e-12)
    for c in range(L // C):     # every chunk starts from a state that holds no write
        sl = slice(c * C, (c + 1) * C)
        o_la, _ = no.gdn_recurrent(x["Q"][sl], x["K"][sl], x["V"][sl], x["alpha"][sl], x["beta"][sl],
                                   np.zeros(C, dtype=np.uint8))
        np.testing.assert_allclose(r["O_la"][sl], o_la, rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["S"], 0.0, atol=0)
    assert r["n_s"] == L


@pytest.mark.parametrize("mode", [0, 1])
def test_c_oracle_matches_numpy_oracle_chunk_routed(mode):
    B, H, L, d, C = 2, 2, 64, 16, 16
    x = make_fwd_inputs(B, H, L, d, "f32", 0.1, seed=11)
    rng = np.random.default_rng(12)
    mc = (rng.random((B, H, L // C)) < 0.4).astype(np.uint8)
    w = rng.random((2, B, H, L)).astype(np.float32)
    S0 = rng.standard_normal((B, H, d, d)) * 0.1
    a = no.hybrid_fwd_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C, mode=mode,
                                   w_nla=w[0], w_la=w[1], S0=S0, la_scale=0.7)
    b = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, mode=mode, w_nla=w[0], w_la=w[1], S0=S0,
                     la_scale=0.7, chunk_routing=C)
    for key in ("O", "O_la", "O_nla", "lse", "S"):
        np.testing.assert_allclose(b[key], a[key], rtol=0, atol=1e-11)
    assert np.array_equal(a["cnt"], b["cnt"]) and np.array_equal(a["n_s"], b["n_s"])
    for bb in range(B):
        for h in range(H):
            n = a["n_s"][bb, h]
            assert np.array_equal(b["idx"][bb, h, :n], a["idx"][bb][h])


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_generation_with_reroll_continues_the_chunk_routed_forward(mode):
    """Prefill by the (pinned) chunk-routed forward, then token-by-token generation with provisional
    updates and a commit per chunk must reproduce the rows of the forward over the longer sequence,
    under every merge (sum, Eq. 21, the single-normalisation ablation)."""
    L0, n_new, d, C = 32, 24, 8, 8
    L = L0 + n_new
    x, mc = _inputs(L, d, 21, C, p=0.5)
    w = np.random.default_rng(22).random((2, L))
    full = no.hybrid_head_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C, la_scale=0.8, mode=mode,
                                       w_nla=w[0], w_la=w[1])
    pre = no.hybrid_head_chunk_routed(x["Q"][:L0], x["K"][:L0], x["V"][:L0], x["alpha"][:L0], x["beta"][:L0],
                                      mc[:L0 // C], C, la_scale=0.8)
    cap = L
    kc, vc = np.zeros((cap, d)), np.zeros((cap, d))
    kc[:pre["n_s"]] = x["K"][pre["idx"]]
    vc[:pre["n_s"]] = x["V"][pre["idx"]]
    st = no.decode_chunk_state(pre["S"], kc, vc, pre["n_s"])
    for t in range(L0, L):
        o, ovf = no.decode_step_chunk_routed(st, x["Q"][t], x["K"][t], x["V"][t], x["alpha"][t], x["beta"][t],
                                             la_scale=0.8, mode=mode, w_nla=w[0, t], w_la=w[1, t])
        assert not ovf
        np.testing.assert_allclose(o, full["O"][t], rtol=0, atol=1e-12)
        if mode == 2:   # the ablation's definition, written out: one RMS norm of the weighted sum
            y = w[0, t] * full["O_nla"][t] + w[1, t] * full["O_la"][t]
            np.testing.assert_allclose(o, y / np.sqrt(np.mean(y * y) + 1e-6), rtol=0, atol=1e-12)
        if (t + 1) % C == 0:
            no.decode_commit_chunk(st, mc[t // C])
    np.testing.assert_allclose(st["S"], full["S"], rtol=0, atol=1e-12)
    assert st["cache_len"] == full["n_s"]
    np.testing.assert_array_equal(st["k_cache"][:full["n_s"]], x["K"][full["idx"]])


def test_chunk_routed_separate_softmax_queries_and_keys():
    """With q_nla, k_nla the softmax branch of the chunk-routed operator is that of (q_nla, k_nla, v), the
    linear branch that of (q, k, v)."""
    import numpy as np
    from nats_inputs import make_fwd_inputs
    from oracle import nats_oracle as no2
    x = make_fwd_inputs(1, 1, 128, 8, "f32", 0.0, seed=31)
    rng = np.random.default_rng(32)
    q, k, v, a, b = x["Q"][0, 0], x["K"][0, 0], x["V"][0, 0], x["alpha"][0, 0], x["beta"][0, 0]
    qn, kn = rng.standard_normal(q.shape), rng.standard_normal(k.shape)
    mc = np.array([1, 0], dtype=np.uint8)
    r = no2.hybrid_head_chunk_routed(q, k, v, a, b, mc, 64, q_nla=qn, k_nla=kn)
    np.testing.assert_allclose(r["O_la"], no2.hybrid_head_chunk_routed(q, k, v, a, b, mc, 64)["O_la"], rtol=1e-12)
    np.testing.assert_allclose(r["O_nla"], no2.hybrid_head_chunk_routed(qn, kn, v, a, b, mc, 64)["O_nla"], rtol=1e-12)


# ---- Section 5, ablation (i): the inner part of a chunk by one operation only -----------------------------------
def _abl_inputs(L=48, d=6, C=8, seed=3):
    from nats_inputs import make_fwd_inputs
    x = make_fwd_inputs(1, 1, L, d, "f32", 0.2, seed=seed)
    mc = (np.random.default_rng(seed + 1).random(L // C) < 0.4).astype(np.uint8)
    return {k: v[0, 0].astype(np.float64) for k, v in x.items() if k != "mask"}, mc, C


def test_inner_part_by_the_linear_operation_only():
    """"GDN Out": the softmax branch is library attention under the mask "column in an earlier softmax chunk"
    (rows that see nothing give zero); the linear branch and the carried state are those of the method."""
    import torch
    x, mc, C = _abl_inputs()
    L = x["Q"].shape[0]
    r = no.hybrid_head_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C, softmax_scale=0.8, inner=2)
    ref = no.hybrid_head_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C, softmax_scale=0.8)
    np.testing.assert_array_equal(r["O_la"], ref["O_la"])
    np.testing.assert_array_equal(r["S"], ref["S"])
    ci = np.arange(L) // C
    allowed = (ci[None, :] < ci[:, None]) & np.repeat(mc != 0, C)[None, :]
    q, k, v = (torch.tensor(x[n][None, None].astype(np.float64)) for n in ("Q", "K", "V"))
    seen = allowed.any(1)
    safe = allowed | ~seen[:, None]          # rows that see nothing: attend to everything, then zeroed
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=torch.tensor(safe)[None, None], scale=0.8)[0, 0].numpy()
    o[~seen] = 0.0
    np.testing.assert_allclose(r["O_nla"], o, rtol=1e-10, atol=1e-12)
    assert np.all(np.isneginf(r["lse"][~seen])) and np.all(np.isfinite(r["lse"][seen]))
    np.testing.assert_allclose(r["O"], r["O_la"] + r["O_nla"], rtol=0, atol=0)


def test_inner_part_by_softmax_attention_only():
    """"SAttn Out": the linear branch's output is that of a run in which the chunk's own tokens write nothing,
    started from the method's carried state at the chunk's start; the softmax branch and the carried state are
    those of the method."""
    x, mc, C = _abl_inputs(seed=5)
    L = x["Q"].shape[0]
    S0 = 0.1 * np.random.default_rng(9).standard_normal((6, 6))
    r = no.hybrid_head_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C, la_scale=1.3, S0=S0, inner=1)
    ref = no.hybrid_head_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, C, la_scale=1.3, S0=S0)
    np.testing.assert_array_equal(r["O_nla"], ref["O_nla"])
    np.testing.assert_array_equal(r["S"], ref["S"])
    S = S0
    for c in range(L // C):
        sl = slice(c * C, (c + 1) * C)
        o, _ = no.gdn_recurrent(x["Q"][sl], x["K"][sl], x["V"][sl], x["alpha"][sl], np.zeros(C), np.zeros(C), S0=S,
                                 la_scale=1.3)
        np.testing.assert_allclose(r["O_la"][sl], o, rtol=1e-12, atol=1e-14)
        # the state the method carries into the next chunk
        _, S_lin = no.gdn_recurrent(x["Q"][sl], x["K"][sl], x["V"][sl], x["alpha"][sl], x["beta"][sl], np.zeros(C), S0=S)
        S = S_lin if mc[c] == 0 else np.prod(x["alpha"][sl]) * S


def test_weights_from_the_input_features():
    """Ablation (v): the same activations as Eq. 22 on W_x x_t, against library linear / softmax / sigmoid."""
    import torch
    rng = np.random.default_rng(4)
    X, W = rng.standard_normal((2, 10, 12)), rng.standard_normal((3, 2, 12))
    logits = torch.nn.functional.linear(torch.tensor(X), torch.tensor(W).reshape(6, 12)).reshape(2, 10, 3, 2).permute(0, 2, 1, 3)
    for act, f in ((0, lambda z: torch.softmax(z, -1)), (1, torch.sigmoid), (2, lambda z: z)):
        wn, wl = no.weights_from_x(X, W, act)
        w = f(logits).numpy()
        np.testing.assert_allclose(wn, w[..., 0], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(wl, w[..., 1], rtol=1e-12, atol=1e-14)
