"""Pins for the CPU oracle: each check ties it to something other than itself --
a library routine, a closed form, an explicit transition-matrix product, the
support pattern of the paper's Fig. 1(c), or brute force -- chosen so that a
dropped term, a wrong sign/index or a transposed operand fails at least one.
Both oracle implementations (numpy and C) run every pin.
"""
import os

import numpy as np
import pytest
import torch

from nats_inputs import make_fwd_inputs
from oracle import c_oracle
from oracle import nats_oracle as npo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --- adapters: one (batch, head) through either implementation ------------- #
def _np_head(q, k, v, alpha, beta, mask, **kw):
    return npo.hybrid_head(q, k, v, alpha, beta, mask, **kw)


def _c_head(q, k, v, alpha, beta, mask, softmax_scale=None, la_scale=1.0, mode=0, w_nla=None,
            w_la=None, eps=1e-6, S0=None):
    f = lambda a: None if a is None else np.asarray(a)[None, None]
    r = c_oracle.fwd(f(q), f(k), f(v), f(alpha), f(beta), f(mask), softmax_scale, la_scale, mode,
                     f(w_nla), f(w_la), eps, f(S0))
    n = int(r["n_s"][0, 0])
    out = {key: r[key][0, 0] for key in ("O", "O_la", "O_nla", "lse", "S", "cnt")}
    out["idx"] = r["idx"][0, 0, :n]
    out["n_s"] = n
    return out


IMPLS = {"numpy": _np_head, "c": _c_head}


@pytest.fixture(params=list(IMPLS))
def head(request):
    return IMPLS[request.param]


def _f32ify(*arrs):
    """Both oracles take float32 inputs; make the test's own arithmetic see the same values."""
    return tuple(np.asarray(a, dtype=np.float32).astype(np.float64) for a in arrs)


def _rand(L, d, seed, p=0.2, dv=None):
    rng = np.random.default_rng(seed)
    dv = d if dv is None else dv
    q = rng.standard_normal((L, d)); k = rng.standard_normal((L, d)); v = rng.standard_normal((L, dv))
    q /= np.linalg.norm(q, axis=1, keepdims=True); k /= np.linalg.norm(k, axis=1, keepdims=True)
    alpha = 1 / (1 + np.exp(-(2 + 0.5 * rng.standard_normal(L))))
    beta = 1 / (1 + np.exp(-rng.standard_normal(L)))
    mask = (rng.random(L) < p).astype(np.uint8)
    q, k, v, alpha, beta = _f32ify(q, k, v, alpha, beta)
    return q, k, v, alpha, beta, mask


# --- softmax branch --------------------------------------------------------- #
def test_all_softmax_is_causal_softmax_attention(head):
    """All tokens softmax: Eq. 11 is textbook causal attention; the state is never written."""
    L, d = 48, 16
    q, k, v, a, b, _ = _rand(L, d, 1)
    mask = np.ones(L, dtype=np.uint8)
    scale = 0.7
    r = head(q, k, v, a, b, mask, softmax_scale=scale)
    tq, tk, tv = (torch.from_numpy(x)[None, None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)[0, 0].numpy()
    np.testing.assert_allclose(r["O_nla"], ref, rtol=0, atol=1e-13)
    assert np.all(r["O_la"] == 0.0) and np.all(r["S"] == 0.0)
    np.testing.assert_allclose(r["O"], ref, rtol=0, atol=1e-13)


def test_general_mask_is_column_masked_attention(head):
    """Eq. 11-12: dense attention with -inf on linear columns and above the diagonal."""
    L, d = 40, 8
    q, k, v, a, b, mask = _rand(L, d, 2, p=0.3)
    mask[0] = 1
    scale = 3.0
    r = head(q, k, v, a, b, mask, softmax_scale=scale)
    allowed = torch.from_numpy((mask[None, :] != 0) & (np.arange(L)[:, None] >= np.arange(L)[None, :]))
    tq, tk, tv = (torch.from_numpy(x)[None, None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=allowed[None, None], scale=scale)
    np.testing.assert_allclose(r["O_nla"], ref[0, 0].numpy(), rtol=0, atol=1e-13)
    logits = torch.where(allowed, scale * (tq[0, 0] @ tk[0, 0].T), torch.tensor(-float("inf"), dtype=torch.float64))
    np.testing.assert_allclose(r["lse"], torch.logsumexp(logits, dim=1).numpy(), rtol=0, atol=1e-13)


def test_empty_softmax_set_gives_zero_and_minus_inf(head):
    L, d = 12, 4
    q, k, v, a, b, _ = _rand(L, d, 3)
    mask = np.zeros(L, dtype=np.uint8); mask[5] = 1
    r = head(q, k, v, a, b, mask)
    assert np.all(r["O_nla"][:5] == 0) and np.all(np.isneginf(r["lse"][:5]))
    # a single visible key: softmax weight 1 -> output is that value row, lse is its logit
    np.testing.assert_allclose(r["O_nla"][5:], np.tile(v[5], (L - 5, 1)), atol=1e-15)
    np.testing.assert_allclose(r["lse"][5:], (q[5:] @ k[5]) / np.sqrt(d), atol=1e-15)


def test_softmax_shift_invariance_and_large_logits(head):
    """Huge logits must not overflow, and softmax weights are convex (rows of V = const -> const)."""
    L, d = 20, 4
    q, k, v, a, b, mask = _rand(L, d, 4, p=0.5)
    mask[0] = 1
    v[:] = 2.5
    r = head(q, k, v, a, b, mask, softmax_scale=5000.0)
    assert np.all(np.isfinite(r["O_nla"]))
    np.testing.assert_allclose(r["O_nla"], 2.5, atol=1e-12)


# --- linear branch: closed forms of the (gated) delta rule ------------------ #
def test_delta_rule_overwrites_with_constant_key(head):
    """alpha=1, beta=1, every key = e_1: S_t = v_t e_1^T, so o_t = v_t * q_t[0] (Eq. 18)."""
    L, d = 10, 6
    q, k, v, a, b, _ = _rand(L, d, 5)
    k[:] = 0; k[:, 0] = 1
    a[:] = 1; b[:] = 1
    r = head(q, k, v, a, b, np.zeros(L, dtype=np.uint8))
    np.testing.assert_allclose(r["O_la"], v * q[:, :1], atol=1e-14)
    np.testing.assert_allclose(r["S"][:, 0], v[-1], atol=1e-14)


def test_orthonormal_keys_give_gated_linear_attention(head):
    """Orthonormal keys: (I - b k k^T) never touches earlier writes, so
    S_t = sum_i (prod_{i<j<=t} alpha_j) beta_i v_i k_i^T  (unrolled Eq. 19)."""
    d = 12; L = d
    q, k, v, a, b, _ = _rand(L, d, 6)
    rot, _ = np.linalg.qr(np.random.default_rng(60).standard_normal((d, d)))
    k = np.asarray(rot.T[:L].astype(np.float32), dtype=np.float64)  # nearly orthonormal after f32 rounding
    r = head(q, k, v, a, b, np.zeros(L, dtype=np.uint8), la_scale=1.0)
    ref = np.zeros((L, d))
    for t in range(L):
        for i in range(t + 1):
            ref[t] += np.prod(a[i + 1:t + 1]) * b[i] * (k[i] @ q[t]) * v[i]
    np.testing.assert_allclose(r["O_la"], ref, atol=5e-7)   # f32 rounding of the keys breaks exact orthogonality


def test_beta_zero_and_retrieval_property(head):
    L, d = 16, 8
    q, k, v, a, b, _ = _rand(L, d, 7)
    z = np.zeros(L, dtype=np.uint8)
    r = head(q, k, v, a, np.zeros(L), z)
    assert np.all(r["O_la"] == 0)
    # beta=1 and unit keys: right after the write, S_t k_t == v_t (query = key reads the value back)
    k64 = k / np.linalg.norm(k, axis=1, keepdims=True)
    r = head(k64, k64, v, a, np.ones(L), z)   # q := k
    np.testing.assert_allclose(r["O_la"], v, atol=2e-6)  # keys are re-rounded to f32 inside -> not exactly unit


def test_transition_matrix_product_form(head):
    """Eq. 19 verbatim with explicit matrices, softmax tokens contributing alpha_t * I (Eq. 14, 20):
    S_t = S_{t-1} (alpha_t (I - beta_t k_t k_t^T)) + beta_t v_t k_t^T."""
    L, d, dv = 9, 5, 5
    q, k, v, a, b, mask = _rand(L, d, 8, p=0.35)
    S0 = np.random.default_rng(80).standard_normal((dv, d))
    r = head(q, k, v, a, b, mask, S0=S0, la_scale=0.5)
    S = S0.copy(); I = np.eye(d)
    for t in range(L):
        if mask[t] == 0:
            S = S @ (a[t] * (I - b[t] * np.outer(k[t], k[t]))) + b[t] * np.outer(v[t], k[t])
        else:
            S = S @ (a[t] * I)
        np.testing.assert_allclose(r["O_la"][t], 0.5 * (S @ q[t]), atol=1e-13)
    np.testing.assert_allclose(r["S"], S, atol=1e-13)


def test_softmax_token_equals_linear_token_with_beta_zero(head):
    L, d = 30, 8
    q, k, v, a, b, mask = _rand(L, d, 9, p=0.4)
    r1 = head(q, k, v, a, b, mask)
    r2 = head(q, k, v, a, b * (mask == 0), np.zeros(L, dtype=np.uint8))
    np.testing.assert_allclose(r1["O_la"], r2["O_la"], atol=1e-14)


def test_decay_applies_on_softmax_tokens():
    """Eq. 20: the state decays on softmax tokens too; the no-decay ablation must differ."""
    L, d = 30, 8
    q, k, v, a, b, mask = _rand(L, d, 10, p=0.4)
    o1, _ = npo.gdn_recurrent(q, k, v, a, b, mask)
    o2, _ = npo.gdn_recurrent(q, k, v, a, b, mask, decay_on_softmax=False)
    assert np.max(np.abs(o1 - o2)) > 1e-3
    # a pure run of softmax tokens after some writes: state shrinks by exactly prod(alpha)
    mask2 = np.zeros(L, dtype=np.uint8); mask2[20:] = 1
    _, S_all = npo.gdn_recurrent(q, k, v, a, b, mask2)
    _, S_20 = npo.gdn_recurrent(q[:20], k[:20], v[:20], a[:20], b[:20], mask2[:20])
    np.testing.assert_allclose(S_all, np.prod(a[20:]) * S_20, atol=1e-15)


@pytest.mark.parametrize("C", [1, 2, 16, 32, 64, 128])
def test_chunkwise_equals_recurrent(head, C):
    """Eq. 6-7: the chunkwise-parallel form reaches the token-recurrent result for any C."""
    L, d = 256, 16
    q, k, v, a, b, mask = _rand(L, d, 11, p=0.1)
    S0 = 0.1 * np.random.default_rng(110).standard_normal((d, d))
    r = head(q, k, v, a, b, mask, S0=S0)
    o_c, S_c = npo.gdn_chunkwise(q, k, v, a, b, mask, C, S0=S0)
    np.testing.assert_allclose(o_c, r["O_la"], atol=1e-12)
    np.testing.assert_allclose(S_c, r["S"], atol=1e-12)


# --- masks / structure ------------------------------------------------------- #
def _read_fig1c():
    blocks, cur = {}, None
    for line in open(os.path.join(GOLDEN, "fig1c_support.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = line.strip("[]"); blocks[cur] = []
        else:
            blocks[cur].append([int(ch) for ch in line])
    return np.array(blocks["nla"]), np.array(blocks["la"])


def test_fig1c_support_pattern(head):
    """Fig. 1(c): 12 tokens, chunk size 2, softmax chunks 1 and 4.  With V = I the branch
    outputs are the attention maps themselves; their supports must be Eq. 12 / Eq. 13."""
    M_nla, M_la = _read_fig1c()
    L = 12
    mask = np.zeros(L, dtype=np.uint8); mask[[0, 1, 6, 7]] = 1
    rng = np.random.default_rng(12)
    k = np.eye(L); q = rng.standard_normal((L, L)) + 3.0     # orthonormal keys, generic queries
    v = np.eye(L); a = np.ones(L); b = np.ones(L)
    r = head(q, k, v, a, b, mask)
    np.testing.assert_array_equal(r["O_nla"] > 0, M_nla.astype(bool))
    np.testing.assert_array_equal(np.abs(r["O_la"]) > 0, M_la.astype(bool))
    # rows of the softmax map sum to one wherever any key is visible
    np.testing.assert_allclose(r["O_nla"].sum(1), 1.0, atol=1e-14)
    # with orthonormal keys and alpha=beta=1 the linear map is exactly q_i . k_j on its support
    np.testing.assert_allclose(r["O_la"], q * M_la, atol=1e-14)


def test_compaction_against_numpy(head):
    L, d = 200, 4
    q, k, v, a, b, mask = _rand(L, d, 13, p=0.15)
    r = head(q, k, v, a, b, mask)
    np.testing.assert_array_equal(r["cnt"], np.cumsum(mask != 0))
    np.testing.assert_array_equal(np.asarray(r["idx"]), np.flatnonzero(mask))
    assert r["n_s"] == int(mask.sum())


# --- merge -------------------------------------------------------------------- #
def test_sum_merge_and_eq21_merge(head):
    L, d = 24, 16
    q, k, v, a, b, mask = _rand(L, d, 14, p=0.3)
    mask[0] = 1
    r0 = head(q, k, v, a, b, mask)
    np.testing.assert_allclose(r0["O"], r0["O_la"] + r0["O_nla"], atol=0)
    rng = np.random.default_rng(140)
    wn = rng.random(L).astype(np.float32).astype(np.float64); wl = 1 - wn
    wl = wl.astype(np.float32).astype(np.float64)
    eps = 1e-6
    r1 = head(q, k, v, a, b, mask, mode=1, w_nla=wn, w_la=wl, eps=eps)
    t = lambda x: torch.from_numpy(x)
    ref = (t(wn)[:, None] * torch.nn.functional.rms_norm(t(r0["O_nla"]), (d,), eps=eps)
           + t(wl)[:, None] * torch.nn.functional.rms_norm(t(r0["O_la"]), (d,), eps=eps)).numpy()
    np.testing.assert_allclose(r1["O"], ref, atol=1e-13)
    # default weights are 0.5 / 0.5
    r2 = head(q, k, v, a, b, mask, mode=1, eps=eps)
    ref2 = 0.5 * (torch.nn.functional.rms_norm(t(r0["O_nla"]), (d,), eps=eps)
                  + torch.nn.functional.rms_norm(t(r0["O_la"]), (d,), eps=eps)).numpy()
    np.testing.assert_allclose(r2["O"], ref2, atol=1e-13)


def test_all_linear_mask_merges_to_pure_gdn(head):
    L, d = 20, 8
    q, k, v, a, b, _ = _rand(L, d, 15)
    r = head(q, k, v, a, b, np.zeros(L, dtype=np.uint8))
    assert np.all(r["O_nla"] == 0)
    np.testing.assert_array_equal(r["O"], r["O_la"])
    assert r["n_s"] == 0


# --- tiny brute force: both branches as explicit L x L attention maps ---------- #
def test_tiny_bruteforce_attention_maps(head):
    """L=6, d=3.  Linear branch as the unrolled sum over writes i<=t of
    beta_i (v_i - S_{i-1}' k_i) k_i^T propagated by explicit transition products."""
    L, d = 6, 3
    q, k, v, a, b, mask = _rand(L, d, 16, p=0.4)
    mask[:] = [1, 0, 0, 1, 0, 0]
    r = head(q, k, v, a, b, mask, softmax_scale=1.0)
    I = np.eye(d)
    P = [a[t] * (I - (b[t] * np.outer(k[t], k[t]) if mask[t] == 0 else 0)) for t in range(L)]
    for t in range(L):
        S = np.zeros((d, d))
        for i in range(t + 1):
            if mask[i]:
                continue
            M = I.copy()
            for j in range(i + 1, t + 1):
                M = M @ P[j]
            S += b[i] * np.outer(v[i], k[i]) @ M
        np.testing.assert_allclose(r["O_la"][t], S @ q[t], atol=1e-14)
        w = np.array([np.exp(q[t] @ k[j]) if (mask[j] and j <= t) else 0.0 for j in range(L)])
        np.testing.assert_allclose(r["O_nla"][t], (w / w.sum()) @ v, atol=1e-14)


# --- decode ---------------------------------------------------------------------- #
def test_decode_continues_prefill():
    """fwd(L) state + compacted cache, then decode steps == the rows of fwd(L + n)."""
    L, n, d = 40, 12, 8
    q, k, v, a, b, mask = _rand(L + n, d, 17, p=0.3)
    mask[0] = 1
    full = npo.hybrid_head(q, k, v, a, b, mask)
    pre = npo.hybrid_head(q[:L], k[:L], v[:L], a[:L], b[:L], mask[:L])
    cap = L + n
    kc = np.zeros((cap, d)); vc = np.zeros((cap, d))
    kc[:pre["n_s"]] = k[pre["idx"]]; vc[:pre["n_s"]] = v[pre["idx"]]
    S, clen = pre["S"], pre["n_s"]
    # same thing through the C oracle's batched decode
    S_c = S[None, None].copy(); kc_c = kc[None, None].astype(np.float32); vc_c = vc[None, None].astype(np.float32)
    clen_c = np.array([[clen]], dtype=np.int32)
    for t in range(L, L + n):
        o, S, kc, vc, clen, ovf = npo.decode_step(S, kc, vc, clen, q[t], k[t], v[t], a[t], b[t], mask[t])
        assert not ovf
        np.testing.assert_allclose(o, full["O"][t], atol=1e-13)
        f = lambda x: np.asarray(x)[None, None]
        o_c, ovf_c = c_oracle.decode(S_c, kc_c, vc_c, clen_c, f(q[t]), f(k[t]), f(v[t]), f(a[t]), f(b[t]), f(mask[t]))
        np.testing.assert_allclose(o_c[0, 0], full["O"][t], atol=1e-13)
        assert ovf_c[0, 0] == 0
    np.testing.assert_allclose(S, full["S"], atol=1e-13)
    assert clen == full["n_s"] and clen_c[0, 0] == full["n_s"]


def test_decode_overflow_flag():
    d, cap = 4, 2
    rng = np.random.default_rng(18)
    S = np.zeros((d, d)); kc = rng.standard_normal((cap, d)); vc = rng.standard_normal((cap, d))
    q, k, v = rng.standard_normal((3, d))
    o, S2, kc2, vc2, n2, ovf = npo.decode_step(S, kc, vc, cap, q, k, v, 0.9, 0.5, 1)
    assert ovf and n2 == cap and np.array_equal(kc2, kc)
    S_c = S[None, None].copy(); kc_c = kc[None, None].astype(np.float32); vc_c = vc[None, None].astype(np.float32)
    n_c = np.array([[cap]], dtype=np.int32)
    f = lambda x: np.asarray(x, dtype=np.float32)[None, None]
    o_c, ovf_c = c_oracle.decode(S_c, kc_c, vc_c, n_c, f(q), f(k), f(v), f(0.9), f(0.5),
                                 np.array([[1]], dtype=np.uint8))
    assert ovf_c[0, 0] == 1 and n_c[0, 0] == cap


# --- the two implementations agree on a batched workload -------------------------- #
def test_c_and_numpy_agree_on_generated_workload():
    x = make_fwd_inputs(2, 3, 96, 16, "bf16", 0.15, seed=99, n_runs=2, run_len=5)
    r_np = npo.hybrid_fwd(**x)
    r_c = c_oracle.fwd(**x)
    for key in ("O", "O_la", "O_nla", "S"):
        np.testing.assert_allclose(r_c[key], r_np[key], atol=1e-13)
    np.testing.assert_allclose(r_c["lse"], r_np["lse"], atol=1e-13)
    np.testing.assert_array_equal(r_c["cnt"], r_np["cnt"])
    np.testing.assert_array_equal(r_c["n_s"], r_np["n_s"])
    for b in range(2):
        for h in range(3):
            n = r_np["n_s"][b, h]
            np.testing.assert_array_equal(r_c["idx"][b, h, :n], r_np["idx"][b][h])


# --- Eq. 22: the merge weights from the queries ---------------------------------------------- #
def test_eq22_weights_against_library_softmax_and_closed_forms():
    rng = np.random.default_rng(5)
    Q = rng.standard_normal((2, 3, 7, 16))
    W = rng.standard_normal((3, 2, 16))
    w_nla, w_la = npo.eq22_weights(Q, W)
    logits = torch.einsum("bhld,hkd->bhlk", torch.from_numpy(Q), torch.from_numpy(W))
    ref = torch.softmax(logits, dim=-1).numpy()
    np.testing.assert_allclose(w_nla, ref[..., 0], rtol=0, atol=1e-15)
    np.testing.assert_allclose(w_la, ref[..., 1], rtol=0, atol=1e-15)
    np.testing.assert_allclose(w_nla + w_la, 1.0, rtol=0, atol=1e-15)
    # equal weight vectors give 1/2 each; swapping the two rows swaps the two weights
    Weq = np.repeat(W[:, :1], 2, axis=1)
    a, b = npo.eq22_weights(Q, Weq)
    np.testing.assert_allclose(a, 0.5, atol=1e-15)
    np.testing.assert_allclose(b, 0.5, atol=1e-15)
    a, b = npo.eq22_weights(Q, W[:, ::-1])
    np.testing.assert_allclose(a, w_la, atol=1e-15)
    np.testing.assert_allclose(b, w_nla, atol=1e-15)
    # a head's weights depend on that head's rows of W only
    W2 = W.copy(); W2[1, 0] += 1.0
    a2, _ = npo.eq22_weights(Q, W2)
    np.testing.assert_allclose(a2[:, 0], w_nla[:, 0], atol=0)
    assert np.abs(a2[:, 1] - w_nla[:, 1]).max() > 1e-3


# --- Eq. 8-9: score layer and routing decision ------------------------------------------------ #
def test_route_chunks_against_library_pooling_and_argmax():
    rng = np.random.default_rng(6)
    B, L, dm, H, C = 2, 48, 24, 3, 8
    X = rng.standard_normal((B, L, dm))
    W = rng.standard_normal((H, 2, dm))
    mask_c, scores = npo.route_chunks(X, W, C)
    pooled = torch.nn.functional.avg_pool1d(torch.from_numpy(X).transpose(1, 2), C).transpose(1, 2)   # [B, L/C, dm]
    ref = torch.nn.functional.linear(pooled, torch.from_numpy(W).reshape(2 * H, dm)).reshape(B, L // C, H, 2).numpy()
    np.testing.assert_allclose(scores, ref, rtol=0, atol=1e-13)
    assert mask_c.shape == (B, H, L // C) and mask_c.dtype == np.uint8
    np.testing.assert_array_equal(mask_c, (ref[..., 0] >= ref[..., 1]).transpose(0, 2, 1))
    # a chunk of identical tokens scores like one of its tokens; scaling one operation's row flips the choice
    Xc = np.repeat(X[:, ::C], C, axis=1)
    _, s2 = npo.route_chunks(Xc, W, C)
    np.testing.assert_allclose(s2, np.einsum("bcd,hkd->bchk", X[:, ::C], W), rtol=0, atol=1e-13)
    W_flip = W.copy(); W_flip[:, 0] = W[:, 1]; W_flip[:, 1] = W[:, 0]
    m_flip, _ = npo.route_chunks(X, W_flip, C)
    assert np.array_equal(m_flip, 1 - mask_c)       # no ties in random data
    m_tie, _ = npo.route_chunks(X, np.repeat(W[:, :1], 2, axis=1), C)
    assert m_tie.min() == 1                          # a tie goes to operation 0, as argmax does


# ---- variants of the linear branch: Mamba2-style gated linear attention, no decay on softmax tokens ----------

def _variant_inputs(L=24, d=6, seed=3, p=0.3):
    rng = np.random.default_rng(seed)
    q, k, v = (rng.standard_normal((L, d)) for _ in range(3))
    k /= np.linalg.norm(k, axis=1, keepdims=True)
    alpha = 1 / (1 + np.exp(-rng.normal(2, 0.5, L)))
    beta = 1 / (1 + np.exp(-rng.standard_normal(L)))
    mask = (rng.random(L) < p).astype(np.uint8)
    return q, k, v, alpha, beta, mask


def test_gated_linear_op_is_masked_decayed_linear_attention():
    """linear_op=1 in closed form: o_t = sum over linear j <= t of (prod_{j<i<=t} alpha_i) beta_j (k_j.q_t) v_j,
    i.e. (Q K^T * decay * column mask) diag(beta) V: Eq. 10 with a decay mask, no delta correction."""
    q, k, v, alpha, beta, mask = _variant_inputs()
    L = len(alpha)
    o, S = npo.gdn_recurrent(q, k, v, alpha, beta, mask, linear_op=1)
    cum = np.cumsum(np.log(alpha))
    A = np.zeros((L, L))
    for t in range(L):
        for j in range(t + 1):
            if mask[j] == 0:
                A[t, j] = np.exp(cum[t] - cum[j]) * beta[j] * (k[j] @ q[t])
    np.testing.assert_allclose(o, A @ v, rtol=1e-10, atol=1e-12)
    S_ref = sum(np.exp(cum[-1] - cum[j]) * beta[j] * np.outer(v[j], k[j]) for j in range(L) if mask[j] == 0)
    np.testing.assert_allclose(S, S_ref, rtol=1e-10, atol=1e-12)
    # the delta rule gives something else as soon as two written keys overlap
    o_gdn, _ = npo.gdn_recurrent(q, k, v, alpha, beta, mask, linear_op=0)
    assert np.abs(o_gdn - o).max() > 1e-3


def test_no_decay_on_softmax_tokens_equals_alpha_one_there():
    q, k, v, alpha, beta, mask = _variant_inputs(seed=4)
    for op in (0, 1):
        o1, S1 = npo.gdn_recurrent(q, k, v, alpha, beta, mask, decay_on_softmax=False, linear_op=op)
        a2 = np.where(mask != 0, 1.0, alpha)
        o2, S2 = npo.gdn_recurrent(q, k, v, a2, beta, mask, linear_op=op)
        np.testing.assert_allclose(o1, o2, rtol=1e-12)
        np.testing.assert_allclose(S1, S2, rtol=1e-12)
        o3, _ = npo.gdn_recurrent(q, k, v, alpha, beta, mask, linear_op=op)
        assert np.abs(o3 - o1).max() > 1e-3


@pytest.mark.parametrize("op,freeze", [(1, 0), (0, 1), (1, 1)])
def test_c_oracle_variants_match_numpy(op, freeze):
    from oracle import c_oracle
    from nats_inputs import make_chunk_mask, make_fwd_inputs
    x = make_fwd_inputs(1, 2, 128, 8, "f32", 0.2, seed=12)
    r = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], linear_op=op, freeze_on_softmax=freeze)
    ref = npo.hybrid_fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], linear_op=op,
                        decay_on_softmax=not freeze)
    np.testing.assert_allclose(r["O"], ref["O"], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(r["S"], ref["S"], rtol=1e-9, atol=1e-11)
    # routing per chunk
    mc = make_chunk_mask(1, 2, 2, 0.5, 5, "alternate")
    r = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, chunk_routing=64, linear_op=op,
                     freeze_on_softmax=freeze)
    ref = npo.hybrid_fwd_chunk_routed(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, 64, linear_op=op,
                                     decay_on_softmax=not freeze)
    np.testing.assert_allclose(r["O"], ref["O"], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(r["S"], ref["S"], rtol=1e-9, atol=1e-11)
    # the defaults are untouched by a variant call before them
    r0 = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"])
    ref0 = npo.hybrid_fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"])
    np.testing.assert_allclose(r0["O"], ref0["O"], rtol=1e-9, atol=1e-11)


def test_chunk_routed_variants_carry_the_per_token_state():
    """Whatever the variant, the state handed from chunk to chunk under routing per chunk is the per-token
    state for the chunk mask expanded to tokens (the fact the kernels rely on)."""
    from nats_inputs import make_fwd_inputs
    x = make_fwd_inputs(1, 1, 192, 8, "f32", 0.2, seed=13)
    mc = np.array([0, 1, 0], dtype=np.uint8)
    for op, keep in ((1, True), (0, False), (1, False)):
        r = npo.hybrid_head_chunk_routed(x["Q"][0, 0], x["K"][0, 0], x["V"][0, 0], x["alpha"][0, 0], x["beta"][0, 0],
                                        mc, 64, linear_op=op, decay_on_softmax=keep)
        _, S = npo.gdn_recurrent(x["Q"][0, 0], x["K"][0, 0], x["V"][0, 0], x["alpha"][0, 0], x["beta"][0, 0],
                                np.repeat(mc, 64), decay_on_softmax=keep, linear_op=op)
        np.testing.assert_allclose(r["S"], S, rtol=1e-10, atol=1e-12)


def test_separate_softmax_queries_and_keys():
    """q_nla, k_nla replace q, k in the softmax branch only: O = O_la(q, k) + O_nla(q_nla, k_nla), each term
    being what the single-input operator gives for that pair; the decode step continues the same sequence."""
    x = make_fwd_inputs(1, 1, 48, 8, "f32", 0.3, seed=21)
    rng = np.random.default_rng(22)
    q, k, v = x["Q"][0, 0], x["K"][0, 0], x["V"][0, 0]
    a, b, m = x["alpha"][0, 0], x["beta"][0, 0], x["mask"][0, 0]
    qn, kn = rng.standard_normal(q.shape), rng.standard_normal(k.shape)
    r = npo.hybrid_head(q, k, v, a, b, m, q_nla=qn, k_nla=kn)
    np.testing.assert_allclose(r["O_la"], npo.hybrid_head(q, k, v, a, b, m)["O_la"], rtol=1e-12)
    np.testing.assert_allclose(r["O_nla"], npo.hybrid_head(qn, kn, v, a, b, m)["O_nla"], rtol=1e-12)
    np.testing.assert_allclose(r["O"], r["O_la"] + r["O_nla"], rtol=1e-12)
    # generation: prefix by the forward, then one token at a time
    L0 = 32
    pre = npo.hybrid_head(q[:L0], k[:L0], v[:L0], a[:L0], b[:L0], m[:L0], q_nla=qn[:L0], k_nla=kn[:L0])
    S, n = pre["S"], int(pre["n_s"])
    kc, vc = np.zeros((48, 8)), np.zeros((48, 8))
    kc[:n], vc[:n] = kn[pre["idx"][:n]], v[pre["idx"][:n]]
    for t in range(L0, 48):
        o, S, kc, vc, n, _ = npo.decode_step(S, kc, vc, n, q[t], k[t], v[t], a[t], b[t], m[t], q_nla=qn[t], k_nla=kn[t])
        np.testing.assert_allclose(o, r["O"][t], rtol=1e-9, atol=1e-11)


def test_merge_weight_activations_of_the_ablation():
    """act = 1: a library sigmoid of each logit; act = 2: the logits; act = 0 stays the softmax over the pair,
    which is the sigmoid of the logits' difference."""
    from scipy.special import expit
    rng = np.random.default_rng(41)
    Q = rng.standard_normal((2, 3, 7, 8))
    W = rng.standard_normal((3, 2, 8))
    logits = np.einsum("bhld,hkd->bhlk", Q, W)
    a1, b1 = npo.eq22_weights(Q, W, act=1)
    np.testing.assert_allclose(a1, expit(logits[..., 0]), rtol=1e-12)
    np.testing.assert_allclose(b1, expit(logits[..., 1]), rtol=1e-12)
    a2, b2 = npo.eq22_weights(Q, W, act=2)
    np.testing.assert_array_equal(a2, logits[..., 0])
    np.testing.assert_array_equal(b2, logits[..., 1])
    a0, b0 = npo.eq22_weights(Q, W)
    np.testing.assert_allclose(a0, expit(logits[..., 0] - logits[..., 1]), rtol=1e-12)
    np.testing.assert_allclose(a0 + b0, 1.0, rtol=1e-12)


def test_single_normalisation_merge_against_library_rms_norm():
    """combine mode 2 (Section 5, ablation (iii)): a library RMS norm of the weighted sum; the C oracle agrees."""
    rng = np.random.default_rng(51)
    o_la, o_nla = rng.standard_normal((9, 16)), rng.standard_normal((9, 16))
    wn, wl = rng.random(9) + 0.5, rng.random(9) + 0.5
    ref = torch.nn.functional.rms_norm(torch.tensor(wn[:, None] * o_nla + wl[:, None] * o_la), (16,), eps=1e-6).numpy()
    np.testing.assert_allclose(npo.combine(o_la, o_nla, 2, wn, wl, 1e-6), ref, rtol=1e-12)
    np.testing.assert_allclose(npo.combine(o_la, o_nla, 2, None, None, 1e-6),
                               torch.nn.functional.rms_norm(torch.tensor(o_nla + o_la), (16,), eps=1e-6).numpy(), rtol=1e-12)
    x = make_fwd_inputs(1, 2, 64, 8, "f32", 0.3, seed=52)
    w = rng.random((2, 1, 2, 64)).astype(np.float32)
    r = c_oracle.fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], mode=2, w_nla=w[0], w_la=w[1])
    ref = npo.hybrid_fwd(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], mode=2, w_nla=w[0], w_la=w[1])
    np.testing.assert_allclose(r["O"], ref["O"], rtol=1e-9, atol=1e-12)
