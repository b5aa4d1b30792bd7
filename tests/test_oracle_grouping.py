"""Pins of the oracle's head grouping (Section 4.3: several softmax heads share the mask of one linear head).

The grouped operator is written with the linear head's wide state (G d value columns).  It must equal
(i) G independent single-head operators on repeated q, k, alpha, beta, mask (rows of the state never mix);
(ii) for the softmax heads, library attention over H G heads with the group's boolean mask repeated;
(iii) for the wide linear head, the product of the transition matrices of Eq. 19 written out here."""
import numpy as np
import pytest
import torch

from nats_inputs import make_chunk_mask, make_fwd_inputs
from oracle import nats_oracle as npo


def grouped_inputs(B, H, G, L, d, p, seed, own_qk=True):
    x = make_fwd_inputs(B, H, L, d, "f32", p, seed=seed)
    rng = np.random.default_rng(seed + 77)
    x["V"] = rng.standard_normal((B, H * G, L, d)).astype(np.float32)
    if own_qk:
        x["Q_nla"] = rng.standard_normal((B, H * G, L, d)).astype(np.float32)
        x["K_nla"] = rng.standard_normal((B, H * G, L, d)).astype(np.float32)
    return x


def rep(a, G):
    return np.repeat(a, G, axis=1)


@pytest.mark.parametrize("G", [1, 2, 3])
@pytest.mark.parametrize("mode", [0, 1])
def test_grouped_equals_independent_heads_with_repeated_mask(G, mode):
    B, H, L, d = 1, 2, 48, 8
    x = grouped_inputs(B, H, G, L, d, 0.2, seed=5 + G)
    rng = np.random.default_rng(3)
    w1, w2 = rng.random((B, H * G, L)), rng.random((B, H * G, L))
    S0 = rng.standard_normal((B, H * G, d, d)) * 0.1
    got = npo.hybrid_fwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], G, mode=mode,
                                 w_nla=w1, w_la=w2, S0=S0, Q_nla=x["Q_nla"], K_nla=x["K_nla"])
    ref = npo.hybrid_fwd(rep(x["Q"], G), rep(x["K"], G), x["V"], rep(x["alpha"], G), rep(x["beta"], G),
                         rep(x["mask"], G), mode=mode, w_nla=w1, w_la=w2, S0=S0, Q_nla=x["Q_nla"], K_nla=x["K_nla"])
    for key in ("O", "O_la", "O_nla", "S"):
        np.testing.assert_allclose(got[key], ref[key], rtol=1e-11, atol=1e-12, err_msg=key)
    np.testing.assert_array_equal(got["cnt"], ref["cnt"][:, ::G])
    np.testing.assert_array_equal(got["n_s"], ref["n_s"][:, ::G])


@pytest.mark.parametrize("G", [2, 3])
def test_grouped_chunk_routing_equals_independent_heads(G):
    B, H, L, d, C = 1, 2, 64, 8, 16
    x = grouped_inputs(B, H, G, L, d, 0.2, seed=11 + G)
    mc = make_chunk_mask(B, H, L // C, 0.4, 9)
    mc[:, :, 0] = 1
    got = npo.hybrid_fwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], mc, G, C=C, Q_nla=x["Q_nla"],
                                 K_nla=x["K_nla"])
    ref = npo.hybrid_fwd_chunk_routed(rep(x["Q"], G), rep(x["K"], G), x["V"], rep(x["alpha"], G), rep(x["beta"], G),
                                      rep(mc, G), C, Q_nla=x["Q_nla"], K_nla=x["K_nla"])
    for key in ("O", "O_la", "O_nla", "S", "lse"):
        np.testing.assert_allclose(got[key], ref[key], rtol=1e-11, atol=1e-12, err_msg=key)


def test_softmax_heads_of_a_group_against_library_attention():
    B, H, G, L, d = 2, 2, 3, 40, 16
    x = grouped_inputs(B, H, G, L, d, 0.25, seed=21)
    x["mask"][:, :, 0] = 1
    got = npo.hybrid_fwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], G, softmax_scale=0.3,
                                 Q_nla=x["Q_nla"], K_nla=x["K_nla"])
    q, k, v = (torch.from_numpy(x[n].astype(np.float64)) for n in ("Q_nla", "K_nla", "V"))
    col = torch.from_numpy(x["mask"] != 0).repeat_interleave(G, dim=1)            # [B, H G, L]: one mask per group
    allowed = col[:, :, None, :] & torch.tril(torch.ones(L, L, dtype=torch.bool))   # column j is a softmax token, j <= i
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=allowed, scale=0.3).numpy()
    np.testing.assert_allclose(got["O_nla"], ref, rtol=1e-10, atol=1e-12)


def test_wide_linear_head_against_transition_matrices():
    """S_t = S_{t-1} alpha_t (I - b_t k_t k_t^T) + b_t v_t k_t^T with b_t = beta_t (1 - m_t) and v_t the G d wide
    value row (Eq. 19, Eq. 14, Eq. 20), multiplied out for a group of three."""
    B, H, G, L, d = 1, 1, 3, 24, 6
    x = grouped_inputs(B, H, G, L, d, 0.3, seed=33, own_qk=False)
    got = npo.hybrid_fwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], G)
    q, k = x["Q"][0, 0].astype(np.float64), x["K"][0, 0].astype(np.float64)
    v = np.concatenate([x["V"][0, g].astype(np.float64) for g in range(G)], axis=-1)
    S = np.zeros((G * d, d))
    o = np.zeros((L, G * d))
    for t in range(L):
        b = float(x["beta"][0, 0, t]) * (1.0 - float(x["mask"][0, 0, t] != 0))
        S = S @ (float(x["alpha"][0, 0, t]) * (np.eye(d) - b * np.outer(k[t], k[t]))) + b * np.outer(v[t], k[t])
        o[t] = S @ q[t]
    for g in range(G):
        np.testing.assert_allclose(got["O_la"][0, g], o[:, g * d:(g + 1) * d], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(got["S"][0, g], S[g * d:(g + 1) * d], rtol=1e-10, atol=1e-12)


# --------------------------------------------------------------------------- #
# backward with head grouping
# --------------------------------------------------------------------------- #
def _grouped_loss(x, G, dO, S0, C=None):
    r = npo.hybrid_fwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], G, C=C, S0=S0)
    return float((r["O"] * dO).sum())


@pytest.mark.parametrize("G,routing_chunk", [(2, False), (3, False), (2, True)])
def test_grouped_backward_against_finite_differences_of_the_grouped_forward(G, routing_chunk):
    """The gradient of a shared input is the sum over the heads of its group: single entries of every gradient
    against central differences of sum(dO . O) of the grouped forward oracle (an independent function: the wide
    state of a linear head, one recurrence for the whole group)."""
    from oracle import nats_oracle_bwd as ob
    from nats_inputs import make_chunk_mask
    B, H, L, d, C = 1, 2, 16, 4, 4
    x = grouped_inputs(B, H, G, L, d, 0.3, seed=40 + G, own_qk=False)
    x = {k: np.asarray(v, dtype=np.float64) for k, v in x.items() if v is not None}
    x["mask"] = x["mask"].astype(np.uint8)
    Cc = None
    if routing_chunk:
        Cc = C
        x["mask"] = make_chunk_mask(B, H, L // C, 0.4, 77)
        x["mask"][:, :, 0] = 1
    rng = np.random.default_rng(5)
    dO = rng.standard_normal((B, H * G, L, d))
    S0 = 0.3 * rng.standard_normal((B, H * G, d, d))
    got = ob.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, C=Cc, S0=S0)
    eps = 1e-6
    for key, name in (("Q", "dQ"), ("K", "dK"), ("V", "dV"), ("alpha", "dalpha"), ("beta", "dbeta")):
        for _ in range(4):
            pos = tuple(int(rng.integers(0, n)) for n in x[key].shape)
            xp = {k: v.copy() for k, v in x.items()}
            xm = {k: v.copy() for k, v in x.items()}
            xp[key][pos] += eps
            xm[key][pos] -= eps
            fd = (_grouped_loss(xp, G, dO, S0, Cc) - _grouped_loss(xm, G, dO, S0, Cc)) / (2 * eps)
            assert abs(fd - got[name][pos]) <= 2e-6 * max(1.0, abs(fd)), (key, pos, fd, got[name][pos])
    for _ in range(4):
        pos = tuple(int(rng.integers(0, n)) for n in S0.shape)
        Sp, Sm = S0.copy(), S0.copy()
        Sp[pos] += eps
        Sm[pos] -= eps
        fd = (_grouped_loss(x, G, dO, Sp, Cc) - _grouped_loss(x, G, dO, Sm, Cc)) / (2 * eps)
        assert abs(fd - got["dS0"][pos]) <= 2e-6 * max(1.0, abs(fd)), (pos, fd, got["dS0"][pos])


def _own_qk_loss(x, G, dO, S0, C=None):
    r = npo.hybrid_fwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], G, C=C, S0=S0,
                               Q_nla=x["Q_nla"], K_nla=x["K_nla"])
    return float((r["O"] * dO).sum())


@pytest.mark.parametrize("G,routing_chunk", [(1, False), (1, True), (2, False), (3, True)])
def test_backward_with_own_softmax_queries_and_keys_against_finite_differences(G, routing_chunk):
    """Softmax heads with queries and keys of their own (Section 4.3): dQ_nla, dK_nla are the softmax branch's
    gradients, dQ, dK the linear branch's alone, dV the sum.  Single entries of each against central differences of
    sum(dO . O) of the forward oracle called with Q_nla, K_nla."""
    from oracle import nats_oracle_bwd as ob
    B, H, L, d, C = 1, 2, 16, 4, 4
    x = grouped_inputs(B, H, G, L, d, 0.3, seed=60 + G, own_qk=True)
    x = {k: np.asarray(v, dtype=np.float64) for k, v in x.items() if v is not None}
    x["mask"] = x["mask"].astype(np.uint8)
    Cc = None
    if routing_chunk:
        Cc = C
        x["mask"] = make_chunk_mask(B, H, L // C, 0.4, 78)
        x["mask"][:, :, 0] = 1
    rng = np.random.default_rng(6)
    dO = rng.standard_normal((B, H * G, L, d))
    S0 = 0.3 * rng.standard_normal((B, H * G, d, d))
    got = ob.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, C=Cc, S0=S0,
                                Q_nla=x["Q_nla"], K_nla=x["K_nla"])
    assert got["dQ_nla"].shape == (B, H * G, L, d) and got["dK_nla"].shape == (B, H * G, L, d)
    eps = 1e-6
    for key, name in (("Q", "dQ"), ("K", "dK"), ("V", "dV"), ("Q_nla", "dQ_nla"), ("K_nla", "dK_nla"),
                      ("alpha", "dalpha"), ("beta", "dbeta")):
        for _ in range(5):
            pos = tuple(int(rng.integers(0, n)) for n in x[key].shape)
            xp = {k: v.copy() for k, v in x.items()}
            xm = {k: v.copy() for k, v in x.items()}
            xp[key][pos] += eps
            xm[key][pos] -= eps
            fd = (_own_qk_loss(xp, G, dO, S0, Cc) - _own_qk_loss(xm, G, dO, S0, Cc)) / (2 * eps)
            assert abs(fd - got[name][pos]) <= 2e-6 * max(1.0, abs(fd)), (key, pos, fd, got[name][pos])
    # with the same tensors given twice the split gradients add up to the shared ones
    if G == 1:
        both = ob.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, C=Cc, S0=S0)
        same = ob.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, C=Cc, S0=S0,
                                     Q_nla=x["Q"], K_nla=x["K"])
        np.testing.assert_allclose(same["dQ"] + same["dQ_nla"], both["dQ"], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(same["dK"] + same["dK_nla"], both["dK"], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("G,mode,routing_chunk", [(2, 1, False), (3, 2, True)])
def test_grouped_backward_through_the_merges_against_finite_differences(G, mode, routing_chunk):
    """Eq. 21 (and its ablation) per output head, weights [B,H G,L]: gradients against central differences of the
    grouped forward oracle run with the same merge."""
    from oracle import nats_oracle_bwd as ob
    B, H, L, d, C = 1, 2, 16, 4, 4
    x = grouped_inputs(B, H, G, L, d, 0.3, seed=70 + G, own_qk=False)
    x = {k: np.asarray(v, dtype=np.float64) for k, v in x.items() if v is not None}
    x["mask"] = x["mask"].astype(np.uint8)
    Cc = None
    if routing_chunk:
        Cc = C
        x["mask"] = make_chunk_mask(B, H, L // C, 0.4, 79)
        x["mask"][:, :, 0] = 1
    rng = np.random.default_rng(8)
    x["w_nla"], x["w_la"] = rng.random((B, H * G, L)) + 0.2, rng.random((B, H * G, L)) + 0.2
    dO = rng.standard_normal((B, H * G, L, d))

    def loss(a):
        r = npo.hybrid_fwd_grouped(a["Q"], a["K"], a["V"], a["alpha"], a["beta"], a["mask"], G, C=Cc, mode=mode,
                                   w_nla=a["w_nla"], w_la=a["w_la"])
        return float((r["O"] * dO).sum())

    got = ob.hybrid_bwd_grouped(x["Q"], x["K"], x["V"], x["alpha"], x["beta"], x["mask"], dO, G, C=Cc, mode=mode,
                                w_nla=x["w_nla"], w_la=x["w_la"])
    eps = 1e-6
    for key, name in (("Q", "dQ"), ("K", "dK"), ("V", "dV"), ("alpha", "dalpha"), ("beta", "dbeta"),
                      ("w_nla", "dw_nla"), ("w_la", "dw_la")):
        for _ in range(4):
            pos = tuple(int(rng.integers(0, n)) for n in x[key].shape)
            xp, xm = {**x, key: x[key].copy()}, {**x, key: x[key].copy()}
            xp[key][pos] += eps
            xm[key][pos] -= eps
            fd = (loss(xp) - loss(xm)) / (2 * eps)
            assert abs(fd - got[name][pos]) <= 3e-6 * max(1.0, abs(fd)), (key, pos, fd, got[name][pos])
