"""Pins of the backward oracle (oracle/nats_oracle_bwd.py) to things other than itself: automatic
differentiation of an independently written forward (plain PyTorch fp64, CPU), a library attention routine,
the derivative with respect to an explicit multiplicative mask (Eq. 15), and central finite differences of
the forward oracle."""
import numpy as np
import pytest
import torch

from oracle import nats_oracle as npo
from oracle import nats_oracle_bwd as nbw


def inputs(L=20, d=5, seed=0, p=0.3):
    rng = np.random.default_rng(seed)
    q, k, v, do = (rng.standard_normal((L, d)) for _ in range(4))
    k /= np.linalg.norm(k, axis=1, keepdims=True)
    alpha = 1 / (1 + np.exp(-rng.normal(2, 0.5, L)))
    beta = 1 / (1 + np.exp(-rng.standard_normal(L)))
    mask = (rng.random(L) < p).astype(np.uint8)
    mask[0] = 1
    S0 = 0.1 * rng.standard_normal((d, d))
    return q, k, v, alpha, beta, mask, do, S0


def torch_forward(q, k, v, alpha, beta, mask, S0, scale, la_scale, linear_op, decay_on_softmax, M=None):
    """The operator's definition written with torch ops (autograd does the rest): Eq. 19 / 14 / 20 token by
    token, Eq. 11-12 as a dense masked softmax.  M: optional multiplicative mask on exp(A) (Eq. 11)."""
    L = q.shape[0]
    S = S0
    o_la = []
    for t in range(L):
        lin = mask[t] == 0
        if lin or decay_on_softmax:
            S = alpha[t] * S
        if lin:
            r = v[t] - (S @ k[t] if linear_op == 0 else 0.0)
            S = S + beta[t] * torch.outer(r, k[t])
        o_la.append(la_scale * (S @ q[t]))
    o_la = torch.stack(o_la)
    A = scale * (q @ k.T)
    vis = torch.tril(torch.ones(L, L, dtype=torch.bool)) & torch.from_numpy(mask != 0)[None, :]
    E = torch.where(vis, torch.exp(A - A.detach().max()), torch.zeros_like(A))
    if M is not None:
        E = E * M
    Z = E.sum(1, keepdim=True)
    P = torch.where(Z > 0, E / torch.where(Z > 0, Z, torch.ones_like(Z)), torch.zeros_like(E))
    return o_la + P @ v, S


@pytest.mark.parametrize("linear_op,decay_on_softmax", [(0, True), (1, True), (0, False), (1, False)])
@pytest.mark.parametrize("seed", [0, 1])
def test_backward_against_autograd(seed, linear_op, decay_on_softmax):
    q, k, v, alpha, beta, mask, do, S0 = inputs(seed=seed)
    scale, la_scale = 0.7, 1.3
    t = {n: torch.tensor(a, dtype=torch.float64, requires_grad=True)
         for n, a in dict(q=q, k=k, v=v, alpha=alpha, beta=beta, S0=S0).items()}
    O, _ = torch_forward(t["q"], t["k"], t["v"], t["alpha"], t["beta"], mask, t["S0"], scale, la_scale, linear_op,
                         decay_on_softmax)
    (O * torch.tensor(do)).sum().backward()
    r = nbw.hybrid_head_bwd(q, k, v, alpha, beta, mask, do, softmax_scale=scale, la_scale=la_scale, S0=S0,
                            linear_op=linear_op, decay_on_softmax=decay_on_softmax)
    for name, key in (("q", "dQ"), ("k", "dK"), ("v", "dV"), ("alpha", "dalpha"), ("beta", "dbeta"), ("S0", "dS0")):
        np.testing.assert_allclose(r[key], t[name].grad.numpy(), rtol=1e-9, atol=1e-11, err_msg=key)
    # the forward written here is the forward oracle's (so the gradients belong to the right function)
    ref = npo.hybrid_head(q, k, v, alpha, beta, mask, softmax_scale=scale, la_scale=la_scale, S0=S0,
                          linear_op=linear_op, decay_on_softmax=decay_on_softmax)
    np.testing.assert_allclose(O.detach().numpy(), ref["O"], rtol=1e-10, atol=1e-12)
    # Section 4.2: k, v of a softmax token get nothing from the linear branch, alpha, beta of it only the decay
    la = nbw.gdn_recurrent_bwd(q, k, v, alpha, beta, mask, do, S0, la_scale, linear_op, decay_on_softmax)
    soft = mask != 0
    assert np.all(la["dk"][soft] == 0) and np.all(la["dv"][soft] == 0) and np.all(la["dbeta"][soft] == 0)
    if not decay_on_softmax:
        assert np.all(la["dalpha"][soft] == 0)


def test_column_sums_are_the_derivative_of_a_multiplicative_mask():
    """Eq. 15: dM_ij = P_ij (dP_ij - do_i . o_i) is dLoss/dM_ij for O = (e^A * M / rowsum(e^A * M)) V at M = 1;
    g_j of the oracle is its column sum (Eq. 16 adds the columns of a chunk)."""
    q, k, v, alpha, beta, mask, do, S0 = inputs(L=16, d=4, seed=3, p=0.5)
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64) for a in (q, k, v))
    M = torch.ones(16, 16, dtype=torch.float64, requires_grad=True)
    O, _ = torch_forward(tq, tk, tv, torch.tensor(alpha), torch.tensor(beta), mask, torch.zeros(4, 4, dtype=torch.float64),
                         0.5, 0.0, 0, True, M=M)
    (O * torch.tensor(do)).sum().backward()
    r = nbw.softmax_branch_bwd(q, k, v, mask, 0.5, do)
    dM = M.grad.numpy()
    np.testing.assert_allclose(r["g"], dM.sum(0), rtol=1e-9, atol=1e-12)
    assert np.all(r["g"][mask == 0] == 0)
    # each row of dM sums to zero (softmax normalisation): so does the total of g
    assert abs(r["g"].sum()) < 1e-10


def test_all_softmax_reduces_to_library_attention_backward():
    q, k, v, alpha, beta, mask, do, S0 = inputs(L=24, d=8, seed=5)
    mask[:] = 1
    tq, tk, tv = (torch.tensor(a[None, None], dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    O = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=0.4)
    (O * torch.tensor(do)[None, None]).sum().backward()
    r = nbw.hybrid_head_bwd(q, k, v, alpha, beta, mask, do, softmax_scale=0.4)
    np.testing.assert_allclose(r["dQ"], tq.grad[0, 0].numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(r["dK"], tk.grad[0, 0].numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(r["dV"], tv.grad[0, 0].numpy(), rtol=1e-9, atol=1e-11)
    assert np.all(r["dbeta"] == 0)       # nothing is ever written


def test_single_entries_against_finite_differences():
    q, k, v, alpha, beta, mask, do, S0 = inputs(L=12, d=4, seed=7)
    r = nbw.hybrid_head_bwd(q, k, v, alpha, beta, mask, do, S0=S0)

    def loss(**over):
        a = dict(q=q, k=k, v=v, alpha=alpha, beta=beta)
        a.update(over)
        return float(np.sum(npo.hybrid_head(a["q"], a["k"], a["v"], a["alpha"], a["beta"], mask, S0=S0)["O"] * do))

    h = 1e-6
    for name, key, pos in (("q", "dQ", (5, 2)), ("k", "dK", (3, 1)), ("k", "dK", (0, 0)), ("v", "dV", (7, 3)),
                           ("alpha", "dalpha", (4,)), ("beta", "dbeta", (6,)), ("alpha", "dalpha", (0,))):
        base = dict(q=q, k=k, v=v, alpha=alpha, beta=beta)[name]
        up, dn = base.copy(), base.copy()
        up[pos] += h
        dn[pos] -= h
        fd = (loss(**{name: up}) - loss(**{name: dn})) / (2 * h)
        assert abs(fd - r[key][pos]) <= 1e-6 * max(1.0, abs(fd)), (name, pos, fd, r[key][pos])


def test_batched_wrapper_stacks_heads():
    rng = np.random.default_rng(9)
    B, H, L, d = 2, 2, 10, 4
    Q, K, V, dO = (rng.standard_normal((B, H, L, d)) for _ in range(4))
    alpha, beta = rng.random((B, H, L)) * 0.5 + 0.5, rng.random((B, H, L))
    mask = (rng.random((B, H, L)) < 0.3).astype(np.uint8)
    r = nbw.hybrid_bwd(Q, K, V, alpha, beta, mask, dO)
    one = nbw.hybrid_head_bwd(Q[1, 0], K[1, 0], V[1, 0], alpha[1, 0], beta[1, 0], mask[1, 0], dO[1, 0])
    for key in ("dQ", "dK", "dV", "dalpha", "dbeta", "g_nla"):
        np.testing.assert_array_equal(r[key][1, 0], one[key])


# --------------------------------------------------------------------------- #
# Eq. 17 and the backward under routing per chunk
# --------------------------------------------------------------------------- #
def test_linear_score_gradient_is_the_derivative_of_a_multiplier_on_the_write():
    """Eq. 14 / Eq. 17: put a multiplier mu_t on what token t adds to the state, S_t = S' + mu_t beta_t r_t k_t^T;
    dLoss/dmu_t at mu = 1 is the oracle's g_la[t] (sum of dS . written), zero for softmax tokens, and the chunk
    sums of Eq. 16-17 are the derivatives with respect to one multiplier per chunk."""
    q, k, v, alpha, beta, mask, do, S0 = inputs(L=24, d=5, seed=11, p=0.3)
    L = 24
    for linear_op in (0, 1):
        mu = torch.ones(L, dtype=torch.float64, requires_grad=True)
        tq, tk, tv, ta, tb = (torch.tensor(a, dtype=torch.float64) for a in (q, k, v, alpha, beta))
        S = torch.tensor(S0)
        o = []
        for t in range(L):
            S = ta[t] * S
            if mask[t] == 0:
                r = tv[t] - (S @ tk[t] if linear_op == 0 else 0.0)
                S = S + mu[t] * tb[t] * torch.outer(r, tk[t])
            o.append(1.3 * (S @ tq[t]))
        (torch.stack(o) * torch.tensor(do)).sum().backward()
        r = nbw.gdn_recurrent_bwd(q, k, v, alpha, beta, mask, do, S0, 1.3, linear_op, True)
        np.testing.assert_allclose(r["g_la"], mu.grad.numpy(), rtol=1e-9, atol=1e-12)
        assert np.all(r["g_la"][mask != 0] == 0)
        np.testing.assert_allclose(r["g_la"], beta * r["dbeta"], rtol=1e-9, atol=1e-12)   # the same number, seen from beta
        C = 8
        _, ds_la = nbw.score_gradients(np.zeros(L), r["g_la"], C)
        np.testing.assert_allclose(ds_la, mu.grad.numpy().reshape(L // C, C).sum(1), rtol=1e-12)


def torch_forward_chunk_routed(q, k, v, alpha, beta, mask_c, C, S0, scale, la_scale, linear_op, decay_on_softmax,
                               M=None, mu=None):
    """Routing per chunk written with torch ops, independently of the oracle: both operations compute the inner
    part of every chunk; between chunks the column mask of Eq. 12 (softmax) and Eq. 14 (linear) act.  M [L,L]:
    optional multiplier on exp(A) for the columns of earlier chunks; mu [L/C]: optional multiplier on what a linear
    chunk adds to the carried state."""
    L = q.shape[0]
    S = S0
    o_la = []
    for c in range(L // C):
        S_c, dec = S, 1.0
        for t in range(c * C, (c + 1) * C):
            S = alpha[t] * S
            dec = dec * alpha[t]
            r = v[t] - (S @ k[t] if linear_op == 0 else 0.0)
            S = S + beta[t] * torch.outer(r, k[t])
            o_la.append(la_scale * (S @ q[t]))
        if mask_c[c]:
            S = (dec if decay_on_softmax else 1.0) * S_c
        elif mu is not None:
            S = dec * S_c + mu[c] * (S - dec * S_c)
    o_la = torch.stack(o_la)
    A = scale * (q @ k.T)
    ci = torch.arange(L) // C
    soft_col = torch.from_numpy(np.repeat(np.asarray(mask_c) != 0, C))
    earlier = (ci[None, :] < ci[:, None]) & soft_col[None, :]
    own = (ci[None, :] == ci[:, None]) & torch.tril(torch.ones(L, L, dtype=torch.bool))
    E = torch.where(earlier | own, torch.exp(A - A.detach().max()), torch.zeros_like(A))
    if M is not None:
        E = torch.where(earlier, E * M, E)
    P = E / E.sum(1, keepdim=True)
    return o_la + P @ v, S


@pytest.mark.parametrize("linear_op,decay_on_softmax", [(0, True), (1, True), (0, False)])
@pytest.mark.parametrize("seed", [0, 1])
def test_chunk_routed_backward_against_autograd(seed, linear_op, decay_on_softmax):
    L, d, C = 24, 5, 4
    q, k, v, alpha, beta, _, do, S0 = inputs(L=L, d=d, seed=20 + seed)
    mask_c = (np.random.default_rng(30 + seed).random(L // C) < 0.4).astype(np.uint8)
    mask_c[0] = 1
    scale, la_scale = 0.6, 1.2
    t = {n: torch.tensor(a, dtype=torch.float64, requires_grad=True)
         for n, a in dict(q=q, k=k, v=v, alpha=alpha, beta=beta, S0=S0).items()}
    M = torch.ones(L, L, dtype=torch.float64, requires_grad=True)
    mu = torch.ones(L // C, dtype=torch.float64, requires_grad=True)
    O, S_end = torch_forward_chunk_routed(t["q"], t["k"], t["v"], t["alpha"], t["beta"], mask_c, C, t["S0"], scale,
                                          la_scale, linear_op, decay_on_softmax, M=M, mu=mu)
    (O * torch.tensor(do)).sum().backward()
    r = nbw.hybrid_head_chunk_routed_bwd(q, k, v, alpha, beta, mask_c, C, do, softmax_scale=scale, la_scale=la_scale,
                                         S0=S0, linear_op=linear_op, decay_on_softmax=decay_on_softmax)
    for name, key in (("q", "dQ"), ("k", "dK"), ("v", "dV"), ("alpha", "dalpha"), ("beta", "dbeta"), ("S0", "dS0")):
        np.testing.assert_allclose(r[key], t[name].grad.numpy(), rtol=1e-9, atol=1e-11, err_msg=key)
    # Eq. 15-16: column sums of the mask gradient, per chunk; Eq. 17: derivative of the chunk's multiplier
    np.testing.assert_allclose(r["dscore_nla"], M.grad.numpy().sum(0).reshape(L // C, C).sum(1), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(r["dscore_la"], mu.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.all(r["dscore_nla"][mask_c == 0] == 0) and np.all(r["dscore_la"][mask_c != 0] == 0)
    # the forward differentiated here is the forward oracle's
    ref = npo.hybrid_head_chunk_routed(q, k, v, alpha, beta, mask_c, C, softmax_scale=scale, la_scale=la_scale, S0=S0,
                                       linear_op=linear_op, decay_on_softmax=decay_on_softmax)
    np.testing.assert_allclose(O.detach().numpy(), ref["O"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(S_end.detach().numpy(), ref["S"], rtol=1e-10, atol=1e-12)


def test_chunk_routed_backward_single_entries_against_finite_differences():
    L, d, C = 16, 4, 4
    q, k, v, alpha, beta, _, do, S0 = inputs(L=L, d=d, seed=41)
    mask_c = np.array([1, 0, 1, 0], dtype=np.uint8)
    r = nbw.hybrid_head_chunk_routed_bwd(q, k, v, alpha, beta, mask_c, C, do, S0=S0)

    def loss(**over):
        a = dict(q=q, k=k, v=v, alpha=alpha, beta=beta)
        a.update(over)
        return float(np.sum(npo.hybrid_head_chunk_routed(a["q"], a["k"], a["v"], a["alpha"], a["beta"], mask_c, C,
                                                         S0=S0)["O"] * do))

    h = 1e-6
    for name, key, pos in (("q", "dQ", (9, 2)), ("k", "dK", (2, 1)), ("k", "dK", (6, 0)), ("v", "dV", (10, 3)),
                           ("alpha", "dalpha", (1,)), ("alpha", "dalpha", (9,)), ("beta", "dbeta", (5,)),
                           ("beta", "dbeta", (8,))):
        base = dict(q=q, k=k, v=v, alpha=alpha, beta=beta)[name]
        up, dn = base.copy(), base.copy()
        up[pos] += h
        dn[pos] -= h
        fd = (loss(**{name: up}) - loss(**{name: dn})) / (2 * h)
        assert abs(fd - r[key][pos]) <= 1e-6 * max(1.0, abs(fd)), (name, pos, fd, r[key][pos])


# --------------------------------------------------------------------------- #
# the normalised, weighted merges (Eq. 21; Section 5, ablation (iii))
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("with_weights", [True, False])
def test_merge_adjoint_against_autograd_of_a_library_rms_norm(mode, with_weights):
    rng = np.random.default_rng(31 + mode)
    L, d, eps = 9, 6, 1e-6
    o_la, o_nla, do = (rng.standard_normal((L, d)) for _ in range(3))
    o_nla[2] = 0.0                                     # a query that sees no softmax token
    wn, wl = (rng.random(L) + 0.1, rng.random(L) + 0.1) if with_weights else (None, None)
    default = 1.0 if mode == 2 else 0.5
    t_la, t_nla = (torch.tensor(a, requires_grad=True) for a in (o_la, o_nla))
    t_wn = torch.tensor(wn if with_weights else np.full(L, default), requires_grad=True)
    t_wl = torch.tensor(wl if with_weights else np.full(L, default), requires_grad=True)
    norm = lambda x: torch.nn.functional.rms_norm(x, (d,), eps=eps)
    if mode == 1:
        o = t_wn[:, None] * norm(t_nla) + t_wl[:, None] * norm(t_la)
    else:
        o = norm(t_wn[:, None] * t_nla + t_wl[:, None] * t_la)
    np.testing.assert_allclose(o.detach().numpy(), npo.combine(o_la, o_nla, mode, wn, wl, eps), rtol=1e-12, atol=1e-13)
    (o * torch.tensor(do)).sum().backward()
    do_la, do_nla, dwn, dwl = nbw.combine_bwd(o_la, o_nla, do, mode, wn, wl, eps)
    for got, want in ((do_la, t_la.grad), (do_nla, t_nla.grad), (dwn, t_wn.grad), (dwl, t_wl.grad)):
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-9, atol=1e-9 * float(want.abs().max()))


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("routing_chunk", [False, True])
def test_backward_through_the_merges_against_finite_differences(mode, routing_chunk):
    """Every gradient (the two weights' included) against central differences of sum(dO . O) of the forward oracle
    run with the same merge; softmax heads with queries and keys of their own in one of the cases."""
    L, d, C = 16, 4, 4
    q, k, v, alpha, beta, mask, do, S0 = inputs(L=L, d=d, seed=50 + mode)
    rng = np.random.default_rng(60 + mode)
    x = dict(q=q, k=k, v=v, alpha=alpha, beta=beta, w_nla=rng.random(L) + 0.2, w_la=rng.random(L) + 0.2)
    own = mode == 2
    if own:
        x["q_nla"], x["k_nla"] = rng.standard_normal((L, d)), rng.standard_normal((L, d))
    mask_c = np.array([1, 0, 1, 0], dtype=np.uint8)

    def forward(a):
        kw = dict(mode=mode, w_nla=a["w_nla"], w_la=a["w_la"], S0=S0, la_scale=1.3, q_nla=a.get("q_nla"),
                  k_nla=a.get("k_nla"))
        if routing_chunk:
            return npo.hybrid_head_chunk_routed(a["q"], a["k"], a["v"], a["alpha"], a["beta"], mask_c, C, **kw)["O"]
        return npo.hybrid_head(a["q"], a["k"], a["v"], a["alpha"], a["beta"], mask, **kw)["O"]

    kw = dict(S0=S0, la_scale=1.3, q_nla=x.get("q_nla"), k_nla=x.get("k_nla"), mode=mode, w_nla=x["w_nla"],
              w_la=x["w_la"])
    if routing_chunk:
        r = nbw.hybrid_head_chunk_routed_bwd(q, k, v, alpha, beta, mask_c, C, do, **kw)
    else:
        r = nbw.hybrid_head_bwd(q, k, v, alpha, beta, mask, do, **kw)
    names = [("q", "dQ"), ("k", "dK"), ("v", "dV"), ("alpha", "dalpha"), ("beta", "dbeta"), ("w_nla", "dw_nla"),
             ("w_la", "dw_la")] + ([("q_nla", "dQ_nla"), ("k_nla", "dK_nla")] if own else [])
    h = 1e-6
    for name, key in names:
        for _ in range(4):
            pos = tuple(int(rng.integers(0, n)) for n in x[name].shape)
            up, dn = {**x, name: x[name].copy()}, {**x, name: x[name].copy()}
            up[name][pos] += h
            dn[name][pos] -= h
            fd = float(np.sum((forward(up) - forward(dn)) * do)) / (2 * h)
            assert abs(fd - r[key][pos]) <= 3e-6 * max(1.0, abs(fd)), (name, pos, fd, r[key][pos])
