"""CPU oracle for the backward pass of the NAtS-L hybrid attention operator (TEST INFRASTRUCTURE ONLY).

Plain fp64 numpy, token by token: the adjoint of the forward oracle's own loops (nats_oracle.py), written
out by hand.  Nothing in the product path may import this file; it shares no code with the HIP kernels.

Given dO = dLoss/dO for the plain-sum merge O = O_la + O_nla (Section 4.1), per (batch, head):

  * linear branch   -- reverse of the recurrence  S <- alpha S;  S <- S + beta (v - S k) k^T  (Eq. 19, written
    for linear tokens only, Eq. 14; decay at every token, Eq. 20);  o = la_scale S q.  Gives dq, dk, dv,
    dalpha, dbeta and the gradient of the initial state.  k and v of a softmax token get nothing from this
    branch (Section 4.2: the gradient is zero for an operation a token is inactive for).
  * softmax branch  -- the usual attention backward over the softmax columns j <= i, and the column sums
    of Eq. 15:  dM_ij = P_ij (dP_ij - do_i . o_i),  g_j = sum_i dM_ij,  which Eq. 16 adds up per chunk into
    the gradient of the softmax score.
  * score gradient of the linear operation (Eq. 17, "sum of dS . S" over a chunk): the linear mask multiplies what a
    token (a chunk) adds to the carried state (Eq. 14), so its gradient is the sum over the state's entries of
    (gradient of the loss with respect to the state after the write) x (what was written); a token or chunk that is
    inactive for an operation gets no score gradient for it (Section 4.2, last paragraph).
  * routing per chunk (hybrid_head_chunk_routed_bwd): the adjoint of nats_oracle.hybrid_head_chunk_routed, in
    which both operations compute every chunk's inner part and the masks act between chunks.
  * the normalised, weighted merges (Eq. 21 and its single-normalisation ablation; combine_bwd): the merge acts on
    the two branches' output rows, so its adjoint turns dO into one gradient per branch (and the gradients of the
    two weights), and each branch's adjoint then runs on its own; the branch outputs it needs are taken from the
    forward oracle.

Parity pins: tests/test_oracle_bwd_pins.py checks every output against automatic differentiation of an
independently written forward (plain PyTorch fp64 on the CPU), the column sums against the derivative with
respect to an explicit multiplicative mask, special cases against a library attention routine, and single
entries against central finite differences of the forward oracle.
"""
from __future__ import annotations

import numpy as np

from . import nats_oracle as _fwd   # the forward oracle's branch outputs, needed by the adjoint of the merge


def combine_bwd(o_la, o_nla, do, mode, w_nla=None, w_la=None, eps=1e-6):
    """Adjoint of nats_oracle.combine for rows o_la, o_nla, do [L,d] and weights [L] (None: the forward's defaults).
    mode 0: the plain sum; 1: Eq. 21, O = w_nla RMSNorm(o_nla) + w_la RMSNorm(o_la); 2: RMSNorm(w_nla o_nla + w_la o_la).
    RMSNorm(x) = x / sqrt(mean(x^2) + eps) without a gain, so for y = x r, r = (mean(x^2) + eps)^(-1/2):
        dx = r (dy - y (y . dy) / d).
    Returns (do_la, do_nla, dw_nla, dw_la); the weight gradients are zero arrays for mode 0."""
    o_la, o_nla, do = (np.asarray(a, dtype=np.float64) for a in (o_la, o_nla, do))
    L, d = o_la.shape
    if mode == 0:
        return do, do, np.zeros(L), np.zeros(L)
    default = 1.0 if mode == 2 else 0.5
    wn = np.full(L, default) if w_nla is None else np.asarray(w_nla, dtype=np.float64)
    wl = np.full(L, default) if w_la is None else np.asarray(w_la, dtype=np.float64)

    def norm_bwd(x, dy):                       # rows: y = x r;  returns (y, dx)
        r = 1.0 / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + eps)
        y = x * r
        return y, r * (dy - y * np.sum(y * dy, axis=1, keepdims=True) / d)

    if mode == 2:
        z = wn[:, None] * o_nla + wl[:, None] * o_la
        _, dz = norm_bwd(z, do)
        return wl[:, None] * dz, wn[:, None] * dz, np.sum(dz * o_nla, axis=1), np.sum(dz * o_la, axis=1)
    y_n, dx_n = norm_bwd(o_nla, wn[:, None] * do)
    y_l, dx_l = norm_bwd(o_la, wl[:, None] * do)
    return dx_l, dx_n, np.sum(do * y_n, axis=1), np.sum(do * y_l, axis=1)


def gdn_recurrent_bwd(q, k, v, alpha, beta, mask, do, S0=None, la_scale=1.0, linear_op=0, decay_on_softmax=True):
    """Adjoint of nats_oracle.gdn_recurrent.  do [L,d_v].

    Returns dict(dq, dk, dv [L,d], dalpha, dbeta [L], dS0 [d_v,d_k])."""
    q, k, v, do = (np.asarray(a, dtype=np.float64) for a in (q, k, v, do))
    alpha = np.asarray(alpha, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    L, d_k = k.shape
    d_v = v.shape[1]
    S = np.zeros((d_v, d_k)) if S0 is None else np.array(S0, dtype=np.float64)
    # forward, keeping what the reverse sweep needs: the state before each token, after its decay, after its write
    S_prev, S_dec, S_new, resid = [], [], [], []
    for t in range(L):
        linear = (mask[t] == 0)
        S_prev.append(S)
        a = alpha[t] if (linear or decay_on_softmax) else 1.0
        S = a * S
        S_dec.append(S)
        r = np.zeros(d_v)
        if linear:
            r = v[t] - (S @ k[t] if linear_op == 0 else 0.0)
            S = S + beta[t] * np.outer(r, k[t])
        resid.append(r)
        S_new.append(S)
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    dalpha, dbeta = np.zeros(L), np.zeros(L)
    g_la = np.zeros(L)                              # Eq. 17 per token: sum(dS . written) for linear tokens
    dS = np.zeros((d_v, d_k))                       # dLoss/dS after token t, from the tokens behind it
    for t in range(L - 1, -1, -1):
        linear = (mask[t] == 0)
        # o_t = la_scale S_t q_t
        dq[t] = la_scale * (S_new[t].T @ do[t])
        dS = dS + la_scale * np.outer(do[t], q[t])
        if linear:                                  # S_t = Sd + beta r k^T,  r = v - Sd k (delta rule) or v
            r = resid[t]
            g_la[t] = np.sum(dS * (S_new[t] - S_dec[t]))   # dS is the gradient w.r.t. the state after the write
            dSk = dS @ k[t]                         # [d_v]
            dbeta[t] = r @ dSk
            dr = beta[t] * dSk
            dk[t] = beta[t] * (dS.T @ r)
            dv[t] = dr
            if linear_op == 0:
                dk[t] -= S_dec[t].T @ dr
                dS = dS - np.outer(dr, k[t])
        if linear or decay_on_softmax:              # Sd = alpha S_{t-1}
            dalpha[t] = np.sum(dS * S_prev[t])
            dS = alpha[t] * dS
    return {"dq": dq, "dk": dk, "dv": dv, "dalpha": dalpha, "dbeta": dbeta, "dS0": dS, "g_la": g_la}


def score_gradients(g_nla, g_la, C):
    """Eq. 16 and Eq. 17 at the granularity of chunks of C tokens: the per-token sums added up per chunk
    (last axis L -> L / C).  Returns (dscore_nla, dscore_la)."""
    g_nla, g_la = np.asarray(g_nla, dtype=np.float64), np.asarray(g_la, dtype=np.float64)
    shp = g_nla.shape[:-1] + (g_nla.shape[-1] // C, C)
    return g_nla.reshape(shp).sum(-1), g_la.reshape(shp).sum(-1)


def softmax_branch_bwd(q, k, v, mask, scale, do):
    """Adjoint of nats_oracle.softmax_branch, plus g [L]: the column sums of Eq. 15 (zero at linear tokens).

    Returns dict(dq, dk, dv, g)."""
    q, k, v, do = (np.asarray(a, dtype=np.float64) for a in (q, k, v, do))
    L = q.shape[0]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    g = np.zeros(L)
    for i in range(L):
        J = np.flatnonzero(np.asarray(mask[:i + 1]) != 0)
        if J.size == 0:
            continue
        s = scale * (k[J] @ q[i])
        p = np.exp(s - s.max())
        p /= p.sum()
        o = p @ v[J]
        dp = v[J] @ do[i]                           # dLoss/dP_ij
        dm = p * (dp - do[i] @ o)                   # Eq. 15; also dLoss/ds_ij
        g[J] += dm
        dv[J] += np.outer(p, do[i])
        dq[i] = scale * (dm @ k[J])
        dk[J] += scale * np.outer(dm, q[i])
    return {"dq": dq, "dk": dk, "dv": dv, "g": g}


def hybrid_head_bwd(q, k, v, alpha, beta, mask, do, softmax_scale=None, la_scale=1.0, S0=None, linear_op=0,
                    decay_on_softmax=True, q_nla=None, k_nla=None, mode=0, w_nla=None, w_la=None, eps=1e-6):
    """Backward of nats_oracle.hybrid_head.  With the plain-sum merge (mode 0) dO goes to both branches as it is; with
    the merges of Eq. 21 (mode 1) and its ablation (mode 2) each branch receives the merge's gradient for its own
    output rows (combine_bwd), and dw_nla, dw_la [L] are returned as well.
    q_nla, k_nla (both or neither; Section 4.3: the two operations normalise the shared projections differently): the
    softmax branch's own queries and keys.  Their gradients are then returned apart as dQ_nla, dK_nla, and dQ, dK are
    the linear branch's alone; V is shared, dV stays the sum."""
    d_k = np.asarray(q).shape[-1]
    scale = (1.0 / np.sqrt(d_k)) if softmax_scale is None else softmax_scale
    do_la = do_nla = do
    merged = {}
    if mode != 0:
        fw = _fwd.hybrid_head(q, k, v, alpha, beta, mask, softmax_scale, la_scale, 0, S0=S0, linear_op=linear_op,
                              decay_on_softmax=decay_on_softmax, q_nla=q_nla, k_nla=k_nla)
        do_la, do_nla, dwn, dwl = combine_bwd(fw["O_la"], fw["O_nla"], do, mode, w_nla, w_la, eps)
        merged = {"dw_nla": dwn, "dw_la": dwl}
    la = gdn_recurrent_bwd(q, k, v, alpha, beta, mask, do_la, S0, la_scale, linear_op, decay_on_softmax)
    out = {"dV": None, "dalpha": la["dalpha"], "dbeta": la["dbeta"], "dS0": la["dS0"], "g_la": la["g_la"]}
    out.update(merged)
    if q_nla is None:
        nla = softmax_branch_bwd(q, k, v, mask, scale, do_nla)
        out.update(dQ=la["dq"] + nla["dq"], dK=la["dk"] + nla["dk"])
    else:
        nla = softmax_branch_bwd(q_nla, k_nla, v, mask, scale, do_nla)
        out.update(dQ=la["dq"], dK=la["dk"], dQ_nla=nla["dq"], dK_nla=nla["dk"])
    out["dV"] = la["dv"] + nla["dv"]
    out["g_nla"] = nla["g"]
    return out


def hybrid_bwd(Q, K, V, alpha, beta, mask, dO, softmax_scale=None, la_scale=1.0, S0=None, linear_op=0,
               decay_on_softmax=True, Q_nla=None, K_nla=None, mode=0, w_nla=None, w_la=None, eps=1e-6):
    """All (b,h) of [B,H,L,d] inputs; returns a dict of stacked fp64 arrays (with Q_nla, K_nla [B,H,L,d] also
    dQ_nla, dK_nla; with mode 1 or 2 and weights [B,H,L] or None also dw_nla, dw_la [B,H,L])."""
    B, H, L, d = np.asarray(Q).shape
    out = {"dQ": np.zeros((B, H, L, d)), "dK": np.zeros((B, H, L, d)), "dV": np.zeros((B, H, L, d)),
           "dalpha": np.zeros((B, H, L)), "dbeta": np.zeros((B, H, L)), "dS0": np.zeros((B, H, d, d)),
           "g_nla": np.zeros((B, H, L)), "g_la": np.zeros((B, H, L))}
    if Q_nla is not None:
        out.update(dQ_nla=np.zeros((B, H, L, d)), dK_nla=np.zeros((B, H, L, d)))
    if mode != 0:
        out.update(dw_nla=np.zeros((B, H, L)), dw_la=np.zeros((B, H, L)))
    for b in range(B):
        for h in range(H):
            r = hybrid_head_bwd(Q[b, h], K[b, h], V[b, h], alpha[b, h], beta[b, h], mask[b, h], dO[b, h],
                                softmax_scale, la_scale, None if S0 is None else S0[b, h], linear_op,
                                decay_on_softmax, None if Q_nla is None else Q_nla[b, h],
                                None if K_nla is None else K_nla[b, h], mode,
                                None if w_nla is None else w_nla[b, h], None if w_la is None else w_la[b, h], eps)
            for key in out:
                out[key][b, h] = r[key]
    return out


# --------------------------------------------------------------------------- #
# routing per chunk (Section 4.1 as stated; Section 4.2 for the score gradients)
# --------------------------------------------------------------------------- #
def hybrid_head_chunk_routed_bwd(q, k, v, alpha, beta, mask_c, C, do, softmax_scale=None, la_scale=1.0, S0=None,
                                 linear_op=0, decay_on_softmax=True, q_nla=None, k_nla=None, mode=0, w_nla=None,
                                 w_la=None, eps=1e-6):
    """Adjoint of nats_oracle.hybrid_head_chunk_routed (plain-sum merge).

    Forward being differentiated, per chunk c with carried state S_c: inside the chunk Eq. 19 runs on every token
    from S_c (the provisional states feed the chunk's own outputs); a linear chunk hands on its last provisional
    state, a softmax chunk hands on decay_c S_c (its writes are dropped).  Query i attends to all tokens of earlier
    softmax chunks and to the tokens j <= i of its own chunk.
    Score gradients (one per chunk): dscore_nla[c] = sum over the columns j of softmax chunk c and the queries i of
    later chunks of dM_ij (Eq. 15-16; the inner part of a chunk is computed whatever its type, no mask stands on
    it); dscore_la[c] = sum(dS_{c+1} . (S_{c+1} - decay_c S_c)) for a linear chunk (Eq. 17); zero where the chunk is
    inactive for the operation.
    q_nla, k_nla (both or neither): the softmax branch's own queries and keys; their gradients come back apart as
    dQ_nla, dK_nla and dQ, dK are the linear branch's alone.
    mode 1, 2 (the merges of Eq. 21 and its ablation, weights w_nla, w_la [L] or None): each branch runs on the
    merge's gradient for its own rows (combine_bwd); dw_nla, dw_la [L] are returned as well.
    Returns dict(dQ, dK, dV [L,d], dalpha, dbeta [L], dS0, dscore_nla, dscore_la [L/C])."""
    q, k, v, do = (np.asarray(a, dtype=np.float64) for a in (q, k, v, do))
    do_la = do_nla = do
    merged = {}
    if mode != 0:
        fw = _fwd.hybrid_head_chunk_routed(q, k, v, alpha, beta, mask_c, C, softmax_scale, la_scale, 0, S0=S0,
                                           linear_op=linear_op, decay_on_softmax=decay_on_softmax, q_nla=q_nla,
                                           k_nla=k_nla)
        do_la, do_nla, dwn, dwl = combine_bwd(fw["O_la"], fw["O_nla"], do, mode, w_nla, w_la, eps)
        merged = {"dw_nla": dwn, "dw_la": dwl}
    own_qk = q_nla is not None
    qn = np.asarray(q_nla, dtype=np.float64) if own_qk else q
    kn = np.asarray(k_nla, dtype=np.float64) if own_qk else k
    alpha = np.asarray(alpha, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    mask_c = np.asarray(mask_c).reshape(-1) != 0
    L, d_k = k.shape
    d_v = v.shape[1]
    n_c = L // C
    scale = (1.0 / np.sqrt(d_k)) if softmax_scale is None else softmax_scale
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    dqn, dkn = (np.zeros_like(q), np.zeros_like(k)) if own_qk else (dq, dk)   # shared: both branches add to dq, dk
    dalpha, dbeta = np.zeros(L), np.zeros(L)
    ds_nla, ds_la = np.zeros(n_c), np.zeros(n_c)

    # ---- softmax branch ----
    earlier = []
    for c in range(n_c):
        for i in range(c * C, (c + 1) * C):
            own = list(range(c * C, i + 1))
            J = np.asarray(earlier + own, dtype=np.int64)
            s = scale * (kn[J] @ qn[i])
            p = np.exp(s - s.max())
            p /= p.sum()
            o = p @ v[J]
            dm = p * (v[J] @ do_nla[i] - do_nla[i] @ o)   # Eq. 15 (also dLoss/ds_ij)
            for jj, j in enumerate(J[:len(earlier)]):      # only these columns stand behind the mask
                ds_nla[j // C] += dm[jj]
            dv[J] += np.outer(p, do_nla[i])
            dqn[i] += scale * (dm @ kn[J])
            dkn[J] += scale * np.outer(dm, qn[i])
        if mask_c[c]:
            earlier += list(range(c * C, (c + 1) * C))

    # ---- linear branch: forward with everything the reverse sweep needs ----
    S = np.zeros((d_v, d_k)) if S0 is None else np.array(S0, dtype=np.float64)
    S_start, S_prev, S_dec, S_new, resid, decay = [], [None] * L, [None] * L, [None] * L, [None] * L, []
    for c in range(n_c):
        S_start.append(S)
        dcy = 1.0
        for t in range(c * C, (c + 1) * C):
            S_prev[t] = S
            S = alpha[t] * S
            dcy *= alpha[t]
            S_dec[t] = S
            r = v[t] - (S @ k[t] if linear_op == 0 else 0.0)
            S = S + beta[t] * np.outer(r, k[t])
            resid[t], S_new[t] = r, S
        decay.append(dcy)
        if mask_c[c]:
            S = (dcy if decay_on_softmax else 1.0) * S_start[c]
    dS_next = np.zeros((d_v, d_k))                     # gradient w.r.t. the state carried into the next chunk
    for c in range(n_c - 1, -1, -1):
        last = (c + 1) * C - 1
        if mask_c[c]:
            dS = np.zeros((d_v, d_k))                  # the provisional states end with the chunk
        else:
            dS = dS_next
            ds_la[c] = np.sum(dS_next * (S_new[last] - decay[c] * S_start[c]))
        for t in range(last, c * C - 1, -1):
            dq[t] += la_scale * (S_new[t].T @ do_la[t])
            dS = dS + la_scale * np.outer(do_la[t], q[t])
            r = resid[t]
            dSk = dS @ k[t]
            dbeta[t] += r @ dSk
            dr = beta[t] * dSk
            dk[t] += beta[t] * (dS.T @ r)
            dv[t] += dr
            if linear_op == 0:
                dk[t] -= S_dec[t].T @ dr
                dS = dS - np.outer(dr, k[t])
            dalpha[t] += np.sum(dS * S_prev[t])
            dS = alpha[t] * dS
        if mask_c[c]:                                  # carried state of a softmax chunk: decay_c S_c
            if decay_on_softmax:
                dd = np.sum(dS_next * S_start[c])      # d/d decay_c, decay_c = prod alpha_t
                for t in range(c * C, (c + 1) * C):
                    dalpha[t] += dd * decay[c] / alpha[t]
                dS = dS + decay[c] * dS_next
            else:
                dS = dS + dS_next
        dS_next = dS
    out = {"dQ": dq, "dK": dk, "dV": dv, "dalpha": dalpha, "dbeta": dbeta, "dS0": dS_next,
           "dscore_nla": ds_nla, "dscore_la": ds_la}
    if own_qk:
        out.update(dQ_nla=dqn, dK_nla=dkn)
    out.update(merged)
    return out


def hybrid_bwd_chunk_routed(Q, K, V, alpha, beta, mask_c, C, dO, softmax_scale=None, la_scale=1.0, S0=None, linear_op=0,
                            decay_on_softmax=True, Q_nla=None, K_nla=None, mode=0, w_nla=None, w_la=None, eps=1e-6):
    """All (b,h) of [B,H,L,d] inputs with mask_c [B,H,L/C]; returns a dict of stacked fp64 arrays (with Q_nla, K_nla
    [B,H,L,d] also dQ_nla, dK_nla)."""
    B, H, L, d = np.asarray(Q).shape
    out = {"dQ": np.zeros((B, H, L, d)), "dK": np.zeros((B, H, L, d)), "dV": np.zeros((B, H, L, d)),
           "dalpha": np.zeros((B, H, L)), "dbeta": np.zeros((B, H, L)), "dS0": np.zeros((B, H, d, d)),
           "dscore_nla": np.zeros((B, H, L // C)), "dscore_la": np.zeros((B, H, L // C))}
    if Q_nla is not None:
        out.update(dQ_nla=np.zeros((B, H, L, d)), dK_nla=np.zeros((B, H, L, d)))
    if mode != 0:
        out.update(dw_nla=np.zeros((B, H, L)), dw_la=np.zeros((B, H, L)))
    for b in range(B):
        for h in range(H):
            r = hybrid_head_chunk_routed_bwd(Q[b, h], K[b, h], V[b, h], alpha[b, h], beta[b, h], mask_c[b, h], C,
                                             dO[b, h], softmax_scale, la_scale, None if S0 is None else S0[b, h],
                                             linear_op, decay_on_softmax, None if Q_nla is None else Q_nla[b, h],
                                             None if K_nla is None else K_nla[b, h], mode,
                                             None if w_nla is None else w_nla[b, h],
                                             None if w_la is None else w_la[b, h], eps)
            for key in out:
                out[key][b, h] = r[key]
    return out


# --------------------------------------------------------------------------- #
# head grouping (Section 4.3)
# --------------------------------------------------------------------------- #
def hybrid_bwd_grouped(Q, K, V, alpha, beta, mask, dO, G, C=None, softmax_scale=None, la_scale=1.0, S0=None,
                       linear_op=0, decay_on_softmax=True, Q_nla=None, K_nla=None, mode=0, w_nla=None, w_la=None,
                       eps=1e-6):
    """Backward of nats_oracle.hybrid_fwd_grouped (the softmax heads of a group use the linear
    head's queries and keys).  Output head h G + g reads Q, K, alpha, beta, mask of linear head h and its own V
    (its block of the wide state's rows never mixes with the other blocks, and its softmax head attends with the
    same Q, K): it is a head of the ungrouped operator.  A shared input's gradient is therefore the sum over g of the
    ungrouped gradients, and dV, dS0 are the members' own.
    Shapes: Q, K [B,H,L,d]; alpha, beta [B,H,L]; mask [B,H,L] (or [B,H,L/C] with C given: routing per chunk);
    V, dO [B,H G,L,d]; S0 [B,H G,d,d].  Returns dQ, dK, dalpha, dbeta and the score gradients per linear head,
    dV [B,H G,L,d], dS0 [B,H G,d,d].  Q_nla, K_nla [B,H G,L,d]: the softmax heads' own queries and keys; their
    gradients dQ_nla, dK_nla [B,H G,L,d] are each member's own, and dQ, dK are the linear branch's, summed over g.
    mode 1, 2: the merges of Eq. 21 and its ablation per output head, weights w_nla, w_la [B,H G,L] (or None); their
    gradients dw_nla, dw_la [B,H G,L] are each member's own."""
    Q, K, V, dO = (np.asarray(a, dtype=np.float64) for a in (Q, K, V, dO))
    B, H, L, d = Q.shape
    assert V.shape == (B, H * G, L, d) and dO.shape == V.shape
    out = None
    dV = np.zeros_like(V)
    dS0 = np.zeros((B, H * G, d, d))
    own = {}
    if Q_nla is not None:
        Q_nla, K_nla = np.asarray(Q_nla, dtype=np.float64), np.asarray(K_nla, dtype=np.float64)
        own = {"dQ_nla": np.zeros_like(V), "dK_nla": np.zeros_like(V)}
    if mode != 0:
        own.update(dw_nla=np.zeros((B, H * G, L)), dw_la=np.zeros((B, H * G, L)))
    mw = dict(mode=mode, eps=eps)
    for g in range(G):
        mw["w_nla"] = None if w_nla is None else np.asarray(w_nla, dtype=np.float64)[:, g::G]
        mw["w_la"] = None if w_la is None else np.asarray(w_la, dtype=np.float64)[:, g::G]
        Vg, dOg = V[:, g::G], dO[:, g::G]                    # heads h G + g, h = 0 .. H - 1
        S0g = None if S0 is None else np.asarray(S0, dtype=np.float64)[:, g::G]
        Qn = None if Q_nla is None else Q_nla[:, g::G]
        Kn = None if K_nla is None else K_nla[:, g::G]
        if C is None:
            r = hybrid_bwd(Q, K, Vg, alpha, beta, mask, dOg, softmax_scale, la_scale, S0g, linear_op, decay_on_softmax,
                           Qn, Kn, **mw)
        else:
            r = hybrid_bwd_chunk_routed(Q, K, Vg, alpha, beta, mask, C, dOg, softmax_scale, la_scale, S0g, linear_op,
                                        decay_on_softmax, Qn, Kn, **mw)
        dV[:, g::G] = r.pop("dV")
        dS0[:, g::G] = r.pop("dS0")
        for key in own:
            own[key][:, g::G] = r.pop(key)
        if out is None:
            out = {k: np.array(v, dtype=np.float64) for k, v in r.items()}
        else:
            for k, v in r.items():
                out[k] += v
    out["dV"], out["dS0"] = dV, dS0
    out.update(own)
    return out
