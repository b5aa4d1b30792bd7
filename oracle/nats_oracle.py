"""CPU oracle for the NAtS-L hybrid attention operator (TEST INFRASTRUCTURE ONLY).

Plain, slow, fp64 numpy.  Nothing in the product path may import this file;
only tests, the smoke check and the benchmark's cpu-baseline leg do.  It shares
no code with the HIP kernels.

What it computes, per (batch, head) independently, for tokens t = 0..L-1 with
q_t, k_t in R^{d_k}, v_t in R^{d_v}, decay alpha_t, write strength beta_t and a
hard routing mask m_t (1 = softmax token, 0 = linear token):

  * linear branch  -- the Gated DeltaNet recurrence of Section 4.3 (Eq. 19),
    written only for linear tokens (Section 4.1, the state-update rule that
    skips non-linear tokens, Eq. 14) while the decay alpha_t is applied at every
    token (Eq. 20); every query reads the state: o_t = S_t q_t (Eq. 5, Eq. 10).
  * softmax branch -- Eq. 11 with the column mask of Eq. 12: query i attends
    to key j iff j is a softmax token and i >= j.
  * merge          -- plain sum (Section 4.1) or the RMS-normalised weighted sum
    of Eq. 21 with caller-supplied weights.

Readings taken where the paper is silent (all listed in the design notes):
routing is applied per token; the state is S[d_v, d_k] and acts as S q; decay
is applied before the write; an empty softmax key set gives output 0 and
lse = -inf; RMSNorm has no gain and Norm(0) = 0.

Parity pins: every function below is pinned by tests/test_oracle_pins.py
(library softmax attention, closed forms of the delta rule, explicit
transition-matrix products, Fig. 1c's support pattern, brute force); the
chunk-routed form at the end of the file by tests/test_oracle_chunk_routing.py
(library attention with explicit masks, and its composition from the pinned
per-token functions).
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------- #
# mask bookkeeping (integer, exactly one correct answer)
# --------------------------------------------------------------------------- #
def compaction(mask):
    """cnt[t] = number of softmax tokens among 0..t; idx[c] = position of the c-th one.

    Column sets t_nla / t_la of Eq. 12-13 as index lists.
    """
    m = (np.asarray(mask).reshape(-1) != 0)
    cnt = np.zeros(m.shape[0], dtype=np.int32)
    idx = []
    running = 0
    for t in range(m.shape[0]):
        if m[t]:
            idx.append(t)
            running += 1
        cnt[t] = running
    return cnt, np.asarray(idx, dtype=np.int32), running


# --------------------------------------------------------------------------- #
# linear branch: token-recurrent Gated DeltaNet (Eq. 19 + Eq. 14 + Eq. 20)
# --------------------------------------------------------------------------- #
def gdn_recurrent(q, k, v, alpha, beta, mask, S0=None, la_scale=1.0, decay_on_softmax=True, linear_op=0):
    """Returns (o_la [L,d_v], S_final [d_v,d_k]).

    decay_on_softmax=False is the ablation that freezes the state on softmax
    tokens (Table 4, the variant without linear-attention decay); the method itself uses True.
    linear_op=1 replaces the delta rule by the gated linear attention of Mamba2,
    S_t = alpha_t S_{t-1} + beta_t v_t k_t^T (appendix "Mixture of SoftmaxAttention and Mamba2
    architecture": the linear operation is exchangeable; B = k, C = q, dt x = beta v, scalar decay).
    """
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    alpha = np.asarray(alpha, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    L, d_k = k.shape
    d_v = v.shape[1]
    S = np.zeros((d_v, d_k)) if S0 is None else np.array(S0, dtype=np.float64)
    o = np.zeros((L, d_v))
    for t in range(L):
        linear = (mask[t] == 0)
        if linear or decay_on_softmax:
            S = alpha[t] * S                       # decay at every token (Eq. 20)
        if linear:                                 # write only linear tokens (Eq. 14)
            pred = S @ k[t] if linear_op == 0 else 0.0   # what the decayed state returns for k_t (delta rule only)
            S = S + beta[t] * np.outer(v[t] - pred, k[t])   # Eq. 19 expanded
        o[t] = la_scale * (S @ q[t])               # Eq. 5
    return o, S


# --------------------------------------------------------------------------- #
# softmax branch: brute force over the softmax-token columns (Eq. 11-12)
# --------------------------------------------------------------------------- #
def softmax_branch(q, k, v, mask, scale):
    """Returns (o_nla [L,d_v], lse [L]); rows with no visible key give 0 / -inf."""
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    L = q.shape[0]
    o = np.zeros((L, v.shape[1]))
    lse = np.full(L, -np.inf)
    for t in range(L):
        J = np.flatnonzero(np.asarray(mask[:t + 1]) != 0)   # softmax columns j <= t
        if J.size == 0:
            continue
        s = scale * (k[J] @ q[t])
        smax = s.max()
        e = np.exp(s - smax)
        z = e.sum()
        o[t] = (e / z) @ v[J]
        lse[t] = smax + np.log(z)
    return o, lse


# --------------------------------------------------------------------------- #
# merge of the two branch outputs (Section 4.1 sum; Eq. 21)
# --------------------------------------------------------------------------- #
def rms_norm_rows(x, eps):
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def combine(o_la, o_nla, mode=0, w_nla=None, w_la=None, eps=1e-6):
    """mode 0: sum (Section 4.1); 1: Eq. 21; 2: the ablation with a single normalisation (Section 5, (iii)),
    RMSNorm(w_nla o_nla + w_la o_la) with weights 1 unless given."""
    if mode == 0:
        return o_la + o_nla
    L = o_la.shape[0]
    if mode == 2:
        wn = np.ones(L) if w_nla is None else np.asarray(w_nla, dtype=np.float64)
        wl = np.ones(L) if w_la is None else np.asarray(w_la, dtype=np.float64)
        return rms_norm_rows(wn[:, None] * o_nla + wl[:, None] * o_la, eps)
    w_nla = np.full(L, 0.5) if w_nla is None else np.asarray(w_nla, dtype=np.float64)
    w_la = np.full(L, 0.5) if w_la is None else np.asarray(w_la, dtype=np.float64)
    return w_nla[:, None] * rms_norm_rows(o_nla, eps) + w_la[:, None] * rms_norm_rows(o_la, eps)


def route_chunks(X, W_s, C):
    """Score layer and routing decision, Eq. 8-9: mean-pool X [B,L,d_model] over chunks of C tokens, map the mean
    with W_s [H,2,d_model] to one score per head and operation (0: softmax attention, 1: linear), give the
    chunk to the operation with the highest score (the first one on a tie, as argmax does).

    Returns (mask_c [B,H,L/C] uint8, scores [B,L/C,H,2])."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W_s, dtype=np.float64)
    B, L, dm = X.shape
    pooled = X.reshape(B, L // C, C, dm).mean(axis=2)
    scores = np.einsum("bcd,hkd->bchk", pooled, W)
    mask_c = (np.argmax(scores, axis=-1) == 0).astype(np.uint8).transpose(0, 2, 1)
    return np.ascontiguousarray(mask_c), scores


def eq22_weights(Q, W_out, act=0):
    """Weights of the merge, Eq. 22: [w_nla, w_la] = softmax([W_nla q_t, W_la q_t]) per token and head.
    act = 1 / 2: the ablation (iv) of Section 5, a sigmoid of each logit / the logits themselves.

    Q [B,H,L,d]; W_out [H,2,d] (row 0: W_nla, row 1: W_la of the head).  Returns (w_nla, w_la) [B,H,L].
    The paper takes "the attention q values"; the Q handed to the operator is used as it is.
    """
    Q = np.asarray(Q, dtype=np.float64)
    W = np.asarray(W_out, dtype=np.float64)
    logits = np.einsum("bhld,hkd->bhlk", Q, W)
    if act == 1:
        w = 1.0 / (1.0 + np.exp(-logits))
        return w[..., 0], w[..., 1]
    if act == 2:
        return logits[..., 0], logits[..., 1]
    logits = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(logits)
    w = e / e.sum(axis=-1, keepdims=True)
    return w[..., 0], w[..., 1]


def weights_from_x(X, W_x, act=0):
    """Section 5, ablation (v): the weights of Eq. 21 computed from the layer's input features instead of the
    queries.  X [B,L,d_model]; W_x [H,2,d_model] (row 0: softmax attention, row 1: the linear operation).
    Returns (w_nla, w_la) [B,H,L], with the activations of eq22_weights."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W_x, dtype=np.float64)
    logits = np.einsum("bld,hkd->bhlk", X, W)
    if act == 1:
        w = 1.0 / (1.0 + np.exp(-logits))
    elif act == 2:
        w = logits
    else:
        e = np.exp(logits - logits.max(axis=-1, keepdims=True))
        w = e / e.sum(axis=-1, keepdims=True)
    return w[..., 0], w[..., 1]


# --------------------------------------------------------------------------- #
# whole operator for one (batch, head), and over [B,H,...]
# --------------------------------------------------------------------------- #
def hybrid_head(q, k, v, alpha, beta, mask, softmax_scale=None, la_scale=1.0, mode=0,
                w_nla=None, w_la=None, eps=1e-6, S0=None, linear_op=0, decay_on_softmax=True,
                q_nla=None, k_nla=None):
    """q_nla, k_nla: the softmax branch's own queries and keys (Section 4.3: the two families share the
    projections but the linear one takes L2-normalised q, k and the softmax one RMS-normalised, possibly
    rotated ones); None: both branches use q, k."""
    d_k = np.asarray(q).shape[-1]
    scale = (1.0 / np.sqrt(d_k)) if softmax_scale is None else softmax_scale
    o_la, S = gdn_recurrent(q, k, v, alpha, beta, mask, S0=S0, la_scale=la_scale,
                            decay_on_softmax=decay_on_softmax, linear_op=linear_op)
    o_nla, lse = softmax_branch(q if q_nla is None else q_nla, k if k_nla is None else k_nla, v, mask, scale)
    o = combine(o_la, o_nla, mode, w_nla, w_la, eps)
    cnt, idx, n_s = compaction(mask)
    return {"O": o, "O_la": o_la, "O_nla": o_nla, "lse": lse, "S": S,
            "cnt": cnt, "idx": idx, "n_s": n_s}


def hybrid_fwd(Q, K, V, alpha, beta, mask, softmax_scale=None, la_scale=1.0, mode=0,
               w_nla=None, w_la=None, eps=1e-6, S0=None, linear_op=0, decay_on_softmax=True, Q_nla=None, K_nla=None):
    """All (b,h) of [B,H,L,d] inputs; returns dict of stacked fp64 arrays (idx as nested lists)."""
    B, H, L, _ = np.asarray(Q).shape
    d_v = np.asarray(V).shape[-1]
    out = {"O": np.zeros((B, H, L, d_v)), "O_la": np.zeros((B, H, L, d_v)),
           "O_nla": np.zeros((B, H, L, d_v)), "lse": np.zeros((B, H, L)),
           "S": np.zeros((B, H, d_v, np.asarray(K).shape[-1])),
           "cnt": np.zeros((B, H, L), dtype=np.int32), "n_s": np.zeros((B, H), dtype=np.int32),
           "idx": [[None] * H for _ in range(B)]}
    for b in range(B):
        for h in range(H):
            r = hybrid_head(Q[b, h], K[b, h], V[b, h], alpha[b, h], beta[b, h], mask[b, h],
                            softmax_scale, la_scale, mode,
                            None if w_nla is None else w_nla[b, h],
                            None if w_la is None else w_la[b, h], eps,
                            None if S0 is None else S0[b, h], linear_op, decay_on_softmax,
                            None if Q_nla is None else Q_nla[b, h], None if K_nla is None else K_nla[b, h])
            for key in ("O", "O_la", "O_nla", "lse", "S", "cnt", "n_s"):
                out[key][b, h] = r[key]
            out["idx"][b][h] = r["idx"]
    return out


# --------------------------------------------------------------------------- #
# one decode step for one (batch, head) (Section 4.1, per-token generation)
# --------------------------------------------------------------------------- #
def decode_step(S, k_cache, v_cache, cache_len, q, k, v, alpha, beta, m,
                softmax_scale=None, la_scale=1.0, mode=0, w_nla=0.5, w_la=0.5, eps=1e-6, linear_op=0,
                decay_on_softmax=True, q_nla=None, k_nla=None):
    """One token.  S [d_v,d_k] fp64; k_cache/v_cache [cap,d] with cache_len live rows.

    Returns (o [d_v], S_new, k_cache, v_cache, cache_len_new, overflow).  A softmax
    token is appended to the cache before attending (it sees itself: Eq. 12, i >= j);
    a linear token is written into the state.  If the cache is full the token is
    not stored and overflow=True; the output then covers the existing rows only.
    """
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    qn = q if q_nla is None else np.asarray(q_nla, dtype=np.float64)   # the softmax branch's own query and key
    kn = k if k_nla is None else np.asarray(k_nla, dtype=np.float64)
    scale = (1.0 / np.sqrt(q.shape[0])) if softmax_scale is None else softmax_scale
    S = (float(alpha) if (m == 0 or decay_on_softmax) else 1.0) * np.array(S, dtype=np.float64)
    overflow = False
    if m == 0:
        S = S + float(beta) * np.outer(v - (S @ k if linear_op == 0 else 0.0), k)
    else:
        if cache_len < k_cache.shape[0]:
            k_cache = np.array(k_cache, dtype=np.float64)
            v_cache = np.array(v_cache, dtype=np.float64)
            k_cache[cache_len] = kn
            v_cache[cache_len] = v
            cache_len = cache_len + 1
        else:
            overflow = True
    o_la = la_scale * (S @ q)
    if cache_len > 0:
        s = scale * (np.asarray(k_cache[:cache_len], dtype=np.float64) @ qn)
        e = np.exp(s - s.max())
        o_nla = (e / e.sum()) @ np.asarray(v_cache[:cache_len], dtype=np.float64)
    else:
        o_nla = np.zeros_like(o_la)
    if mode == 0:
        o = o_la + o_nla
    elif mode == 2:
        o = rms_norm_rows((w_nla * o_nla + w_la * o_la)[None], eps)[0]
    else:
        o = (w_nla * rms_norm_rows(o_nla[None], eps)[0] + w_la * rms_norm_rows(o_la[None], eps)[0])
    return o, S, k_cache, v_cache, cache_len, overflow


# --------------------------------------------------------------------------- #
# second, independent form of the linear branch: chunkwise (Eq. 6-7 shape)
# --------------------------------------------------------------------------- #
def gdn_chunkwise(q, k, v, alpha, beta, mask, C, S0=None, la_scale=1.0):
    """Chunkwise-parallel form of the same recurrence (Section 3, Eq. 6-7).

    With b'_t = beta_t * (1 - m_t) and, inside a chunk, g_r = sum_{i<=r} log alpha_i:
      D[r,i] = exp(g_r - g_i) (i <= r),  A = strict_lower(diag(b') (K K^T . D)),
      T = (I + A)^{-1},  U~ = T diag(b') V,  W = T diag(b' exp(g)) K,
      U = U~ - W S0^T,  O = diag(exp(g)) Q S0^T + ((Q K^T) . D) U,
      S1 = exp(g_C) S0 + U^T diag(exp(g_C - g)) K.
    Used only to pin "chunkwise == token-recurrent" and independence of C.
    """
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    alpha = np.asarray(alpha, dtype=np.float64)
    bp = np.asarray(beta, dtype=np.float64) * (np.asarray(mask) == 0)
    L, d_k = k.shape
    d_v = v.shape[1]
    assert L % C == 0
    S = np.zeros((d_v, d_k)) if S0 is None else np.array(S0, dtype=np.float64)
    o = np.zeros((L, d_v))
    for c0 in range(0, L, C):
        sl = slice(c0, c0 + C)
        Kc, Vc, Qc = k[sl], v[sl], q[sl]
        g = np.cumsum(np.log(alpha[sl]))
        D = np.tril(np.exp(g[:, None] - g[None, :]))
        A = np.tril(bp[sl][:, None] * (Kc @ Kc.T) * D, -1)
        T = np.linalg.inv(np.eye(C) + A)
        Ut = T @ (bp[sl][:, None] * Vc)
        W = T @ ((bp[sl] * np.exp(g))[:, None] * Kc)
        U = Ut - W @ S.T
        o[sl] = la_scale * (np.exp(g)[:, None] * (Qc @ S.T) + ((Qc @ Kc.T) * D) @ U)
        S = np.exp(g[-1]) * S + U.T @ (np.exp(g[-1] - g)[:, None] * Kc)
    return o, S


# --------------------------------------------------------------------------- #
# chunk-level routing (Section 4.1 as the paper states it: the type is chosen per
# chunk, after the whole chunk has been seen)
# --------------------------------------------------------------------------- #
def hybrid_head_chunk_routed(q, k, v, alpha, beta, mask_c, C, softmax_scale=None, la_scale=1.0, mode=0,
                             w_nla=None, w_la=None, eps=1e-6, S0=None, linear_op=0, decay_on_softmax=True,
                             q_nla=None, k_nla=None, inner=0):
    """One (batch, head) with one routing decision per chunk of C tokens (mask_c[c] = 1: softmax chunk).

    Section 4.1: a chunk's type is known only once the whole chunk has been seen, so both
    operations compute the intra-chunk part of every chunk, and afterwards the state of the
    operation that was not chosen is rolled back (per-token generation paragraph):
      * linear branch  -- inside every chunk the Gated DeltaNet recurrence (Eq. 19) runs on all of
        its tokens, starting from the state at the chunk's start; after a linear chunk the state is
        kept (Eq. 14), after a softmax chunk it is reset to the chunk-start state times the chunk's
        decay (the writes are dropped, the decay of Eq. 20 stays);
      * softmax branch -- query t attends to every token of earlier softmax chunks (column mask of
        Eq. 12 at chunk granularity) and, causally, to the tokens j <= t of its own chunk whatever
        its type.
    cnt / idx / n_s describe the compaction of the tokens of softmax chunks.
    linear_op, decay_on_softmax: the variants of gdn_recurrent (without decay on softmax chunks the state
    after such a chunk is the chunk-start state itself).
    inner: which operation computes the inner part of a chunk (Section 5, ablation (i)): 0 both (the method);
    1 softmax attention only ("SAttn Out": the linear branch's output reads the carried state of the chunk's
    start, decayed up to the query, and nothing of the chunk's own tokens); 2 the linear operation only ("GDN
    Out": a query attends to the tokens of earlier softmax chunks and to nothing of its own chunk; a query with
    nothing visible gets o_nla = 0, lse = -inf).  The carried state and the cache are the same in all three.
    """
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    qn = q if q_nla is None else np.asarray(q_nla, dtype=np.float64)   # the softmax branch's own queries and keys
    kn = k if k_nla is None else np.asarray(k_nla, dtype=np.float64)
    alpha = np.asarray(alpha, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    mask_c = np.asarray(mask_c).reshape(-1) != 0
    L, d_k = k.shape
    d_v = v.shape[1]
    assert L % C == 0 and mask_c.shape[0] == L // C
    scale = (1.0 / np.sqrt(d_k)) if softmax_scale is None else softmax_scale
    S = np.zeros((d_v, d_k)) if S0 is None else np.array(S0, dtype=np.float64)
    o_la = np.zeros((L, d_v))
    o_nla = np.zeros((L, d_v))
    lse = np.full(L, -np.inf)
    earlier = []                                   # tokens of earlier softmax chunks
    for c in range(L // C):
        S_start, decay = S.copy(), 1.0
        for t in range(c * C, (c + 1) * C):
            S = alpha[t] * S
            decay *= alpha[t]
            pred = S @ k[t] if linear_op == 0 else 0.0
            S = S + beta[t] * np.outer(v[t] - pred, k[t])            # Eq. 19, every token of the chunk
            o_la[t] = la_scale * ((S if inner != 1 else decay * S_start) @ q[t])
            own = list(range(c * C, t + 1)) if inner != 2 else []
            J = np.asarray(earlier + own, dtype=np.int64)
            if J.size == 0:
                continue
            s = scale * (kn[J] @ qn[t])
            smax = s.max()
            e = np.exp(s - smax)
            z = e.sum()
            o_nla[t] = (e / z) @ v[J]
            lse[t] = smax + np.log(z)
        if mask_c[c]:
            S = (decay if decay_on_softmax else 1.0) * S_start   # softmax chunk: its writes are rolled back
            earlier += list(range(c * C, (c + 1) * C))
    o = combine(o_la, o_nla, mode, w_nla, w_la, eps)
    cnt, idx, n_s = compaction(np.repeat(mask_c, C))
    return {"O": o, "O_la": o_la, "O_nla": o_nla, "lse": lse, "S": S, "cnt": cnt, "idx": idx, "n_s": n_s}


def hybrid_fwd_chunk_routed(Q, K, V, alpha, beta, mask_c, C, softmax_scale=None, la_scale=1.0, mode=0,
                            w_nla=None, w_la=None, eps=1e-6, S0=None, linear_op=0, decay_on_softmax=True,
                            Q_nla=None, K_nla=None, inner=0):
    """All (b,h) of [B,H,L,d] inputs with mask_c [B,H,L/C]; same result layout as hybrid_fwd."""
    B, H, L, _ = np.asarray(Q).shape
    d_v = np.asarray(V).shape[-1]
    out = {"O": np.zeros((B, H, L, d_v)), "O_la": np.zeros((B, H, L, d_v)),
           "O_nla": np.zeros((B, H, L, d_v)), "lse": np.zeros((B, H, L)),
           "S": np.zeros((B, H, d_v, np.asarray(K).shape[-1])),
           "cnt": np.zeros((B, H, L), dtype=np.int32), "n_s": np.zeros((B, H), dtype=np.int32),
           "idx": [[None] * H for _ in range(B)]}
    for b in range(B):
        for h in range(H):
            r = hybrid_head_chunk_routed(Q[b, h], K[b, h], V[b, h], alpha[b, h], beta[b, h], mask_c[b, h], C,
                                         softmax_scale, la_scale, mode,
                                         None if w_nla is None else w_nla[b, h],
                                         None if w_la is None else w_la[b, h], eps,
                                         None if S0 is None else S0[b, h], linear_op, decay_on_softmax,
                                         None if Q_nla is None else Q_nla[b, h], None if K_nla is None else K_nla[b, h],
                                         inner)
            for key in ("O", "O_la", "O_nla", "lse", "S", "cnt", "n_s"):
                out[key][b, h] = r[key]
            out["idx"][b][h] = r["idx"]
    return out


# --------------------------------------------------------------------------- #
# generation with routing per chunk (Section 4.1, per-token generation): provisional
# updates inside the open chunk, rollback of the unchosen operation when it is settled
# --------------------------------------------------------------------------- #
def decode_chunk_state(S, k_cache, v_cache, cache_len):
    """State of one (batch, head) between tokens: settled rows [0, cache_len) of the caches."""
    return {"S": np.array(S, dtype=np.float64), "S_start": np.array(S, dtype=np.float64), "decay": 1.0,
            "pos": 0, "k_cache": np.array(k_cache, dtype=np.float64), "v_cache": np.array(v_cache, dtype=np.float64),
            "cache_len": int(cache_len)}


def decode_step_chunk_routed(st, q, k, v, alpha, beta, softmax_scale=None, la_scale=1.0, mode=0,
                             w_nla=0.5, w_la=0.5, eps=1e-6, linear_op=0):
    """One token inside an open chunk.  Both operations take it: the state is updated by Eq. 19 and (k, v)
    goes to the cache at row cache_len + pos; the output reads the state and every row up to that one
    (earlier softmax chunks, and the own chunk causally).  Returns (o, overflow); st is updated in place.
    A full cache leaves the token out of the cache (overflow=True)."""
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    scale = (1.0 / np.sqrt(q.shape[0])) if softmax_scale is None else softmax_scale
    if st["pos"] == 0:
        st["S_start"] = st["S"].copy()
        st["decay"] = 1.0
    S = float(alpha) * st["S"]
    st["decay"] *= float(alpha)
    S = S + float(beta) * np.outer(v - (S @ k if linear_op == 0 else 0.0), k)
    st["S"] = S
    n = st["cache_len"] + st["pos"]
    overflow = n >= st["k_cache"].shape[0]
    if not overflow:
        st["k_cache"][n] = k
        st["v_cache"][n] = v
        n += 1
    st["pos"] += 1
    o_la = la_scale * (S @ q)
    if n > 0:
        s = scale * (st["k_cache"][:n] @ q)
        e = np.exp(s - s.max())
        o_nla = (e / e.sum()) @ st["v_cache"][:n]
    else:
        o_nla = np.zeros_like(o_la)
    # the merge of the forward, on this one row (mode 0: sum; 1: Eq. 21; 2: one normalisation of the weighted sum)
    o = combine(o_la[None], o_nla[None], mode, None if w_nla is None else np.array([w_nla]),
                None if w_la is None else np.array([w_la]), eps)[0]
    return o, overflow


def decode_commit_chunk(st, m, decay_on_softmax=True):
    """Settles the open chunk: a softmax chunk (m != 0) keeps its cache rows and sets the state back to
    (chunk decay) x (chunk-start state), or to the chunk-start state itself in the variant without decay on
    softmax chunks; a linear chunk keeps the state and drops the rows."""
    if m:
        st["cache_len"] = min(st["cache_len"] + st["pos"], st["k_cache"].shape[0])
        st["S"] = (st["decay"] if decay_on_softmax else 1.0) * st["S_start"]
    st["pos"] = 0


# --------------------------------------------------------------------------- #
# head grouping (Section 4.3; appendix "Experimental details": 2 or 3 softmax heads per Gated DeltaNet head)
# --------------------------------------------------------------------------- #
def hybrid_fwd_grouped(Q, K, V, alpha, beta, mask, G, C=None, softmax_scale=None, la_scale=1.0, mode=0,
                       w_nla=None, w_la=None, eps=1e-6, S0=None, linear_op=0, decay_on_softmax=True,
                       Q_nla=None, K_nla=None):
    """G softmax heads share the routing mask (and so the set of softmax tokens) of one linear head.

    The linear family uses fewer, wider heads than the softmax family, so every linear head h is matched by the
    G softmax heads h G .. h G + G - 1, which "share the same set of attention types and the corresponding masks";
    each linear head has its own mask.  Shapes: Q, K [B,H,L,d] (linear head: its queries and keys), alpha, beta,
    mask [B,H,L] (mask [B,H,L/C] with routing per chunk, C given); V [B,H G,L,d]: the value columns of linear head
    h are the G blocks V[:, h G + g] side by side, i.e. its state is S in R^{(G d) x d}, and softmax head h G + g
    attends with the g-th block as its values; Q_nla, K_nla [B,H G,L,d] are the softmax heads' queries and keys
    (None: every softmax head of a group uses the linear head's).  Output head h G + g merges the g-th block of
    the linear head's output columns with softmax head h G + g (sum, or Eq. 21 with the normalisations over the d
    columns of the block and weights w [B,H G,L]).
    Returns the dict of hybrid_fwd with H G heads (S [B,H G,d,d]: row blocks of the wide states); cnt, n_s, idx
    per linear head."""
    Q, K, V = (np.asarray(a, dtype=np.float64) for a in (Q, K, V))
    B, H, L, d = Q.shape
    assert V.shape[:3] == (B, H * G, L)
    dv = V.shape[-1]
    out = {"O": np.zeros((B, H * G, L, dv)), "O_la": np.zeros((B, H * G, L, dv)), "O_nla": np.zeros((B, H * G, L, dv)),
           "lse": np.zeros((B, H * G, L)), "S": np.zeros((B, H * G, dv, d)),
           "cnt": np.zeros((B, H, L), dtype=np.int32), "n_s": np.zeros((B, H), dtype=np.int32),
           "idx": [[None] * H for _ in range(B)]}
    for b in range(B):
        for h in range(H):
            hs = slice(h * G, (h + 1) * G)
            v_wide = np.concatenate(list(V[b, hs]), axis=-1)                       # [L, G d]
            s0_wide = None if S0 is None else np.concatenate(list(np.asarray(S0, dtype=np.float64)[b, hs]), axis=0)
            if C is None:
                tok_mask = np.asarray(mask[b, h])
                o_la, S = gdn_recurrent(Q[b, h], K[b, h], v_wide, alpha[b, h], beta[b, h], tok_mask, S0=s0_wide,
                                        la_scale=la_scale, decay_on_softmax=decay_on_softmax, linear_op=linear_op)
            else:
                r = hybrid_head_chunk_routed(Q[b, h], K[b, h], v_wide, alpha[b, h], beta[b, h], mask[b, h], C,
                                             softmax_scale, la_scale, 0, S0=s0_wide, linear_op=linear_op,
                                             decay_on_softmax=decay_on_softmax)
                o_la, S = r["O_la"], r["S"]
                tok_mask = np.repeat(np.asarray(mask[b, h]).reshape(-1) != 0, C)
            cnt, idx, n_s = compaction(tok_mask)
            out["cnt"][b, h], out["n_s"][b, h] = cnt, n_s
            out["idx"][b][h] = idx
            for g in range(G):
                hg = h * G + g
                qn = Q[b, h] if Q_nla is None else np.asarray(Q_nla[b, hg], dtype=np.float64)
                kn = K[b, h] if K_nla is None else np.asarray(K_nla[b, hg], dtype=np.float64)
                scale = (1.0 / np.sqrt(d)) if softmax_scale is None else softmax_scale
                if C is None:
                    o_nla, lse = softmax_branch(qn, kn, V[b, hg], tok_mask, scale)
                else:   # the softmax side of the chunk-routed head (its linear side is not used)
                    r = hybrid_head_chunk_routed(qn, kn, V[b, hg], alpha[b, h], beta[b, h], mask[b, h], C, scale)
                    o_nla, lse = r["O_nla"], r["lse"]
                o_la_g = o_la[:, g * dv:(g + 1) * dv]
                out["O"][b, hg] = combine(o_la_g, o_nla, mode, None if w_nla is None else w_nla[b, hg],
                                          None if w_la is None else w_la[b, hg], eps)
                out["O_la"][b, hg], out["O_nla"][b, hg], out["lse"][b, hg] = o_la_g, o_nla, lse
                out["S"][b, hg] = S[g * dv:(g + 1) * dv]
    return out
