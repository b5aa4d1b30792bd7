/* nats.h -- C ABI of the NAtS-L hybrid attention operator for AMD MI355X (gfx950).
 *
 * One layer of token-level hybrid attention (paper Section 4.1 and 4.3): a hard
 * per-token routing mask m (1 = softmax token, 0 = linear token) sends each
 * key/value either into a Gated DeltaNet state (Eq. 19; written only for linear
 * tokens, Eq. 14; decayed at every token, Eq. 20) or into the softmax key set
 * (Eq. 11 under the column mask of Eq. 12).  Every query reads both, and the
 * two outputs are merged by a plain sum (Section 4.1) or by Eq. 21.
 *
 * Conventions common to every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates no memory, frees nothing and never synchronises the host: all
 *     work is ordered after what the given HIP stream (a hipStream_t passed as
 *     void*, NULL = the default stream) held at the call, is complete when that
 *     stream reaches the end of what the call enqueued, and the call returns
 *     immediately.  Every kernel of a call runs on the given stream (legal
 *     under stream capture).  Two calls that overlap in time need different
 *     workspaces.
 *   - Arguments are validated on the host before anything is launched; a bad
 *     argument returns a negative nats_status and launches nothing.
 *     nats_last_error() then describes the problem (thread-local string).
 *   - Tensors are dense, row-major, in the layouts written below; data pointers
 *     must be 16-byte aligned; outputs must not alias inputs.
 *   - Data-dependent sizes (the number of softmax tokens per head) stay on the
 *     device; nothing is read back to the host.
 *   - Results are deterministic: no floating-point atomics.
 */
#ifndef NATS_H_
#define NATS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum nats_status {
    NATS_OK = 0,
    NATS_ERR_NULL = -1,        /* a required pointer is NULL */
    NATS_ERR_SHAPE = -2,       /* a size is out of range (e.g. L % C != 0) */
    NATS_ERR_DTYPE = -3,       /* unknown dtype code */
    NATS_ERR_ALIGN = -4,       /* a data pointer is not 16-byte aligned */
    NATS_ERR_WORKSPACE = -5,   /* workspace missing or smaller than *_workspace_bytes() */
    NATS_ERR_UNSUPPORTED = -6, /* legal request this build has no kernel for */
    NATS_ERR_HIP = -7          /* a HIP launch failed; message holds hipGetErrorString */
} nats_status;

typedef enum nats_dtype { NATS_F32 = 0, NATS_BF16 = 1 } nats_dtype;

/* Arithmetic used inside the kernels.
 *   NATS_MATH_AUTO : f32 tensors -> fp32 kernels; bf16 tensors -> chunkwise bf16 MFMA kernels
 *                    with fp32 state and accumulation.
 *   NATS_MATH_FP32 : fp32 arithmetic for either tensor dtype (token-recurrent state update,
 *                    fp32 dot products); slower, used for tight-tolerance work. */
typedef enum nats_math { NATS_MATH_AUTO = 0, NATS_MATH_FP32 = 1 } nats_math;

/* ------------------------------------------------------------------------- *
 * Prefill / training forward
 * ------------------------------------------------------------------------- */
/* Granularity of the routing decision (Section 4.1).
 *   NATS_ROUTE_TOKEN: mask is [B,H,L], one decision per token.  A softmax token is never written into
 *       the linear state (it only decays it) and is a key of the softmax branch; a linear token is
 *       written into the state and is no key.
 *   NATS_ROUTE_CHUNK: mask is [B,H,L/C], one decision per chunk of C tokens, as the paper states it:
 *       a chunk's type is known only after the chunk has been seen, so both operations compute
 *       the intra-chunk part of every chunk.  Linear branch: Eq. 19 runs on all tokens of a chunk from
 *       the state at its start; after a softmax chunk the state is set back to that state times the
 *       chunk's decay (Eq. 14, Eq. 20).  Softmax branch: a query sees the tokens of earlier softmax
 *       chunks (Eq. 12) and, causally, the tokens of its own chunk whatever its type.  n_s, idx, cnt,
 *       Kc, Vc then describe the tokens of softmax chunks. */
typedef enum nats_routing { NATS_ROUTE_TOKEN = 0, NATS_ROUTE_CHUNK = 1 } nats_routing;

/* The linear operation (the search space's linear member is exchangeable: Section 4.3 uses Gated DeltaNet,
 * the appendix "Mixture of SoftmaxAttention and Mamba2 architecture" Mamba2):
 *   NATS_LINEAR_GDN  : S <- alpha S;  S <- S + beta (v - S k) k^T          (Eq. 19, the delta rule)
 *   NATS_LINEAR_GATED: S <- alpha S;  S <- S + beta v k^T                  (Mamba2's recurrence with scalar
 *                      decay per head: B = k, C = q, dt x = beta v; no correction by the state)  */
typedef enum nats_linear_op { NATS_LINEAR_GDN = 0, NATS_LINEAR_GATED = 1 } nats_linear_op;

/* What turns the two logits W_out q of Eq. 22 into the weights of Eq. 21: the softmax over the pair (the
 * method), or, as in the ablation "(iv)" of Section 5, a sigmoid of each logit, or the logits themselves. */
typedef enum nats_weight_act { NATS_WEIGHTS_SOFTMAX = 0, NATS_WEIGHTS_SIGMOID = 1, NATS_WEIGHTS_LINEAR = 2 } nats_weight_act;

typedef struct nats_fwd_params {
    int32_t B, H;          /* batch, heads (each (b,h) has its own mask: Section 4.3)          */
    int32_t L;             /* tokens; must be a positive multiple of C                          */
    int32_t d;             /* head dim, d_k = d_v = d, 64 or 128                                */
    int32_t C;             /* chunk size, 64 or 128.  Routing per token: the result does not depend on it (the
                              chunkwise form of Eq. 6-7 is exact; the kernels use their own chunk of 64).
                              Routing per chunk: tokens per routing decision (mask [B,H,L/C]); C = 128 (the chunk-size
                              ablation of Section 5) runs the forward on the token-by-token kernels, whatever the
                              dtype; the backward covers C = 64                                    */
    int32_t dtype;         /* nats_dtype of Q, K, V, O                                          */
    float softmax_scale;   /* logits = scale * q.k ; <= 0 selects 1/sqrt(d)                     */
    float la_scale;        /* o_la = la_scale * S q (Eq. 5 has none); <= 0 selects 1            */
    int32_t combine_mode;  /* 0: O = O_la + O_nla (Section 4.1).  1: Eq. 21,
                              O = w_nla * RMSNorm(O_nla) + w_la * RMSNorm(O_la), no gain.
                              2: the ablation with one normalisation (Section 5, (iii)):
                              O = RMSNorm(w_nla * O_nla + w_la * O_la), weights NULL -> 1       */
    float rms_eps;         /* RMSNorm epsilon for combine_mode 1; <= 0 selects 1e-6             */
    int32_t math;          /* nats_math                                                         */
    int32_t routing;       /* nats_routing: granularity of the routing mask                     */
    int32_t linear_op;     /* nats_linear_op                                                    */
    int32_t freeze_on_softmax; /* 0: the decay acts on the state at every token (Eq. 20).  1: the ablation
                              without linear-attention decay (Section 5, Ablation Study (ii)): softmax
                              tokens, or softmax chunks as a whole, leave the carried state unchanged  */
    int32_t weight_act;    /* nats_weight_act, used where the weights come from W_out                     */
    int32_t gdn_segments;  /* bf16 path: segments the sequence of every (batch, head) is cut into, which then
                              run side by side (the recurrence over chunks is affine in the state, so the
                              segments' start states are composed afterwards); 0 chooses automatically
                              (about 256 / (B*H), at least 4 chunks per segment).  The result does not depend
                              on it beyond rounding                                                          */
    int32_t group;         /* head grouping (Section 4.3; the appendix's model sizes use 2 and 3): G = group
                              softmax heads share the mask of one linear head, 0 counts as 1, at most 8.
                              H stays the number of linear heads: Q, K, alpha, beta, mask, cnt, idx, n_s are
                              [B,H,...].  Everything else has B, H*G heads, output head h*G + g belonging to
                              linear head h: V (the linear head's value columns are the G blocks V[:, h*G + g]
                              side by side, i.e. its state is (G d) x d, and softmax head h*G + g attends with
                              block g), O, Q_nla, K_nla (absent: the softmax heads of a group use the linear
                              head's Q, K), w_nla, w_la, W_out [H*G,2,d] (applied to the linear head's query),
                              initial_state, final_state [B,H*G,d,d] (row blocks of the wide states), Kc, Vc,
                              O_la, O_nla, lse.  Output head h*G + g is the merge of block g of the linear
                              head's output with softmax head h*G + g (Eq. 21: norms over the d columns of the
                              block).  The result equals that of group = 1 on H*G heads with Q, K, alpha, beta
                              and the mask repeated G times; the integers and the per-chunk work of the linear
                              branch that does not depend on V are done once per linear head.  A generation
                              step (nats_hybrid_attn_decode) is a call on H*G heads with the linear head's
                              q, k, alpha, beta, mask repeated.  Not available in the backward pass          */
    int32_t inner_chunk;   /* routing per chunk only (else 0): which operation computes the inner part of a chunk.
                              0: both (the method, Section 4.1).  The ablation (i) of Section 5:
                              1: softmax attention only: the linear branch's output reads the state carried into
                                 the chunk, decayed up to the query, and nothing the chunk's own tokens wrote;
                              2: the linear operation only: a query attends to earlier softmax chunks only (a
                                 query that then sees nothing gets O_nla = 0, lse = -inf).
                              The carried state and the cache are the same in all three.  Forward only          */
} nats_fwd_params;

/* Optional inputs / outputs of nats_hybrid_attn_fwd_ex; any pointer may be NULL. */
typedef struct nats_fwd_extra {
    const float* w_nla;         /* in  [B,H,L] weights of Eq. 21 (NULL -> 0.5)                   */
    const float* w_la;          /* in  [B,H,L]                    (NULL -> 0.5)                   */
    const float* initial_state; /* in  [B,H,d,d] f32 state S[d_v][d_k] before token 0 (NULL -> 0)*/
    float* final_state;         /* out [B,H,d,d] f32 state after token L-1                       */
    void* Kc;                   /* out [B,H,cap,d] softmax-token keys in order of position:      */
    void* Vc;                   /* out [B,H,cap,d] the decode KV cache (rows >= cap are dropped) */
    int32_t cap;                /* rows per (b,h) in Kc / Vc                                     */
    int32_t* n_s;               /* out [B,H]   number of softmax tokens                          */
    int32_t* idx;               /* out [B,H,L] idx[c] = position of the c-th softmax token;
                                   entries c >= n_s are left untouched                           */
    int32_t* cnt;               /* out [B,H,L] cnt[t] = number of softmax tokens among 0..t      */
    float* O_la;                /* out [B,H,L,d] f32 linear-branch output (Eq. 10)               */
    float* O_nla;               /* out [B,H,L,d] f32 softmax-branch output (Eq. 11)              */
    float* lse;                 /* out [B,H,L] f32 log-sum-exp of the visible logits; -inf where
                                   no softmax token is visible (then O_nla = 0)                  */
    const float* W_out;         /* in  [H,2,d] f32 or NULL.  With combine_mode 1: the weights of Eq. 21
                                   are computed from Q by Eq. 22, [w_nla, w_la] = softmax([W_out[h,0] . q_t,
                                   W_out[h,1] . q_t]); w_nla and w_la must then be NULL                  */
    const void* Q_nla;          /* in  [B,H,L,d] dtype or NULL: queries and keys of the softmax branch when  */
    const void* K_nla;          /* in  they differ from the linear branch's (Section 4.3: L2-normalised q, k for
                                   the linear operation, RMS-normalised and possibly rotated ones for softmax
                                   attention; V is shared).  Both or neither.  Kc then holds rows of K_nla.   */
} nats_fwd_extra;

/* Bytes of device workspace nats_hybrid_attn_fwd{,_ex} needs for these params
 * (0 if the params are invalid).  Host-only; touches no device. */
size_t nats_hybrid_attn_fwd_workspace_bytes(const nats_fwd_params* p);

/* O = merge(GDN branch, softmax branch) as defined above.
 *   Q, K, V : in  [B,H,L,d]  dtype p->dtype.  The paper L2-normalises q,k for the linear
 *             branch (Section 4.3); the caller does that, the library uses them as given.
 *   alpha   : in  [B,H,L] f32 decay in (0,1]           (Eq. 19)
 *   beta    : in  [B,H,L] f32 write strength in [0,1]  (Eq. 19)
 *   mask    : in  [B,H,L] u8 (routing = NATS_ROUTE_TOKEN) or [B,H,L/C] u8 (NATS_ROUTE_CHUNK), non-zero =
 *             softmax token / chunk (Eq. 12-13)
 *   O       : out [B,H,L,d] dtype p->dtype
 *   workspace, workspace_bytes : device scratch of at least *_workspace_bytes(p); contents
 *             are undefined afterwards; two calls in flight must not share it.
 * Value range of the bf16 path: its products take fp16 operands (fp32 sums, fp32 carried state), so
 * V, the carried state, the rows V - S k that the delta rule writes and both branches' output rows are
 * rounded to fp16 on their way into a product.  Magnitudes up to 65504 are represented; anything
 * beyond saturates at +-65504 (the hardware's fp16 clamp is on, no infinity or NaN arises) and no
 * status reports it.  alpha is clamped below at 1e-30 per token.  The fp32 path (NATS_F32 tensors,
 * or math = NATS_MATH_F32) has neither limit.
 * Returns NATS_OK once everything is enqueued. */
nats_status nats_hybrid_attn_fwd(const nats_fwd_params* p, const void* Q, const void* K, const void* V,
                                 const float* alpha, const float* beta, const uint8_t* mask, void* O,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* Same, with the optional inputs (Eq. 21 weights, initial state) and optional outputs
 * (final state, compacted KV cache and its integer bookkeeping, per-branch outputs)
 * that tests and the prefill -> decode hand-off need.  extra may be NULL. */
nats_status nats_hybrid_attn_fwd_ex(const nats_fwd_params* p, const void* Q, const void* K, const void* V,
                                    const float* alpha, const float* beta, const uint8_t* mask, void* O,
                                    const nats_fwd_extra* extra, void* workspace, size_t workspace_bytes,
                                    void* hip_stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): nats_hybrid_attn_fwd with the workspace taken from a buffer of NATS_NOALLOC_SCRATCH_BYTES that is
 * part of the library's device code, one copy per GPU, held from the moment the library is loaded until the
 * process ends.  The call allocates nothing and frees nothing (no hipMalloc, no allocating library routine); its
 * first call on a device looks up the buffer's address (no stream operation).  Problems whose
 * nats_hybrid_attn_fwd_workspace_bytes() exceeds NATS_NOALLOC_SCRATCH_BYTES return NATS_ERR_WORKSPACE and
 * launch nothing.  Every call on a GPU shares that GPU's buffer: calls that overlap in time on one GPU (two
 * streams, two threads) race; calls ordered on one stream do not.  The buffer keeps the last call's contents;
 * no kernel needs it cleared.  Arguments and result as nats_hybrid_attn_fwd. */
#define NATS_NOALLOC_SCRATCH_BYTES (32u << 20)
nats_status nats_hybrid_attn_fwd_noalloc(const nats_fwd_params* p, const void* Q, const void* K, const void* V,
                                         const float* alpha, const float* beta, const uint8_t* mask, void* O,
                                         void* hip_stream);

/* ------------------------------------------------------------------------- *
 * Backward pass (Section 4.2), any of the three merges, fp32 results
 * ------------------------------------------------------------------------- */
typedef struct nats_bwd_extra {
    const float* initial_state; /* in  [B,H,d,d] f32, the state the forward started from (NULL -> 0)         */
    float* d_initial_state;     /* out [B,H,d,d] f32, gradient of that state                                 */
    float* g_nla;               /* out [B,H,L] f32: g_j = sum_i dM_ij of Eq. 15 for softmax tokens j, 0 for
                                   linear tokens; Eq. 16 (the gradient of a chunk's softmax score) is the sum
                                   of g over the chunk's tokens                                              */
    float* g_la;                /* out [B,H,L] f32: the linear operation's counterpart (Eq. 17, "sum of dS . S"):
                                   for a linear token, the sum over the state's entries of (gradient of the loss
                                   with respect to the state after the token's write) x (what the token wrote),
                                   i.e. the derivative with respect to a multiplier on the write of Eq. 14;
                                   0 for softmax tokens.  With routing per chunk: not available (NULL)          */
    float* dscore_nla;          /* out [B,H,L/C] f32: Eq. 16, gradient of a chunk's softmax score                */
    float* dscore_la;           /* out [B,H,L/C] f32: Eq. 17, gradient of a chunk's linear score.  Routing per
                                   token: the sums of g_nla and g_la over the chunk's tokens.  Routing per chunk:
                                   the mask gradients between chunks (the inner part of a chunk is computed by
                                   both operations whatever its type, no mask stands on it); a chunk gets no
                                   gradient for the operation it is inactive for (Section 4.2)                   */
    const void* Q_nla;          /* in  [B,H*G,L,d] dtype p->dtype: queries and keys of the softmax branch given apart */
    const void* K_nla;          /*     (as nats_fwd_extra.Q_nla, K_nla; both or neither, NULL = the branch uses Q, K) */
    float* dQ_nla;              /* out [B,H*G,L,d] f32: their gradients (required with Q_nla, K_nla).  dQ and dK are     */
    float* dK_nla;              /*     then the linear branch's gradients alone                                        */
    const float* w_nla;         /* in  [B,H*G,L] f32: the weights of the merge, p->combine_mode 1 (Eq. 21) and 2 (its      */
    const float* w_la;          /*     ablation with one normalisation); NULL: 0.5 (mode 1) or 1 (mode 2) as in the forward */
    float* dw_nla;              /* out [B,H*G,L] f32: their gradients (each optional); the caller takes them through        */
    float* dw_la;               /*     Eq. 22 (or whatever made the weights).  All four must be NULL with combine_mode 0    */
} nats_bwd_extra;

size_t nats_hybrid_attn_bwd_workspace_bytes(const nats_fwd_params* p);

/* Gradients of nats_hybrid_attn_fwd's O with respect to its inputs, given dO = dLoss/dO.  For O = O_la + O_nla:
 * the adjoint of the recurrence of Eq. 19 / 14 / 20 (or of the gated operation) for the linear branch, and the
 * attention backward over the softmax columns of Eq. 12 with the mask gradients of Eq. 15.  k and v of a
 * softmax token get nothing from the linear branch and vice versa (Section 4.2).
 *   p->combine_mode 1 (Eq. 21) and 2 (Section 5, the ablation with one normalisation): the merge acts on the two
 *             branches' output rows, so its adjoint turns dO into one gradient per branch, and each branch then runs
 *             as for the plain sum.  The pass recomputes both branches' rows in fp32 (the linear branch's token by
 *             token), takes p->rms_eps and extra->w_nla, w_la, and returns extra->dw_nla, dw_la.  These per-branch
 *             gradients are fp32, so bf16 tensors are widened first and the whole pass runs on fp32 tensors
 *             (slower than combine_mode 0, and a workspace larger by the fp32 copies).
 *   Q, K, V, alpha, beta, mask : as in the forward (either routing).
 *             With routing per chunk the function differentiated is the one the
 *             forward computes there: both operations compute every chunk's inner part, the masks act between
 *             chunks, a softmax chunk hands on (its decay) x (the state at its start).  Every sum is fp32 and the recurrence's adjoint is fp32 throughout.
 *             p->math: with NATS_MATH_AUTO the linear branch's adjoint runs by chunks of 64
 *             tokens on fp32 matrix instructions (the chunk form of Eq. 19 / 20 and its derivative; the states
 *             at the chunk starts, then the state gradients behind every chunk, then all chunks in parallel);
 *             dalpha then comes through the logarithms of the decays and needs alpha > 0 (an alpha of exactly 0
 *             gets dalpha = 0).  NATS_MATH_FP32 takes the adjoint token by token (the workspace is larger).
 *             For bf16 tensors the softmax branch's dQ, dK, dV products run on the matrix cores: Q, K, V, dO
 *             enter exactly (they are bf16), the probabilities and dS enter as the sum of two fp16 terms,
 *             so the gradients keep fp32-level accuracy; for f32 tensors those products are fp32 too
 *   dO      : in  [B,H,L,d] dtype p->dtype
 *   dQ, dK, dV : out [B,H,L,d] f32 (whatever p->dtype);  dalpha, dbeta : out [B,H,L] f32
 *   extra   : optional, may be NULL
 *   head grouping (p->group = G > 1, Section 4.3; the softmax heads of a group use the linear head's Q and K, or
 *             their own, extra->Q_nla, K_nla with H*G heads):
 *             V, dO, dV are [B,H*G,L,d] and initial_state, d_initial_state [B,H*G,d,d], head h*G + g the member g
 *             of linear head h as in the forward; Q, K, alpha, beta, mask and their gradients, g_nla, g_la and the
 *             score gradients stay [B,H,...]: a shared input's gradient is the sum over the G heads that read it.
 *             The pass runs once per member (G times the work and a workspace larger by one member's tensors)
 *   workspace : at least nats_hybrid_attn_bwd_workspace_bytes(p); nothing is kept from the forward call, the
 *             backward recomputes what it needs (the state is checkpointed once per 64 tokens)
 * Sums over (batch, head)-internal blocks are taken in a fixed order: results are deterministic. */
nats_status nats_hybrid_attn_bwd(const nats_fwd_params* p, const void* Q, const void* K, const void* V,
                                 const float* alpha, const float* beta, const uint8_t* mask, const void* dO,
                                 float* dQ, float* dK, float* dV, float* dalpha, float* dbeta,
                                 const nats_bwd_extra* extra, void* workspace, size_t workspace_bytes,
                                 void* hip_stream);

/* ------------------------------------------------------------------------- *
 * Single-token decode (Section 4.1, per-token generation, with per-token routing)
 * ------------------------------------------------------------------------- */
typedef struct nats_dec_params {
    int32_t B, H;
    int32_t d;             /* 64 or 128                                                         */
    int32_t cap;           /* rows per (b,h) in the KV cache                                    */
    int32_t dtype;         /* nats_dtype of q, k, v, o and of the KV cache                      */
    float softmax_scale;   /* as in nats_fwd_params                                             */
    float la_scale;
    int32_t combine_mode;
    float rms_eps;
    int32_t linear_op;         /* as in nats_fwd_params */
    int32_t freeze_on_softmax; /* as in nats_fwd_params (routing per chunk: applied by the commit) */
    const void* q_nla;         /* [B,H,d] dtype or NULL: the softmax branch's own query and key of this token  */
    const void* k_nla;         /* (see nats_fwd_extra.Q_nla); both or neither; k_nla is what the cache receives */
    void* workspace;           /* NULL, or device scratch of nats_hybrid_attn_decode_workspace_bytes(p) bytes for    */
    size_t workspace_bytes;    /* nats_hybrid_attn_decode: the step then runs as many blocks of equal size (state
                                  rows and cache rows of a (b,h) spread over blocks, partial results merged by a
                                  second kernel) instead of one block per (b,h); same result up to the order of
                                  the softmax sums.  Worth it when cache lengths differ across the batch.
                                  Contents undefined afterwards; calls in flight must not share it             */
} nats_dec_params;

/* Bytes of the optional workspace of nats_hybrid_attn_decode (0 if the params are invalid).  Host-only. */
size_t nats_hybrid_attn_decode_workspace_bytes(const nats_dec_params* p);

/* For every (b,h):  S <- alpha S;  linear token: S <- S + beta (v - S k) k^T;  softmax token:
 * (k,v) appended to the cache first (it sees itself, Eq. 12 i >= j);  then
 * o = merge(la_scale * S q, softmax(scale * q.K_cache^T) V_cache).
 *   state     : in/out [B,H,d,d] f32, S[d_v][d_k], updated in place
 *   k_cache, v_cache : in/out [B,H,cap,d]; row cache_len[b,h] is written for a softmax token
 *   cache_len : in/out [B,H] i32, incremented for a softmax token
 *   q, k, v   : in  [B,H,d];  alpha, beta : in [B,H] f32;  mask : in [B,H] u8
 *   w_nla, w_la : in [B,H] f32 or NULL (0.5), used by combine_mode 1
 *   o         : out [B,H,d]
 *   err_flags : out [B,H] i32 or NULL; set to 1 where a softmax token found its cache full
 *               (the token is then not stored and o covers the existing rows), else 0.
 * Needs no workspace (p->workspace = NULL); with one it balances uneven cache lengths, see nats_dec_params. */
nats_status nats_hybrid_attn_decode(const nats_dec_params* p, float* state, void* k_cache, void* v_cache,
                                    int32_t* cache_len, const void* q, const void* k, const void* v,
                                    const float* alpha, const float* beta, const uint8_t* mask,
                                    const float* w_nla, const float* w_la, void* o, int32_t* err_flags,
                                    void* hip_stream);

/* Routing decision per chunk by the score layer (Section 4.1, Eq. 8-9): the layer's input features are
 * mean-pooled over each chunk of C tokens, one linear layer maps the mean to a score per head and
 * operation, and the operation with the higher score gets the chunk.
 *   X      : in  [B,L,d_model] dtype (NATS_F32 or NATS_BF16); d_model a multiple of 8, at most 65536
 *   W_s    : in  [H,2,d_model] f32; row 0 of a head scores softmax attention, row 1 the linear operation
 *   scores : out [B,L/C,H,2] f32 or NULL
 *   mask_c : out [B,H,L/C] u8, 1 = softmax chunk (score 0 >= score 1, decided on the fp32 scores), the
 *            mask nats_hybrid_attn_fwd takes with routing = NATS_ROUTE_CHUNK
 * L must be a multiple of C; H at most 32. */
nats_status nats_route_chunks(int32_t B, int32_t L, int32_t C, int32_t d_model, int32_t H, int32_t dtype,
                              const void* X, const float* W_s, float* scores, uint8_t* mask_c, void* hip_stream);

/* Weights of the merge by Eq. 22 as a call of its own (the forward does the same when W_out is given):
 *   Q [B,H,L,d] dtype p->dtype (L = 1 for a generation step; only B, H, L, d, dtype, weight_act of p are used),
 *   W_out [H,2,d] f32  ->  w_nla, w_la [B,H,L] f32,  [w_nla, w_la] = softmax([W_out[h,0] . q, W_out[h,1] . q]).
 * The paper maps "the attention q values" to the weights; the Q given here is used as it is. */
/* The ablation (v) of Section 5, "Weights From X": the merge weights from the layer's input features instead of
 * the queries.  X [B,L,d_model] dtype (d_model a multiple of 8, at most 65536), W_x [H,2,d_model] f32 (row 0:
 * softmax attention, row 1: the linear operation; H at most 32)  ->  w_nla, w_la [B,H,L] f32 =
 * weight_act([W_x[h,0] . x_t, W_x[h,1] . x_t]), to be passed to the forward as its w_nla, w_la. */
nats_status nats_merge_weights_from_x(int32_t B, int32_t L, int32_t d_model, int32_t H, int32_t dtype, const void* X,
                                      const float* W_x, int32_t weight_act, float* w_nla, float* w_la, void* hip_stream);

nats_status nats_merge_weights(const nats_fwd_params* p, const void* Q, const float* W_out, float* w_nla,
                               float* w_la, void* hip_stream);

/* ------------------------------------------------------------------------- *
 * Generation with routing per chunk (Section 4.1, per-token generation)
 * ------------------------------------------------------------------------- */
/* The type of a chunk is known only after its last token, so inside an open chunk both operations
 * are updated provisionally and one of them is rolled back when the chunk is settled:
 *   every token:  S <- alpha S + beta (v - alpha S k) k^T  (Eq. 19) and (k, v) appended to the cache at
 *                 row cache_len + chunk_pos;  o = merge(la_scale * S q, softmax over rows
 *                 [0, cache_len + chunk_pos] of the cache)  -- the token sees earlier softmax chunks
 *                 and, causally, its own chunk;
 *   first token of a chunk (chunk_pos == 0): state_start <- S (before the update), chunk_decay <- 1;
 *   nats_hybrid_attn_decode_commit, after the chunk: a softmax chunk keeps its rows (cache_len +=
 *                 chunk_pos) and sets S <- chunk_decay * state_start (writes dropped, Eq. 14; decay
 *                 kept, Eq. 20); a linear chunk keeps S and drops the rows; chunk_pos <- 0.
 * All members are DEVICE pointers owned by the caller, updated in place. */
typedef struct nats_dec_chunk_state {
    float* state;         /* [B,H,d,d] f32 S[d_v][d_k], with the open chunk's provisional writes       */
    float* state_start;   /* [B,H,d,d] f32 state at the start of the open chunk                         */
    float* chunk_decay;   /* [B,H]     f32 product of alpha over the open chunk's tokens so far         */
    int32_t* chunk_pos;   /* [B,H]     i32 tokens of the open chunk seen so far                         */
    void* k_cache;        /* [B,H,cap,d] rows [0,cache_len) settled, [cache_len, +chunk_pos) provisional */
    void* v_cache;
    int32_t* cache_len;   /* [B,H]     i32 settled rows                                                 */
} nats_dec_chunk_state;

/* One token for every (b,h).  q, k, v [B,H,d]; alpha, beta [B,H]; w_nla, w_la [B,H] or NULL (0.5);
 * o [B,H,d]; err_flags [B,H] or NULL: 1 where the cache was full (the token is then not stored and o
 * covers the rows that are there).  The cache needs room for cache_len + C rows. */
nats_status nats_hybrid_attn_decode_chunk(const nats_dec_params* p, const nats_dec_chunk_state* s, const void* q,
                                          const void* k, const void* v, const float* alpha, const float* beta,
                                          const float* w_nla, const float* w_la, void* o, int32_t* err_flags,
                                          void* hip_stream);

/* Settles the open chunk of every (b,h) with its routing decision mask_c [B,H] u8 (non-zero = softmax
 * chunk), as described above.  err_flags [B,H] or NULL: 1 where rows of a softmax chunk had not fitted. */
nats_status nats_hybrid_attn_decode_commit(const nats_dec_params* p, const nats_dec_chunk_state* s,
                                           const uint8_t* mask_c, int32_t* err_flags, void* hip_stream);

/* Host-side message for the last non-OK status returned on this thread ("" if none). */
const char* nats_last_error(void);

/* ABI version of this header: major * 100 + minor. */
int nats_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NATS_H_ */
