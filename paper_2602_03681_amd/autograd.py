"""torch.autograd wrapper over the two C-ABI calls nats_hybrid_attn_fwd_ex and nats_hybrid_attn_bwd.

Argument marshalling only: the forward is one call of the forward entry point, the backward one call of the
backward entry point (which recomputes what it needs; nothing but the inputs is kept between the two).  The
routing mask is a hard decision and gets no gradient of its own; the paper trains the score layer that makes it
with a straight-through estimator (Section 4.2): pass `score_nla` / `score_la` ([B,H,L/C] tensors that require
grad; their values are not read) and their .grad receives the chunk score gradients of Eq. 16 / Eq. 17.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as nb


class _HybridAttn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, opts, Q, K, V, alpha, beta, mask, initial_state, w_nla, w_la, Q_nla, K_nla, score_nla, score_la):
        r = nb.hybrid_attn_fwd_ex(Q, K, V, alpha, beta, mask, opts["C"], softmax_scale=opts["softmax_scale"],
                                  la_scale=opts["la_scale"], combine_mode=opts["combine_mode"], rms_eps=opts["rms_eps"],
                                  routing=opts["routing"], linear_op=opts["linear_op"],
                                  freeze_on_softmax=opts["freeze_on_softmax"], w_nla=w_nla, w_la=w_la,
                                  initial_state=initial_state, Q_nla=Q_nla, K_nla=K_nla, group=opts["group"])
        ctx.opts = opts
        ctx.save_for_backward(Q, K, V, alpha, beta, mask, initial_state, w_nla, w_la, Q_nla, K_nla)
        ctx.score_shapes = tuple(None if s is None else (s.shape, s.dtype) for s in (score_nla, score_la))
        return r["O"]

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, alpha, beta, mask, initial_state, w_nla, w_la, Q_nla, K_nla = ctx.saved_tensors
        o = ctx.opts
        need = ctx.needs_input_grad   # index 0 is `opts`
        want = []
        if initial_state is not None and need[7]: want.append("d_initial_state")
        if ctx.score_shapes[0] is not None and need[12]: want.append("dscore_nla")
        if ctx.score_shapes[1] is not None and need[13]: want.append("dscore_la")
        r = nb.hybrid_attn_bwd(Q, K, V, alpha, beta, mask, dO.to(Q.dtype).contiguous(), o["C"],
                               softmax_scale=o["softmax_scale"], la_scale=o["la_scale"], linear_op=o["linear_op"],
                               freeze_on_softmax=o["freeze_on_softmax"], initial_state=initial_state, want=tuple(want),
                               routing=o["routing"], group=o["group"], Q_nla=Q_nla, K_nla=K_nla,
                               combine_mode=o["combine_mode"], rms_eps=o["rms_eps"], w_nla=w_nla, w_la=w_la)

        def g(key, like, wanted):
            return r[key].to(like.dtype) if (wanted and like is not None and key in r) else None

        grads = [None,
                 g("dQ", Q, need[1]), g("dK", K, need[2]), g("dV", V, need[3]), g("dalpha", alpha, need[4]),
                 g("dbeta", beta, need[5]), None, g("d_initial_state", initial_state, need[7]),
                 g("dw_nla", w_nla, need[8]), g("dw_la", w_la, need[9]), g("dQ_nla", Q_nla, need[10]),
                 g("dK_nla", K_nla, need[11])]
        for key, meta, wanted in (("dscore_nla", ctx.score_shapes[0], need[12]),
                                  ("dscore_la", ctx.score_shapes[1], need[13])):
            grads.append(r[key].to(meta[1]).reshape(meta[0]) if (meta is not None and wanted) else None)
        return tuple(grads)


def hybrid_attn(Q, K, V, alpha, beta, mask, C: int = 64, *, softmax_scale: float = 0.0, la_scale: float = 0.0,
                combine_mode: int = 0, rms_eps: float = 0.0, routing: int = nb.NATS_ROUTE_TOKEN,
                linear_op: int = nb.NATS_LINEAR_GDN, freeze_on_softmax: bool = False, group: int = 1,
                initial_state: Optional[torch.Tensor] = None, w_nla: Optional[torch.Tensor] = None,
                w_la: Optional[torch.Tensor] = None, Q_nla: Optional[torch.Tensor] = None,
                K_nla: Optional[torch.Tensor] = None, score_nla: Optional[torch.Tensor] = None,
                score_la: Optional[torch.Tensor] = None) -> torch.Tensor:
    """O of nats_hybrid_attn_fwd_ex as a differentiable function of Q, K, V, alpha, beta, initial_state, the merge
    weights and the softmax branch's own queries and keys (arguments as in binding.hybrid_attn_fwd_ex and
    binding.hybrid_attn_bwd; what the backward entry point does not cover, it rejects).  score_nla, score_la: see the
    module's note on the straight-through estimator."""
    opts = dict(C=C, softmax_scale=softmax_scale, la_scale=la_scale, combine_mode=combine_mode, rms_eps=rms_eps,
                routing=routing, linear_op=linear_op, freeze_on_softmax=freeze_on_softmax, group=group)
    return _HybridAttn.apply(opts, Q, K, V, alpha, beta, mask, initial_state, w_nla, w_la, Q_nla, K_nla, score_nla,
                             score_la)
