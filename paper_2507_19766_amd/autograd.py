"""torch.autograd entry points over the binding, so that the fused objective (Sec. 3.2.2) can sit in
a training script where a log-softmax / gather / clipped-ratio chain would otherwise be:

    loss = ulorl.autograd.token_loss(logits, token_ids, cu_seqlens, advantages, old_logp, params)
    loss.backward()                     # logits.grad holds dlogits

Nothing here computes: every function forwards tensors to the library calls of ``binding`` and
hands their results to autograd.  There is no CPU path.

Two ways to run the logits path:
  * ``fused=False`` (default): ``ulorl_token_loss_fwd`` in forward, ``ulorl_token_loss_bwd`` in
    backward with the upstream gradient as ``grad_out``.  Any upstream scale is honoured.
  * ``fused=True``: ``ulorl_token_loss_fwd_bwd`` in forward (the logits are read once and the
    gradient of an upstream 1 is written in the same pass); backward hands that gradient out and
    refuses any other upstream gradient.  ``in_place=True`` lets the gradient overwrite ``logits``.

The upstream gradient is a 0-dim device tensor; reading it (``float()``) synchronises the stream
once per backward, as ``grad_out`` is a host scalar of the C ABI.
"""
from typing import Optional

import torch

from . import binding
from .binding import FwdResult, Launch, Params


class _TokenLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, logits, token_ids, cu_seqlens, advantages, old_logp, params, segment_ids, fused, in_place,
                launch, sink):
        ctx.fused = bool(fused)
        if fused:
            res, dlogits = binding.token_loss_fwd_bwd(logits, token_ids, cu_seqlens, advantages, old_logp, params,
                                                      segment_ids=segment_ids, grad_out=1.0, inplace=bool(in_place),
                                                      launch=launch)
            ctx.dlogits = dlogits
        else:
            if in_place:
                raise ValueError("in_place needs fused=True (the two-call path reads the logits again in backward)")
            res = binding.token_loss_fwd(logits, token_ids, cu_seqlens, advantages, old_logp, params,
                                         segment_ids=segment_ids, launch=launch)
            ctx.save_for_backward(logits, token_ids, res.lse, res.gcoef)
        if sink is not None:
            sink.append(res)
        return res.loss.reshape(())

    @staticmethod
    def backward(ctx, grad_loss):
        g = float(grad_loss)
        if ctx.fused:
            if g != 1.0:
                raise RuntimeError("token_loss(fused=True) computed the gradient of an upstream 1 in its forward pass; "
                                   "got an upstream gradient of %r: scale through Params.denominator or use fused=False" % g)
            d = ctx.dlogits
            ctx.dlogits = None
        else:
            logits, token_ids, lse, gcoef = ctx.saved_tensors
            d = binding.token_loss_bwd(logits, token_ids, lse, gcoef, grad_out=g)
        return (d,) + (None,) * 10


def token_loss(logits: torch.Tensor, token_ids, cu_seqlens, advantages, old_logp=None, params: Optional[Params] = None,
               segment_ids=None, fused: bool = False, in_place: bool = False, launch: Optional[Launch] = None,
               results: Optional[list] = None) -> torch.Tensor:
    """The masked, clipped policy-gradient loss of Sec. 3.2.2 as a differentiable 0-dim tensor (gradient
    to ``logits`` only).  ``results``: a list that receives the call's ``FwdResult`` (per-token
    log-probs, entropies, mask, ratio, counters)."""
    return _TokenLoss.apply(logits, token_ids, cu_seqlens, advantages, old_logp, params, segment_ids, fused, in_place,
                            launch, results)


class _LmheadTokenLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, hidden, weight, token_ids, cu_seqlens, advantages, old_logp, params, segment_ids, vocab_chunk,
                launch, sink):
        res = binding.lmhead_token_loss_fwd(hidden, weight, token_ids, cu_seqlens, advantages, old_logp, params,
                                            segment_ids=segment_ids, vocab_chunk=vocab_chunk, launch=launch)
        ctx.save_for_backward(hidden, weight, token_ids, res.lse, res.gcoef)
        ctx.vocab_chunk = vocab_chunk
        ctx.launch = launch
        if sink is not None:
            sink.append(res)
        return res.loss.reshape(())

    @staticmethod
    def backward(ctx, grad_loss):
        hidden, weight, token_ids, lse, gcoef = ctx.saved_tensors
        d_hidden, d_weight = binding.lmhead_token_loss_bwd(hidden, weight, token_ids, lse, gcoef, grad_out=float(grad_loss),
                                                           vocab_chunk=ctx.vocab_chunk, launch=ctx.launch)
        return (d_hidden, d_weight) + (None,) * 9


def lmhead_token_loss(hidden: torch.Tensor, weight: torch.Tensor, token_ids, cu_seqlens, advantages, old_logp=None,
                      params: Optional[Params] = None, segment_ids=None, vocab_chunk: int = 8192,
                      launch: Optional[Launch] = None, results: Optional[list] = None) -> torch.Tensor:
    """The same loss from the last hidden states and the lm_head weight [hidden, vocabulary], the
    logits never materialised; gradients to ``hidden`` and ``weight`` (both computed, bf16)."""
    return _LmheadTokenLoss.apply(hidden, weight, token_ids, cu_seqlens, advantages, old_logp, params, segment_ids,
                                  vocab_chunk, launch, results)


__all__ = ["token_loss", "lmhead_token_loss", "FwdResult"]
