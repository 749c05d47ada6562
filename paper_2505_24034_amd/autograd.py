"""torch.autograd glue over the three entry points, for a PyTorch trainer that wants the path as one differentiable
op: `aipo_loss(H, W, ...)` returns the scalar loss (paper Sec. 6 update, as a loss: see `llamarl_offpolicy_loss_fwd`
in include/llamarl.h) and the statistics; `loss.backward()` fills `H.grad` and `W.grad` through
`llamarl_offpolicy_loss_bwd`.  No arithmetic happens here: the forward chains `llamarl_token_logprobs` and
`llamarl_offpolicy_loss_fwd`, keeps `lse` and `coef`, and the backward hands them to the library.

The upstream gradient of the loss reaches the C ABI as a host float, so `backward` reads it from the device once
(one synchronisation per backward; it is 1.0 when the loss is the root of the graph)."""
import torch

from . import binding as L


class _AipoLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, H, W, targets, mu_logp, adv, mask, rho, norm_mode, clip_mode, eps_lo, eps_hi, dW_dtype):
        B, T = mask.shape
        logp, lse = L.token_logprobs(H, W, targets, mask.reshape(-1))
        loss, coef, stats = L.offpolicy_loss_fwd(logp, mu_logp, adv, mask, B, T, rho=rho, norm_mode=norm_mode,
                                                 clip_mode=clip_mode, eps_lo=eps_lo, eps_hi=eps_hi, targets=targets,
                                                 V=W.shape[0])
        ctx.save_for_backward(H, W, targets, lse, coef)
        ctx.dW_dtype = dW_dtype
        ctx.mark_non_differentiable(stats, logp)
        return loss.reshape(()), stats, logp

    @staticmethod
    def backward(ctx, g_loss, _g_stats, _g_logp):
        H, W, targets, lse, coef = ctx.saved_tensors
        dH, dW = L.offpolicy_loss_bwd(H, W, targets, lse, coef, grad_loss=float(g_loss), dW_dtype=ctx.dW_dtype)
        if dW.dtype != W.dtype:
            dW = dW.to(W.dtype)
        return (dH, dW) + (None,) * 10


def aipo_loss(H, W, targets, mu_logp, adv, mask, rho=2.0, norm_mode=L.NORM_TOKEN_MEAN, clip_mode=L.CLIP_AIPO,
              eps_lo=0.2, eps_hi=0.2, dW_dtype=None):
    """H [N,d], W [V,d] (bf16 or fp32, contiguous, on the GPU), targets int32 [N], mu_logp float32 [N],
    adv float32 [B] or [B,T], mask uint8 [B,T] with B*T = N.  Returns (loss (0-dim), stats [5], logp [N]); only
    the loss carries gradient, to H and W.  dW_dtype=torch.float32 accumulates the head's gradient in fp32 inside
    the library before it is cast to W's dtype for autograd."""
    return _AipoLoss.apply(H, W, targets, mu_logp, adv, mask, float(rho), int(norm_mode), int(clip_mode),
                           float(eps_lo), float(eps_hi), dW_dtype)
