"""torch.autograd glue over the C ABI (marshalling only): the forward keeps the int32 argmax the kernels
emit (Sec. "Closed-Form Gradients"), the backward hands it with the upstream gradient to maxsim_backward.
Nothing is computed here; every step runs in the HIP kernels, and there is no CPU fallback."""
import torch

from . import binding as M


class _MaxSim(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, D):
        scores, argmax = M.maxsim_forward(Q, D, want_argmax=True)
        ctx.save_for_backward(Q, D, argmax)
        return scores

    @staticmethod
    def backward(ctx, dscore):
        Q, D, argmax = ctx.saved_tensors
        dQ, dD = M.maxsim_backward(Q, D, argmax, dscore.contiguous().float())
        return dQ.to(Q.dtype), dD.to(D.dtype)


class _MaxSimRagged(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, D_packed, doc_offsets):
        scores, argmax = M.maxsim_forward_ragged(Q, D_packed, doc_offsets, want_argmax=True)
        ctx.save_for_backward(Q, D_packed, doc_offsets, argmax)
        return scores

    @staticmethod
    def backward(ctx, dscore):
        Q, D_packed, doc_offsets, argmax = ctx.saved_tensors
        dQ, dD = M.maxsim_backward_ragged(Q, D_packed, doc_offsets, argmax, dscore.contiguous().float())
        return dQ.to(Q.dtype), dD.to(D_packed.dtype), None


def maxsim(Q, D, doc_offsets=None):
    """Differentiable scores [n_q, b] of Q [n_q,l_q,d] against D [b,l_d,d], or against a packed corpus
    D [T,d] with int32 doc_offsets [b+1] (all on the GPU; d as the forward and backward entry points take it).  An empty ragged document scores -inf and receives no gradient."""
    if doc_offsets is None:
        return _MaxSim.apply(Q, D)
    return _MaxSimRagged.apply(Q, D, doc_offsets)
