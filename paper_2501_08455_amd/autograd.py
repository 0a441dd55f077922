"""The signature as a differentiable torch operation: sig_compute forward, sig_backward backward.

Marshalling only: both directions run in libsig's kernels (include/sig.h).  This is what lets the layer sit
between trainable layers as in the paper's model (Section 4.2, Eq. 11).
"""
import torch

from . import binding


class _Signature(torch.autograd.Function):
    @staticmethod
    def forward(ctx, path, depth, stream):
        path = path.contiguous()
        out = binding.signature(path, depth, stream=stream)
        ctx.save_for_backward(path, out)
        ctx.depth = int(depth)
        ctx.stream = bool(stream)
        return out

    @staticmethod
    def backward(ctx, grad_out):
        path, out = ctx.saved_tensors
        grad_path = torch.empty_like(path)
        rc = binding.sig_backward(binding.default_ctx(), path, ctx.depth, int(ctx.stream), out,
                                  grad_out.contiguous(), grad_path)
        if rc != binding.SIG_OK:
            raise binding.SigError(rc, "sig_backward")
        return grad_path, None, None


def signature(path, depth, stream=False):
    """Depth-`depth` signatures of `path` (float32 CUDA tensor [B, L, d]) with gradient support:
    [B, D], or [B, L-1, D] with stream=True."""
    return _Signature.apply(path, depth, stream)
