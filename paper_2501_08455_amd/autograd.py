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


def capture(step_fn, warmup=3):
    """One call of `step_fn()` as a HIP graph: (graph, what the captured call returned).

    A training step of the paper's model at batch 128 is a few dozen short kernels, and launching them one by one costs
    several times what they take to run; replayed as a graph the step is one launch.  `step_fn` must read its inputs from
    tensors that stay where they are (copy each batch into them before `graph.replay()`) and may update its parameters
    in place.  It is first run `warmup` times outside the graph, on a side stream of default priority, so that libsig has
    sized its context scratch and torch its workspaces: neither may allocate while the capture is on.
    """
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(warmup):
            step_fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = step_fn()
    return graph, out
