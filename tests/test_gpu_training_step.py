"""One training step of the paper's model (Section 4.2, Eq. 11): Dense(20 -> d, tanh) -> signature of depth N ->
Dense(D -> 10), mean squared error.  On the GPU the two Dense layers are torch and the signature layer is libsig
(sig_compute forward, sig_backward backward, through paper_2501_08455_amd/autograd.py); the expected loss and the four
parameter gradients come from the same chain written out in fp64 numpy around the two oracles (oracle.signature and
oracle.signature_backward).  Batches: the full 128, and the ragged last batch of an epoch over 12,765 samples -- the
paper states 65, while 12,765 - 99 x 128 = 93; both are run.  Shapes (L, d, N): the three that bench.py times.

The activation is not named in the paper; tanh is used on both sides.  Gate: relative Frobenius error 1e-4 on the loss
and on every gradient (the forward transform's tolerance; the Dense layers run in fp32 on the GPU).
"""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 1e-4


def say(msg):
    print(msg)
    sys.stdout.flush()


def reference_step(oracle, X, Y, W1, b1, W2, b2, depth):
    """Loss and gradients (dW1, db1, dW2, db2) of the model in fp64, the signature layer through the oracles."""
    X, Y, W1, b1, W2, b2 = (np.asarray(a, dtype=np.float64) for a in (X, Y, W1, b1, W2, b2))
    A = X @ W1 + b1                                   # [B, L, d]
    Z = np.tanh(A)
    # the layer sees what the GPU layer sees: the fp32 hidden paths (the oracle widens them exactly)
    Z32 = Z.astype(np.float32)
    S = oracle.signature(Z32, depth)                  # [B, D]
    P = S @ W2 + b2                                   # [B, 10]
    R = P - Y
    loss = np.mean(R ** 2)
    dP = 2.0 * R / R.size
    dW2 = S.T @ dP
    db2 = dP.sum(axis=0)
    dS = dP @ W2.T                                    # [B, D]
    dZ = oracle.signature_backward(Z32, depth, dS)    # [B, L, d]
    dA = dZ * (1.0 - Z ** 2)
    dW1 = np.einsum("blc,bld->cd", X, dA)
    db1 = dA.sum(axis=(0, 1))
    return loss, dW1, db1, dW2, db2


@pytest.mark.parametrize("L,d,depth", [(100, 5, 4), (200, 6, 3), (500, 4, 4)])
@pytest.mark.parametrize("B", [128, 93, 65])
def test_training_step_gradients(oracle, L, d, depth, B):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2501_08455_amd import autograd, workloads
    D = workloads.sig_size(d, depth)
    rng = np.random.default_rng(1000 * L + 10 * d + depth + B)
    X = (np.cumsum(rng.normal(size=(B, L, 20)), axis=1) / np.sqrt(L)).astype(np.float32)
    Y = rng.normal(size=(B, 10)).astype(np.float32)
    W1 = (rng.normal(size=(20, d)) * 0.2).astype(np.float32)
    b1 = (rng.normal(size=d) * 0.1).astype(np.float32)
    W2 = (rng.normal(size=(D, 10)) * 0.05).astype(np.float32)
    b2 = (rng.normal(size=10) * 0.1).astype(np.float32)
    say("training step B=%d L=%d d=%d depth=%d (D=%d)" % (B, L, d, depth, D))

    dev = "cuda"
    Xt, Yt = torch.from_numpy(X).to(dev), torch.from_numpy(Y).to(dev)
    params = [torch.from_numpy(a).to(dev).requires_grad_(True) for a in (W1, b1, W2, b2)]
    W1t, b1t, W2t, b2t = params
    # keep the GEMMs in plain fp32 (no reduced-precision matmul modes)
    torch.backends.cuda.matmul.allow_tf32 = False
    Z = torch.tanh(Xt @ W1t + b1t)
    S = autograd.signature(Z, depth)
    loss = ((S @ W2t + b2t - Yt) ** 2).mean()
    grads = torch.autograd.grad(loss, params)
    torch.cuda.synchronize()

    want = reference_step(oracle, X, Y, W1, b1, W2, b2, depth)
    got = [float(loss.detach())] + [g.cpu().numpy().astype(np.float64) for g in grads]
    names = ["loss", "dW1", "db1", "dW2", "db2"]
    errs = []
    for name, g, w in zip(names, got, want):
        g, w = np.asarray(g), np.asarray(w)
        assert g.shape == w.shape and np.all(np.isfinite(g)), name
        errs.append(np.linalg.norm(g - w) / np.linalg.norm(w))
    say("  rel err: " + "  ".join("%s %.2e" % (n, e) for n, e in zip(names, errs)))
    assert max(errs) <= TOL, dict(zip(names, errs))


def test_an_epoch_over_the_ragged_set_runs_and_lowers_the_loss(oracle):
    """A short run of plain gradient descent over a set whose size is not a multiple of the batch (the layer is called
    with 128 and then with the remainder, again and again, as in an epoch of the paper's experiment): the loss of the
    full set falls, and the last step's gradients agree with the fp64 chain."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2501_08455_amd import autograd, workloads
    L, d, depth, n, batch = 50, 4, 3, 128 * 3 + 65, 128
    D = workloads.sig_size(d, depth)
    rng = np.random.default_rng(7)
    X = (np.cumsum(rng.normal(size=(n, L, 20)), axis=1) / np.sqrt(L)).astype(np.float32)
    Wtrue = rng.normal(size=(D, 10)) * 0.3
    W1 = (rng.normal(size=(20, d)) * 0.2).astype(np.float32)
    b1 = np.zeros(d, dtype=np.float32)
    # targets a linear read-out of the signatures can reach
    S0 = oracle.signature(np.tanh(X.astype(np.float64) @ W1 + b1).astype(np.float32), depth)
    Y = (S0 @ Wtrue).astype(np.float32)
    Xt, Yt = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda()
    params = [torch.from_numpy(a).cuda().requires_grad_(True)
              for a in (W1, b1, np.zeros((D, 10), dtype=np.float32), np.zeros(10, dtype=np.float32))]

    def full_loss():
        with torch.no_grad():
            Z = torch.tanh(Xt @ params[0] + params[1])
            return float((((autograd.signature(Z, depth) @ params[2] + params[3]) - Yt) ** 2).mean())

    before = full_loss()
    for epoch in range(3):
        for lo in range(0, n, batch):
            hi = min(lo + batch, n)
            Z = torch.tanh(Xt[lo:hi] @ params[0] + params[1])
            loss = ((autograd.signature(Z, depth) @ params[2] + params[3] - Yt[lo:hi]) ** 2).mean()
            grads = torch.autograd.grad(loss, params)
            if epoch == 2 and hi == n:
                snap = [p.detach().cpu().numpy().copy() for p in params]
                want = reference_step(oracle, X[lo:hi], Y[lo:hi], *snap, depth)
                for name, g, w in zip(["dW1", "db1", "dW2", "db2"], grads, want[1:]):
                    err = np.linalg.norm(g.cpu().numpy() - w) / np.linalg.norm(w)
                    assert err <= TOL, (name, err)
            with torch.no_grad():
                for p_, g_ in zip(params, grads):
                    p_ -= 0.05 * g_
    after = full_loss()
    say("  loss over the set: %.4f -> %.4f" % (before, after))
    assert after < before
