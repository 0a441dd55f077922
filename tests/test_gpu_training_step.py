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


@pytest.mark.parametrize("L,d,depth,B", [(100, 5, 4, 128), (200, 6, 3, 93)])
def test_training_step_as_a_graph_replays_like_the_eager_step(L, d, depth, B):
    """The whole step (both Dense layers, the signature layer forward and backward, the update) captured once as a HIP
    graph and replayed on four different batches, with eager work and synchronisation between the replays: after every
    replay the parameters equal those of the same steps run eagerly from the same start."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2501_08455_amd import autograd, workloads
    D = workloads.sig_size(d, depth)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5 + L)
    batches = [(torch.randn((B, L, 20), device="cuda", generator=gen).cumsum(1) / L ** 0.5,
                torch.randn((B, 10), device="cuda", generator=gen)) for _ in range(4)]
    start = [torch.randn((20, d), device="cuda", generator=gen) * 0.2, torch.zeros(d, device="cuda"),
             torch.randn((D, 10), device="cuda", generator=gen) * 0.05, torch.zeros(10, device="cuda")]

    def make(params, xb, yb):
        def step():
            Z = torch.tanh(xb @ params[0] + params[1])
            S = autograd.signature(Z, depth)
            loss = ((S @ params[2] + params[3] - yb) ** 2).mean()
            grads = torch.autograd.grad(loss, params)
            with torch.no_grad():
                for p_, g_ in zip(params, grads):
                    p_ -= 1e-2 * g_
            return loss
        return step

    eager = [p.clone().requires_grad_(True) for p in start]
    graphed = [p.clone().requires_grad_(True) for p in start]
    xb, yb = batches[0][0].clone(), batches[0][1].clone()
    graph_step = make(graphed, xb, yb)
    say("capturing the step L=%d d=%d depth=%d B=%d" % (L, d, depth, B))
    graph, loss_g = autograd.capture(graph_step)
    with torch.no_grad():                      # the warm-up and the capture moved the parameters: start again
        for p_, s_ in zip(graphed, start):
            p_.copy_(s_)
    for i, (x, y) in enumerate(batches):
        say("replay %d" % i)
        xb.copy_(x)
        yb.copy_(y)
        graph.replay()
        loss_e = make(eager, x, y)()           # the program's own eager work between the replays
        torch.cuda.synchronize()
        lg, le = float(loss_g.detach()), float(loss_e.detach())
        assert np.isfinite(lg) and abs(lg - le) <= 1e-5 * abs(le)
        for pg, pe in zip(graphed, eager):
            err = float((pg - pe).norm() / pe.norm().clamp_min(1e-30))
            assert err <= 1e-5, (i, err)
