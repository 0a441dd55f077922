"""Pins of the gradient oracle (oracle/sig_grad_oracle.c) to facts other than itself.

The paper prints no gradient values (it differentiates Eqs. 2-5 automatically, Section 4.2), so the pins are:
central finite differences of the forward oracle, the analytic derivative of the brute-force iterated sums
with explicit indices, closed forms (depth 1, one segment), and invariances.  All CPU, fp64.
"""
import itertools
import math

import numpy as np
import pytest


def rand_path(rng, L, d, scale=0.5):
    return np.cumsum(rng.normal(size=(L, d)) * scale, axis=0)


def finite_difference(oracle, x, N, g, stream, h=1e-6):
    fd = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp = x.copy(); xp[idx] += h
        xm = x.copy(); xm[idx] -= h
        fd[idx] = ((oracle.signature(xp, N, stream) - oracle.signature(xm, N, stream)) * g).sum() / (2 * h)
    return fd


# ---------------------------------------------------------------- 1. finite differences of the forward oracle
@pytest.mark.parametrize("B,L,d,N,stream", [(2, 5, 3, 3, False), (2, 5, 3, 3, True), (1, 2, 2, 4, False),
                                            (3, 7, 2, 4, True), (1, 4, 4, 2, False), (2, 6, 1, 5, True)])
def test_matches_central_finite_differences(oracle, B, L, d, N, stream):
    rng = np.random.default_rng(10 * B + L + d + N)
    x = np.stack([rand_path(rng, L, d) for _ in range(B)])
    D = oracle.sig_size(d, N)
    g = rng.normal(size=(B, L - 1, D) if stream else (B, D))
    got = oracle.signature_backward(x, N, g, stream)
    want = finite_difference(oracle, x, N, g, stream)
    np.testing.assert_allclose(got, want, rtol=2e-7, atol=2e-8)


# ---------------------------------------------------------------- 2. analytic derivative of the brute-force sums
def brute_force_gradient(x, N, glevels):
    """d/dx of sum_n <G_n, level n of the iterated integrals of the piecewise-linear path>, term by term.

    Level n is the sum over weakly increasing segment indices k_1 <= ... <= k_n of
    prod_r dx[k_r, i_r] / prod(run lengths)!; the derivative with respect to dx[k, i] removes one factor.
    """
    dx = np.diff(x, axis=0)
    K, d = dx.shape
    gdx = np.zeros_like(dx)
    for n in range(1, N + 1):
        G = glevels[n - 1].reshape((d,) * n)
        for ks in itertools.combinations_with_replacement(range(K), n):
            weight = 1.0
            for _, run in itertools.groupby(ks):
                weight /= math.factorial(len(list(run)))
            for word in itertools.product(range(d), repeat=n):
                for r in range(n):
                    rest = weight * G[word]
                    for s in range(n):
                        if s != r:
                            rest *= dx[ks[s], word[s]]
                    gdx[ks[r], word[r]] += rest
    gx = np.zeros_like(x)
    gx[1:] += gdx
    gx[:-1] -= gdx
    return gx


@pytest.mark.parametrize("L,d,N", [(2, 2, 4), (4, 2, 3), (5, 3, 3), (6, 2, 4), (3, 3, 4)])
def test_matches_derivative_of_brute_force_sums(oracle, L, d, N):
    rng = np.random.default_rng(300 + L + d + N)
    x = rand_path(rng, L, d)
    D = oracle.sig_size(d, N)
    g = rng.normal(size=(1, D))
    glevels = [g[0, s] for s in oracle.level_slices(d, N)]
    got = oracle.signature_backward(x[None], N, g)[0]
    np.testing.assert_allclose(got, brute_force_gradient(x, N, glevels), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- 3. closed forms
def test_depth_one_gradient(oracle):
    rng = np.random.default_rng(5)
    x = rand_path(rng, 6, 3)[None]
    g = rng.normal(size=(1, 3))
    got = oracle.signature_backward(x, 1, g)
    want = np.zeros_like(x)
    want[0, -1] = g[0]
    want[0, 0] = -g[0]
    np.testing.assert_allclose(got, want, atol=1e-14)
    gs = rng.normal(size=(1, 5, 3))  # stream: row k is X_{k+1} - X_0
    got = oracle.signature_backward(x, 1, gs, stream=True)
    want = np.zeros_like(x)
    want[0, 1:] = gs[0]
    want[0, 0] = -gs[0].sum(axis=0)
    np.testing.assert_allclose(got, want, atol=1e-14)


@pytest.mark.parametrize("d,N", [(2, 4), (3, 3), (1, 5)])
def test_single_segment_gradient(oracle, d, N):
    """One segment: level n is v^{(x)n}/n! (Eq. 2), whose derivative is written out with explicit indices."""
    rng = np.random.default_rng(7 + d + N)
    x = rand_path(rng, 2, d)
    v = x[1] - x[0]
    D = oracle.sig_size(d, N)
    g = rng.normal(size=(1, D))
    gv = np.zeros(d)
    for n, sl in enumerate(oracle.level_slices(d, N), start=1):
        G = g[0, sl].reshape((d,) * n)
        for word in itertools.product(range(d), repeat=n):
            for r in range(n):
                gv[word[r]] += G[word] * np.prod([v[word[s]] for s in range(n) if s != r]) / math.factorial(n)
    got = oracle.signature_backward(x[None], N, g)[0]
    np.testing.assert_allclose(got[1], gv, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got[0], -gv, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- 4. invariances
def test_translation_invariance_and_linearity(oracle):
    rng = np.random.default_rng(11)
    x = np.stack([rand_path(rng, 7, 3) for _ in range(2)])
    D = oracle.sig_size(3, 3)
    for stream in (False, True):
        shape = (2, 6, D) if stream else (2, D)
        g1, g2 = rng.normal(size=shape), rng.normal(size=shape)
        a = oracle.signature_backward(x, 3, g1, stream)
        b = oracle.signature_backward(x, 3, g2, stream)
        c = oracle.signature_backward(x, 3, 2.0 * g1 - 3.0 * g2, stream)
        np.testing.assert_allclose(c, 2.0 * a - 3.0 * b, rtol=1e-11, atol=1e-12)
        # the signature does not change when the whole path is shifted: gradients over the points sum to zero
        np.testing.assert_allclose(a.sum(axis=1), 0.0, atol=1e-12)
        shifted = oracle.signature_backward(x + 5.0, 3, g1, stream)
        np.testing.assert_allclose(shifted, a, rtol=1e-9, atol=1e-10)


def test_homogeneity_under_scaling(oracle):
    """Level n is homogeneous of degree n in the path, so its gradient is homogeneous of degree n - 1."""
    rng = np.random.default_rng(13)
    d, N, lam = 2, 4, 1.7
    x = rand_path(rng, 6, d)[None]
    D = oracle.sig_size(d, N)
    for n, sl in enumerate(oracle.level_slices(d, N), start=1):
        g = np.zeros((1, D))
        g[0, sl] = rng.normal(size=d ** n)
        a = oracle.signature_backward(x, N, g)
        b = oracle.signature_backward(lam * x, N, g)
        np.testing.assert_allclose(b, lam ** (n - 1) * a, rtol=1e-10, atol=1e-12)


def test_stream_gradient_is_sum_of_prefix_gradients(oracle):
    rng = np.random.default_rng(17)
    d, N, L = 3, 3, 6
    x = rand_path(rng, L, d)[None]
    D = oracle.sig_size(d, N)
    gs = rng.normal(size=(1, L - 1, D))
    want = np.zeros_like(x)
    for k in range(L - 1):
        want[:, :k + 2] += oracle.signature_backward(x[:, :k + 2], N, gs[:, k])
    got = oracle.signature_backward(x, N, gs, stream=True)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)


def test_batch_entries_are_independent(oracle):
    rng = np.random.default_rng(19)
    x = np.stack([rand_path(rng, 5, 2) for _ in range(3)])
    D = oracle.sig_size(2, 3)
    g = rng.normal(size=(3, D))
    whole = oracle.signature_backward(x, 3, g)
    for b in range(3):
        np.testing.assert_allclose(whole[b], oracle.signature_backward(x[b:b + 1], 3, g[b:b + 1])[0], atol=0)


def test_repeated_point_gets_a_gradient_and_bad_shapes_raise(oracle):
    rng = np.random.default_rng(23)
    x = rand_path(rng, 5, 2)[None]
    x[0, 2] = x[0, 1]
    D = oracle.sig_size(2, 3)
    g = rng.normal(size=(1, D))
    np.testing.assert_allclose(oracle.signature_backward(x, 3, g), finite_difference(oracle, x, 3, g, False),
                               rtol=2e-7, atol=2e-8)
    with pytest.raises(ValueError):
        oracle.signature_backward(x, 3, g[:, :-1])
    with pytest.raises(ValueError):
        oracle.signature_backward(x[:, :1], 3, g)
