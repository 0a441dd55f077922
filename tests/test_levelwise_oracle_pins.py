"""Pins of the level-by-level oracle (oracle/sig_levelwise.py, Section 3.2, Eqs. 6-10 in the corrected reading).

The expected side of every check is a closed form, a hand-worked value, an explicit-index brute force or the
separately written fold of Section 3.1 (oracle/sig_oracle.c, pinned on its own in test_oracle_pins.py): never the
level-by-level routine itself.  A dropped term of the inner sum, a wrong factorial, an inclusive instead of an
exclusive prefix, or swapped tensor factors each break at least one of them.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2501_08455_amd import workloads
from test_oracle_pins import brute_force_signature, levels, rand_path

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def levelwise(oracle):
    return oracle.signature_levelwise


@pytest.mark.parametrize("d,N", [(1, 6), (2, 5), (3, 4)])
def test_single_segment_is_tensor_exponential(levelwise, d, N):
    rng = np.random.default_rng(21)
    x0, delta = rng.normal(size=d), rng.normal(size=d)
    sig = levelwise(np.stack([x0, x0 + delta])[None], N)[0]
    power = np.ones(())
    for n, lev in enumerate(levels(sig, d, N), start=1):
        power = np.multiply.outer(power, delta)
        np.testing.assert_allclose(lev, power / math.factorial(n), rtol=1e-12, atol=1e-15)


def test_hand_worked_two_segment_example(levelwise):
    want = {}
    with open(os.path.join(HERE, "golden", "two_segment_2d.txt")) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                word, frac = line.split()
                want[tuple(int(ch) for ch in word)] = float(Fraction(frac))
    x = np.array([[0.0, 0.0], [1.0, 0.0], [1.0, 1.0]])
    got = levels(levelwise(x[None], 3)[0], 2, 3)
    for word, value in want.items():
        assert got[len(word) - 1][word] == pytest.approx(value, abs=1e-15), word


@pytest.mark.parametrize("L,d,N", [(3, 2, 4), (4, 2, 4), (6, 3, 3), (5, 3, 4)])
def test_brute_force_iterated_sums(levelwise, L, d, N):
    rng = np.random.default_rng(300 + L + d + N)
    x = rand_path(rng, L, d)
    got = levels(levelwise(x[None], N)[0], d, N)
    for g, w in zip(got, brute_force_signature(x, N)):
        np.testing.assert_allclose(g, w, rtol=1e-11, atol=1e-13)


def test_collinear_path_is_one_exponential(levelwise):
    rng = np.random.default_rng(23)
    d, N = 3, 5
    v = rng.normal(size=d)
    c = rng.normal(size=7)
    x = np.concatenate([np.zeros((1, d)), np.cumsum(c[:, None] * v[None, :], axis=0)])
    sig = levels(levelwise(x[None], N)[0], d, N)
    power, total = np.ones(()), c.sum() * v
    for n, lev in enumerate(sig, start=1):
        power = np.multiply.outer(power, total)
        np.testing.assert_allclose(lev, power / math.factorial(n), rtol=1e-10, atol=1e-13)


def test_one_channel(levelwise):
    rng = np.random.default_rng(24)
    x = rand_path(rng, 12, 1)
    t = x[-1, 0] - x[0, 0]
    np.testing.assert_allclose(levelwise(x[None], 6)[0], [t ** n / math.factorial(n) for n in range(1, 7)],
                               rtol=1e-11, atol=1e-14)


def test_stream_rows_are_prefix_signatures(levelwise):
    rng = np.random.default_rng(25)
    d, N, L = 3, 3, 8
    x = np.stack([rand_path(rng, L, d) for _ in range(3)])
    st = levelwise(x, N, stream=True)
    assert st.shape == (3, L - 1, 3 + 9 + 27)
    for k in range(L - 1):
        np.testing.assert_allclose(st[:, k], levelwise(x[:, :k + 2], N), rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(st[:, -1], levelwise(x, N))


@pytest.mark.parametrize("shape,N", [((4, 16, 2), 3), ((3, 40, 5), 4), ((2, 33, 4), 4), ((2, 9, 3), 6), ((5, 7, 7), 2)])
@pytest.mark.parametrize("stream", [False, True])
def test_agrees_with_the_fold(oracle, levelwise, shape, N, stream):
    rng = np.random.default_rng(26 + N)
    x = np.cumsum(rng.normal(0, 0.3, size=shape), axis=1)
    want = oracle.signature(x, N, stream=stream)
    got = levelwise(x, N, stream=stream)
    assert got.shape == want.shape
    for sl in oracle.level_slices(shape[2], N):
        den = np.linalg.norm(want[..., sl])
        assert np.linalg.norm(got[..., sl] - want[..., sl]) <= 1e-13 * den


def test_agrees_with_the_fold_on_the_small_config(oracle, levelwise):
    x = workloads.make_paths("C1")
    np.testing.assert_allclose(levelwise(x, 3), oracle.signature(x, 3), rtol=1e-12, atol=1e-15)


def test_bad_shapes(levelwise):
    with pytest.raises(ValueError):
        levelwise(np.zeros((1, 1, 2)), 2)
    with pytest.raises(ValueError):
        levelwise(np.zeros((1, 3, 2)), 0)
