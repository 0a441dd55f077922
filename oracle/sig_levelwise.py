"""fp64 CPU oracle of the paper's level-by-level formulation (test infrastructure only).

TEST INFRASTRUCTURE ONLY: nothing in the product imports this module.

What it computes.  Section 3.2 of the paper ("GPU-Optimized Approach") reorganises the recursion of
Section 3.1 so that time is handled by one cumulative sum per level (Eqs. 6-10): level n of every prefix
signature is the running sum over time of a per-step term built from the lower levels and from powers of
the step's increment divided by factorials (Eq. 7).  This module takes those steps in the paper's order,
with whole-tensor numpy operations of shape (batch, time, d^n) exactly as the section describes them
(batched outer products that keep the batch and time axes, Eq. 9; `cumsum` along time; concatenation of
the levels, Eq. 10).  No fold over time, no product of two signatures: a different algorithm from
sig_oracle.c, which is what makes the agreement of the two a check of both.

Reading of Eq. 8 taken here (the printed form cannot be used as it stands): the printed terms put the
increment on the left of the running level, use the running level of the same step inside the sum that
defines it, and divide the increment itself by n! instead of its n-th tensor power.  The form that agrees
with Eq. 3 summed over time, and with Eq. 1 (earlier time is the left factor), is

    S_{n,i} = sum_{j <= i}  sum_{m=0}^{n-1}  S_{m,j-1} (x) dX_j^{(x)(n-m)} / (n-m)!,      S_{0,.} = 1,

with S_{m,j-1} the level-m signature of the path BEFORE step j (zero for m >= 1 when j is the first
step).  Eq. 7 is read as P_r = dX^{(x)r} / r!, built by one more factor on the right and a division by r.

Pins (tests/test_levelwise_oracle_pins.py): the closed form of a single segment, the hand-worked
two-segment example, brute-force iterated sums with explicit indices, collinear paths, stream rows
against truncated paths, and agreement with the fold of sig_oracle.c to rounding.
"""
import numpy as np


def _outer(a, b):
    """Eq. 9: (a (x) b)[b, k] = a[b, k] (x) b[b, k]; a on the left is the slow index."""
    B, K = a.shape[:2]
    return (a[:, :, :, None] * b[:, :, None, :]).reshape(B, K, a.shape[2] * b.shape[2])


def signature_levelwise(path, depth, stream=False):
    """Depth-`depth` signatures of `path` ([B, L, d]) by the level-by-level cumulative sums of Eqs. 6-10.

    Returns float64 [B, D] (final) or [B, L-1, D] (stream), the same rows as oracle.signature.
    """
    x = np.ascontiguousarray(path, dtype=np.float64)
    if x.ndim != 3 or x.shape[1] < 2 or depth < 1:
        raise ValueError("path must be [B, L >= 2, d] and depth >= 1")
    B, L, d = x.shape
    K = L - 1
    dX = x[:, 1:, :] - x[:, :-1, :]                      # [B, K, d]
    # Eq. 7: P[r] = dX^{(x) r} / r!
    P = [np.ones((B, K, 1)), dX]
    for r in range(2, depth + 1):
        P.append(_outer(P[r - 1], dX) / r)
    # level 0 of every prefix is 1
    S = [np.ones((B, K, 1))]
    for n in range(1, depth + 1):
        term = np.zeros((B, K, d ** n))
        for m in range(n):
            before = np.zeros_like(S[m])                 # S_{m, j-1}: shifted one step along time
            before[:, 1:, :] = S[m][:, :-1, :]
            if m == 0:
                before[:, 0, :] = 1.0
            term += _outer(before, P[n - m])
        S.append(np.cumsum(term, axis=1))                # Eq. 8: the only dependence along time
    rows = np.concatenate(S[1:], axis=2)                 # Eq. 10
    return rows if stream else np.ascontiguousarray(rows[:, -1, :])
