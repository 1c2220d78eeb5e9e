"""Gradient-coding matrices for one sibling group.  TEST INFRASTRUCTURE ONLY.

Section II-C: n workers share k = n data partitions; the encoding matrix B
(n x n) has one row per worker whose non-zeros mark the s+1 partitions that
worker holds, and for every set of s stragglers there is a decoding row a_f,
supported on the n-s survivors, with a_f B = (1,...,1).  The decoding matrix A
stacks the F = C(n,s) rows.

The paper cites the gradient-coding construction without restating it, so this
module states one as mathematics:

* support of row i is the cyclic window {i, i+1, ..., i+s} mod n (the printed
  matrix of the (3,2) example has this support);
* pick H (s x n) with generic entries whose rows sum to zero; every row b_i of
  B is the vector on that support with H b_i^T = 0, found from an s x s solve.
  All rows then live in null(H), which has dimension n-s and contains the
  all-ones vector, so any n-s rows generically span it;
* rows are scaled to unit 2-norm (row scaling does not change what can be
  decoded);
* a decoding row solves the consistent system  x B_I = 1  on the survivor set I.

The paper is silent on conditioning.  `search_encoding_matrix` draws K
candidates for H from a counter-based generator (splitmix64; entry (r, j) of
candidate c uses counter (c*s + r)*(n-1) + j) and keeps the candidate with the
smallest amplification  gamma = max_f sum_i |a_fi| ||b_i||_2 / sqrt(n).
`design_code` adds the fall-back used when even the best cyclic candidate is
too badly conditioned for fp32 messages: the fractional-repetition design
(another published gradient code; needs s+1 | n), whose decode rows are 0/1.

Exact-rational variants (fractions.Fraction) serve the brute-force tests.
"""
from __future__ import annotations

import itertools
import math
from fractions import Fraction

import numpy as np

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
DEFAULT_CANDIDATES = 2048


# --------------------------------------------------------------------------
# counter-based uniform numbers (the published splitmix64 output function)
# --------------------------------------------------------------------------
def splitmix64_at(seed: int, counter: int) -> int:
    """Output number `counter` (0-based) of the splitmix64 stream started at `seed`."""
    z = (seed + (counter + 1) * _GOLDEN) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def uniform_pm1(seed: int, counter: int) -> float:
    """Uniform double in [-1, 1) from the top 53 bits of the stream output."""
    return (splitmix64_at(seed, counter) >> 11) * (2.0 ** -53) * 2.0 - 1.0


def candidate_H(n: int, s: int, seed: int, c: int) -> np.ndarray:
    """Candidate number c of the s x n matrix H; each row sums to zero."""
    H = np.zeros((s, n))
    for r in range(s):
        for j in range(n - 1):
            H[r, j] = uniform_pm1(seed, (c * s + r) * (n - 1) + j)
        H[r, n - 1] = -math.fsum(H[r, : n - 1])
    return H


# --------------------------------------------------------------------------
# floating-point construction
# --------------------------------------------------------------------------
def cyclic_support(n: int, s: int, i: int) -> list[int]:
    return [(i + t) % n for t in range(s + 1)]


def encoding_from_H(H: np.ndarray) -> np.ndarray:
    """Rows b_i on the cyclic support with H b_i^T = 0, unit 2-norm, b_i(i) > 0."""
    s, n = H.shape
    B = np.zeros((n, n))
    for i in range(n):
        supp = cyclic_support(n, s, i)
        others = supp[1:]
        B[i, i] = 1.0
        if s > 0:
            B[i, others] = np.linalg.solve(H[:, others], -H[:, i])
        B[i] /= np.linalg.norm(B[i])
    return B


def straggler_sets(n: int, s: int) -> list[tuple[int, ...]]:
    """All straggler sets of size exactly s, in lexicographic order (row order of A)."""
    return list(itertools.combinations(range(n), s))


def decoding_row(B: np.ndarray, stragglers) -> np.ndarray:
    """Row a with zeros on `stragglers` and a B = 1 (least-squares solve of the consistent system)."""
    n = B.shape[0]
    I = [i for i in range(n) if i not in set(stragglers)]
    x, *_ = np.linalg.lstsq(B[I].T, np.ones(B.shape[1]), rcond=None)
    a = np.zeros(n)
    a[I] = x
    return a


def decoding_matrix(B: np.ndarray, s: int) -> np.ndarray:
    n = B.shape[0]
    return np.array([decoding_row(B, T) for T in straggler_sets(n, s)])


def amplification(B: np.ndarray, A: np.ndarray) -> float:
    """gamma = max_f sum_i |a_fi| ||b_i||_2 / sqrt(n)."""
    n = B.shape[0]
    norms = np.linalg.norm(B, axis=1)
    return float(np.max(np.abs(A) @ norms) / math.sqrt(n))


def candidate_count(n: int, s: int) -> int:
    """K = min(2048, max(16, 2^20 // C(n,s))): fewer candidates when every one needs many decode rows."""
    return min(DEFAULT_CANDIDATES, max(16, (1 << 20) // math.comb(n, s)))


def fractional_repetition_matrix(n: int, s: int) -> np.ndarray:
    """s+1 groups of n/(s+1) workers; worker j of every group holds the j-th window of s+1 partitions (unit-norm rows).
    s stragglers cannot break all s+1 groups, and the members of an intact group sum to the whole."""
    assert n % (s + 1) == 0
    per_group = n // (s + 1)
    B = np.zeros((n, n))
    for g in range(s + 1):
        for j in range(per_group):
            B[g * per_group + j, j * (s + 1):(j + 1) * (s + 1)] = 1.0 / math.sqrt(s + 1)
    return B


def design_code(n: int, s: int, L: int, seed: int):
    """The code a plan uses by default: best cyclic candidate, unless its rounding amplification over L levels is too
    large for fp32 messages (gamma^L > 256) and s+1 divides n; then the fractional-repetition design if its gamma is
    smaller.  Returns (B, A, gamma, candidate) with candidate = -2 for fractional repetition."""
    B, A, gamma, c = search_encoding_matrix(n, s, seed, candidates=None)
    if s > 0 and n % (s + 1) == 0 and not (gamma ** L <= 256.0):
        FR = fractional_repetition_matrix(n, s)
        A_fr = decoding_matrix(FR, s)
        g_fr = amplification(FR, A_fr)
        if g_fr < gamma:
            return FR, A_fr, g_fr, -2
    return B, A, gamma, c


def search_encoding_matrix(n: int, s: int, seed: int, candidates: int | None = None):
    """Best-of-K cyclic construction (K from candidate_count unless given).  Returns (B, A, gamma, index of the winning candidate)."""
    if candidates is None:
        candidates = candidate_count(n, s)
    if s == 0:
        B = np.eye(n)
        A = np.ones((1, n))
        return B, A, amplification(B, A), 0
    if s == n - 1:
        # every worker holds every partition: null(H) is the line through the all-ones vector, all candidates coincide
        B = np.full((n, n), 1.0 / math.sqrt(n))
        A = decoding_matrix(B, s)
        return B, A, amplification(B, A), 0
    sets = straggler_sets(n, s)
    surv = np.array([[i for i in range(n) if i not in T] for T in sets])  # F x (n-s)
    ones = np.ones(n)
    best = None
    for c in range(candidates):
        H = candidate_H(n, s, seed, c)
        try:
            B = encoding_from_H(H)
        except np.linalg.LinAlgError:
            continue
        # all F survivor systems at once: x = pinv(B_I^T) 1
        BT = np.transpose(B[surv], (0, 2, 1))            # F x n x (n-s)
        X = np.linalg.pinv(BT) @ ones                    # F x (n-s)
        A = np.zeros((len(sets), n))
        np.put_along_axis(A, surv, X, axis=1)
        if not np.all(np.isfinite(A)) or np.max(np.abs(A @ B - 1.0)) > 1e-10:
            continue
        g = amplification(B, A)
        if best is None or g < best[2]:
            best = (B, A, g, c)
    if best is None:
        raise RuntimeError("no usable candidate")
    return best


# --------------------------------------------------------------------------
# exact-rational construction (tiny cases)
# --------------------------------------------------------------------------
def solve_exact(M, rhs):
    """Solve M x = rhs over the rationals (M: r x c list of lists, r >= c, consistent, full column rank)."""
    r, c = len(M), len(M[0])
    aug = [[Fraction(v) for v in row] + [Fraction(b)] for row, b in zip(M, rhs)]
    piv_row = 0
    for col in range(c):
        p = next((k for k in range(piv_row, r) if aug[k][col] != 0), None)
        if p is None:
            raise ValueError("rank deficient")
        aug[piv_row], aug[p] = aug[p], aug[piv_row]
        pv = aug[piv_row][col]
        aug[piv_row] = [v / pv for v in aug[piv_row]]
        for k in range(r):
            if k != piv_row and aug[k][col] != 0:
                f = aug[k][col]
                aug[k] = [vk - f * vp for vk, vp in zip(aug[k], aug[piv_row])]
        piv_row += 1
    for k in range(c, r):
        if aug[k][c] != 0:
            raise ValueError("inconsistent system")
    return [aug[k][c] for k in range(c)]


def encoding_from_H_exact(H):
    """Exact B (leading entry 1, no normalisation) from an integer/rational H whose rows sum to zero."""
    s, n = len(H), len(H[0])
    B = [[Fraction(0)] * n for _ in range(n)]
    for i in range(n):
        supp = cyclic_support(n, s, i)
        others = supp[1:]
        B[i][i] = Fraction(1)
        if s > 0:
            M = [[Fraction(H[r][j]) for j in others] for r in range(s)]
            x = solve_exact(M, [-Fraction(H[r][i]) for r in range(s)])
            for j, v in zip(others, x):
                B[i][j] = v
    return B


def decoding_row_exact(B, stragglers):
    n, k = len(B), len(B[0])
    I = [i for i in range(n) if i not in set(stragglers)]
    M = [[Fraction(B[i][col]) for i in I] for col in range(k)]     # B_I^T, k x (n-s)
    x = solve_exact(M, [Fraction(1)] * k)
    a = [Fraction(0)] * n
    for i, v in zip(I, x):
        a[i] = v
    return a
