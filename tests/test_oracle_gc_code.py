"""Pins for the oracle's gradient-coding matrices (Section II-C): printed values, exact identities, structure."""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import gc_code

PAIRS = [(3, 1), (4, 1), (4, 2), (5, 2), (6, 2), (8, 2), (7, 3)]


def _example(golden_dir):
    with open(os.path.join(golden_dir, "cr_example_3_2_1.json")) as f:
        return json.load(f)


def test_printed_B_gives_printed_A_exactly(golden_dir):
    ex = _example(golden_dir)
    B = [[Fraction(v).limit_denominator(4) for v in row] for row in ex["B"]]
    for f, T in enumerate(gc_code.straggler_sets(3, 1)):
        assert gc_code.decoding_row_exact(B, T) == [Fraction(v) for v in ex["A"][f]]
    A = gc_code.decoding_matrix(np.array(ex["B"], dtype=float), 1)
    np.testing.assert_allclose(A, np.array(ex["A"], dtype=float), atol=1e-14)
    # dyadic entries: the identity holds exactly in floating point with the printed matrices
    assert np.array_equal(np.array(ex["A"], dtype=float) @ np.array(ex["B"], dtype=float), np.ones((3, 3)))


def test_gc_example_identity(golden_dir):
    with open(os.path.join(golden_dir, "gc_example_3_1.json")) as f:
        ex = json.load(f)
    rng = np.random.default_rng(0)
    g = rng.standard_normal((3, 5))
    msgs = np.array(ex["worker_messages"]) @ g
    np.testing.assert_allclose(np.array(ex["decode"]) @ msgs, g.sum(0), atol=1e-14)
    # the same two messages are rows 1,2 of the printed B of the (3,2) example and the decode is its row for straggler 3
    B = np.array([[0.5, 1, 0], [0, 1, -1], [0.5, 0, 1]])
    np.testing.assert_allclose(gc_code.decoding_row(B, (2,)), [2, -1, 0], atol=1e-14)


def test_splitmix64_reference_values():
    # first outputs of the published splitmix64 generator for seed 0 and seed 1234567
    assert gc_code.splitmix64_at(0, 0) == 0xE220A8397B1DCDAF
    assert gc_code.splitmix64_at(0, 1) == 0x6E789E6AA1B965F4
    assert gc_code.splitmix64_at(1234567, 0) == 6457827717110365317
    assert gc_code.splitmix64_at(1234567, 1) == 3203168211198807973
    u = [gc_code.uniform_pm1(7, c) for c in range(1000)]
    assert -1.0 <= min(u) and max(u) < 1.0 and abs(np.mean(u)) < 0.1


@pytest.mark.parametrize("n,s", PAIRS)
def test_structure_and_identity(n, s):
    B, A, gamma, _ = gc_code.search_encoding_matrix(n, s, seed=2024, candidates=64)
    sets = gc_code.straggler_sets(n, s)
    assert A.shape == (len(sets), n) and len(sets) == len(list(itertools.combinations(range(n), s)))
    for i in range(n):                                   # cyclic support, s+1 non-zeros per row
        supp = set(gc_code.cyclic_support(n, s, i))
        assert {j for j in range(n) if B[i, j] != 0} == supp
        assert abs(np.linalg.norm(B[i]) - 1) < 1e-12 and B[i, i] > 0
    assert all(np.count_nonzero(B[:, k]) == s + 1 for k in range(n))   # each partition sits in s+1 workers
    for f, T in enumerate(sets):
        assert all(A[f, j] == 0 for j in T)              # stragglers are not used
    assert np.max(np.abs(A @ B - 1)) <= 1e-10            # a_f B = 1 for every straggler set
    assert gamma == pytest.approx(gc_code.amplification(B, A))
    # the rows of B lie in an (n-s)-dimensional space that contains the all-ones vector
    assert np.linalg.matrix_rank(B, tol=1e-9) == n - s


@pytest.mark.parametrize("n,s", [(3, 1), (4, 1), (5, 2), (6, 2), (6, 3)])
def test_exact_rational_identity(n, s):
    # small-integer H with zero row sums; generic enough for every s x s minor used to be non-singular
    rng = np.random.default_rng(100 * n + s)
    for _ in range(50):
        H = [[int(v) for v in rng.integers(-7, 8, size=n - 1)] for _ in range(s)]
        H = [row + [-sum(row)] for row in H]
        try:
            B = gc_code.encoding_from_H_exact(H)
            rows = [gc_code.decoding_row_exact(B, T) for T in gc_code.straggler_sets(n, s)]
        except ValueError:
            continue
        for T, a in zip(gc_code.straggler_sets(n, s), rows):
            assert all(a[j] == 0 for j in T)
            for k in range(n):
                assert sum(a[i] * B[i][k] for i in range(n)) == 1
        # the floating-point routines agree with the exact ones (up to the row scaling of B)
        Bf = gc_code.encoding_from_H(np.array(H, dtype=float))
        Be = np.array([[float(v) for v in row] for row in B])
        np.testing.assert_allclose(Bf, Be / np.linalg.norm(Be, axis=1, keepdims=True), atol=1e-10)
        return
    pytest.fail("no non-singular integer H found")


@pytest.mark.parametrize("n,s", [(4, 1), (6, 2), (12, 3), (12, 5), (10, 4)])
def test_fractional_repetition_decodes_every_straggler_set(n, s):
    B = gc_code.fractional_repetition_matrix(n, s)
    assert np.all(np.count_nonzero(B, axis=0) == s + 1) and np.all(np.count_nonzero(B, axis=1) == s + 1)
    A = gc_code.decoding_matrix(B, s)
    assert np.max(np.abs(A @ B - 1)) <= 1e-12
    for f, T in enumerate(gc_code.straggler_sets(n, s)):
        assert all(A[f, j] == 0 for j in T)
    # pigeonhole: some group of n/(s+1) replicas is intact, so a 0/1 row (times the row norm) always exists
    per_group = n // (s + 1)
    for T in gc_code.straggler_sets(n, s):
        intact = [g for g in range(s + 1) if not any(g * per_group <= j < (g + 1) * per_group for j in T)]
        assert intact
        a = np.zeros(n)
        a[intact[0] * per_group:(intact[0] + 1) * per_group] = np.sqrt(s + 1)
        np.testing.assert_allclose(a @ B, 1.0, atol=1e-12)
    assert gc_code.amplification(B, A) <= 2.0 + 1e-9     # all-positive 0/1-like rows: no cancellation to amplify


def test_candidate_count_rule():
    assert gc_code.candidate_count(3, 1) == 2048 and gc_code.candidate_count(12, 3) == 2048
    assert gc_code.candidate_count(12, 5) == (1 << 20) // 792 and gc_code.candidate_count(20, 5) == 67
    assert gc_code.candidate_count(24, 12) == 16


def test_zero_stragglers_is_identity():
    B, A, gamma, _ = gc_code.search_encoding_matrix(5, 0, seed=1)
    assert np.array_equal(B, np.eye(5)) and np.array_equal(A, np.ones((1, 5)))
    assert gamma == pytest.approx(np.sqrt(5))


def test_search_picks_the_minimum_and_is_deterministic():
    n, s, seed = 6, 2, 99
    B, A, gamma, c = gc_code.search_encoding_matrix(n, s, seed, candidates=40)
    B2, A2, gamma2, c2 = gc_code.search_encoding_matrix(n, s, seed, candidates=40)
    assert c == c2 and np.array_equal(B, B2) and gamma == gamma2
    for cand in range(40):
        Bc = gc_code.encoding_from_H(gc_code.candidate_H(n, s, seed, cand))
        Ac = gc_code.decoding_matrix(Bc, s)
        assert gc_code.amplification(Bc, Ac) >= gamma - 1e-9
    Bw = gc_code.encoding_from_H(gc_code.candidate_H(n, s, seed, c))
    np.testing.assert_allclose(Bw, B, atol=1e-13)
    # rows of every candidate H sum to zero
    assert np.max(np.abs(gc_code.candidate_H(n, s, seed, 3).sum(axis=1))) < 1e-15


def test_amplification_budget_for_benchmark_trees():
    # fp32 message rounding (2^-24) amplified by gamma per level must stay well inside the 1e-4 parity bar
    for (n, s, L) in [(3, 1, 2), (4, 1, 2), (4, 1, 3), (8, 2, 2), (6, 2, 3)]:
        _, _, gamma, _ = gc_code.search_encoding_matrix(n, s, seed=190201981)
        assert gamma ** L * 6e-8 < 2e-5, (n, s, L, gamma)
