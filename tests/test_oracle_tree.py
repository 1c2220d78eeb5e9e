"""Pins for the oracle's tree, allocation and execution (Section III, Algorithms 1-2, Theorem 1)."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from cr_inputs import workloads as wl
from oracle import cr_tree, gc_code

B_PRINTED = np.array([[0.5, 1, 0], [0, 1, -1], [0.5, 0, 1]])


def _data(m, d, seed=0, model=cr_tree.LINEAR):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((m, d)).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    if model == cr_tree.LINEAR:
        y = (X @ rng.standard_normal(d) + 0.01 * rng.standard_normal(m)).astype(np.float32)
    else:
        y = (rng.random(m) < 0.5).astype(np.float32)
    return X, y, w


# ------------------------------------------------------------------ tree and load
def test_tree_counts_and_numbering():
    for n, L in [(3, 2), (4, 2), (4, 3), (8, 2), (6, 3), (12, 2)]:
        N = cr_tree.num_workers(n, L)
        assert N == sum(n ** l for l in range(1, L + 1))
        groups = cr_tree.sibling_groups(n, L)
        assert len(groups) == N // n
        for g, grp in enumerate(groups):                 # level-order numbering: group g is a block of n ids
            assert grp == list(range(g * n, (g + 1) * n))
        assert wl.num_workers(n, L) == N
    assert [cr_tree.num_workers(*a) for a in [(3, 2), (4, 2), (4, 3), (8, 2), (6, 3), (12, 2)]] == [12, 20, 84, 72, 258, 156]
    assert cr_tree.children(3, 2, 0) == [3, 4, 5] and cr_tree.children(3, 2, 2) == [9, 10, 11] and cr_tree.children(3, 2, 5) == []


def test_computation_load_closed_form(golden_dir):
    with open(os.path.join(golden_dir, "computation_load.json")) as f:
        gold = json.load(f)
    for case in gold["cases"]:
        assert cr_tree.computation_load(case["n"], case["L"], case["s"]) == Fraction(*case["r"])
    # remark after Theorem 1: half the children may straggle; one layer versus three layers
    n = 1000
    r1 = cr_tree.computation_load(n, 1, n // 2)
    r3 = cr_tree.computation_load(n, 3, n // 2)
    assert float(r1 / r3) == pytest.approx(gold["remark_alpha_half"]["ratio_L1_over_L3"], rel=0.02)


@pytest.mark.parametrize("L,n,s,m", [(2, 3, 1, 1200), (2, 4, 1, 100_000), (3, 4, 1, 252_000), (2, 8, 2, 88), (3, 6, 2, 2_064_000),
                                     (1, 5, 2, 1000), (3, 3, 1, 977), (2, 4, 0, 4000)])
def test_allocation_sizes(L, n, s, m):
    B = gc_code.search_encoding_matrix(n, s, 7, candidates=8)[0]
    own, subtree = cr_tree.cr_allocate(L, n, s, m, B)
    r = cr_tree.computation_load(n, L, s)
    rows = [cr_tree.set_size(o) for o in own]
    assert max(rows) - min(rows) <= (0 if (r * m).denominator == 1 else 2)
    assert all(abs(k - float(r * m)) < 2.0 for k in rows)             # every worker holds r_CR m points (Theorem 1), up to integer cuts
    for i in range(n):                                               # |D^T(1,i)| = (s+1) m / n  (proof of Theorem 1)
        assert abs(cr_tree.set_size(subtree[i]) - (s + 1) * m / n) <= s + 1
    cover = np.zeros(m, dtype=int)                                   # each point lies in exactly s+1 level-1 sub-trees
    for i in range(n):
        for b, e, _ in subtree[i]:
            cover[b:e] += 1
    assert np.all(cover == s + 1)
    for node in range(len(own)):                                     # keep + rest = sub-tree set, in order
        kids = cr_tree.children(n, L, node)
        W = subtree[node]
        k = cr_tree.set_size(own[node])
        assert own[node] == cr_tree.take(W, 0, k)
        if kids:
            rest = cr_tree.take(W, k, cr_tree.set_size(W))
            assert [subtree[c] for c in kids] == cr_tree.comp_alloc(rest, B)
        else:
            assert k == cr_tree.set_size(W)


def test_sizes_of_benchmark_trees():
    expect = {(2, 3, 1, 1200): (27, 3840), (2, 4, 1, 100_000): (36, 333_332), (3, 4, 1, 252_000): (148, 1_512_000),
              (2, 8, 2, 88): (248, 648), (3, 6, 2, 2_064_000): (780, 38_036_556)}
    for (L, n, s, m), (S, visits) in expect.items():
        B = gc_code.search_encoding_matrix(n, s, 7, candidates=4)[0]
        own, _ = cr_tree.cr_allocate(L, n, s, m, B)
        assert len(cr_tree.slabs_of(own)) == S
        assert sum(cr_tree.set_size(o) for o in own) == visits


def test_printed_allocation_of_the_example(golden_dir):
    with open(os.path.join(golden_dir, "cr_example_3_2_1.json")) as f:
        ex = json.load(f)
    own, subtree = cr_tree.cr_allocate(2, 3, 1, ex["m_for_row_units"], B_PRINTED)
    assert subtree[0] == [(0, 5, 0.5), (5, 10, 1.0)]                  # D^T(1,1) = 1/2 D_1 u D_2
    for node, segs in ex["own_rows_m15"].items():
        if node == "comment":
            continue
        assert [list(t) for t in own[int(node)]] == segs
    assert cr_tree.computation_load(3, 2, 1) * 15 == 4


def test_comp_alloc_is_algorithm_1():
    W = [(0, 12, 1.0)]
    alloc = cr_tree.comp_alloc(W, B_PRINTED)
    assert alloc[0] == [(0, 4, 0.5), (4, 8, 1.0)]
    assert alloc[1] == [(4, 8, 1.0), (8, 12, -1.0)]
    assert alloc[2] == [(0, 4, 0.5), (8, 12, 1.0)]
    # a part may straddle two coefficients
    W = [(0, 3, 2.0), (10, 13, 4.0)]
    alloc = cr_tree.comp_alloc(W, B_PRINTED)
    assert alloc[1] == [(2, 3, 2.0), (10, 11, 4.0), (11, 13, -4.0)]


# ------------------------------------------------------------------ gradients
def test_partial_gradient_closed_forms():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((200, 7)).astype(np.float32)
    ws = rng.standard_normal(7).astype(np.float32)
    y = (X.astype(np.float64) @ ws.astype(np.float64))
    # least squares: zero residual at the true model
    g = cr_tree.partial_gradient(X, y, ws, 0, 200, cr_tree.LINEAR)
    assert np.max(np.abs(g)) < 1e-10
    # segments add up to the whole; transposed-operand mistakes would break the shape or this sum
    w = rng.standard_normal(7).astype(np.float32)
    parts = sum(cr_tree.partial_gradient(X, y, w, b, b + 50, cr_tree.LINEAR) for b in range(0, 200, 50))
    np.testing.assert_allclose(parts, cr_tree.full_gradient(X, y, w, cr_tree.LINEAR, block=64), rtol=1e-12)
    # per-point definition: sum_j x_j (x_j.w - y_j)
    brute = np.zeros(7)
    for j in range(200):
        xj = X[j].astype(np.float64)
        brute += xj * (xj @ w.astype(np.float64) - y[j])
    np.testing.assert_allclose(parts, brute, rtol=1e-12)


def test_logistic_gradient_is_derivative_of_the_loss():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((60, 5)).astype(np.float32)
    t = (rng.random(60) < 0.4).astype(np.float32)
    w = (0.5 * rng.standard_normal(5)).astype(np.float32)

    def loss(wv):                                        # sum_j log(1+e^{z_j}) - t_j z_j
        z = X.astype(np.float64) @ wv
        return float(np.sum(np.logaddexp(0.0, z) - t * z))

    g = cr_tree.partial_gradient(X, t, w, 0, 60, cr_tree.LOGISTIC)
    w64 = w.astype(np.float64)
    for k in range(5):
        e = np.zeros(5)
        e[k] = 1e-6
        fd = (loss(w64 + e) - loss(w64 - e)) / 2e-6
        assert g[k] == pytest.approx(fd, rel=1e-6, abs=1e-7)
    z = np.array([-800.0, -30.0, 0.0, 30.0, 800.0])      # stable at both tails
    np.testing.assert_allclose(cr_tree.phi(z, cr_tree.LOGISTIC), [0.0, 9.357622968840175e-14, 0.5, 1 - 9.357622968840175e-14, 1.0], atol=1e-15)


# ------------------------------------------------------------------ execution
def test_example_message_identities():
    X, y, w = _data(15 * 8, 6, seed=11)
    m = X.shape[0]
    own, subtree = cr_tree.cr_allocate(2, 3, 1, m, B_PRINTED)
    grads = [cr_tree.local_coded_gradient(X, y, w, segs) for segs in own]
    gD = [cr_tree.partial_gradient(X, y, w, k * m // 3, (k + 1) * m // 3) for k in range(3)]
    mask = np.zeros(12, dtype=np.uint8)
    mask[5] = 1                      # child (2,3) of node (1,1) straggles -> row [2,-1,0]
    mask[1] = 1                      # child (1,2) of the master straggles -> row [1,0,1]
    msgs, g = cr_tree.cr_execute(2, 3, 1, grads, mask, lambda T: gc_code.decoding_row(B_PRINTED, T))
    np.testing.assert_allclose(msgs[0], 2 * msgs[3] - msgs[4] + grads[0], rtol=1e-12)
    np.testing.assert_allclose(msgs[0], 0.5 * gD[0] + gD[1], rtol=1e-10, atol=1e-9)
    np.testing.assert_allclose(msgs[2], 0.5 * gD[0] + gD[2], rtol=1e-10, atol=1e-9)
    np.testing.assert_allclose(g, msgs[0] + msgs[2], rtol=1e-12)
    np.testing.assert_allclose(g, cr_tree.full_gradient(X, y, w), rtol=1e-10, atol=1e-9)
    assert msgs[1] is None and msgs[5] is None


@pytest.mark.parametrize("L,n,s,model", [(2, 3, 1, cr_tree.LINEAR), (2, 3, 1, cr_tree.LOGISTIC)])
def test_every_mask_decodes_to_the_full_gradient(L, n, s, model):
    X, y, w = _data(240, 9, seed=5, model=model)
    B = gc_code.search_encoding_matrix(n, s, 31, candidates=16)[0]
    own, subtree = cr_tree.cr_allocate(L, n, s, 240, B)
    grads = [cr_tree.local_coded_gradient(X, y, w, segs, model) for segs in own]
    sub_grads = [cr_tree.local_coded_gradient(X, y, w, W, model) for W in subtree]
    gstar = cr_tree.full_gradient(X, y, w, model)
    rows = {T: gc_code.decoding_row(B, T) for T in gc_code.straggler_sets(n, s)}
    count = 0
    for mask in wl.enumerate_masks(L, n, s):
        msgs, g = cr_tree.cr_execute(L, n, s, grads, mask, rows.__getitem__)
        assert np.linalg.norm(g - gstar) <= 1e-12 * np.linalg.norm(gstar)
        for node, mm in enumerate(msgs):                 # a node's message is the coded gradient of its whole sub-tree set
            assert (mm is None) == bool(mask[node])
            if mm is not None:
                assert np.linalg.norm(mm - sub_grads[node]) <= 1e-11 * (1 + np.linalg.norm(sub_grads[node]))
        count += 1
    assert count == 256                                   # 4 groups x (1 + 3) choices


def test_all_masks_two_level_four_children():
    L, n, s = 2, 4, 1
    X, y, w = _data(600, 5, seed=6)
    B = gc_code.search_encoding_matrix(n, s, 8, candidates=16)[0]
    own, _ = cr_tree.cr_allocate(L, n, s, 600, B)
    grads = [cr_tree.local_coded_gradient(X, y, w, segs) for segs in own]
    gstar = cr_tree.full_gradient(X, y, w)
    rows = {T: gc_code.decoding_row(B, T) for T in gc_code.straggler_sets(n, s)}
    count = 0
    for mask in wl.enumerate_masks(L, n, s):
        _, g = cr_tree.cr_execute(L, n, s, grads, mask, rows.__getitem__)
        assert np.linalg.norm(g - gstar) <= 1e-12 * np.linalg.norm(gstar)
        count += 1
    assert count == 5 ** 5


@pytest.mark.parametrize("L,n,s", [(2, 4, 2), (3, 3, 1), (2, 6, 2), (1, 5, 2), (3, 2, 1)])
def test_sampled_masks_deeper_and_wider(L, n, s):
    m = 50 * cr_tree.num_workers(n, L) + 13
    X, y, w = _data(m, 6, seed=L * 100 + n * 10 + s)
    B = gc_code.search_encoding_matrix(n, s, 5, candidates=64)[0]
    own, _ = cr_tree.cr_allocate(L, n, s, m, B)
    grads = [cr_tree.local_coded_gradient(X, y, w, segs) for segs in own]
    gstar = cr_tree.full_gradient(X, y, w)
    rows = {T: gc_code.decoding_row(B, T) for T in gc_code.straggler_sets(n, s)}
    rng = np.random.default_rng(1)
    N = cr_tree.num_workers(n, L)
    for trial in range(200):
        mask = np.zeros(N, dtype=np.uint8)
        for g in range(N // n):
            k = rng.integers(0, s + 1)
            mask[g * n + rng.choice(n, size=k, replace=False)] = 1
        _, g = cr_tree.cr_execute(L, n, s, grads, mask, rows.__getitem__)
        assert np.linalg.norm(g - gstar) <= 1e-10 * np.linalg.norm(gstar)


def test_exact_arithmetic_brute_force():
    """Integer data and rational codes: the decoded gradient equals the plain sum exactly, for every mask."""
    L, n, s, m, d = 2, 3, 1, 45, 4
    rng = np.random.default_rng(9)
    X = rng.integers(-3, 4, size=(m, d)).astype(np.float32)
    y = rng.integers(-5, 6, size=m).astype(np.float32)
    w = rng.integers(-2, 3, size=d).astype(np.float32)
    H = [[3, -5, 2]]
    B = gc_code.encoding_from_H_exact(H)                 # entries 1, 3/5, 5/2, 2/3-like rationals, not dyadic
    own, _ = cr_tree.cr_allocate(L, n, s, m, B, one=Fraction(1))
    gstar = cr_tree.full_gradient(X, y, w)
    assert np.array_equal(gstar, np.round(gstar))        # integer data: fp64 is exact here

    def exact(vec):
        return np.array([Fraction(int(v)) for v in vec], dtype=object)

    grads = []
    for segs in own:
        acc = exact(np.zeros(d))
        for b, e, c in segs:
            acc = acc + c * exact(cr_tree.partial_gradient(X, y, w, b, e))
        grads.append(acc)
    rows = {T: np.array(gc_code.decoding_row_exact(B, T), dtype=object) for T in gc_code.straggler_sets(n, s)}
    for mask in wl.enumerate_masks(L, n, s):
        _, g = cr_tree.cr_execute(L, n, s, grads, mask, rows.__getitem__)
        assert list(g) == list(exact(gstar))


def test_zero_stragglers_is_a_plain_tree_sum():
    L, n, s, m = 2, 3, 0, 1200
    X, y, w = _data(m, 5, seed=2)
    B = np.eye(n)
    own, _ = cr_tree.cr_allocate(L, n, s, m, B)
    N = cr_tree.num_workers(n, L)
    assert cr_tree.computation_load(n, L, 0) == Fraction(1, N)
    cover = np.zeros(m, dtype=int)
    for segs in own:
        assert len(segs) == 1 and segs[0][2] == 1.0 and segs[0][1] - segs[0][0] == m // N
        cover[segs[0][0]:segs[0][1]] += 1
    assert np.all(cover == 1)                            # a disjoint even split
    grads = [cr_tree.local_coded_gradient(X, y, w, segs) for segs in own]
    msgs, g = cr_tree.cr_execute(L, n, s, grads, np.zeros(N, dtype=np.uint8), lambda T: np.ones(n))
    np.testing.assert_allclose(g, sum(grads), rtol=1e-12)
    np.testing.assert_allclose(g, cr_tree.full_gradient(X, y, w), rtol=1e-11)


def test_one_layer_is_master_worker_gradient_coding():
    n, s, m = 3, 1, 300
    X, y, w = _data(m, 4, seed=8)
    own, subtree = cr_tree.cr_allocate(1, n, s, m, B_PRINTED)
    assert own == subtree                                # leaves keep everything
    assert own[0] == [(0, 100, 0.5), (100, 200, 1.0)] and own[1] == [(100, 200, 1.0), (200, 300, -1.0)]
    g1, g2, g3 = (cr_tree.partial_gradient(X, y, w, 100 * k, 100 * (k + 1)) for k in range(3))
    grads = [cr_tree.local_coded_gradient(X, y, w, segs) for segs in own]
    mask = np.array([0, 0, 1], dtype=np.uint8)
    _, g = cr_tree.cr_execute(1, n, s, grads, mask, lambda T: gc_code.decoding_row(B_PRINTED, T))
    np.testing.assert_allclose(g, 2 * (0.5 * g1 + g2) - (g2 - g3), rtol=1e-12)
    np.testing.assert_allclose(g, g1 + g2 + g3, rtol=1e-11, atol=1e-10)


def test_padding_rule_and_failure():
    assert cr_tree.padded_straggler_set([0, 1, 0, 0, 0, 0], 2) == (1, 5)
    assert cr_tree.padded_straggler_set([0, 0, 0, 0, 0, 1], 2) == (4, 5)
    assert cr_tree.padded_straggler_set([0, 0, 0], 1) == (2,)
    assert cr_tree.padded_straggler_set([1, 0, 1], 2) == (0, 2)
    with pytest.raises(cr_tree.Undecodable):
        cr_tree.padded_straggler_set([1, 1, 0], 1)
    grads = [np.ones(2)] * 12
    mask = np.zeros(12, dtype=np.uint8)
    mask[[6, 7]] = 1                                     # two stragglers among the children of node (1,2)
    with pytest.raises(cr_tree.Undecodable):
        cr_tree.cr_execute(2, 3, 1, grads, mask, lambda T: gc_code.decoding_row(B_PRINTED, T))


def test_gd_trajectory_equals_uncoded_gd():
    cfg = wl.config("cfg1")
    data = wl.make_dataset(cfg)
    X, y = data["X"], data["y"]
    B = gc_code.search_encoding_matrix(cfg["n"], cfg["s"], cfg["seed"], candidates=32)[0]
    rng = wl.mask_stream(cfg)
    w_cr = data["w0"].astype(np.float64)
    w_gd = w_cr.copy()
    ner = []
    for step in range(8):
        mask = wl.draw_mask(rng, cfg["L"], cfg["n"], cfg["s"])
        assert all(mask[g * 3:(g + 1) * 3].sum() == 1 for g in range(4))
        _, _, _, g = cr_tree.coded_reduce(cfg["L"], cfg["n"], cfg["s"], X, y, w_cr, mask, B)
        w_cr = w_cr - 2e-4 * g
        w_gd = w_gd - 2e-4 * cr_tree.full_gradient(X, y, w_gd)
        ner.append(np.sum((w_cr - data["w_star"]) ** 2) / np.sum(data["w_star"].astype(np.float64) ** 2))
    np.testing.assert_allclose(w_cr, w_gd, rtol=1e-9, atol=1e-12)
    assert all(b < a for a, b in zip(ner, ner[1:]))       # normalised error rate, eq. (8), falls monotonically
