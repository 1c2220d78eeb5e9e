"""CodedReduce on an (n,L)-regular tree, written out literally.  TEST INFRASTRUCTURE ONLY.

Follows Section III-A (scheme description), Algorithm 1 (CompAlloc) and
Algorithm 2 (CR.Allocate / CR.Execute) in the paper's order and notation, plus
the plain definition of the result, eq. (3):  g = sum over all data points of
the per-point loss gradient.  Per-point gradients are those of least squares,
grad = x (x^T w - y), and of logistic regression with targets in {0,1},
grad = x (sigma(x^T w) - y); stacked over a row range [b,e) of the data matrix
that is  X[b:e]^T (phi(X[b:e] w) - y[b:e]).

Notation: m data points (the paper's d), model dimension d (the paper's p),
n children per parent, L layers, s stragglers tolerated per sibling group.
Nodes are numbered 0-based: node (l,i), l in 1..L, i in 0..n^l-1, has flat id
off_l + i with off_l = n + ... + n^(l-1); its children are (l+1, n*i + j).

A *weighted set* is an ordered list of segments (row_begin, row_end, coef):
the data points X[row_begin:row_end], each carrying the scalar `coef`
(the paper's "b D" notation).  Coefficients may be floats or Fractions.

Readings where the paper is silent:
  * k = n partitions per CompAlloc call, cut by position at floor(kappa*|W|/n);
  * a child's parts are concatenated in ascending partition index;
  * a node keeps the FIRST `own` positions of its sub-tree set, where
    own = round_half_up(|W| / Q_l), Q_l = sum_{j=0}^{L-l} (n/(s+1))^j, which is
    r_CR * m whenever that is an integer; leaves keep everything;
  * with fewer than s stragglers in a group the straggler set is padded with the
    highest-index survivors and that decoding row is used;
  * more than s stragglers in any sibling group is an error;
  * a straggler sends no message; every other node does.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

from . import gc_code

LINEAR = 0
LOGISTIC = 1


class Undecodable(Exception):
    """A sibling group has more than s stragglers (the scheme cannot recover)."""


# --------------------------------------------------------------------------
# tree
# --------------------------------------------------------------------------
def num_workers(n: int, L: int) -> int:
    return sum(n ** l for l in range(1, L + 1))


def level_offset(n: int, l: int) -> int:
    return sum(n ** j for j in range(1, l))


def node_id(n: int, l: int, i: int) -> int:
    return level_offset(n, l) + i


def node_level_index(n: int, L: int, node: int) -> tuple[int, int]:
    for l in range(1, L + 1):
        off = level_offset(n, l)
        if node < off + n ** l:
            return l, node - off
    raise ValueError(node)


def children(n: int, L: int, node: int) -> list[int]:
    l, i = node_level_index(n, L, node)
    if l == L:
        return []
    return [node_id(n, l + 1, n * i + j) for j in range(n)]


def sibling_groups(n: int, L: int) -> list[list[int]]:
    """Group 0 = the master's children; then the children of every inner node, in node order."""
    groups = [[node_id(n, 1, j) for j in range(n)]]
    for node in range(num_workers(n, L)):
        kids = children(n, L, node)
        if kids:
            groups.append(kids)
    return groups


def computation_load(n: int, L: int, s: int) -> Fraction:
    """r_CR of Theorem 1."""
    q = Fraction(n, s + 1)
    return 1 / sum(q ** l for l in range(1, L + 1))


# --------------------------------------------------------------------------
# allocation (Algorithm 1 and the first half of Algorithm 2)
# --------------------------------------------------------------------------
def set_size(W) -> int:
    return sum(e - b for b, e, _ in W)


def take(W, lo: int, hi: int):
    """Positions [lo, hi) of the weighted set W, as a weighted set."""
    out, pos = [], 0
    for b, e, c in W:
        a0, a1 = max(lo, pos), min(hi, pos + (e - b))
        if a1 > a0:
            out.append((b + (a0 - pos), b + (a1 - pos), c))
        pos += e - b
    return out


def comp_alloc(W, B):
    """Algorithm 1: uniform partition of W into k = n parts; worker i gets the union over kappa of b_ik W_k."""
    n = len(B)
    size = set_size(W)
    cuts = [(kappa * size) // n for kappa in range(n + 1)]
    parts = [take(W, cuts[k], cuts[k + 1]) for k in range(n)]
    alloc = []
    for i in range(n):
        Di = []
        for kappa in range(n):
            bik = B[i][kappa]
            if bik != 0:
                Di.extend((b, e, c * bik) for b, e, c in parts[kappa])
        alloc.append(Di)
    return alloc


def own_count(size: int, n: int, L: int, s: int, l: int) -> int:
    if l == L:
        return size
    Q = sum(Fraction(n, s + 1) ** j for j in range(0, L - l + 1))
    x = Fraction(size) / Q
    return int((2 * x.numerator + x.denominator) // (2 * x.denominator))  # round half up


def cr_allocate(L: int, n: int, s: int, m: int, B, one=1.0):
    """CR.Allocate.  Returns (own, subtree): per node, its local weighted set D(l,i) and its sub-tree set D^T(l,i)."""
    N = num_workers(n, L)
    own = [None] * N
    subtree = [None] * N
    # remainder set handed to the children of each parent; the master hands down the whole data set
    rest_of_parent = {None: [(0, m, one)]}
    for l in range(1, L + 1):
        parents = [None] if l == 1 else [node_id(n, l - 1, i) for i in range(n ** (l - 1))]
        for pi, parent in enumerate(parents):
            sets = comp_alloc(rest_of_parent[parent], B)
            for j in range(n):
                subtree[node_id(n, l, n * pi + j)] = sets[j]
        for i in range(n ** l):
            node = node_id(n, l, i)
            W = subtree[node]
            size = set_size(W)
            k = own_count(size, n, L, s, l)
            own[node] = take(W, 0, k)
            rest_of_parent[node] = take(W, k, size)
    return own, subtree


def slabs_of(own):
    """Flatten per-node segments into the slab list: (node, row_begin, row_end, coef), node-major."""
    return [(node, b, e, c) for node, segs in enumerate(own) for (b, e, c) in segs]


# --------------------------------------------------------------------------
# gradients
# --------------------------------------------------------------------------
def phi(z, model: int):
    if model == LINEAR:
        return z
    z = np.asarray(z, dtype=np.float64)
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    ez = np.exp(z[~pos])
    out[~pos] = ez / (1.0 + ez)
    return out


def partial_gradient(X, y, w, b: int, e: int, model: int = LINEAR):
    """X[b:e]^T (phi(X[b:e] w) - y[b:e]) in fp64 (inputs converted exactly)."""
    Xs = np.asarray(X[b:e], dtype=np.float64)
    r = phi(Xs @ np.asarray(w, dtype=np.float64), model) - np.asarray(y[b:e], dtype=np.float64)
    return Xs.T @ r


def full_gradient(X, y, w, model: int = LINEAR, block: int = 8192):
    """eq. (3): the sum of per-point gradients over the whole data set."""
    m = X.shape[0]
    g = np.zeros(X.shape[1])
    for b in range(0, m, block):
        g += partial_gradient(X, y, w, b, min(m, b + block), model)
    return g


def local_coded_gradient(X, y, w, segments, model: int = LINEAR):
    """g_{D(l,i)}: sum over the node's segments of coef times that segment's partial gradient."""
    g = np.zeros(X.shape[1])
    for b, e, c in segments:
        g = g + float(c) * partial_gradient(X, y, w, b, e, model)
    return g


# --------------------------------------------------------------------------
# execution (second half of Algorithm 2)
# --------------------------------------------------------------------------
def padded_straggler_set(flags, s: int) -> tuple[int, ...]:
    """Straggler set of a sibling group padded to size s with the highest-index survivors."""
    T = [j for j, f in enumerate(flags) if f]
    if len(T) > s:
        raise Undecodable(f"{len(T)} stragglers in a group that tolerates {s}")
    j = len(flags) - 1
    while len(T) < s:
        if j not in T:
            T.append(j)
        j -= 1
    return tuple(sorted(T))


def cr_execute(L: int, n: int, s: int, node_grads, mask, decode_row):
    """CR.Execute.  node_grads[node] = g_{D(l,i)}; mask[node] true = straggler;
    decode_row(straggler_tuple) -> length-n coefficient row.
    Returns (messages, g): messages[node] is None for stragglers."""
    N = num_workers(n, L)
    groups = sibling_groups(n, L)
    for grp in groups:                                   # any group beyond tolerance: the scheme fails
        padded_straggler_set([mask[k] for k in grp], s)
    msg = [None] * N
    for l in range(L, 0, -1):
        for i in range(n ** l):
            node = node_id(n, l, i)
            if mask[node]:
                continue
            if l == L:
                msg[node] = node_grads[node]
                continue
            kids = children(n, L, node)
            a = decode_row(padded_straggler_set([mask[k] for k in kids], s))
            acc = node_grads[node]
            for j, k in enumerate(kids):
                if a[j] != 0:
                    acc = acc + a[j] * msg[k]
            msg[node] = acc
    top = groups[0]
    a = decode_row(padded_straggler_set([mask[k] for k in top], s))
    g = None
    for j, k in enumerate(top):
        if a[j] != 0:
            g = a[j] * msg[k] if g is None else g + a[j] * msg[k]
    return msg, g


def coded_reduce(L, n, s, X, y, w, mask, B, model: int = LINEAR):
    """One whole iteration: allocate, compute every node's coded gradient, execute.  Returns (own, node_grads, messages, g)."""
    B = np.asarray(B, dtype=np.float64)
    own, _ = cr_allocate(L, n, s, X.shape[0], B)
    node_grads = [local_coded_gradient(X, y, w, segs, model) for segs in own]
    msgs, g = cr_execute(L, n, s, node_grads, mask, lambda T: gc_code.decoding_row(B, T))
    return own, node_grads, msgs, g
