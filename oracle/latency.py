"""Run-time model of one CodedReduce iteration.  TEST INFRASTRUCTURE ONLY.

Section III-C ("Latency Performance"): a worker holding d_i data points finishes its local computation after a
shifted-exponential time, eq. (5):  P[T_i <= t] = 1 - exp(-(mu/d_i)(t - a d_i)) for t >= a d_i; a node receives from one
child at a time and one message takes t_c (single-port model).  A parent needs any n-s of its children's messages.

The paper analyses this model only asymptotically (Theorem 2); the simulation below states it operationally.  Readings:
  * T_i = a d_i + (d_i/mu) * (-ln(1-u_i)) with u_i uniform on [0,1): the inverse of eq. (5);
  * all nodes start computing at time 0 (CR.Execute step 1) and compute while they receive;
  * a parent serves its children in order of readiness (ties: lower index first); the transfer of a child starts when the
    child is ready and the parent's port is free, and lasts t_c;
  * the parent decodes when its (n-s)-th transfer completes; the s children not yet received are this iteration's
    stragglers; the parent's own message is ready at max(own computation finished, decode time); a leaf's at T_i;
  * the iteration ends when the master has decoded.
Uniforms come from the same counter-based generator as the code search: u(node) = top 53 bits of splitmix64 output number
iteration*N + node of the stream started at `seed`.
"""
from __future__ import annotations

import math

from . import cr_tree, gc_code


def uniform01(seed: int, counter: int) -> float:
    return (gc_code.splitmix64_at(seed, counter) >> 11) * (2.0 ** -53)


def compute_time(u: float, rows: int, a: float, mu: float) -> float:
    """Inverse CDF of eq. (5) for a worker holding `rows` data points."""
    return a * rows + (rows / mu) * (-math.log1p(-u))


def expected_order_statistic(n: int, s: int, rows: float, a: float, mu: float) -> float:
    """E[T_(n-s)] of n i.i.d. shifted exponentials (Appendix D): (rows/mu)(H_n - H_s) + a rows."""
    H = lambda k: sum(1.0 / i for i in range(1, k + 1))
    return (rows / mu) * (H(n) - H(s)) + a * rows


def receive(ready, n_needed: int, t_c: float):
    """Single-port reception.  ready[j] = time child j can start sending.  Returns (decode_time, received_order)."""
    order = sorted(range(len(ready)), key=lambda j: (ready[j], j))
    port_free = 0.0
    done = []
    for j in order[:n_needed]:
        start = max(ready[j], port_free)
        port_free = start + t_c
        done.append(j)
    return port_free, done


def simulate_iteration(L: int, n: int, s: int, rows_per_node, a: float, mu: float, t_c: float, uniforms):
    """Returns (mask, ready, total): mask[node] = 1 for this iteration's stragglers, ready[node] = time its message is
    ready to send, total = time the master has decoded."""
    N = cr_tree.num_workers(n, L)
    T = [compute_time(uniforms[k], rows_per_node[k], a, mu) for k in range(N)]
    ready = [0.0] * N
    mask = [0] * N
    for l in range(L, 0, -1):
        for i in range(n ** l):
            node = cr_tree.node_id(n, l, i)
            kids = cr_tree.children(n, L, node)
            if not kids:
                ready[node] = T[node]
                continue
            decode, got = receive([ready[k] for k in kids], n - s, t_c)
            for j, k in enumerate(kids):
                if j not in got:
                    mask[k] = 1
            ready[node] = max(T[node], decode)
    top = [cr_tree.node_id(n, 1, j) for j in range(n)]
    total, got = receive([ready[k] for k in top], n - s, t_c)
    for j, k in enumerate(top):
        if j not in got:
            mask[k] = 1
    return mask, ready, total


def simulate(L, n, s, rows_per_node, a, mu, t_c, seed: int, iteration: int):
    N = cr_tree.num_workers(n, L)
    u = [uniform01(seed, iteration * N + k) for k in range(N)]
    return simulate_iteration(L, n, s, rows_per_node, a, mu, t_c, u)
