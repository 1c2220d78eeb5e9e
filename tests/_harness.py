"""Shared plumbing for the GPU parity tests: runs the HIP path through the C-ABI binding and the oracle on the same inputs."""
from __future__ import annotations

import numpy as np

import paper_1902_01981_amd as cr
from oracle import cr_tree, gc_code, native

TOL = {cr.CR_F32: 1e-4, cr.CR_BF16: 5e-3}      # relative L2 bars of the parity contract


# Regression gates, an order of magnitude under the contract: what fp32 accumulation of these sums really leaves (observed
# 4e-8 to 3e-6, the same for bf16 data since both sides widen identical bits) with some room.  A message or a decoded gradient
# also carries the fp32 rounding of the messages below it, amplified by the code's gamma once per level.
GATE = 1e-5
WORST = {}                                     # what the gates saw, by kind of row: printed by the tests that want a record


def gate_for(gamma: float = 1.0, L: int = 1) -> float:
    return max(GATE, 8.0 * gamma ** L * 2.0 ** -24)


def rel_l2(a, b) -> float:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def max_over_rms(a, b) -> float:
    """Largest element-wise deviation in units of the reference's root mean square."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    rms = max(float(np.sqrt(np.mean(b * b))), 1e-300)
    return float(np.max(np.abs(a - b))) / rms


def assert_close(got, ref, tol, gate, what):
    """The parity contract (relative L2 <= tol), the regression gate (relative L2 <= gate) and an element-wise bound: no single
    entry off by more than 10 gates of the row's rms (one bad column in ten thousand passes a relative L2 unnoticed)."""
    err, worst = rel_l2(got, ref), max_over_rms(got, ref)
    kind = what[0] if isinstance(what, tuple) else what
    seen = WORST.setdefault(kind, [0.0, 0.0])
    seen[0], seen[1] = max(seen[0], err), max(seen[1], worst)
    assert err <= tol, (what, "contract", err)
    assert err <= gate, (what, "regression gate", err, gate)
    assert worst <= 10.0 * gate, (what, "element-wise", worst, 10.0 * gate)


class HipPath:
    """One plan + workspace + device copies of the inputs."""

    def __init__(self, L, n, s, X, y, model, x_dtype, B=None, teams=None):
        import torch

        self.torch = torch
        m, d = X.shape
        self.plan = cr.cr_plan_ex(L, n, s, m, d, model=model, x_dtype=x_dtype, B=B)
        if teams is not None:
            cr.cr_plan_set_split(self.plan, *teams) if isinstance(teams, tuple) else cr.cr_plan_set_split(self.plan, cr.CR_SPLIT_EQUAL_RANGES, teams)
        self.ws = cr.Workspace(self.plan)
        self.info = self.ws.info
        if X.dtype == np.uint16:
            self.X = torch.from_numpy(X.view(np.int16)).cuda()
        else:
            self.X = torch.from_numpy(X).cuda()
        self.y = torch.from_numpy(np.ascontiguousarray(y, dtype=np.float32)).cuda()
        self.g = torch.empty(d, dtype=torch.float32, device="cuda")

    def gradient(self, w_dev, mask):
        cr.cr_partial_grads(self.plan, self.X, self.y, w_dev)
        cr.cr_encode_tree(self.plan, mask)
        cr.cr_decode_root(self.plan, self.g)
        cr.cr_synchronize(self.plan)
        return self.g.cpu().numpy()

    def close(self):
        cr.cr_synchronize(self.plan)
        cr.cr_plan_destroy(self.plan)


_CODES = {}


def oracle_code(n, s, L):
    """The oracle's own code design for (n, s, L); the search over wide groups takes a while, so one per process."""
    key = (n, s, L)
    if key not in _CODES:
        _CODES[key] = gc_code.design_code(n, s, L, cr.DEFAULT_SEED)[0]
    return _CODES[key]


class OraclePath:
    """The CR tree literally, in fp64, with the oracle's own code design and allocation."""

    def __init__(self, L, n, s, X, y, model, B=None, use_native=False):
        self.L, self.n, self.s, self.X, self.y, self.model = L, n, s, X, y, model
        self.B = np.asarray(B, dtype=np.float64) if B is not None else oracle_code(n, s, L)
        self.own, self.subtree = cr_tree.cr_allocate(L, n, s, X.shape[0], self.B)
        self.slabs = cr_tree.slabs_of(self.own)
        self.native = use_native or X.dtype == np.uint16
        self._rows = {}

    def decode_row(self, T):
        if T not in self._rows:
            self._rows[T] = gc_code.decoding_row(self.B, T)
        return self._rows[T]

    def seg_grad(self, w, b, e):
        if self.native:
            return native.segment_gradient(self.X, self.y, w, b, e, self.model)
        return cr_tree.partial_gradient(self.X, self.y, w, b, e, self.model)

    def slab_grads(self, w):
        return [self.seg_grad(w, b, e) for (_, b, e, _) in self.slabs]

    def node_grads(self, slab_grads):
        d = self.X.shape[1]
        out = [np.zeros(d) for _ in self.own]
        for (node, _, _, c), gp in zip(self.slabs, slab_grads):
            out[node] = out[node] + float(c) * gp
        return out

    def execute(self, node_grads, mask):
        return cr_tree.cr_execute(self.L, self.n, self.s, node_grads, mask, self.decode_row)

    def full_gradient(self, w):
        if self.native:
            return native.full_gradient(self.X, self.y, w, self.model)
        return cr_tree.full_gradient(self.X, self.y, w, self.model)
