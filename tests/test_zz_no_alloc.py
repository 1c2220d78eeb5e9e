"""cr_aggregate_static -- aggregation out of the library's own device array, for callers that cannot allocate -- against the
workspace path (cr_load_partial_grads, cr_encode_tree, cr_decode_root) on the same slab gradients and masks: same kernels, same
program, so the decoded gradients must agree bit for bit; and against the oracle.  Two calls in a row share the array, the second
on a smaller problem."""
import numpy as np
import pytest

import paper_1902_01981_amd as cr
from cr_inputs import workloads as wl
from _harness import OraclePath, assert_close, gate_for

pytestmark = pytest.mark.gpu


def _problem(torch, L, n, s, m, d, seed):
    plan = cr.cr_plan_ex(L, n, s, m, d, model=cr.CR_AGGREGATE_ONLY)
    orc = OraclePath(L, n, s, np.zeros((m, 1), dtype=np.float32), np.zeros(m, dtype=np.float32), cr.CR_LINEAR)
    cuts, member = wl.atoms_of([b for (_, b, _, _) in orc.slabs], [e for (_, _, e, _) in orc.slabs])
    atoms = wl.atom_vectors(seed, len(cuts) - 1, 0, d)
    G = np.stack([atoms[idx].sum(axis=0, dtype=np.float32) for idx in member])
    ng = [np.zeros(d) for _ in orc.own]
    for q, (nd, _, _, c) in enumerate(orc.slabs):
        ng[nd] += float(c) * G[q].astype(np.float64)
    return plan, orc, torch.from_numpy(G).cuda(), ng


def test_static_aggregation_matches_the_workspace_path():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    stream = torch.cuda.current_stream().cuda_stream
    # the paper's network on its (12,2) tree: 73.5 MB of messages, close to what the array holds; then a small tree
    problems = [(2, 12, 3, 156 * 40, 117_706, 11), (2, 3, 1, 1_200, 1_003, 12)]
    built = [_problem(torch, *args) for args in problems]
    rng = np.random.default_rng(7)
    for round_ in range(2):                              # big, small, big, small: each call finds the other's leftovers
        for (L, n, s, m, d, _), (plan, orc, G_dev, ng) in zip(problems, built):
            mask = wl.draw_mask(rng, L, n, s)
            if round_ == 1:
                mask[::n] = 0                            # fewer than s stragglers in every group
            g_static = torch.full((d,), float("nan"), dtype=torch.float32, device="cuda")
            cr.cr_aggregate_static(plan, G_dev, mask, g_static, stream)
            torch.cuda.synchronize()
            ws = cr.Workspace(plan)                      # the existing entry points, on a workspace of their own
            g_ws = torch.empty(d, dtype=torch.float32, device="cuda")
            cr.cr_load_partial_grads(plan, G_dev)
            cr.cr_encode_tree(plan, mask)
            cr.cr_decode_root(plan, g_ws)
            cr.cr_synchronize(plan)
            assert torch.equal(g_static, g_ws), (round_, d)
            _, g_ref = orc.execute(ng, mask)
            assert_close(g_static.cpu().numpy(), g_ref, 1e-4, gate_for(ws.info.gamma, L), "decoded gradient")
            del ws
    for plan, _, _, _ in built:
        cr.cr_plan_destroy(plan)
