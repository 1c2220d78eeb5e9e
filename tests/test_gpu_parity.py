"""HIP path vs oracle, element by element, on seeded inputs that span several tiles and ragged tails.
Bars: relative L2 <= 1e-4 (fp32 X) or 5e-3 (bf16 X) for the decoded gradient, every slab and every message."""
import numpy as np
import pytest

import paper_1902_01981_amd as cr
from cr_inputs import workloads as wl
from _harness import TOL, WORST, HipPath, OraclePath, assert_close, gate_for, rel_l2

pytestmark = pytest.mark.gpu
B_PRINTED = np.array([[0.5, 1, 0], [0, 1, -1], [0.5, 0, 1]])


def _torch():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def _check_iteration(hip, orc, w, mask, tol, check_rows=True):
    torch = _torch()
    w_dev = torch.from_numpy(w).cuda()
    g = hip.gradient(w_dev, mask)
    sg = orc.slab_grads(w)
    ng = orc.node_grads(sg)
    msgs, g_cr = orc.execute(ng, mask)
    gstar = orc.full_gradient(w)
    assert rel_l2(g_cr, gstar) < 1e-9                    # the oracle's tree result is the plain definition
    gate = gate_for(hip.info.gamma, hip.info.L)
    assert_close(g, gstar, tol, gate, "decoded gradient")
    if check_rows:
        G = hip.ws.slab_grads().cpu().numpy()
        for q, ref in enumerate(sg):
            assert_close(G[q], ref, tol, gate_for(), ("slab", q))
        M = hip.ws.messages().cpu().numpy()
        for node, ref in enumerate(msgs):
            if ref is not None:
                assert_close(M[node], ref, tol, gate, ("message", node))
    return g


def test_cfg1_every_mask():
    """Tiny tree (L=2, n=3, s=1), 1200 x 100 linear regression: all 256 masks with at most one straggler per group."""
    torch = _torch()
    cfg = wl.config("cfg1")
    data = wl.make_dataset(cfg)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    orc = OraclePath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR)
    assert hip.info.num_slabs == 27 and hip.info.row_visits == 3840
    w = data["w0"]
    w_dev = torch.from_numpy(w).cuda()
    sg = orc.slab_grads(w)
    ng = orc.node_grads(sg)
    gstar = orc.full_gradient(w)
    count = 0
    for mask in wl.enumerate_masks(cfg["L"], cfg["n"], cfg["s"]):
        g = hip.gradient(w_dev, mask)
        assert_close(g, gstar, 1e-4, gate_for(hip.info.gamma, 2), "decoded gradient")
        if count % 16 == 0:
            msgs, _ = orc.execute(ng, mask)
            M = hip.ws.messages().cpu().numpy()
            for node, ref in enumerate(msgs):
                if ref is not None:
                    assert_close(M[node], ref, 1e-4, gate_for(hip.info.gamma, 2), ("message", node))
        count += 1
    assert count == 256
    G = hip.ws.slab_grads().cpu().numpy()
    for q, ref in enumerate(sg):
        assert_close(G[q], ref, 1e-4, gate_for(), ("slab", q))
    hip.close()


def test_printed_code_of_the_example():
    """The (3,2) example with the printed B: messages are the printed combinations of partition gradients."""
    cfg = wl.config("cfg1", m=1500, d=52)
    data = wl.make_dataset(cfg)
    hip = HipPath(2, 3, 1, data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32, B=B_PRINTED)
    orc = OraclePath(2, 3, 1, data["X"], data["y"], cr.CR_LINEAR, B=B_PRINTED)
    mask = np.zeros(12, dtype=np.uint8)
    mask[[1, 5]] = 1
    g = _check_iteration(hip, orc, data["w0"], mask, 1e-4)
    gD = [orc.seg_grad(data["w0"], 500 * k, 500 * (k + 1)) for k in range(3)]
    M = hip.ws.messages().cpu().numpy()
    assert rel_l2(M[0], 0.5 * gD[0] + gD[1]) <= 1e-4 and rel_l2(M[2], 0.5 * gD[0] + gD[2]) <= 1e-4
    assert rel_l2(g, gD[0] + gD[1] + gD[2]) <= 1e-4
    hip.close()


CASES = [
    # name, L, n, s, m, d, model, x_dtype, teams
    ("cfg2-shape", 2, 4, 1, 6_007, 10_000, cr.CR_LINEAR, cr.CR_F32, None),       # 256-thread teams, 10 chunks per thread, ragged last chunk
    ("cfg2-few-teams", 2, 4, 1, 3_001, 10_000, cr.CR_LINEAR, cr.CR_F32, 37),      # pieces crossing slab boundaries
    ("cfg2-row-cells", 2, 4, 1, 3_001, 10_000, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_ROW_CELLS, 48)),  # holders of a cell run side by side
    ("cfg3-shape", 3, 4, 1, 8_400, 4_096, cr.CR_LOGISTIC, cr.CR_F32, None),
    ("cfg5-row-cells", 3, 6, 2, 25_801, 1_024, cr.CR_LINEAR, cr.CR_BF16, (cr.CR_SPLIT_ROW_CELLS, 100)),
    ("cfg5-shape", 3, 6, 2, 25_801, 1_024, cr.CR_LINEAR, cr.CR_BF16, None),       # one wavefront per row, bf16 x8 chunks
    ("bf16-wide", 2, 3, 1, 2_000, 8_192, cr.CR_LOGISTIC, cr.CR_BF16, None),       # bf16 with 256-thread teams
    ("odd-d-fp32", 2, 3, 1, 1_111, 1_003, cr.CR_LINEAR, cr.CR_F32, None),         # d % 4 != 0: the last chunk overlaps its neighbour
    ("odd-d-bf16", 2, 3, 1, 1_111, 270, cr.CR_LINEAR, cr.CR_BF16, None),
    ("odd-d-cfg2", 2, 4, 1, 2_003, 9_999, cr.CR_LOGISTIC, cr.CR_F32, None),       # rows not 16-byte aligned, 10 chunks per thread
    ("odd-d-bf16-k3", 2, 3, 1, 1_500, 1_027, cr.CR_LINEAR, cr.CR_BF16, None),     # rows on odd 2-byte boundaries, last thread chunk mostly inert
    ("bf16-k3-buffers", 2, 3, 1, 1_503, 1_536, cr.CR_LOGISTIC, cr.CR_BF16, None),  # buffer loads, three chunks per lane, pieces that end inside a trip of four rows
    ("bf16-k4-buffers", 3, 3, 2, 2_001, 2_042, cr.CR_LINEAR, cr.CR_BF16, (cr.CR_SPLIT_ROW_CELLS, 7)),   # rows on 4-byte (not 16-byte) boundaries, last chunk moved back, cells of 7 rows
    ("bf16-k1-buffers", 1, 6, 3, 999, 72, cr.CR_LOGISTIC, cr.CR_BF16, (cr.CR_SPLIT_EQUAL_RANGES, 13)),    # one chunk per lane, most lanes idle, pieces across slab boundaries
    ("d-5", 2, 3, 1, 600, 5, cr.CR_LINEAR, cr.CR_F32, None),                      # two chunks sharing three columns
    ("d-9-bf16", 2, 3, 1, 600, 9, cr.CR_LOGISTIC, cr.CR_BF16, None),              # two chunks sharing seven columns
    ("d-3", 2, 3, 1, 600, 3, cr.CR_LINEAR, cr.CR_F32, None),                      # shorter than one chunk: one column per lane
    ("d-7-bf16", 1, 4, 1, 600, 7, cr.CR_LINEAR, cr.CR_BF16, None),
    ("tiny-d", 1, 5, 2, 333, 4, cr.CR_LINEAR, cr.CR_F32, None),                   # one layer: master-worker gradient coding
    ("s0-plain-tree", 2, 4, 0, 4_000, 256, cr.CR_LINEAR, cr.CR_F32, None),
    ("deep", 4, 2, 1, 3_000, 520, cr.CR_LOGISTIC, cr.CR_F32, None),
    ("big-team", 2, 3, 1, 700, 16_384, cr.CR_LINEAR, cr.CR_F32, None),            # 1024-thread teams
    ("m-equals-N", 2, 3, 1, 12, 64, cr.CR_LINEAR, cr.CR_F32, None),               # one row per worker
    ("gc-master-worker", 1, 10, 4, 10_000, 512, cr.CR_LINEAR, cr.CR_F32, None),   # one layer, 10 workers, 4 stragglers (fractional repetition)
    ("uncoded-master-worker", 1, 10, 0, 10_000, 512, cr.CR_LINEAR, cr.CR_F32, None),
    ("wide-rows-fp32", 2, 3, 1, 400, 30_000, cr.CR_LINEAR, cr.CR_F32, None),      # beyond one team's registers: two-pass stage 1
    ("wide-rows-bf16", 2, 4, 1, 500, 50_008, cr.CR_LOGISTIC, cr.CR_BF16, None),
    ("wide-rows-odd", 1, 3, 1, 200, 25_001, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_EQUAL_RANGES, 40)),
    ("cr-12x2-s3", 2, 12, 3, 31_200, 320, cr.CR_LOGISTIC, cr.CR_F32, None),       # the paper's (12,2) tree, 156 workers, 3 stragglers per group
    ("cr-12x2-s2", 2, 12, 2, 15_611, 1_000, cr.CR_LINEAR, cr.CR_F32, None),       # ... 2 per group
    ("cr-12x2-s5", 2, 12, 5, 49_920, 432, cr.CR_LOGISTIC, cr.CR_F32, None),       # ... 5 per group (resiliency 5/12, 49 920 points as in the network experiment): 36 holders per row
    # rows staged through LDS and shared by the holders in one workgroup
    ("direct-4-holders", 2, 4, 1, 3_001, 10_000, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 37)),      # rows loaded straight into LDS, weights in LDS too, 10 chunks per thread, cells of 2 and 4 holders
    ("direct-4-holders-k8", 2, 3, 1, 2_501, 8_192, cr.CR_LOGISTIC, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 3)),    # 2048 chunks: no partial wavefront in the fetch; cells shorter than the ring
    ("direct-4-holders-8", 3, 4, 1, 2_400, 6_500, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 20)),      # 8, 4 and 2 holders: cells of two workgroups (kept in the L2) and of one (streamed)
    ("direct-3-holders", 1, 4, 2, 3_001, 10_000, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 37)),      # three holders per row and workgroup, weights in registers; every row streamed
    ("direct-6-holders-5", 1, 10, 4, 2_000, 9_000, cr.CR_LOGISTIC, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 11)),   # five holders in one workgroup: three teams that work for two holders each, one of them for one
    ("direct-6-holders-6", 1, 12, 5, 1_800, 7_000, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 5)),      # six holders, seven chunks per thread, cells shorter than the ring
    ("direct-3-holders-k9", 1, 6, 2, 2_000, 8_196, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 1)),      # single-row cells: the ring runs across items; last fetch wavefronts idle
    ("direct-widest", 2, 4, 1, 1_500, 10_232, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 16)),          # 2558 chunks: the ring and the weights fill LDS to the last byte
    ("direct-default", 2, 4, 1, 70_000, 6_400, cr.CR_LINEAR, cr.CR_F32, None),                                  # large enough for the default split to pick it
    ("staged-2-holders", 1, 4, 1, 3_001, 10_000, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 37)),      # two holders per row: register-staged kernel, 10 chunks per thread
    ("staged-2-holders-odd-d", 2, 4, 1, 2_003, 9_999, cr.CR_LOGISTIC, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 64)),
    ("staged-4-holders", 2, 4, 1, 5_003, 2_052, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 50)),       # four 256-thread teams, two rows per step
    ("staged-4-holders-k6", 2, 3, 1, 2_000, 5_640, cr.CR_LOGISTIC, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 90)),
    ("staged-8-holders", 3, 4, 1, 8_400, 4_096, cr.CR_LOGISTIC, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 33)),     # eight one-wavefront teams, 16 chunks per thread
    ("staged-8-holders-1-row", 3, 3, 1, 2_500, 3_001, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 1)),  # cells of a single row
    ("staged-3-holders", 1, 5, 2, 4_001, 3_001, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 100)),      # one idle team per workgroup of four
    ("staged-k12", 2, 3, 1, 900, 12_288, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 1000)),            # the widest staged rows
    ("staged-default", 2, 4, 1, 140_000, 1_100, cr.CR_LINEAR, cr.CR_F32, None),                               # large enough for the staged default
    ("staged-queue-gaps", 3, 2, 1, 3_000, 7_000, cr.CR_LINEAR, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 40)),      # cells of 1, 2 and 4 workgroups in gangs of 4
    ("staged-wide-gang", 4, 3, 2, 2_400, 6_200, cr.CR_LOGISTIC, cr.CR_F32, (cr.CR_SPLIT_SHARED_CELLS, 25)),     # 81 holders: more workgroups per cell than one L2 domain has slots
]


@pytest.mark.parametrize("name,L,n,s,m,d,model,x_dtype,teams", CASES, ids=[c[0] for c in CASES])
def test_shapes_and_kernel_variants(name, L, n, s, m, d, model, x_dtype, teams):
    base = "cfg3" if model == cr.CR_LOGISTIC else ("cfg5" if x_dtype == cr.CR_BF16 else "cfg2")
    cfg = wl.config(base, L=L, n=n, s=s, m=m, d=d, model=model, x_dtype=x_dtype, w0_std=None if model == cr.CR_LOGISTIC else 1.0)
    data = wl.make_dataset(cfg)
    hip = HipPath(L, n, s, data["X"], data["y"], model, x_dtype, teams=teams)
    orc = OraclePath(L, n, s, data["X"], data["y"], model)
    rng = wl.mask_stream(cfg)
    N = wl.num_workers(n, L)
    masks = [np.zeros(N, dtype=np.uint8)] + [wl.draw_mask(rng, L, n, s) for _ in range(3)]
    for mask in masks:
        _check_iteration(hip, orc, data["w0"], mask, TOL[x_dtype])
    hip.close()


def test_gd_trajectory_cfg1():
    """Gradient descent with a fresh mask per step: the HIP path is fed its own w; the oracle is given the same w each step."""
    torch = _torch()
    cfg = wl.config("cfg1")
    data = wl.make_dataset(cfg)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    orc = OraclePath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR)
    rng = wl.mask_stream(cfg)
    w_dev = torch.from_numpy(data["w0"]).cuda()
    ner = []
    for step in range(10):
        mask = wl.draw_mask(rng, cfg["L"], cfg["n"], cfg["s"])
        w_host = w_dev.cpu().numpy()
        g = hip.gradient(w_dev, mask)
        assert rel_l2(g, orc.full_gradient(w_host)) <= 1e-4
        cr.cr_gd_update(hip.plan, w_dev, hip.g, 2e-4)
        cr.cr_synchronize(hip.plan)
        np.testing.assert_allclose(w_dev.cpu().numpy(), w_host - np.float32(2e-4) * g, rtol=1e-6, atol=1e-7)
        ner.append(float(np.sum((w_dev.cpu().numpy() - data["w_star"]) ** 2) / np.sum(data["w_star"] ** 2)))
    assert all(b < a for a, b in zip(ner, ner[1:]))
    hip.close()


def test_device_resident_gd_loop_and_run_time_model_masks():
    """cr_gd_run against the step-by-step calls (bit-identical models) and against uncoded fp64 GD; masks come from the
    run-time model (the s slowest children of every group under shifted-exponential compute times)."""
    torch = _torch()
    cfg = wl.config("cfg1")
    data = wl.make_dataset(cfg)
    L, n, s = cfg["L"], cfg["n"], cfg["s"]
    hip = HipPath(L, n, s, data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    orc = OraclePath(L, n, s, data["X"], data["y"], cr.CR_LINEAR)
    steps, lr = 12, 2e-4
    masks = np.stack([cr.cr_simulate_iteration(hip.plan, 5e-5, 2e4, 0.05, 42, t)[0] for t in range(steps)])
    assert all(masks[t, g * n:(g + 1) * n].sum() == s for t in range(steps) for g in range(4)) and len({m.tobytes() for m in masks}) > 1
    # step by step
    w_a = torch.from_numpy(data["w0"]).cuda()
    for t in range(steps):
        hip.gradient(w_a, masks[t])
        cr.cr_gd_update(hip.plan, w_a, hip.g, lr)
    # one call, with the convergence measures
    w_b = torch.from_numpy(data["w0"]).cuda()
    w_star = torch.from_numpy(data["w_star"]).cuda()
    metrics = torch.zeros(steps, 2, dtype=torch.float32, device="cuda")
    cr.cr_gd_run(hip.plan, hip.X, hip.y, w_b, hip.g, masks, lr, w_star, metrics)
    cr.cr_synchronize(hip.plan)
    assert torch.equal(w_a, w_b)
    # and without them (plain update kernel)
    w_c = torch.from_numpy(data["w0"]).cuda()
    cr.cr_gd_run(hip.plan, hip.X, hip.y, w_c, hip.g, masks, lr)
    cr.cr_synchronize(hip.plan)
    assert torch.equal(w_a, w_c)
    # uncoded fp64 gradient descent (the oracle) gives the same trajectory and the same measures
    w = data["w0"].astype(np.float64)
    ws = data["w_star"].astype(np.float64)
    ref = []
    for t in range(steps):
        w_new = w - lr * orc.full_gradient(w)
        ref.append([np.sum((w_new - w) ** 2) / np.sum(w ** 2), np.sum((w_new - ws) ** 2) / np.sum(ws ** 2)])
        w = w_new
    assert rel_l2(w_b.cpu().numpy(), w) <= 1e-5
    np.testing.assert_allclose(metrics.cpu().numpy(), np.array(ref), rtol=2e-3)
    assert np.all(np.diff(metrics.cpu().numpy()[:, 1]) < 0)            # normalised error rate falls
    bad = masks.copy()
    bad[5, 3:5] = 1
    with pytest.raises(cr.CodedReduceError) as ei:
        cr.cr_gd_run(hip.plan, hip.X, hip.y, w_c, hip.g, bad, lr)
    assert ei.value.status == cr.CR_E_UNDECODABLE
    cr.cr_synchronize(hip.plan)
    assert torch.equal(w_a, w_c)                         # nothing was enqueued
    hip.close()


@pytest.mark.parametrize("d,m,model", [(5, 900, cr.CR_LINEAR), (1_003, 2_400, cr.CR_LOGISTIC), (9_999, 2_003, cr.CR_LINEAR), (10, 480, cr.CR_LINEAR)])
def test_gd_run_fused_step_with_ragged_widths(d, m, model):
    """cr_gd_run without the convergence measures lets the gradient step ride in the decode launch.  With d not a multiple of 4 the
    row's last chunk overlaps its neighbour and only the owner of a column may step it: compared bit for bit with separate decode
    and update calls, and with uncoded fp64 gradient descent from the oracle."""
    torch = _torch()
    L, n, s = 2, 3, 1
    cfg = wl.config("cfg3" if model == cr.CR_LOGISTIC else "cfg2", L=L, n=n, s=s, m=m, d=d, model=model,
                    w0_std=None if model == cr.CR_LOGISTIC else 1.0, seed=31_000 + d)
    data = wl.make_dataset(cfg)
    hip = HipPath(L, n, s, data["X"], data["y"], model, cr.CR_F32)
    orc = OraclePath(L, n, s, data["X"], data["y"], model)
    steps = 9
    lr = 0.5 / (m * (1 + np.sqrt(d / m)) ** 2) * (4.0 if model == cr.CR_LOGISTIC else 1.0)      # inside 2 / lambda_max(X^T X)
    rng = wl.mask_stream(cfg)
    masks = np.stack([wl.draw_mask(rng, L, n, s) for _ in range(steps)])
    w_a = torch.from_numpy(data["w0"]).cuda()
    for t in range(steps):                               # separate calls: decode, then the update kernel
        hip.gradient(w_a, masks[t])
        cr.cr_gd_update(hip.plan, w_a, hip.g, lr)
    g_a = hip.g.clone()
    w_b = torch.from_numpy(data["w0"]).cuda()
    cr.cr_gd_run(hip.plan, hip.X, hip.y, w_b, hip.g, masks[:4], lr)       # two calls: the loop can be resumed
    cr.cr_gd_run(hip.plan, hip.X, hip.y, w_b, hip.g, masks[4:], lr)
    cr.cr_synchronize(hip.plan)
    assert torch.equal(w_a, w_b) and torch.equal(g_a, hip.g)
    w = data["w0"].astype(np.float64)
    for t in range(steps):
        w = w - lr * orc.full_gradient(w)
    assert rel_l2(w_b.cpu().numpy(), w) <= 1e-5, rel_l2(w_b.cpu().numpy(), w)
    assert rel_l2(w_b.cpu().numpy(), data["w0"]) > 1e-3                   # and the model did move
    hip.close()


def test_aggregation_only():
    """Partition gradients supplied as vectors (L=2, n=8, s=2): encode + decode alone, 20 masks."""
    torch = _torch()
    L, n, s, d = 2, 8, 2, 70_004                        # several 1024-column blocks and a ragged one
    cfg = wl.config("cfg4", d=d)
    plan = cr.cr_plan_ex(L, n, s, cfg["m"], d, model=cr.CR_AGGREGATE_ONLY)
    ws = cr.Workspace(plan)
    assert ws.info.num_slabs == 248 and ws.info.num_workers == 72
    orc = OraclePath(L, n, s, np.zeros((cfg["m"], 1), dtype=np.float32), np.zeros(cfg["m"], dtype=np.float32), cr.CR_LINEAR)
    rb = [b for (_, b, _, _) in orc.slabs]
    re_ = [e for (_, _, e, _) in orc.slabs]
    cuts, member = wl.atoms_of(rb, re_)
    assert len(cuts) - 1 == 56
    atoms = wl.atom_vectors(cfg["seed"], len(cuts) - 1, 0, d)
    G = np.stack([atoms[idx].sum(axis=0, dtype=np.float32) for idx in member])   # redundant copies of a row range agree
    G_dev = torch.from_numpy(G).cuda()
    g_dev = torch.empty(d, dtype=torch.float32, device="cuda")
    slab_grads = [G[q].astype(np.float64) for q in range(len(member))]
    ng = []
    for node in range(72):
        acc = np.zeros(d)
        for q, (nd, _, _, c) in enumerate(orc.slabs):
            if nd == node:
                acc += float(c) * slab_grads[q]
        ng.append(acc)
    rng = wl.mask_stream(cfg)
    for trial in range(20):
        mask = wl.draw_mask(rng, L, n, s)
        cr.cr_load_partial_grads(plan, G_dev)
        cr.cr_encode_tree(plan, mask)
        cr.cr_decode_root(plan, g_dev)
        cr.cr_synchronize(plan)
        msgs, g_ref = orc.execute(ng, mask)
        assert rel_l2(g_dev.cpu().numpy(), g_ref) <= 1e-4, (trial, rel_l2(g_dev.cpu().numpy(), g_ref))
        if trial % 5 == 0:
            M = ws.messages().cpu().numpy()
            for node, ref in enumerate(msgs):
                if ref is not None:
                    assert rel_l2(M[node], ref) <= 1e-4
    # the decoded vector is the sum of all atoms, whatever the mask
    assert rel_l2(g_dev.cpu().numpy(), atoms.astype(np.float64).sum(0)) <= 1e-4
    cr.cr_plan_destroy(plan)


@pytest.mark.parametrize("s", [1, 2, 3, 5])
def test_aggregation_only_network_sized(s):
    """(12,2) tree, 156 workers, 1 to 5 stragglers per group (5 = the resiliency 5/12 of the network experiment), vectors of the
    size of the paper's CNN (117 706 parameters, not a multiple of 4)."""
    torch = _torch()
    L, n, d = 2, 12, 117_706
    m = 156 * 40
    plan = cr.cr_plan_ex(L, n, s, m, d, model=cr.CR_AGGREGATE_ONLY)
    ws = cr.Workspace(plan)
    info = ws.info
    orc = OraclePath(L, n, s, np.zeros((m, 1), dtype=np.float32), np.zeros(m, dtype=np.float32), cr.CR_LINEAR)
    assert info.num_slabs == len(orc.slabs) and info.num_workers == 156
    cuts, member = wl.atoms_of([b for (_, b, _, _) in orc.slabs], [e for (_, _, e, _) in orc.slabs])
    atoms = wl.atom_vectors(1234 + s, len(cuts) - 1, 0, d)
    G = np.stack([atoms[idx].sum(axis=0, dtype=np.float32) for idx in member])
    G_dev = torch.from_numpy(G).cuda()
    g_dev = torch.empty(d, dtype=torch.float32, device="cuda")
    ng = [np.zeros(d) for _ in range(156)]
    for q, (nd, _, _, c) in enumerate(orc.slabs):
        ng[nd] += float(c) * G[q].astype(np.float64)
    rng = np.random.default_rng(s)
    for trial in range(6):
        mask = wl.draw_mask(rng, L, n, s)
        cr.cr_load_partial_grads(plan, G_dev)
        cr.cr_encode_tree(plan, mask)
        cr.cr_decode_root(plan, g_dev)
        cr.cr_synchronize(plan)
        msgs, g_ref = orc.execute(ng, mask)
        gate = gate_for(info.gamma, L)
        assert_close(g_dev.cpu().numpy(), g_ref, 1e-4, gate, "decoded gradient")
        M = ws.messages().cpu().numpy()
        for node, ref in enumerate(msgs):
            if ref is not None:
                assert_close(M[node], ref, 1e-4, gate, ("message", node))
    cr.cr_plan_destroy(plan)


def test_aggregate_run_matches_the_three_calls():
    """cr_aggregate_run over 37 masks (three program uploads) against cr_load_partial_grads + cr_encode_tree + cr_decode_root per mask:
    the same bits, with one set of slab gradients for all steps and with one per step; and a bad mask enqueues nothing."""
    torch = _torch()
    L, n, s, d, steps = 2, 12, 5, 1_003, 37
    m = 156 * 8
    plan = cr.cr_plan_ex(L, n, s, m, d, model=cr.CR_AGGREGATE_ONLY)
    ws = cr.Workspace(plan)
    S = ws.info.num_slabs
    rng = np.random.default_rng(99)
    masks = np.stack([wl.draw_mask(rng, L, n, s) for _ in range(steps)])
    masks[5, ::n] = 0                                    # fewer than s stragglers in every group of one step
    stride = (S * d + 3) // 4 * 4                        # per-step slab sets, 16-byte aligned
    G_all = torch.randn(steps * stride, dtype=torch.float32, device="cuda")
    for per_step in (False, True):
        g_ref = torch.empty(steps, d, dtype=torch.float32, device="cuda")
        for t in range(steps):
            off = t * stride if per_step else 0
            cr.cr_load_partial_grads(plan, G_all[off:off + S * d])
            cr.cr_encode_tree(plan, masks[t])
            cr.cr_decode_root(plan, g_ref[t])
        M_ref = ws.messages().clone()
        g_run = torch.full((steps, d), float("nan"), dtype=torch.float32, device="cuda")
        cr.cr_aggregate_run(plan, G_all, masks, g_run, G_step_stride=stride if per_step else 0, g_step_stride=d)
        cr.cr_synchronize(plan)
        assert torch.equal(g_run, g_ref) and torch.equal(ws.messages(), M_ref), per_step
        if per_step:
            assert not torch.equal(g_run[0], g_run[1])
        else:
            last_same_slabs = g_ref[-1].clone()
    g_one = torch.empty(d, dtype=torch.float32, device="cuda")
    cr.cr_aggregate_run(plan, G_all, masks, g_one)       # stride 0: every step overwrites the same vector; the last one stays
    cr.cr_synchronize(plan)
    assert torch.equal(g_one, last_same_slabs)
    before = g_one.clone()
    bad = masks.copy()
    bad[20, 0:6] = 1
    with pytest.raises(cr.CodedReduceError) as ei:
        cr.cr_aggregate_run(plan, G_all, bad, g_one)
    assert ei.value.status == cr.CR_E_UNDECODABLE
    cr.cr_synchronize(plan)
    assert torch.equal(g_one, before)
    cr.cr_plan_destroy(plan)


def test_gd_run_across_program_batches():
    """40 steps in one cr_gd_run call (three uploads of encode programs) against the step-by-step calls: bit-identical models and
    convergence measures; then the same masks in two calls of 23 and 17."""
    torch = _torch()
    cfg = wl.config("cfg1")
    data = wl.make_dataset(cfg)
    L, n, s = cfg["L"], cfg["n"], cfg["s"]
    hip = HipPath(L, n, s, data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    steps, lr = 40, 1e-4
    rng = wl.mask_stream(cfg)
    masks = np.stack([wl.draw_mask(rng, L, n, s) for _ in range(steps)])
    w_a = torch.from_numpy(data["w0"]).cuda()
    for t in range(steps):
        hip.gradient(w_a, masks[t])
        cr.cr_gd_update(hip.plan, w_a, hip.g, lr)
    w_b = torch.from_numpy(data["w0"]).cuda()
    metrics = torch.zeros(steps, 2, dtype=torch.float32, device="cuda")
    cr.cr_gd_run(hip.plan, hip.X, hip.y, w_b, hip.g, masks, lr, None, metrics)
    w_c = torch.from_numpy(data["w0"]).cuda()
    cr.cr_gd_run(hip.plan, hip.X, hip.y, w_c, hip.g, masks[:23], lr)
    cr.cr_gd_run(hip.plan, hip.X, hip.y, w_c, hip.g, masks[23:], lr)
    cr.cr_synchronize(hip.plan)
    assert torch.equal(w_a, w_b) and torch.equal(w_a, w_c)
    rel = metrics.cpu().numpy()[:, 0]
    assert np.all(rel > 0) and np.all(metrics.cpu().numpy()[:, 1] == -1)
    hip.close()


LAYERS = [("conv1.weight", 3 * 16 * 3 * 3), ("conv1.bias", 16), ("conv2.weight", 16 * 64 * 4 * 4), ("conv2.bias", 64),
          ("fc1.weight", 64 * 384), ("fc1.bias", 384), ("fc2.weight", 384 * 192), ("fc2.bias", 192), ("fc3.weight", 192 * 10),
          ("fc3.bias", 10)]


@pytest.mark.parametrize("s", [2, 5])
def test_aggregation_per_layer_of_the_simulated_network(s):
    """The network of the paper's simulation (two convolutions, three dense layers: 117 706 parameters) aggregated layer by layer,
    as a training framework hands gradients over: ten vectors of 10 to 73 728 entries, several shorter than one workgroup's
    columns, some not multiples of 4, each through its own plan on the (12,2) tree over 49 920 data points."""
    torch = _torch()
    L, n, m = 2, 12, 49_920
    assert sum(size for _, size in LAYERS) == 117_706
    orc = OraclePath(L, n, s, np.zeros((m, 1), dtype=np.float32), np.zeros(m, dtype=np.float32), cr.CR_LINEAR)
    cuts, member = wl.atoms_of([b for (_, b, _, _) in orc.slabs], [e for (_, _, e, _) in orc.slabs])
    rng = np.random.default_rng(50 + s)
    masks = [wl.draw_mask(rng, L, n, s) for _ in range(3)]
    masks[2][::n] = 0                                    # fewer than s stragglers in every group: the padded decode rows
    B_plan = None
    for k, (name, d) in enumerate(LAYERS):
        # the first plan searches the code; the others are handed its B (the search does not depend on d)
        plan = cr.cr_plan_ex(L, n, s, m, d, model=cr.CR_AGGREGATE_ONLY, B=B_plan)
        if B_plan is None:
            B_plan = cr.cr_plan_get_B(plan)
            np.testing.assert_allclose(B_plan, orc.B, atol=1e-12)
        ws = cr.Workspace(plan)
        assert ws.info.num_slabs == len(orc.slabs)
        atoms = wl.atom_vectors(7_000 + 10 * s + k, len(cuts) - 1, 0, d)
        G = np.stack([atoms[idx].sum(axis=0, dtype=np.float32) for idx in member])
        G_dev = torch.from_numpy(G).cuda()
        g_dev = torch.empty(d, dtype=torch.float32, device="cuda")
        ng = [np.zeros(d) for _ in range(156)]
        for q, (nd, _, _, c) in enumerate(orc.slabs):
            ng[nd] += float(c) * G[q].astype(np.float64)
        gate = gate_for(ws.info.gamma, L)
        for mask in masks:
            cr.cr_load_partial_grads(plan, G_dev)
            cr.cr_encode_tree(plan, mask)
            cr.cr_decode_root(plan, g_dev)
            cr.cr_synchronize(plan)
            msgs, g_ref = orc.execute(ng, mask)
            assert_close(g_dev.cpu().numpy(), g_ref, 1e-4, gate, ("decoded gradient", name))
            assert_close(g_dev.cpu().numpy(), atoms.astype(np.float64).sum(0), 1e-4, gate, ("sum of all atoms", name))
            M = ws.messages().cpu().numpy()
            for node, ref in enumerate(msgs):
                if ref is not None:
                    assert_close(M[node], ref, 1e-4, gate, ("message", name, node))
        cr.cr_plan_destroy(plan)


def test_aggregation_only_long_vectors():
    """Vectors long enough for the wide encode shape (128 KB pieces per workgroup, fp32 accumulation), ragged last workgroup."""
    torch = _torch()
    L, n, s = 2, 8, 2
    d = (1 << 20) + 8192 * 3 + 36
    cfg = wl.config("cfg4", d=d)
    plan = cr.cr_plan_ex(L, n, s, cfg["m"], d, model=cr.CR_AGGREGATE_ONLY)
    ws = cr.Workspace(plan)
    orc = OraclePath(L, n, s, np.zeros((cfg["m"], 1), dtype=np.float32), np.zeros(cfg["m"], dtype=np.float32), cr.CR_LINEAR)
    cuts, member = wl.atoms_of([b for (_, b, _, _) in orc.slabs], [e for (_, _, e, _) in orc.slabs])
    atoms_dev = torch.from_numpy(wl.atom_vectors(cfg["seed"], len(cuts) - 1, 0, d)).cuda()
    G_dev = torch.stack([atoms_dev[idx].sum(dim=0) for idx in member])           # input preparation (copies of a row range agree)
    G = G_dev.cpu().numpy()
    g_dev = torch.empty(d, dtype=torch.float32, device="cuda")
    cols = np.r_[0:64, 8192 * 7 - 32:8192 * 7 + 32, d - 100:d]                   # sampled columns, incl. workgroup seams and the tail
    ng = []
    for node in range(72):
        acc = np.zeros(len(cols))
        for q, (nd, _, _, c) in enumerate(orc.slabs):
            if nd == node:
                acc += float(c) * G[q, cols].astype(np.float64)
        ng.append(acc)
    rng = wl.mask_stream(cfg)
    for trial in range(4):
        mask = wl.draw_mask(rng, L, n, s)
        cr.cr_load_partial_grads(plan, G_dev)
        cr.cr_encode_tree(plan, mask)
        cr.cr_decode_root(plan, g_dev)
        cr.cr_synchronize(plan)
        msgs, g_ref = orc.execute(ng, mask)
        assert rel_l2(g_dev.cpu().numpy()[cols], g_ref) <= 1e-4
        M = ws.messages()[:, torch.from_numpy(cols).cuda()].cpu().numpy()
        for node, ref in enumerate(msgs):
            if ref is not None:
                assert rel_l2(M[node], ref) <= 1e-4
    # whole vector: the decoded gradient is the sum of all atoms, whatever the mask
    total = atoms_dev.double().sum(dim=0)
    err = (g_dev.double() - total).norm() / total.norm()
    assert float(err) <= 1e-4
    cr.cr_plan_destroy(plan)


def test_failure_paths_leave_state_alone():
    torch = _torch()
    cfg = wl.config("cfg1")
    data = wl.make_dataset(cfg)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    w_dev = torch.from_numpy(data["w0"]).cuda()
    lib = cr.load_library()
    ok = np.zeros(12, dtype=np.uint8)
    with pytest.raises(cr.CodedReduceError) as ei:       # encode before any gradients
        cr.cr_encode_tree(hip.plan, ok)
    assert ei.value.status == cr.CR_E_STATE
    g_ok = hip.gradient(w_dev, ok).copy()
    M_before = hip.ws.messages().cpu().numpy().copy()
    bad = ok.copy()
    bad[[3, 4]] = 1                                      # two stragglers among the children of node (1,1)
    with pytest.raises(cr.CodedReduceError) as ei:
        cr.cr_encode_tree(hip.plan, bad)
    assert ei.value.status == cr.CR_E_UNDECODABLE
    cr.cr_decode_root(hip.plan, hip.g)                   # the previous messages are still in place
    cr.cr_synchronize(hip.plan)
    assert np.array_equal(hip.g.cpu().numpy(), g_ok) and np.array_equal(hip.ws.messages().cpu().numpy(), M_before)
    cr.cr_partial_grads(hip.plan, hip.X, hip.y, w_dev)
    with pytest.raises(cr.CodedReduceError) as ei:       # decode before the new encode
        cr.cr_decode_root(hip.plan, hip.g)
    assert ei.value.status == cr.CR_E_STATE
    assert lib.cr_partial_grads(hip.plan, hip.X.data_ptr() + 4, hip.y.data_ptr(), w_dev.data_ptr()) == cr.CR_E_INVAL
    hip.close()


def test_repeat_runs_are_bit_identical():
    torch = _torch()
    cfg = wl.config("cfg2", m=4_000, d=2_048)
    data = wl.make_dataset(cfg)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    w_dev = torch.from_numpy(data["w0"]).cuda()
    mask = wl.draw_mask(wl.mask_stream(cfg), cfg["L"], cfg["n"], cfg["s"])
    a = hip.gradient(w_dev, mask).copy()
    b = hip.gradient(w_dev, mask).copy()
    assert np.array_equal(a, b)                          # fixed reduction order, no floating-point atomics
    hip.close()


def test_random_small_problems():
    """Seeded sweep over trees, widths, dtypes, models and work splits (each picks its own kernel variant)."""
    rng = np.random.default_rng(77)
    widths = [4, 20, 100, 260, 1000, 1032, 2052, 3000, 5001, 12_288]
    for trial in range(24):
        L = int(rng.integers(1, 4))
        n = int(rng.integers(2, 6))
        s = int(rng.integers(0, n))
        N = wl.num_workers(n, L)
        d = int(widths[trial % len(widths)])
        m = int(N + rng.integers(1, max(2, 600_000 // d)))
        model = cr.CR_LOGISTIC if trial % 3 == 0 else cr.CR_LINEAR
        x_dtype = cr.CR_BF16 if trial % 4 == 1 else cr.CR_F32
        base = "cfg3" if model == cr.CR_LOGISTIC else "cfg2"
        cfg = wl.config(base, L=L, n=n, s=s, m=m, d=d, model=model, x_dtype=x_dtype, w0_std=None if model == cr.CR_LOGISTIC else 1.0,
                        seed=1000 + trial)
        data = wl.make_dataset(cfg)
        split = [None, (cr.CR_SPLIT_EQUAL_RANGES, int(rng.integers(1, 2000))), (cr.CR_SPLIT_ROW_CELLS, int(rng.integers(1, 300)))][trial % 3]
        if s > 0 and x_dtype == cr.CR_F32 and 1024 < d <= 12_288 and trial % 2 == 0:
            split = (cr.CR_SPLIT_SHARED_CELLS, int(rng.integers(1, 300)))
        print(f"trial {trial}: L={L} n={n} s={s} m={m} d={d} model={model} x_dtype={x_dtype} split={split}", flush=True)
        hip = HipPath(L, n, s, data["X"], data["y"], model, x_dtype, teams=split)
        orc = OraclePath(L, n, s, data["X"], data["y"], model)
        mask = np.zeros(N, dtype=np.uint8)
        for g in range(N // n):
            k = int(rng.integers(0, s + 1))
            mask[g * n + rng.choice(n, size=k, replace=False)] = 1
        _check_iteration(hip, orc, data["w0"], mask, TOL[x_dtype])
        hip.close()


def test_random_sweep_of_staged_kernels():
    """Seeded sweep over the staged stage-1 kernels: every chunk count of the one-wavefront family and of both four-wavefront
    families, odd widths, trees with 2 to 27 holders per row, random cell heights, fewer than s stragglers in some groups."""
    rng = np.random.default_rng(4242)
    chunk_counts = list(range(257, 1025, 64)) + [1024, 1100, 1536, 1700, 2304, 2900, 3072]      # 16-byte chunks per row
    for trial, nq in enumerate(chunk_counts):
        L = int(rng.integers(1, 4))
        n = int(rng.integers(2, 5))
        s = int(rng.integers(1, n))
        N = wl.num_workers(n, L)
        d = 4 * nq - int(rng.integers(0, 4))              # any remainder modulo the chunk width
        m = int(N * int(rng.integers(8, 40)) + rng.integers(0, max(60, 1_500_000 // d)))
        model = cr.CR_LOGISTIC if trial % 2 else cr.CR_LINEAR
        cfg = wl.config("cfg3" if model == cr.CR_LOGISTIC else "cfg2", L=L, n=n, s=s, m=m, d=d, model=model, x_dtype=cr.CR_F32,
                        w0_std=None if model == cr.CR_LOGISTIC else 1.0, seed=5000 + trial)
        data = wl.make_dataset(cfg)
        split = (cr.CR_SPLIT_SHARED_CELLS, int(rng.integers(1, 60)))
        print(f"trial {trial}: L={L} n={n} s={s} m={m} d={d} model={model} split={split}", flush=True)
        hip = HipPath(L, n, s, data["X"], data["y"], model, cr.CR_F32, teams=split)
        assert hip.info.stage1_staged == 1
        orc = OraclePath(L, n, s, data["X"], data["y"], model)
        mask = np.zeros(N, dtype=np.uint8)
        for g in range(N // n):
            k = int(rng.integers(0, s + 1))
            mask[g * n + rng.choice(n, size=k, replace=False)] = 1
        _check_iteration(hip, orc, data["w0"], mask, TOL[cr.CR_F32])
        hip.close()


def test_read_bandwidth_probe_reads_every_word():
    torch = _torch()
    n = (1 << 24) + 12                                    # floats; not a multiple of the probe's stride
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    sink = torch.zeros(16384, dtype=torch.float32, device="cuda")
    gbps = cr.cr_probe_read_bandwidth(src, n * 4, sink, launches=3)
    assert float(sink.double().sum()) == n               # every word was read exactly once in the last launch
    assert gbps > 100.0
    with pytest.raises(cr.CodedReduceError):
        cr.cr_probe_read_bandwidth(src, 1024, sink)



def test_zz_report_what_the_gates_saw():
    """Not a check: prints the largest relative L2 error and element-wise deviation every kind of row showed in this session."""
    for kind, (err, worst) in sorted(WORST.items()):
        print(f"{kind}: worst rel-L2 {err:.2e}, worst max|delta|/rms {worst:.2e}", flush=True)
