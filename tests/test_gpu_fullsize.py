"""The benchmark configurations at full size, in the launch configuration bench.py times (default work split, default code).

Each test runs the HIP path through the C-ABI on the full synthetic workload and checks it against the oracle: the decoded
gradient at several GD steps (the oracle is handed the GPU's current model, so the two cannot drift apart), every slab gradient and
every message at the first step, and properties of the whole trajectory.  Bars: relative L2 <= 1e-4 (fp32 X), 5e-3 (bf16 X).

Where the model has converged (late steps of a fast-converging run) the gradient is the difference of large cancelling terms and a
relative error of the gradient says nothing; there the models themselves are compared with an uncoded fp64 GD trajectory.
"""
import time

import numpy as np
import pytest

import paper_1902_01981_amd as cr
from cr_inputs import workloads as wl
from _harness import TOL, WORST, HipPath, OraclePath, assert_close, gate_for, rel_l2

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def _torch():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def _full_first_step(hip, orc, w, mask, tol):
    """All slabs, all messages and the decoded gradient against the CR tree computed literally by the oracle."""
    torch = _torch()
    g = hip.gradient(torch.from_numpy(w).cuda(), mask)
    sg = orc.slab_grads(w)
    msgs, g_cr = orc.execute(orc.node_grads(sg), mask)
    gstar = orc.full_gradient(w)
    assert rel_l2(g_cr, gstar) < 1e-9
    gate = gate_for(hip.info.gamma, hip.info.L)
    assert_close(g, gstar, tol, gate, "decoded gradient")
    G = hip.ws.slab_grads().cpu().numpy()
    for q, ref in enumerate(sg):
        assert_close(G[q], ref, tol, gate_for(), ("slab", q))
    M = hip.ws.messages().cpu().numpy()
    for node, ref in enumerate(msgs):
        if ref is not None:
            assert_close(M[node], ref, tol, gate, ("message", node))


def _gd_steps(hip, orc, cfg, data, steps, check_at, tol):
    torch = _torch()
    rng = wl.mask_stream(cfg)
    w_dev = torch.from_numpy(data["w0"]).cuda()
    lr = float(cfg["lr"])
    ner = []
    ws = float(np.sum(data["w_star"].astype(np.float64) ** 2))
    for step in range(steps):
        mask = wl.draw_mask(rng, cfg["L"], cfg["n"], cfg["s"])
        if step in check_at:
            w_host = w_dev.cpu().numpy()
            g = hip.gradient(w_dev, mask)
            ref = orc.full_gradient(w_host)
            print(f"step {step}: rel-L2 {rel_l2(g, ref):.2e}", flush=True)
            assert_close(g, ref, tol, gate_for(hip.info.gamma, hip.info.L), ("decoded gradient", step))
        else:
            hip.gradient(w_dev, mask)
        cr.cr_gd_update(hip.plan, w_dev, hip.g, lr)
        ner.append(float(np.sum((w_dev.cpu().numpy().astype(np.float64) - data["w_star"]) ** 2)) / ws)
    return w_dev.cpu().numpy(), ner


def test_cfg2_full():
    """L=2, n=4, s=1 (20 workers); linear regression fp32, 100 000 x 10 000; 50 GD steps, lr 1e-6, random mask per step."""
    cfg = wl.config("cfg2")
    t0 = time.time()
    data = wl.make_dataset(cfg, threads=16)
    print(f"data {time.time() - t0:.1f}s", flush=True)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    orc = OraclePath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, use_native=True)
    assert hip.info.num_slabs == 36 and hip.info.row_visits == 333_332
    _full_first_step(hip, orc, data["w0"], wl.draw_mask(wl.mask_stream(cfg), 2, 4, 1), 1e-4)
    _, ner = _gd_steps(hip, orc, cfg, data, 50, {0, 1, 2, 10, 25, 49}, 1e-4)
    assert all(b < a for a, b in zip(ner, ner[1:]))      # normalised error rate, eq. (8), falls at every step
    assert ner[-1] < 0.05 * ner[0]
    hip.close()


def test_cfg2_gd_run_full():
    """The call the benchmark times: cr_gd_run on configuration 2 at full size, the gradient step riding in the decode launch.
    After every batch of four steps the model equals, bit for bit, the one the step-by-step calls (gradients, encode, decode,
    update kernel) produce, and follows uncoded fp64 gradient descent from the oracle."""
    from oracle import native

    torch = _torch()
    cfg = wl.config("cfg2")
    data = wl.make_dataset(cfg, threads=16)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    assert (hip.info.split_kind, hip.info.stage1_staged) == (cr.CR_SPLIT_SHARED_CELLS, 1) and hip.info.l2_sharing == 1
    rng = wl.mask_stream(cfg)
    lr = float(cfg["lr"])
    w_run = torch.from_numpy(data["w0"]).cuda()
    w_steps = torch.from_numpy(data["w0"]).cuda()
    g_run = torch.empty_like(hip.g)
    w_ref = data["w0"].astype(np.float64)
    for batch in range(3):
        masks = np.stack([wl.draw_mask(rng, cfg["L"], cfg["n"], cfg["s"]) for _ in range(4)])
        cr.cr_gd_run(hip.plan, hip.X, hip.y, w_run, g_run, masks, lr)
        for mask in masks:
            hip.gradient(w_steps, mask)
            cr.cr_gd_update(hip.plan, w_steps, hip.g, lr)
        cr.cr_synchronize(hip.plan)
        assert torch.equal(w_run, w_steps) and torch.equal(g_run, hip.g), batch
        for _ in masks:                                  # exact gradient descent; the oracle's row loop takes the model in fp32
            w_ref = w_ref - lr * native.full_gradient(data["X"], data["y"], w_ref.astype(np.float32), cr.CR_LINEAR)
        err = rel_l2(w_run.cpu().numpy(), w_ref)
        print(f"after {4 * (batch + 1)} steps: model rel-L2 vs uncoded fp64 GD {err:.2e}", flush=True)
        assert err <= 1e-5, (batch, err)
    assert rel_l2(w_run.cpu().numpy(), data["w0"]) > 1e-2
    hip.close()


def test_cfg3_full():
    """L=3, n=4, s=1 (84 workers); logistic regression fp32, 252 000 x 4 096; 20 GD steps."""
    cfg = wl.config("cfg3")
    data = wl.make_dataset(cfg, threads=16)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LOGISTIC, cr.CR_F32)
    orc = OraclePath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LOGISTIC, use_native=True)
    assert hip.info.num_slabs == 148 and hip.info.row_visits == 1_512_000
    _full_first_step(hip, orc, data["w0"], wl.draw_mask(wl.mask_stream(cfg), 3, 4, 1), 1e-4)
    w, _ = _gd_steps(hip, orc, cfg, data, 20, {0, 1, 2, 10, 19}, 1e-4)
    # the model has moved towards the generating direction: training accuracy rises well above chance
    torch = _torch()
    z = (hip.X[:20000].float() @ torch.from_numpy(w).cuda()).cpu().numpy()     # harness-side evaluation only
    acc = float(np.mean((z >= 0) == (data["labels"][:20000] > 0)))
    assert acc > 0.9, acc
    hip.close()


def test_cfg5_full():
    """L=3, n=6, s=2 (258 workers); linear regression, X bf16 / fp32 accumulate, 2 064 000 x 1 024; 100 GD steps, lr 4e-7."""
    from oracle import native

    cfg = wl.config("cfg5")
    data = wl.make_dataset(cfg, threads=16)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_BF16)
    orc = OraclePath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, use_native=True)
    assert hip.info.num_slabs == 780 and hip.info.row_visits == 38_036_556
    _full_first_step(hip, orc, data["w0"], wl.draw_mask(wl.mask_stream(cfg), 3, 6, 2), 5e-3)
    # lr * lambda_max(X^T X) is about 0.85, so the run converges within a dozen steps: gradient parity where the gradient is
    # well conditioned (steps 0-2), model parity against uncoded fp64 gradient descent afterwards (steps 10, 50, 99)
    torch = _torch()
    rng = wl.mask_stream(cfg)
    w_dev = torch.from_numpy(data["w0"]).cuda()
    w_ref = data["w0"].astype(np.float64)
    lr = float(cfg["lr"])
    snap = {}
    for step in range(100):
        mask = wl.draw_mask(rng, 3, 6, 2)
        if step <= 2:
            w_host = w_dev.cpu().numpy()
            g = hip.gradient(w_dev, mask)
            err = rel_l2(g, orc.full_gradient(w_host))
            print(f"step {step}: rel-L2 {err:.2e}", flush=True)
            assert err <= 5e-3
        else:
            hip.gradient(w_dev, mask)
        cr.cr_gd_update(hip.plan, w_dev, hip.g, lr)
        if step < 12:
            w_ref = w_ref - lr * native.full_gradient(data["X"], data["y"], w_ref.astype(np.float32), cr.CR_LINEAR)
        if step in (10, 50, 99):
            snap[step] = w_dev.cpu().numpy().astype(np.float64)
    assert rel_l2(snap[10], w_ref) <= 1e-4                # same iterate as exact uncoded GD (to the fp32 model's resolution)
    assert rel_l2(snap[50], snap[99]) <= 1e-5 and rel_l2(snap[99], w_ref) <= 1e-4      # stationary at the least-squares solution
    assert rel_l2(snap[99], data["w_star"]) <= 1e-3       # which is the generating model up to the noise
    hip.close()


def test_four_holders_two_workgroups_per_unit_full():
    """A (2,4,1) tree over 366 000 x 2 048 fp32 (3 GB): the staged kernel with four holders per workgroup and, rows being 8 KB,
    two workgroups per compute unit."""
    cfg = wl.config("cfg2", m=366_000, d=2_048, lr=3e-7)
    data = wl.make_dataset(cfg, threads=16)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    orc = OraclePath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, use_native=True)
    assert (hip.info.split_kind, hip.info.stage1_staged, hip.info.stage1_teams_per_group) == (cr.CR_SPLIT_SHARED_CELLS, 1, 4)
    assert 256 * 4 < hip.info.num_teams <= 512 * 4         # more than one workgroup per unit
    _full_first_step(hip, orc, data["w0"], wl.draw_mask(wl.mask_stream(cfg), 2, 4, 1), 1e-4)
    _, ner = _gd_steps(hip, orc, cfg, data, 6, {0, 1, 5}, 1e-4)
    assert all(b < a for a, b in zip(ner, ner[1:]))
    hip.close()


def test_gradient_coding_twenty_workers_full():
    """One layer, 20 workers, 4 stragglers tolerated, on configuration 2's data: five holders per row, all in one workgroup of three
    teams that work for two holders each, so that every row is fetched once and streamed."""
    cfg = wl.config("gc20")
    data = wl.make_dataset(cfg, threads=16)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    orc = OraclePath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, use_native=True)
    assert (hip.info.split_kind, hip.info.stage1_staged, hip.info.stage1_teams_per_group) == (cr.CR_SPLIT_SHARED_CELLS, 1, 6)
    assert hip.info.row_visits == 5 * cfg["m"]
    _full_first_step(hip, orc, data["w0"], wl.draw_mask(wl.mask_stream(cfg), 1, 20, 4), 1e-4)
    _, ner = _gd_steps(hip, orc, cfg, data, 4, {0, 3}, 1e-4)
    assert all(b < a for a, b in zip(ner, ner[1:]))
    hip.close()


def test_uncoded_twenty_workers_full():
    """One layer, 20 workers, no redundancy, on configuration 2's data (4 GB): nobody else reads a row, so the register kernel
    fetches every row with the non-temporal hint (only data sets of 1 GiB and more take that path)."""
    cfg = wl.config("umw20")
    data = wl.make_dataset(cfg, threads=16)
    hip = HipPath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    orc = OraclePath(cfg["L"], cfg["n"], cfg["s"], data["X"], data["y"], cr.CR_LINEAR, use_native=True)
    assert (hip.info.split_kind, hip.info.stage1_staged) == (cr.CR_SPLIT_EQUAL_RANGES, 0) and hip.info.row_visits == cfg["m"]
    _full_first_step(hip, orc, data["w0"], np.zeros(20, dtype=np.uint8), 1e-4)
    _, ner = _gd_steps(hip, orc, cfg, data, 3, {0, 2}, 1e-4)
    assert all(b < a for a, b in zip(ner, ner[1:]))
    hip.close()


@pytest.mark.parametrize("L,n,s,m,d,holders", [(1, 4, 2, 30_000, 10_000, 3), (1, 4, 1, 30_000, 10_000, 2), (1, 6, 2, 70_000, 4_096, 4)])
def test_streamed_cells_full(L, n, s, m, d, holders):
    """Data sets of 1.1 to 1.2 GB whose every cell belongs to one workgroup: three holders loaded straight into LDS, two and
    three holders (one idle team) staged through registers, all fetched with the non-temporal hint."""
    cfg = wl.config("cfg2", L=L, n=n, s=s, m=m, d=d, lr=3e-7)
    data = wl.make_dataset(cfg, threads=16)
    hip = HipPath(L, n, s, data["X"], data["y"], cr.CR_LINEAR, cr.CR_F32)
    orc = OraclePath(L, n, s, data["X"], data["y"], cr.CR_LINEAR, use_native=True)
    assert (hip.info.split_kind, hip.info.stage1_staged, hip.info.stage1_teams_per_group) == (cr.CR_SPLIT_SHARED_CELLS, 1, holders)
    rng = wl.mask_stream(cfg)
    _full_first_step(hip, orc, data["w0"], wl.draw_mask(rng, L, n, s), 1e-4)
    hip.close()


def test_cfg4_full():
    """Aggregation only: L=2, n=8, s=2 (72 workers), 248 partition-gradient vectors of length 2^24, 20 random masks.  The decoded
    vector is checked on every column under every mask (it is the sum of all atoms whatever the mask); for the first two masks
    every message and the decoded vector are compared on every column with the oracle, run in column chunks on the host."""
    from concurrent.futures import ThreadPoolExecutor

    torch = _torch()
    cfg = wl.config("cfg4")
    L, n, s, d = cfg["L"], cfg["n"], cfg["s"], cfg["d"]
    plan = cr.cr_plan_ex(L, n, s, cfg["m"], d, model=cr.CR_AGGREGATE_ONLY)
    ws = cr.Workspace(plan)
    orc = OraclePath(L, n, s, np.zeros((cfg["m"], 1), dtype=np.float32), np.zeros(cfg["m"], dtype=np.float32), cr.CR_LINEAR)
    cuts, member = wl.atoms_of([b for (_, b, _, _) in orc.slabs], [e for (_, _, e, _) in orc.slabs])
    atoms_dev = torch.empty((len(cuts) - 1, d), dtype=torch.float32, device="cuda")
    for lo in range(0, d, 1 << 22):
        atoms_dev[:, lo:lo + (1 << 22)] = torch.from_numpy(wl.atom_vectors(cfg["seed"], len(cuts) - 1, lo, min(d, lo + (1 << 22)))).cuda()
    G_dev = torch.empty((len(member), d), dtype=torch.float32, device="cuda")
    for q, idx in enumerate(member):                     # input preparation: copies of a row range agree
        G_dev[q] = atoms_dev[idx].sum(dim=0)
    total = atoms_dev.double().sum(dim=0)
    del atoms_dev
    g_dev = torch.empty(d, dtype=torch.float32, device="cuda")
    rng = wl.mask_stream(cfg)
    gate = gate_for(ws.info.gamma, L)
    kept = []                                            # (mask, messages, decoded vector) of the first two masks, on the host
    for trial in range(20):
        mask = wl.draw_mask(rng, L, n, s)
        cr.cr_load_partial_grads(plan, G_dev)
        cr.cr_encode_tree(plan, mask)
        cr.cr_decode_root(plan, g_dev)
        cr.cr_synchronize(plan)
        err = float((g_dev.double() - total).norm() / total.norm())        # all 2^24 columns: the sum of all atoms, whatever the mask
        worst = float((g_dev.double() - total).abs().max() / total.square().mean().sqrt())
        assert err <= gate and worst <= 10 * gate, (trial, err, worst)
        if trial < 2:
            kept.append((mask, ws.messages().cpu().numpy(), g_dev.cpu().numpy()))
    G = G_dev.cpu().numpy()
    cr.cr_plan_destroy(plan)

    def check(lo):
        hi = min(d, lo + (1 << 18))
        ng = [np.zeros(hi - lo) for _ in range(72)]
        for q, (nd, _, _, c) in enumerate(orc.slabs):
            ng[nd] += float(c) * G[q, lo:hi].astype(np.float64)
        seen = 0.0
        for mask, M, g in kept:
            msgs, g_ref = orc.execute(ng, mask)
            assert rel_l2(g[lo:hi], g_ref) <= gate, (lo, "decoded")
            for node, ref in enumerate(msgs):
                if ref is not None:
                    err = rel_l2(M[node, lo:hi], ref)
                    dev = float(np.max(np.abs(M[node, lo:hi] - ref)) / np.sqrt(np.mean(ref * ref)))
                    assert err <= gate and dev <= 10 * gate, (lo, node, err, dev)
                    seen = max(seen, err)
        return seen

    with ThreadPoolExecutor(max_workers=16) as ex:       # numpy releases the interpreter lock; chunks are independent
        seen = list(ex.map(check, range(0, d, 1 << 18)))
    print(f"all {sum(int(m is not None) for m in orc.execute([np.zeros(1)] * 72, kept[0][0])[0])} messages x 2^24 columns x 2 masks: "
          f"worst chunk rel-L2 {max(seen):.2e}", flush=True)


def test_zz_report_what_the_gates_saw():
    """Not a check: prints the largest relative L2 error and element-wise deviation every kind of row showed in this session."""
    for kind, (err, worst) in sorted(WORST.items()):
        print(f"{kind}: worst rel-L2 {err:.2e}, worst max|delta|/rms {worst:.2e}", flush=True)
