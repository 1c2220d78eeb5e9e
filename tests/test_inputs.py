"""The seeded input recipes: shapes, determinism, mask structure."""
import numpy as np

from cr_inputs import workloads as wl


def test_dataset_is_deterministic_and_shaped():
    cfg = wl.config("cfg1")
    a, b = wl.make_dataset(cfg, threads=1), wl.make_dataset(cfg, threads=4)
    for k in ("X", "y", "w_star", "w0"):
        assert np.array_equal(a[k], b[k])
    assert a["X"].shape == (1200, 100) and a["X"].dtype == np.float32 and a["y"].dtype == np.float32
    resid = a["y"] - a["X"].astype(np.float64) @ a["w_star"].astype(np.float64)
    assert 0.005 < resid.std() < 0.02                    # noise N(0, 0.01^2)
    assert abs(a["X"].mean()) < 0.01 and abs(a["X"].std() - 1) < 0.01


def test_logistic_and_bf16_recipes():
    cfg = wl.config("cfg3", m=4000, d=64)
    data = wl.make_dataset(cfg)
    assert set(np.unique(data["labels"])) == {-1.0, 1.0} and set(np.unique(data["y"])) == {0.0, 1.0}
    assert np.array_equal(data["y"], (data["labels"] + 1) / 2)
    assert abs(np.linalg.norm(data["w0"]) - 1.0) < 0.3    # w0 ~ N(0, 1/d)
    cfg = wl.config("cfg5", m=3000, d=32)
    data = wl.make_dataset(cfg)
    assert data["X"].dtype == np.uint16
    Xr = wl.bf16_bits_to_f32(data["X"])
    resid = data["y"] - Xr.astype(np.float64) @ data["w_star"].astype(np.float64)
    assert resid.std() < 0.02                            # y is formed from the rounded values


def test_masks():
    cfg = wl.config("cfg4")
    rng = wl.mask_stream(cfg)
    seen = set()
    for _ in range(50):
        mask = wl.draw_mask(rng, cfg["L"], cfg["n"], cfg["s"])
        assert mask.shape == (72,) and all(mask[g * 8:(g + 1) * 8].sum() == 2 for g in range(9))
        seen.add(mask.tobytes())
    assert len(seen) == 50
    assert sum(1 for _ in wl.enumerate_masks(2, 3, 1)) == 256
    assert sum(1 for _ in wl.enumerate_masks(2, 3, 1, exactly_s=True)) == 81


def test_atoms():
    cuts, member = wl.atoms_of([0, 4, 4, 2], [4, 9, 6, 9])
    assert cuts == [0, 2, 4, 6, 9] and member == [[0, 1], [2, 3], [2], [1, 2, 3]]
    v = wl.atom_vectors(5, 3, 0, 1000)
    v2 = wl.atom_vectors(5, 3, 0, 1000)
    assert np.array_equal(v, v2) and v.shape == (3, 1000) and abs(v.std() - 1) < 0.1


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "one GPU" in res.stderr and res.stdout.strip() == ""
