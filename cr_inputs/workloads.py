"""Workload recipes: Gaussian regression / classification data, bf16 storage, straggler masks.

The paper's experiments use Gaussian linear regression (features and true model
N(0, I), additive Gaussian noise) and logistic regression on a real data set
that is not available here; Gaussian stand-ins of the configured shapes take its
place.  All draws come from numpy PCG64 streams spawned from one base seed, so
the same arrays reach the GPU path and the oracle.
"""
from __future__ import annotations

import itertools
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 190201981
ROW_BLOCK = 16384          # rows per independent random stream (fixed: results do not depend on thread count)
COL_BLOCK = 1 << 20        # columns per independent stream for long vectors

LINEAR, LOGISTIC, AGGREGATE_ONLY = 0, 1, 2
F32, BF16 = 0, 1

# name -> recipe.  Shapes, trees and step counts are the benchmark configurations; lr / w0 are harness choices
# inside 2/lambda_max of X^T X for the sum-of-gradients convention.
CONFIGS = {
    "cfg1": dict(L=2, n=3, s=1, m=1_200, d=100, model=LINEAR, x_dtype=F32, noise=0.01, steps=1, lr=1e-4, w0_std=1.0),
    "cfg2": dict(L=2, n=4, s=1, m=100_000, d=10_000, model=LINEAR, x_dtype=F32, noise=0.01, steps=50, lr=1e-6, w0_std=1.0),
    "cfg3": dict(L=3, n=4, s=1, m=252_000, d=4_096, model=LOGISTIC, x_dtype=F32, noise=0.1, steps=20, lr=1e-5, w0_std=None),
    "cfg4": dict(L=2, n=8, s=2, m=88, d=1 << 24, model=AGGREGATE_ONLY, x_dtype=F32, noise=0.0, steps=20, lr=0.0, w0_std=1.0),
    # the paper's simulated network training: (12,2) tree, 156 workers, resiliency 5/12, 49 920 data points, about 120 000 parameters
    # (5 layers: 3x16x3x3, 16x64x4x4, 64x384, 384x192, 192x10 weights plus biases = 117 706), aggregation only
    "nn12": dict(L=2, n=12, s=5, m=49_920, d=117_706, model=AGGREGATE_ONLY, x_dtype=F32, noise=0.0, steps=20, lr=0.0, w0_std=1.0),
    # configuration 2's data with 20 workers under one master instead of a (4,2) tree: gradient coding with the same resiliency
    # (4 of 20 = 1 of 4 children may straggle) and the uncoded split.  Section III-C compares their computation loads.
    "gc20": dict(L=1, n=20, s=4, m=100_000, d=10_000, model=LINEAR, x_dtype=F32, noise=0.01, steps=50, lr=1e-6, w0_std=1.0),
    "umw20": dict(L=1, n=20, s=0, m=100_000, d=10_000, model=LINEAR, x_dtype=F32, noise=0.01, steps=50, lr=1e-6, w0_std=1.0),
    # the paper's own linear-regression experiment: 84 workers as a (4,3) tree, one straggler in four, (d,p) = (7644, 6500)
    "paper84": dict(L=3, n=4, s=1, m=7_644, d=6_500, model=LINEAR, x_dtype=F32, noise=1.0, steps=300, lr=2e-5, w0_std=1.0),
    "cfg5": dict(L=3, n=6, s=2, m=2_064_000, d=1_024, model=LINEAR, x_dtype=BF16, noise=0.01, steps=100, lr=4e-7, w0_std=1.0),
}


def config(name: str, **overrides) -> dict:
    cfg = dict(CONFIGS[name])
    cfg["name"] = name
    cfg["seed"] = BASE_SEED + {"nn12": 12, "gc20": 2, "umw20": 2, "paper84": 84}.get(name, int(name[3:]) if name.startswith("cfg") else 0)
    cfg.update(overrides)
    return cfg


def _streams(seed: int, count: int):
    return np.random.SeedSequence(seed).spawn(count)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def gaussian_matrix(seed_seq, m: int, d: int, threads: int = 8) -> np.ndarray:
    """m x d standard normal fp32, generated in independent row blocks."""
    X = np.empty((m, d), dtype=np.float32)
    nblk = (m + ROW_BLOCK - 1) // ROW_BLOCK
    seqs = seed_seq.spawn(nblk)

    def fill(i):
        b, e = i * ROW_BLOCK, min(m, (i + 1) * ROW_BLOCK)
        np.random.Generator(np.random.PCG64(seqs[i])).standard_normal((e - b, d), dtype=np.float32, out=X[b:e])

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(fill, range(nblk)))
    return X


def _matvec64(X: np.ndarray, v: np.ndarray, is_bf16: bool) -> np.ndarray:
    out = np.empty(X.shape[0], dtype=np.float64)
    v64 = v.astype(np.float64)
    step = max(1, (1 << 24) // max(1, X.shape[1]))
    for b in range(0, X.shape[0], step):
        blk = X[b:b + step]
        blk = bf16_bits_to_f32(blk) if is_bf16 else blk
        out[b:b + step] = blk.astype(np.float64) @ v64
    return out


def make_dataset(cfg: dict, threads: int = 8) -> dict:
    """X (fp32, or uint16 bf16 bits), y (fp32 targets), w_star, w0 for a regression / classification recipe.

    Linear:   y = X w* + noise * N(0,1).
    Logistic: labels = sign(X w* + noise * N(0,1)) in {-1,+1}; y holds the {0,1} targets (labels+1)/2.
    With bf16 storage X is rounded first and y is formed from the rounded values.
    """
    m, d = cfg["m"], cfg["d"]
    sx, sw, sn, s0 = _streams(cfg["seed"], 4)
    X = gaussian_matrix(sx, m, d, threads)
    is_bf16 = cfg["x_dtype"] == BF16
    if is_bf16:
        Xb = np.empty((m, d), dtype=np.uint16)
        for b in range(0, m, ROW_BLOCK):
            Xb[b:b + ROW_BLOCK] = to_bf16_bits(X[b:b + ROW_BLOCK])
        X = Xb
    w_star = np.random.Generator(np.random.PCG64(sw)).standard_normal(d).astype(np.float32)
    noise = np.random.Generator(np.random.PCG64(sn)).standard_normal(m)
    z = _matvec64(X, w_star, is_bf16) + cfg["noise"] * noise
    out = dict(X=X, w_star=w_star)
    if cfg["model"] == LOGISTIC:
        labels = np.where(z >= 0, 1.0, -1.0).astype(np.float32)
        out["labels"] = labels
        out["y"] = ((labels + 1.0) * 0.5).astype(np.float32)
    else:
        out["y"] = z.astype(np.float32)
    std = cfg["w0_std"] if cfg["w0_std"] is not None else 1.0 / np.sqrt(d)
    out["w0"] = (std * np.random.Generator(np.random.PCG64(s0)).standard_normal(d)).astype(np.float32)
    return out


# --------------------------------------------------------------------------
# straggler masks.  Workers are numbered level by level, so sibling group g is ids [g*n, (g+1)*n).
# --------------------------------------------------------------------------
def num_workers(n: int, L: int) -> int:
    return sum(n ** l for l in range(1, L + 1))


def draw_mask(rng: np.random.Generator, L: int, n: int, s: int) -> np.ndarray:
    """Exactly s stragglers in every sibling group, each size-s subset equally likely."""
    N = num_workers(n, L)
    mask = np.zeros((N // n, n), dtype=np.uint8)
    if s > 0:
        # the s smallest of n i.i.d. uniforms sit at a uniformly random size-s subset
        pick = np.argpartition(rng.random((N // n, n)), s - 1, axis=1)[:, :s]
        np.put_along_axis(mask, pick, 1, axis=1)
    return mask.reshape(N)


def mask_stream(cfg: dict) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(cfg["seed"]).spawn(5)[4]))


def enumerate_masks(L: int, n: int, s: int, exactly_s: bool = False):
    """Every mask with at most (or exactly) s stragglers per sibling group."""
    N = num_workers(n, L)
    sizes = [s] if exactly_s else range(s + 1)
    per_group = [T for k in sizes for T in itertools.combinations(range(n), k)]
    for combo in itertools.product(per_group, repeat=N // n):
        mask = np.zeros(N, dtype=np.uint8)
        for g, T in enumerate(combo):
            for j in T:
                mask[g * n + j] = 1
        yield mask


# --------------------------------------------------------------------------
# aggregation-only inputs: partition gradients handed in as vectors
# --------------------------------------------------------------------------
def atoms_of(row_begin, row_end):
    """Common refinement of the slab row ranges.  Returns (cuts, member) where atom t = [cuts[t], cuts[t+1]) and
    member[p] lists the atoms slab p is made of."""
    cuts = sorted(set(int(v) for v in row_begin) | set(int(v) for v in row_end))
    index = {c: i for i, c in enumerate(cuts)}
    member = [list(range(index[int(b)], index[int(e)])) for b, e in zip(row_begin, row_end)]
    return cuts, member


def atom_vectors(seed: int, n_atoms: int, col_lo: int, col_hi: int) -> np.ndarray:
    """Columns [col_lo, col_hi) of the n_atoms seeded N(0,1) fp32 vectors (col_lo, col_hi multiples of COL_BLOCK or the end)."""
    assert col_lo % COL_BLOCK == 0
    out = np.empty((n_atoms, col_hi - col_lo), dtype=np.float32)
    root = np.random.SeedSequence(seed)
    for t in range(n_atoms):
        for cb in range(col_lo // COL_BLOCK, (col_hi + COL_BLOCK - 1) // COL_BLOCK):
            lo, hi = cb * COL_BLOCK, min(col_hi, (cb + 1) * COL_BLOCK)
            ss = np.random.SeedSequence(entropy=root.entropy, spawn_key=(t, cb))
            out[t, lo - col_lo:hi - col_lo] = np.random.Generator(np.random.PCG64(ss)).standard_normal(hi - lo, dtype=np.float32)
    return out
