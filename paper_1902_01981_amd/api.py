"""ctypes binding with the names of include/codedreduce.h.

Every function marshals its arguments and calls the C-ABI entry point of the same name; all arithmetic of the
path runs in the HIP library.  Device buffers are torch tensors (their data_ptr() is passed) or raw integer
addresses.  The library must have been built (paper_1902_01981_amd/build.py); nothing here falls back to
another implementation.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcodedreduce.so")

CR_OK, CR_E_INVAL, CR_E_UNDECODABLE, CR_E_STATE, CR_E_HIP, CR_E_NOMEM = 0, -1, -2, -3, -4, -5
CR_LINEAR, CR_LOGISTIC, CR_AGGREGATE_ONLY = 0, 1, 2
CR_F32, CR_BF16 = 0, 1
CR_K_PARTIAL_GRADS, CR_K_REDUCE_PIECES, CR_K_ENCODE, CR_K_DECODE, CR_K_UPDATE, CR_K_COUNT = 0, 1, 2, 3, 4, 5
CR_PROFILE_ALL = (1 << CR_K_COUNT) - 1
CR_SPLIT_EQUAL_RANGES, CR_SPLIT_ROW_CELLS, CR_SPLIT_SHARED_CELLS = 0, 1, 2
DEFAULT_SEED = 190201981

EXPORTS = [
    "cr_plan", "cr_plan_ex", "cr_plan_destroy", "cr_plan_info", "cr_plan_get_B", "cr_plan_get_A", "cr_plan_get_segments",
    "cr_plan_decode_row", "cr_plan_set_split", "cr_plan_get_pieces", "cr_simulate_iteration", "cr_workspace_bytes", "cr_bind_workspace",
    "cr_partial_grads", "cr_load_partial_grads", "cr_encode_tree", "cr_decode_root", "cr_gd_update", "cr_gd_run", "cr_get_slab_grads",
    "cr_get_messages", "cr_profile_enable", "cr_profile_read", "cr_last_algorithmic_bytes", "cr_synchronize", "cr_last_error",
    "cr_probe_read_bandwidth", "cr_aggregate_static", "cr_profile_samples", "cr_aggregate_run",
]


class CodedReduceError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"status {status}: {message}")
        self.status = status


class cr_plan_info_t(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in ("L", "n", "s", "model", "x_dtype", "num_workers", "num_groups", "num_slabs",
                                              "num_decode_rows", "code_candidate", "num_teams", "num_pieces", "split_kind",
                                              "stage1_team_size", "stage1_teams_per_group", "stage1_staged")] + \
               [(k, ctypes.c_int64) for k in ("m", "d", "row_visits", "min_rows", "max_rows", "split_value")] + \
               [("gamma", ctypes.c_double), ("r_cr", ctypes.c_double)] + \
               [(k, ctypes.c_int32) for k in ("l2_domains", "unit_slots", "l2_sharing", "code_warning")]


_lib = None


def load_library():
    """Loads the built shared library; raises if it is missing (there is no other implementation to fall back to)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python paper_1902_01981_amd/build.py`")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, c_int = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.cr_last_error.restype = ctypes.c_char_p
        lib.cr_plan_destroy.restype = None
        lib.cr_plan.argtypes = [c_int, c_int, c_int, i64, i64, ctypes.POINTER(vp)]
        lib.cr_plan_ex.argtypes = [c_int, c_int, c_int, i64, i64, c_int, c_int, ctypes.c_uint64, vp, ctypes.POINTER(vp)]
        lib.cr_plan_destroy.argtypes = [vp]
        lib.cr_plan_info.argtypes = [vp, ctypes.POINTER(cr_plan_info_t)]
        lib.cr_plan_get_B.argtypes = [vp, vp]
        lib.cr_plan_get_A.argtypes = [vp, vp]
        lib.cr_plan_get_segments.argtypes = [vp, vp, vp, vp, vp]
        lib.cr_plan_decode_row.argtypes = [vp, vp, vp]
        lib.cr_plan_set_split.argtypes = [vp, c_int, i64]
        lib.cr_plan_get_pieces.argtypes = [vp, vp, vp, vp, vp]
        lib.cr_simulate_iteration.argtypes = [vp, ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_uint64, i64, vp, vp,
                                              ctypes.POINTER(ctypes.c_double)]
        lib.cr_workspace_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
        lib.cr_bind_workspace.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.cr_partial_grads.argtypes = [vp, vp, vp, vp]
        lib.cr_load_partial_grads.argtypes = [vp, vp]
        lib.cr_encode_tree.argtypes = [vp, vp]
        lib.cr_decode_root.argtypes = [vp, vp]
        lib.cr_gd_update.argtypes = [vp, vp, vp, ctypes.c_float]
        lib.cr_gd_run.argtypes = [vp, vp, vp, vp, vp, vp, c_int, ctypes.c_float, vp, vp]
        lib.cr_aggregate_static.argtypes = [vp, vp, vp, vp, vp]
        lib.cr_aggregate_run.argtypes = [vp, vp, i64, vp, c_int, vp, i64]
        lib.cr_get_slab_grads.argtypes = [vp, ctypes.POINTER(vp)]
        lib.cr_get_messages.argtypes = [vp, ctypes.POINTER(vp)]
        lib.cr_profile_enable.argtypes = [vp, c_int]
        lib.cr_profile_read.argtypes = [vp, c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64), ctypes.POINTER(i64)]
        lib.cr_profile_samples.argtypes = [vp, c_int, vp, i64, ctypes.POINTER(i64)]
        lib.cr_last_algorithmic_bytes.argtypes = [vp, c_int, ctypes.POINTER(i64)]
        lib.cr_synchronize.argtypes = [vp]
        lib.cr_probe_read_bandwidth.argtypes = [vp, ctypes.c_size_t, vp, c_int, vp, ctypes.POINTER(ctypes.c_double)]
        _lib = lib
    return _lib


def cr_last_error() -> str:
    return load_library().cr_last_error().decode()


def _check(status: int) -> None:
    if status != CR_OK:
        raise CodedReduceError(status, cr_last_error())


def _ptr(buf) -> int:
    """Address of a host numpy array, or an integer address passed through."""
    if buf is None:
        return 0
    if isinstance(buf, int):
        return buf
    if isinstance(buf, np.ndarray):
        return buf.ctypes.data
    raise TypeError("expected a numpy array or an integer address")


_TORCH_DTYPES = {"f32": ("torch.float32",), "x_f32": ("torch.float32",), "x_bf16": ("torch.bfloat16", "torch.int16", "torch.uint16")}


def _dev(buf, name: str, kind: str, numel: int, optional: bool = False) -> int:
    """Address of a device buffer for the argument `name`.  A torch tensor is checked (on the GPU, element type `kind`, contiguous,
    at least `numel` elements): a wrong buffer must become a Python error here, not a memory fault in a kernel.  A plain integer is
    taken to be a device address the caller vouches for."""
    if buf is None:
        if optional:
            return 0
        raise ValueError(f"{name} is required")
    if isinstance(buf, int):
        return buf
    if isinstance(buf, np.ndarray):
        raise ValueError(f"{name} must be a device buffer, not a host numpy array")
    if not getattr(buf, "is_cuda", False):
        raise ValueError(f"{name} must live on the GPU")
    if str(buf.dtype) not in _TORCH_DTYPES[kind]:
        raise ValueError(f"{name} has dtype {buf.dtype}, expected {_TORCH_DTYPES[kind][0]}")
    if not buf.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if buf.numel() < numel:
        raise ValueError(f"{name} has {buf.numel()} elements, the plan needs {numel}")
    return buf.data_ptr()


def _x_kind(info) -> str:
    return "x_bf16" if info.x_dtype == CR_BF16 else "x_f32"


# ---- plan ------------------------------------------------------------------------------------------------------------
def cr_plan(L: int, n: int, s: int, m: int, d: int) -> int:
    out = ctypes.c_void_p()
    _check(load_library().cr_plan(L, n, s, m, d, ctypes.byref(out)))
    return out.value


def cr_plan_ex(L: int, n: int, s: int, m: int, d: int, model: int = CR_LINEAR, x_dtype: int = CR_F32,
               seed: int = DEFAULT_SEED, B=None) -> int:
    out = ctypes.c_void_p()
    Bc = None if B is None else np.ascontiguousarray(B, dtype=np.float64)
    if Bc is not None and Bc.shape != (n, n):
        raise ValueError("B must be n x n")
    _check(load_library().cr_plan_ex(L, n, s, m, d, model, x_dtype, seed, _ptr(Bc), ctypes.byref(out)))
    return out.value


def cr_plan_destroy(plan: int) -> None:
    load_library().cr_plan_destroy(plan)


def cr_plan_info(plan: int) -> cr_plan_info_t:
    info = cr_plan_info_t()
    _check(load_library().cr_plan_info(plan, ctypes.byref(info)))
    return info


def cr_plan_get_B(plan: int) -> np.ndarray:
    n = cr_plan_info(plan).n
    B = np.empty((n, n), dtype=np.float64)
    _check(load_library().cr_plan_get_B(plan, B.ctypes.data))
    return B


def cr_plan_get_A(plan: int) -> np.ndarray:
    info = cr_plan_info(plan)
    A = np.empty((info.num_decode_rows, info.n), dtype=np.float64)
    _check(load_library().cr_plan_get_A(plan, A.ctypes.data))
    return A


def cr_plan_get_segments(plan: int):
    """Returns (row_begin, row_end, coef, worker), S entries each."""
    S = cr_plan_info(plan).num_slabs
    worker = np.empty(S, dtype=np.int32)
    rb, re = np.empty(S, dtype=np.int64), np.empty(S, dtype=np.int64)
    coef = np.empty(S, dtype=np.float64)
    _check(load_library().cr_plan_get_segments(plan, rb.ctypes.data, re.ctypes.data, coef.ctypes.data, worker.ctypes.data))
    return rb, re, coef, worker


def cr_plan_decode_row(plan: int, flags) -> np.ndarray:
    n = cr_plan_info(plan).n
    f = np.ascontiguousarray(flags, dtype=np.uint8)
    if f.shape != (n,):
        raise ValueError("flags must have n entries")
    a = np.empty(n, dtype=np.float64)
    _check(load_library().cr_plan_decode_row(plan, f.ctypes.data, a.ctypes.data))
    return a


def cr_plan_set_split(plan: int, kind: int, value: int) -> None:
    _check(load_library().cr_plan_set_split(plan, kind, value))


def cr_plan_get_pieces(plan: int):
    P = cr_plan_info(plan).num_pieces
    slab, team = np.empty(P, dtype=np.int32), np.empty(P, dtype=np.int32)
    rb, re = np.empty(P, dtype=np.int64), np.empty(P, dtype=np.int64)
    _check(load_library().cr_plan_get_pieces(plan, slab.ctypes.data, rb.ctypes.data, re.ctypes.data, team.ctypes.data))
    return slab, rb, re, team


def cr_simulate_iteration(plan: int, a: float, mu: float, t_c: float, seed: int, iteration: int):
    """Returns (mask uint8[N], ready float64[N], total)."""
    N = cr_plan_info(plan).num_workers
    mask = np.zeros(N, dtype=np.uint8)
    ready = np.zeros(N, dtype=np.float64)
    total = ctypes.c_double()
    _check(load_library().cr_simulate_iteration(plan, a, mu, t_c, seed, iteration, mask.ctypes.data, ready.ctypes.data, ctypes.byref(total)))
    return mask, ready, total.value


# ---- device binding and the hot path --------------------------------------------------------------------------------
def cr_workspace_bytes(plan: int) -> int:
    out = ctypes.c_size_t()
    _check(load_library().cr_workspace_bytes(plan, ctypes.byref(out)))
    return out.value


def cr_bind_workspace(plan: int, workspace, nbytes: int, stream: int = 0) -> None:
    if not isinstance(workspace, int):
        raise TypeError("workspace is a device address (see Workspace for a torch-owned block)")
    _check(load_library().cr_bind_workspace(plan, workspace, nbytes, stream))


def cr_partial_grads(plan: int, X, y, w) -> None:
    info = cr_plan_info(plan)
    _check(load_library().cr_partial_grads(plan, _dev(X, "X", _x_kind(info), info.m * info.d), _dev(y, "y", "f32", info.m),
                                           _dev(w, "w", "f32", info.d)))


def cr_load_partial_grads(plan: int, G) -> None:
    info = cr_plan_info(plan)
    _check(load_library().cr_load_partial_grads(plan, _dev(G, "G", "f32", info.num_slabs * info.d)))


def cr_encode_tree(plan: int, straggler_mask) -> None:
    mask = np.ascontiguousarray(straggler_mask, dtype=np.uint8)
    if mask.shape != (cr_plan_info(plan).num_workers,):
        raise ValueError("mask must have one byte per worker")
    _check(load_library().cr_encode_tree(plan, mask.ctypes.data))


def cr_decode_root(plan: int, g) -> None:
    _check(load_library().cr_decode_root(plan, _dev(g, "g", "f32", cr_plan_info(plan).d)))


def cr_gd_update(plan: int, w, g, lr: float) -> None:
    d = cr_plan_info(plan).d
    _check(load_library().cr_gd_update(plan, _dev(w, "w", "f32", d), _dev(g, "g", "f32", d), lr))


def cr_gd_run(plan: int, X, y, w, g, masks, lr: float, w_star=None, metrics=None) -> None:
    m = np.ascontiguousarray(masks, dtype=np.uint8)
    if m.ndim != 2 or m.shape[1] != cr_plan_info(plan).num_workers:
        raise ValueError("masks must be steps x N bytes")
    info = cr_plan_info(plan)
    _check(load_library().cr_gd_run(plan, _dev(X, "X", _x_kind(info), info.m * info.d), _dev(y, "y", "f32", info.m),
                                    _dev(w, "w", "f32", info.d), _dev(g, "g", "f32", info.d), m.ctypes.data, m.shape[0], lr,
                                    _dev(w_star, "w_star", "f32", info.d, optional=True),
                                    _dev(metrics, "metrics", "f32", 2 * m.shape[0], optional=True)))


def cr_aggregate_run(plan: int, G, masks, g, G_step_stride: int = 0, g_step_stride: int = 0) -> None:
    info = cr_plan_info(plan)
    m = np.ascontiguousarray(masks, dtype=np.uint8)
    if m.ndim != 2 or m.shape[1] != info.num_workers:
        raise ValueError("masks must be steps x N bytes")
    steps = m.shape[0]
    need_G = info.num_slabs * info.d + max(0, steps - 1) * G_step_stride
    need_g = info.d + max(0, steps - 1) * g_step_stride
    _check(load_library().cr_aggregate_run(plan, _dev(G, "G", "f32", need_G), G_step_stride, m.ctypes.data, steps,
                                           _dev(g, "g", "f32", need_g), g_step_stride))


CR_STATIC_SCRATCH_BYTES = 96 << 20


def cr_aggregate_static(plan: int, G, straggler_mask, g, stream: int = 0) -> None:
    info = cr_plan_info(plan)
    mask = np.ascontiguousarray(straggler_mask, dtype=np.uint8)
    if mask.shape != (info.num_workers,):
        raise ValueError("mask must have one byte per worker")
    _check(load_library().cr_aggregate_static(plan, _dev(G, "G", "f32", info.num_slabs * info.d), mask.ctypes.data,
                                              _dev(g, "g", "f32", info.d), stream))


def cr_get_slab_grads(plan: int) -> int:
    out = ctypes.c_void_p()
    _check(load_library().cr_get_slab_grads(plan, ctypes.byref(out)))
    return out.value


def cr_get_messages(plan: int) -> int:
    out = ctypes.c_void_p()
    _check(load_library().cr_get_messages(plan, ctypes.byref(out)))
    return out.value


def cr_profile_enable(plan: int, kernels) -> None:
    """kernels: True = all, False = none, or a mask with bit k set for kernel id k."""
    mask = (CR_PROFILE_ALL if kernels else 0) if isinstance(kernels, bool) else int(kernels)
    _check(load_library().cr_profile_enable(plan, mask))


def cr_profile_read(plan: int, kernel: int):
    ms, n, b = ctypes.c_double(), ctypes.c_int64(), ctypes.c_int64()
    _check(load_library().cr_profile_read(plan, kernel, ctypes.byref(ms), ctypes.byref(n), ctypes.byref(b)))
    return ms.value, n.value, b.value


def cr_profile_samples(plan: int, kernel: int) -> np.ndarray:
    """Milliseconds of every timed launch of one kernel id since profiling was last switched on."""
    n = ctypes.c_int64()
    _check(load_library().cr_profile_samples(plan, kernel, 0, 0, ctypes.byref(n)))
    out = np.empty(n.value, dtype=np.float32)
    if n.value:
        _check(load_library().cr_profile_samples(plan, kernel, out.ctypes.data, n.value, ctypes.byref(n)))
    return out


def cr_last_algorithmic_bytes(plan: int, kernel: int) -> int:
    b = ctypes.c_int64()
    _check(load_library().cr_last_algorithmic_bytes(plan, kernel, ctypes.byref(b)))
    return b.value


def cr_synchronize(plan: int) -> None:
    _check(load_library().cr_synchronize(plan))


def cr_probe_read_bandwidth(src, nbytes: int, sink, launches: int = 10, stream: int = 0) -> float:
    """GB/s of a plain streaming read of src[0:nbytes] (device buffers; sink holds at least 16384 floats)."""
    gbps = ctypes.c_double()
    if not isinstance(src, int) and src.numel() * src.element_size() < nbytes:
        raise ValueError("src is shorter than nbytes")
    sp = src if isinstance(src, int) else (src.data_ptr() if getattr(src, "is_cuda", False) and src.is_contiguous() else None)
    if sp is None:
        raise ValueError("src must be a contiguous device buffer")
    _check(load_library().cr_probe_read_bandwidth(sp, nbytes, _dev(sink, "sink", "f32", 16384), launches, stream, ctypes.byref(gbps)))
    return gbps.value


# ---- memory plumbing (torch owns device memory and the stream) ------------------------------------------------------
class Workspace:
    """A plan bound to a torch-owned workspace on the current device and stream.  Holds memory only; no arithmetic."""

    def __init__(self, plan: int, device="cuda"):
        import torch

        self.plan = plan
        self.info = cr_plan_info(plan)
        nbytes = cr_workspace_bytes(plan)
        self.buffer = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        base = self.buffer.data_ptr()
        self.base = (base + 255) // 256 * 256
        self.nbytes = nbytes
        self.stream = torch.cuda.current_stream().cuda_stream
        cr_bind_workspace(plan, self.base, nbytes, self.stream)
        self.info = cr_plan_info(plan)

    def _view(self, addr: int, rows: int):
        import torch

        d = self.info.d
        off = addr - self.buffer.data_ptr()
        assert 0 <= off and off + rows * d * 4 <= self.buffer.numel()
        return self.buffer[off:off + rows * d * 4].view(torch.float32).view(rows, d)

    def messages(self):
        """M[N][d] as a torch view of the workspace (rows of stragglers hold stale data)."""
        return self._view(cr_get_messages(self.plan), self.info.num_workers)

    def slab_grads(self):
        """G[S][d] as a torch view of the workspace (only when stage 1 produced them)."""
        return self._view(cr_get_slab_grads(self.plan), self.info.num_slabs)
