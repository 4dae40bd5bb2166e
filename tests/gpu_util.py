"""Helpers for the GPU parity tests: upload/download and the comparison bars."""
import sys

import numpy as np
import torch

from paper_2407_02327_amd import qsync as Q

GRAN = {"tensor": Q.PER_TENSOR, "row": Q.PER_ROW, "col": Q.PER_COL}
RND = {"nearest": Q.ROUND_NEAREST, "stochastic": Q.ROUND_STOCHASTIC, "floor": Q.ROUND_FLOOR}


def say(*a):
    """Name the case before touching the GPU, so a lost box still tells which case ran."""
    print("[gpu-case]", *a, flush=True)
    sys.stdout.flush()


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def empty(shape, dtype):
    return torch.empty(shape, dtype=dtype, device="cuda")


def ws(nbytes: int):
    """Workspace for a C-ABI call: zero-filled once, as qsync_absmax_scale requires of its counters."""
    return torch.zeros(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def assert_bits_equal(got: np.ndarray, want: np.ndarray, what: str):
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if got.dtype.kind == "f":
        g = got.view({2: np.uint16, 4: np.uint32}[got.dtype.itemsize])
        w = want.astype(got.dtype).view(g.dtype)
    else:
        g, w = got, want.astype(got.dtype)
    bad = np.flatnonzero(g.reshape(-1) != w.reshape(-1))
    assert bad.size == 0, f"{what}: {bad.size} of {g.size} differ, first at flat index {bad[:5]}: " \
                          f"got {got.reshape(-1)[bad[:5]]}, want {want.reshape(-1)[bad[:5]]}"


def assert_close(got: np.ndarray, want: np.ndarray, what: str, rtol=1e-3, atol_rel=1e-3):
    """|got - want| <= rtol*|want| + atol_rel*max|want|  (the bar for FP16 and dequantized outputs)."""
    assert got.shape == want.shape, (what, got.shape, want.shape)
    g, w = got.astype(np.float64), want.astype(np.float64)
    bound = rtol * np.abs(w) + atol_rel * (np.abs(w).max() if w.size else 0.0)
    err = np.abs(g - w)
    bad = np.flatnonzero((err > bound).reshape(-1))
    assert bad.size == 0, f"{what}: {bad.size} of {g.size} outside tolerance; worst err {err.max():.3e} " \
                          f"(bound there {bound.reshape(-1)[err.argmax()]:.3e}), max|want| {np.abs(w).max():.3e}"
