"""Helpers shared by the GPU parity tests (comparison metrics and small fixtures)."""
import os
import time

import numpy as np
import torch

TOL = 1e-4  # max relative error for fp32 outputs and gradients

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def progress(msg: str):
    """A progress line of a long test: printed, and appended to gpurun_out/test_progress.log when that folder
    exists (pytest holds printed output back until the test ends; a run that stays silent for minutes looks hung)."""
    line = f"[{time.strftime('%H:%M:%S')}] {msg}"
    print(line, flush=True)
    d = os.path.join(_ROOT, "gpurun_out")
    if os.path.isdir(d):
        try:
            with open(os.path.join(d, "test_progress.log"), "a") as f:
                f.write(line + "\n")
        except OSError:
            pass


def rel_err(got, want) -> float:
    """Normwise max error: max|got - want| / max|want| (the stated parity bar's denominator)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    denom = float(np.max(np.abs(want)))
    return float(np.max(np.abs(got - want))) / (denom if denom > 0 else 1.0)


def assert_close(got, want, what: str, tol: float = TOL):
    e = rel_err(got, want)
    assert np.all(np.isfinite(np.asarray(got))), f"{what}: non-finite values"
    assert e <= tol, f"{what}: max relative error {e:.3e} > {tol:.1e}"
    return e


def dev(a, dtype=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(a)).to(device="cuda", dtype=dtype)


def padded(a: np.ndarray, ld: int) -> torch.Tensor:
    """Device copy of a 2-D array with leading dimension ld; returns the n x w view."""
    n, w = a.shape
    buf = torch.zeros((n, ld), dtype=torch.float32, device="cuda")
    buf[:, :w] = torch.as_tensor(a, dtype=torch.float32)
    return buf[:, :w]


def messy_edges(n, m, rng):
    """Directed pairs with repeats, both orientations and self pairs mixed in."""
    src = rng.integers(0, n, size=m)
    dst = rng.integers(0, n, size=m)
    rep = rng.integers(0, max(m, 1), size=m // 3)
    src = np.concatenate([src, src[rep], dst[rep][: m // 6], np.arange(min(n, 5))])
    dst = np.concatenate([dst, dst[rep], src[rep][: m // 6], np.arange(min(n, 5))])
    return src.astype(np.int64), dst.astype(np.int64)


def hub_edges(n, m, hubs, hub_deg, rng):
    """Random pairs plus a few very high-degree vertices (rows longer than one segment)."""
    src, dst = messy_edges(n, m, rng)
    hs, hd = [], []
    for h in hubs:
        nb = rng.choice(n, size=min(hub_deg, n - 1), replace=False)
        hs.append(np.full(nb.size, h)); hd.append(nb)
    return np.concatenate([src] + hs).astype(np.int64), np.concatenate([dst] + hd).astype(np.int64)


def unpack_mask(words: np.ndarray, w_out: int) -> np.ndarray:
    """n x mask_words int32 -> n x w_out 0/1."""
    u = words.astype(np.uint32)
    cols = np.arange(w_out)
    return ((u[:, cols // 32] >> (cols % 32).astype(np.uint32)) & 1).astype(np.uint8)


def pack_mask(bits: np.ndarray) -> np.ndarray:
    n, w = bits.shape
    mw = (w + 31) // 32
    out = np.zeros((n, mw), dtype=np.uint32)
    for j in range(w):
        out[:, j // 32] |= (bits[:, j].astype(np.uint32) & 1) << np.uint32(j % 32)
    return out.view(np.int32)
