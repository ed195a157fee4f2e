"""Helpers shared by the GPU parity tests (device upload, tolerance checks)."""
import numpy as np
import torch

import os
import sys
import time

F32_TOL = 1e-4      # fp32 paths: relative error bound stated for the build
BF16_TOL = 2e-2     # paths with bf16 inputs


def dev(a: np.ndarray, dtype: str = "f32") -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    if dtype == "bf16":
        t = t.to(torch.bfloat16)        # exact: the values already lie on the bf16 grid
    return t.contiguous()


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got: np.ndarray, ref: np.ndarray):
    """(||got-ref||_2 / ||ref||_2, max|got-ref| / max|ref|) -- element-wise ratios are
    meaningless near zero crossings, so closeness is judged per tensor."""
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all()
    nref = np.linalg.norm(ref)
    mref = np.abs(ref).max() if ref.size else 0.0
    if nref == 0.0:
        return float(np.linalg.norm(got - ref)), float(np.abs(got - ref).max() if got.size else 0.0)
    return float(np.linalg.norm(got - ref) / nref), float(np.abs(got - ref).max() / mref)


def assert_close(got, ref, tol, what=""):
    l2, mx = rel_err(got, ref)
    assert l2 <= tol and mx <= tol, f"{what}: rel l2 {l2:.3e}, rel max {mx:.3e} > {tol:.1e}"
    return l2, mx


_PROGRESS = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")


def progress(msg: str):
    """A line of progress from a long test: printed, and appended to test_progress.log in the run's output folder
    when that folder exists (output of a passing test is captured, a file is visible while the test still runs)."""
    line = f"[{time.strftime('%H:%M:%S')}] {msg}"
    print(line, flush=True)
    if os.path.isdir(_PROGRESS):
        with open(os.path.join(_PROGRESS, "test_progress.log"), "a") as f:
            f.write(line + "\n")
