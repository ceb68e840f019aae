"""Helpers shared by the GPU parity tests."""
import sys

import numpy as np


def say(msg: str) -> None:
    """Name the case before the GPU step that runs it, flushed, so a fault can be traced."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def first_mismatch(got: np.ndarray, want: np.ndarray) -> str:
    if got.shape != want.shape:
        return f"shape {got.shape} != {want.shape}"
    bad = np.argwhere(got != want)
    if bad.size == 0:
        return ""
    idx = tuple(int(v) for v in bad[0])
    return (f"{len(bad)} of {got.size} elements differ; first at {idx}: "
            f"got 0x{int(got[idx]):016x} want 0x{int(want[idx]):016x}")
