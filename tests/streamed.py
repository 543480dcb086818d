"""Whole-buffer parity at full size: every index of a large buffer streamed through the checker.

The path is element-wise in the parameter index, so a chunk's result does not depend on the rest
and comparing chunk after chunk is exact, not sampling.  The checker is single-threaded NumPy; to
cover 10^9 indices in tens of seconds the CHUNKS are handed to a pool of threads (NumPy and torch
release the interpreter lock inside their array loops).  The checker itself is untouched.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

CHUNK = 1 << 21          # parameter indices per chunk: a few GB of float64 temporaries per worker at M = 8


def workers():
    return max(1, min(12, (os.cpu_count() or 4) - 2))


def f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a GPU fp32 / bf16 slice to float64 on the host."""
    return t.to("cpu").to(torch.float64).numpy()


def stream_chunks(n: int, process, chunk: int = CHUNK):
    """process(lo, hi) -> {buffer: error / tolerance} for every chunk [lo, hi) of [0, n); returns the
    worst ratio per buffer and the number of indices covered.  The last chunk is ragged."""
    bounds = [(lo, min(lo + chunk, n)) for lo in range(0, n, chunk)]
    worst = {}
    covered = 0
    with ThreadPoolExecutor(max_workers=workers()) as pool:
        for (lo, hi), res in zip(bounds, pool.map(lambda b: process(*b), bounds)):
            covered += hi - lo
            for k, v in res.items():
                worst[k] = max(worst.get(k, 0.0), v)
    assert covered == n
    return worst, covered
