"""Shared helpers of the parity tests: the error metric and its tolerances."""
import numpy as np

# fp32 buffers: max relative error 1e-6; bf16 buffers: 4e-3 (one bf16 ulp is 2^-8 = 3.9e-3
# relative, round-to-nearest-even costs at most half of it).
TOL_F32 = 1e-6
TOL_BF16 = 4e-3


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max_i |got_i - want_i| / (|want_i| + rms(want)).

    Plain relative error is undefined where the exact result passes through zero (a mean of
    sign-random outer gradients does, somewhere in 10^9 elements); the rms of the buffer is
    the floor.  For a buffer of one magnitude this is within a factor 2 of max relative error.
    """
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    assert np.isfinite(got).all(), "non-finite values in the result"
    rms = float(np.sqrt(np.mean(want * want)))
    if rms == 0.0:
        return float(np.max(np.abs(got - want)))
    return float(np.max(np.abs(got - want) / (np.abs(want) + rms)))


def assert_close(got, want, tol, what=""):
    e = rel_err(got, want)
    assert e <= tol, f"{what}: error {e:.3e} above tolerance {tol:.1e}"
    return e
