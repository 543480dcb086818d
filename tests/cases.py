"""Seeded draws of valid argument combinations for the sweep tests.

The draws hold no arithmetic of the method; they live here (not in the GPU test module) so that a
CPU test can regenerate any case of the GPU sweeps by its (chunk, draw) coordinates.
"""
import numpy as np

EAGER_SWEEP_SEED, EAGER_SWEEP_DRAWS, EAGER_STATE_SEED = 1000, 25, 300
STANDARD_SWEEP_SEED, STANDARD_SWEEP_DRAWS, STANDARD_STATE_SEED, ADAMW_STATE_SEED = 2000, 20, 400, 500

LAUNCH_SHAPES = [(0, 0, -1), (64, 1, 2), (256, 0, 0), (128, 1, 3), (512, 0, 1)]


def random_eager_case(rng):
    M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 11, 17, 42]))
    n = int(rng.choice([1, 3, 4, 63, 64, 257, 1000, 4097, 8191, 8192, 8193, 20_001]))
    variant = str(rng.choice(["eager", "delayed"]))
    case = dict(M=M, n=n, variant=variant, apply=bool(rng.integers(0, 2)), nesterov=bool(rng.integers(0, 2)),
                bf16=bool(rng.integers(0, 2)), packed=bool(rng.integers(0, 2)), pad=int(rng.choice([0, 1, 4, 6])),
                comm=[None, "bf16", (2, 1, 11), (4, 3, 16), (5, 2, 24)][int(rng.integers(0, 5))],
                no_mean=bool(rng.integers(0, 2)) and variant == "eager",
                shape=LAUNCH_SHAPES[int(rng.integers(0, 5))],
                eta=float(rng.choice([0.7, 1.0, 0.1])), mu=float(rng.choice([0.9, 0.0, 0.5])))
    case["misalign"] = 0 if case["packed"] else int(rng.choice([0, 0, 1, 2]))
    return case


def random_standard_adamw_case(rng):
    """One standard-outer-step call and one AdamW call on the same shapes."""
    M = int(rng.choice([1, 2, 3, 4, 7, 8, 9, 12, 16, 33]))
    n = int(rng.choice([1, 3, 4, 64, 257, 4097, 8193, 20_001]))
    bf16, mis, pad = bool(rng.integers(0, 2)), int(rng.choice([0, 0, 1, 3])), int(rng.choice([0, 1, 4]))
    comm = [None, "bf16", (2, 1, 11), (4, 3, 16)][int(rng.integers(0, 4))]
    shape = LAUNCH_SHAPES[int(rng.integers(0, 5))]
    eta, mu, nest = float(rng.choice([0.7, 1.0])), float(rng.choice([0.9, 0.0])), bool(rng.integers(0, 2))
    grad_bf16 = bool(bf16 and rng.integers(0, 2))
    step = int(rng.choice([1, 2, 31, 1000]))
    return dict(M=M, n=n, bf16=bf16, misalign=mis, pad=pad, comm=comm, shape=shape, eta=eta, mu=mu,
                nesterov=nest, grad_bf16=grad_bf16, step=step)


def standard_sweep_case(chunk, draw):
    """Case `draw` of chunk `chunk` of the standard / AdamW sweep."""
    rng = np.random.default_rng(STANDARD_SWEEP_SEED + chunk)
    for _ in range(draw + 1):
        c = random_standard_adamw_case(rng)
    return c


def oracle_comm(comm):
    """Wire format of a case in the checker's spelling."""
    return "f32" if comm is None else ("bf16" if comm == "bf16" else ("exmy",) + tuple(comm))
