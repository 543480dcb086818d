"""Writes tests/golden/checker_trajectories.txt from the CPU checker alone.

The file freezes what the checker computes today on a few tiny seeded runs (hexadecimal floats,
so the comparison is exact).  It pins nothing to the paper: its purpose is that a later change to
the checker's arithmetic cannot go unnoticed (tests/test_oracle_pins.py compares), and has to be
made on purpose, by re-running this script and saying in the commit which passage of the paper
justifies it.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import diloco_oracle as O  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "checker_trajectories.txt")


def runs():
    """name -> flat float64 array; every input is drawn from numpy's PCG64 with a fixed seed."""
    out = {}
    for variant in ("standard", "eager", "delayed"):
        rng = np.random.default_rng(20250218)
        M, n, H, phases = 3, 5, 2, 3
        a0 = rng.standard_normal(n) * 0.02
        theta = np.tile(a0, (M, 1))
        m1, m2 = np.zeros((M, n)), np.zeros((M, n))
        a = a0.copy() if variant == "standard" else np.tile(a0, (M, 1))
        u = np.zeros_like(a)
        P, D = np.zeros((M, n)), np.zeros(n)
        t = 0
        for k in range(phases):
            for _ in range(H):
                t += 1
                g = rng.standard_normal((M, n)) * 1e-2
                O.adamw_step(theta, m1, m2, g, t, 4e-4, 0.9, 0.95, 1e-8, 0.1)
            if variant == "standard":
                O.outer_standard(theta, a, u, 0.7, 0.9, True)
            elif variant == "eager":
                O.outer_eager(theta, a, u, P, D, 0.7, 0.9, True, k > 0, comm="bf16" if k == 2 else "f32")
            else:
                O.outer_delayed(theta, a, u, P, D, 0.7, 0.9, True, k > 0)
        out[f"{variant}.theta"] = theta.ravel()
        out[f"{variant}.outer"] = np.ravel(a)
        out[f"{variant}.velocity"] = np.ravel(u)
        out[f"{variant}.m2"] = m2.ravel()
        if variant != "standard":
            out[f"{variant}.prev_local"] = P.ravel()
            out[f"{variant}.prev_mean"] = D.ravel()
    x = np.float32([0.3, -1.26, 2.5, 1e-4, 7.0, 0.7499999, 0.75])
    out["exmy.e2m1_bias1"] = O.round_to_exmy(x, 2, 1, 1)
    out["exmy.e4m3_bias7"] = O.round_to_exmy(x, 4, 3, 7)
    out["bf16"] = O.round_to_bf16(x)
    idx = np.arange(6, dtype=np.int64)
    out["noise.seed7_step3_replica1"] = O.standard_normal(7, 3, 1, idx)
    ref, losses = O.run_quadratic("eager", 2, 3, 3, np.float64([0.5, 0.1, 1.0, 0.01]),
                                  np.float64([1.0, -1.0, 0.5, 2.0]), 11, 0.1, 1e-2, 0.9, 0.95, 1e-8, 0.0,
                                  0.7, 0.9)
    out["quadratic.eager.losses"] = np.float64(losses)
    out["quadratic.eager.theta"] = ref["theta"].ravel()
    return out


def render():
    lines = ["# written by tests/golden/make_golden.py from oracle/diloco_oracle.py alone; hexadecimal float64"]
    for name, arr in runs().items():
        lines.append(name + " " + " ".join(float(v).hex() for v in np.asarray(arr, dtype=np.float64)))
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    with open(OUT, "w") as f:
        f.write(render())
    print("wrote", OUT)
