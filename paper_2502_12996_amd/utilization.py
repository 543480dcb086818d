"""Compute-utilisation calculator for overlapped communication in DiLoCo (CPU arithmetic only).

Section 3.1 of the paper ("Compute utilization simulation") and its appendix table "Simulation"
report, per training method, the bandwidth between replicas needed to keep the accelerators
computing a given fraction of the time.  The paper's figures come from a simulator that walks a
DAG of forward and backward nodes, described in a cited work and not in the paper; what the paper
itself fixes is the bookkeeping around it, and that is what this module computes in closed form:

  * how long a transfer may take before it delays computation (the "tolerated latency" of the
    table "Communication overlap", Section 3.2): nothing without overlap, one inner step with the
    1-inner-step overlap, H inner steps with naive delayed or eager outer gradients (Algorithms 2
    and 3), 2H with the two-outer-steps overlap;
  * how many bits cross the link: the parameters' worth at the wire width, every step for
    Data-Parallel, every H steps for DiLoCo (hence "H x (16 / 4) = 400x fewer bits" for H = 100 and
    float4 against 16-bit gradients, caption of the table "Overtraining");
  * compute utilisation = compute time / (compute time + communication time that nothing hides),
    and the smallest bandwidth reaching a target utilisation, exactly and on the paper's grid of
    50 log-spaced bandwidths from 0.1 to 1000 Gbit/s.

Model (this build's reading, stated where the paper is silent): one link between the replicas
carries, per exchange, `params * wire_bits * 2 (M - 1) / M` bits (ring all-reduce; 1x for the
paper's M = 2); all fragments of Streaming DiLoCo share that link, so over H steps it carries one
model's worth whatever the fragmentation; a transfer hides behind `window` seconds of computation
and only its remainder stalls the replicas.  No DAG, no overlap of a data-parallel all-reduce with
the backward pass: for the methods whose figures depend on those (Data-Parallel, un-overlapped
Streaming DiLoCo, the 1-inner-step overlap) the bandwidths printed in the paper are NOT
reproduced, and parity with them is unpinned (the closed form lands within a factor 4 of the printed
1-outer-step rows and above the rows of the methods that overlap with the backward pass); see
tests/test_utilization.py for what is pinned.

    python -m paper_2502_12996_amd.utilization            # the table for 1B / 10B / 100B
"""
from __future__ import annotations

import argparse
import math
from typing import List, Sequence

METHODS = ("dp", "diloco", "inner1", "outer1", "outer2")
CU_TARGETS = (0.50, 0.80, 0.90, 0.95, 0.99)
# Section 3.1: models of 1, 10 and 100 billion parameters with step times of 0.1, 0.8 and 4.9 s
PAPER_MODELS = (("1B", 1e9, 0.1), ("10B", 1e10, 0.8), ("100B", 1e11, 4.9))


def bandwidth_grid() -> List[float]:
    """The 50 log-spaced bandwidths from 1e-1 to 1e3 Gbit/s that every value printed in the
    appendix table lies on (Section 3.1 names the range; the count follows from the printed values)."""
    return [10.0 ** (-1.0 + 4.0 * k / 49.0) for k in range(50)]


def exchange_period(method: str, H: int) -> int:
    """Inner steps between two exchanges: 1 for Data-Parallel, H for every DiLoCo variant."""
    _check(method)
    return 1 if method == "dp" else H


def overlap_window(method: str, H: int, step_time: float) -> float:
    """Seconds of computation a transfer may hide behind (the tolerated latency)."""
    _check(method)
    return {"dp": 0.0, "diloco": 0.0, "inner1": step_time, "outer1": H * step_time,
            "outer2": 2 * H * step_time}[method]


def bits_per_exchange(params: float, wire_bits: float, replicas: int = 2) -> float:
    """Bits one link carries per exchange: a ring all-reduce of `params` values of `wire_bits` bits."""
    if replicas < 1:
        raise ValueError("replicas >= 1")
    return params * wire_bits * 2.0 * (replicas - 1) / replicas


def total_bits(method: str, params: float, steps: int, H: int, wire_bits: float, replicas: int = 2) -> float:
    """Bits exchanged over a run of `steps` inner steps."""
    return (steps // exchange_period(method, H)) * bits_per_exchange(params, wire_bits, replicas)


def compute_utilization(method: str, params: float, step_time: float, H: int, gbit_per_s: float,
                        wire_bits: float, replicas: int = 2) -> float:
    """Fraction of wall-clock time spent computing at the given bandwidth."""
    if gbit_per_s <= 0 or step_time <= 0 or H < 1:
        raise ValueError("bandwidth and step time must be positive, H >= 1")
    period = exchange_period(method, H)
    compute = period * step_time
    transfer = bits_per_exchange(params, wire_bits, replicas) / (gbit_per_s * 1e9)
    exposed = max(0.0, transfer - overlap_window(method, H, step_time))
    return compute / (compute + exposed)


def required_bandwidth(method: str, params: float, step_time: float, H: int, cu: float, wire_bits: float,
                       replicas: int = 2) -> float:
    """Smallest bandwidth in Gbit/s at which compute_utilization(...) >= cu (closed form): the
    transfer may take the overlap window plus the stall a utilisation of cu leaves room for."""
    if not 0.0 < cu <= 1.0:
        raise ValueError("0 < cu <= 1")
    period = exchange_period(method, H)
    allowed = overlap_window(method, H, step_time) + period * step_time * (1.0 / cu - 1.0)
    if allowed <= 0.0:
        return math.inf                     # no overlap and cu = 1: no finite bandwidth does it
    return bits_per_exchange(params, wire_bits, replicas) / allowed / 1e9


def on_grid(gbit_per_s: float, grid: Sequence[float] | None = None) -> float:
    """Smallest grid bandwidth >= the given one (inf beyond the grid), as the paper's table reports."""
    for w in (grid or bandwidth_grid()):
        if w >= gbit_per_s * (1.0 - 1e-12):
            return w
    return math.inf


def hours_at_bandwidth(method: str, params: float, step_time: float, H: int, steps: int, gbit_per_s: float,
                       wire_bits: float, replicas: int = 2) -> float:
    """Wall-clock hours of a run of `steps` inner steps."""
    cu = compute_utilization(method, params, step_time, H, gbit_per_s, wire_bits, replicas)
    return steps * step_time / cu / 3600.0


def _check(method: str) -> None:
    if method not in METHODS:
        raise ValueError(f"method must be one of {METHODS}")


def table(H_values=(30, 100), wire_bits_dp=16.0, wire_bits_diloco=4.0) -> List[dict]:
    rows = []
    for name, params, step in PAPER_MODELS:
        cases = [("dp", 1, wire_bits_dp), ("diloco", 100, wire_bits_dp)]
        for method in ("inner1", "outer1", "outer2"):
            cases += [(method, H, wire_bits_diloco) for H in H_values]
        for method, H, bits in cases:
            exact = [required_bandwidth(method, params, step, H, cu, bits) for cu in CU_TARGETS]
            rows.append(dict(model=name, step_time=step, method=method, H=H, wire_bits=bits,
                             gbit_per_s=exact, gbit_per_s_on_grid=[on_grid(w) for w in exact],
                             tolerated_latency_s=overlap_window(method, H, step)))
    return rows


def main() -> None:
    ap = argparse.ArgumentParser(description="Bandwidth needed for a target compute utilisation (closed form).")
    ap.add_argument("--wire-bits-dp", type=float, default=16.0)
    ap.add_argument("--wire-bits-diloco", type=float, default=4.0)
    args = ap.parse_args()
    print("model step[s] method  H   bits  tolerated latency [s]   Gbit/s for CU = " + " / ".join(f"{c:.0%}" for c in CU_TARGETS)
          + "   (exact | on the paper's 50-point grid)")
    for r in table(wire_bits_dp=args.wire_bits_dp, wire_bits_diloco=args.wire_bits_diloco):
        exact = " ".join(f"{w:9.3f}" for w in r["gbit_per_s"])
        grid = " ".join(("    inf" if math.isinf(w) else f"{w:7.1f}") for w in r["gbit_per_s_on_grid"])
        print(f"{r['model']:5s} {r['step_time']:5.1f}  {r['method']:7s} {r['H']:3d} {r['wire_bits']:5.0f} "
              f"{r['tolerated_latency_s']:12.2f}          {exact} | {grid}")


if __name__ == "__main__":
    main()
