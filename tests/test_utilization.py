"""The compute-utilisation calculator against what the paper prints (CPU only).

Pinned to the paper: the tolerated latencies of the table "Communication overlap" (Section 3.2),
the "400x fewer bits" and the proportionality of the terabytes exchanged in the table
"Overtraining" (Section 3), the equality of its hours at 1 Gbit/s and at unlimited bandwidth for
the 1-outer-step overlap, the 1,177x / 336x quoted in Section 3.1, and the bandwidth grid every
value of the appendix table "Simulation" lies on.  PARITY UNPINNED: the bandwidths of that table
themselves: they come from a DAG simulator defined in a cited work; the closed form here lands
within a factor 4 of the 1-outer-step rows and above the rows whose methods overlap with the
backward pass, which is checked as a sanity bound, not as agreement.
"""
import math
import os

import pytest

from paper_2502_12996_amd import utilization as U

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
PARAMS = {"1B": 1e9, "10B": 1e10, "100B": 1e11}


def simulation_rows():
    rows = []
    with open(os.path.join(GOLDEN, "paper_simulation_table.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                p = line.split()
                rows.append(dict(model=p[0], step=float(p[1]), method=p[2], H=int(p[3]), gbit=[float(x) for x in p[4:]]))
    assert len(rows) == 18 and all(len(r["gbit"]) == 5 for r in rows)
    return rows


def other_rows(kind):
    out = []
    with open(os.path.join(GOLDEN, "paper_overlap_and_overtraining.txt")) as f:
        for line in f:
            if line.startswith(kind + " "):
                out.append(line.split()[1:])
    return out


def _printable(grid):
    """One-decimal renderings of the grid's points: rounded, or cut off either way (the printed table
    is not consistent about it: 86.851 appears as 86.8, 323.75 as 323.8, 2.947 as 3.0)."""
    out = set()
    for g in grid:
        out |= {round(g, 1), math.floor(g * 10) / 10, math.ceil(g * 10) / 10}
    return out


def test_every_printed_bandwidth_lies_on_the_fifty_point_grid():
    grid = U.bandwidth_grid()
    assert len(grid) == 50 and abs(grid[0] - 0.1) < 1e-15 and abs(grid[-1] - 1000.0) < 1e-9
    ok = _printable(grid)
    values = sorted({v for r in simulation_rows() for v in r["gbit"]})
    assert all(v in ok for v in values), [v for v in values if v not in ok]
    # the three-to-four-digit values fix the spacing: grids of other sizes over the range Section 3.1
    # names do not hold them
    large = [v for v in values if v > 50]
    assert len(large) >= 9
    for count in (25, 40, 45, 48, 49, 51, 52, 55, 60, 75, 101):
        other = _printable([10.0 ** (-1 + 4 * k / (count - 1)) for k in range(count)])
        assert not all(v in other for v in large), count


def test_tolerated_latency_is_the_overlap_window():
    step, H = 0.08, 30                     # the table's 500M model: one step in 0.08 s, H = 30
    for method, want in other_rows("latency"):
        assert U.overlap_window(method, H, step) == pytest.approx(float(want), rel=1e-12, abs=1e-15), method
    assert U.overlap_window("dp", H, step) == 0.0


def test_four_hundred_times_fewer_bits_and_terabytes_follow_the_token_budget():
    claims = dict((k, float(v)) for k, v in other_rows("claim"))
    H = 100
    ratio = U.total_bits("dp", 1e9, 10 * H, H, 16.0) / U.total_bits("outer1", 1e9, 10 * H, H, 4.0)
    assert ratio == claims["fewer_bits"] == H * 16 / 4
    rows = other_rows("overtrain")
    tb = {(m, int(b)): float(t) for m, b, _, _, t in rows}
    for budget in (25, 100, 250):
        assert tb[("dp", budget)] / tb[("outer1", budget)] == pytest.approx(400.0, rel=5e-3)     # printed to 3 digits
        assert tb[("inner1", budget)] == tb[("outer1", budget)]                                 # same bits, other timing
        for m in ("dp", "outer1"):
            assert tb[(m, budget)] / tb[(m, 25)] == pytest.approx(budget / 25, rel=5e-3)          # bits ~ steps ~ tokens
    assert U.total_bits("outer1", 1e9, 250, 100, 4.0) == 2 * U.bits_per_exchange(1e9, 4.0)       # whole exchanges only


def test_one_outer_step_overlap_hides_the_exchange_at_one_gbit_per_second():
    """Table "Overtraining": with the 1-outer-step overlap the hours at 1 Gbit/s equal the hours at
    unlimited bandwidth.  1B parameters in float4 are 4 Gbit per exchange; H = 100 steps of 0.1 s
    (the 1B model of Section 3.1) give 10 s to send them: utilisation 1."""
    for m, budget, h_inf, h_1g, _ in other_rows("overtrain"):
        if m == "outer1":
            assert h_inf == h_1g
    assert U.compute_utilization("outer1", 1e9, 0.1, 100, 1.0, 4.0) == 1.0
    steps = 1000
    assert U.hours_at_bandwidth("outer1", 1e9, 0.1, 100, steps, 1.0, 4.0) == pytest.approx(steps * 0.1 / 3600)
    # data-parallel at the same bandwidth spends almost all its time communicating, as the table's 109 h vs 0.67 h
    assert U.compute_utilization("dp", 1e9, 0.1, 100, 1.0, 16.0) < 0.01
    # and the one-inner-step overlap sits in between (0.88 h vs 0.67 h printed)
    cu = U.compute_utilization("inner1", 1e9, 0.1, 100, 1.0, 4.0)
    assert U.compute_utilization("dp", 1e9, 0.1, 100, 1.0, 16.0) < cu < 1.0


def test_the_ratios_quoted_in_the_text_are_those_of_the_table():
    rows = {(r["model"], r["method"], r["H"]): r["gbit"] for r in simulation_rows()}
    claims = dict((k, float(v)) for k, v in other_rows("claim"))
    dp, outer, inner = rows[("100B", "dp", 0)][4], rows[("100B", "outer1", 100)][4], rows[("100B", "inner1", 100)][4]
    assert (dp, outer, inner) == (471.5, 0.4, 1.4)
    assert abs(dp / outer - claims["ratio_outer1_vs_dp_100B"]) < 2      # 1178.75 printed as 1,177
    assert abs(dp / inner - claims["ratio_inner1_vs_dp_100B"]) < 1      # 336.8 printed as 336


@pytest.mark.parametrize("method", U.METHODS)
@pytest.mark.parametrize("H", [1, 30, 100])
def test_required_bandwidth_is_the_threshold_of_the_utilisation(method, H):
    for name, params, step in U.PAPER_MODELS:
        bits = 16.0 if method in ("dp", "diloco") else 4.0
        last = 0.0
        for cu in U.CU_TARGETS:
            w = U.required_bandwidth(method, params, step, H, cu, bits)
            assert w > 0 and w >= last                                   # more utilisation, more bandwidth
            last = w
            assert U.compute_utilization(method, params, step, H, w * (1 + 1e-9), bits) >= cu - 1e-12
            assert U.compute_utilization(method, params, step, H, w * (1 - 1e-6), bits) < cu
            # the grid search the paper's table reports: first grid bandwidth that reaches the target
            brute = next((g for g in U.bandwidth_grid()
                          if U.compute_utilization(method, params, step, H, g, bits) >= cu - 1e-12), math.inf)
            assert U.on_grid(w) == brute
    # a longer window never needs more bandwidth
    args = (1e9, 0.1, 30, 0.95, 4.0)
    need = [U.required_bandwidth(m, *args) for m in ("diloco", "inner1", "outer1", "outer2")]
    assert need == sorted(need, reverse=True)
    assert U.required_bandwidth("outer1", 1e9, 0.1, 100, 0.9, 4.0) < U.required_bandwidth("outer1", 1e9, 0.1, 30, 0.9, 4.0)


def test_worked_examples_by_hand():
    # 1B parameters, float4, H = 100, 0.1 s per step: 4 Gbit every 10 s of computation
    assert U.bits_per_exchange(1e9, 4.0) == 4e9
    assert U.bits_per_exchange(1e9, 4.0, replicas=8) == 4e9 * 2 * 7 / 8
    assert U.bits_per_exchange(1e9, 4.0, replicas=1) == 0.0
    assert U.required_bandwidth("outer1", 1e9, 0.1, 100, 1.0, 4.0) == pytest.approx(0.4)       # 4 Gbit in 10 s
    assert U.required_bandwidth("outer2", 1e9, 0.1, 100, 1.0, 4.0) == pytest.approx(0.2)       # ... in 20 s
    assert U.required_bandwidth("inner1", 1e9, 0.1, 100, 1.0, 4.0) == pytest.approx(40.0)      # ... in one step
    assert math.isinf(U.required_bandwidth("diloco", 1e9, 0.1, 100, 1.0, 4.0))
    # no overlap, 50 %: the transfer may take as long as the computation between two exchanges
    assert U.required_bandwidth("diloco", 1e9, 0.1, 100, 0.5, 16.0) == pytest.approx(16e9 / 10.0 / 1e9)
    assert U.required_bandwidth("dp", 1e9, 0.1, 100, 0.5, 16.0) == pytest.approx(160.0)
    assert U.compute_utilization("outer1", 1e9, 0.1, 100, 0.2, 4.0) == pytest.approx(10.0 / (10.0 + 10.0))
    assert U.on_grid(0.1) == pytest.approx(0.1) and math.isinf(U.on_grid(1001.0))
    for bad in (lambda: U.overlap_window("ring", 1, 1.0), lambda: U.compute_utilization("dp", 1e9, 0.1, 1, 0.0, 16.0),
                lambda: U.required_bandwidth("dp", 1e9, 0.1, 1, 0.0, 16.0), lambda: U.bits_per_exchange(1e9, 4.0, 0)):
        with pytest.raises(ValueError):
            bad()


def test_sanity_bounds_against_the_unpinned_rows_of_the_simulation_table():
    """Not agreement, only bounds (the table's own figures come from a DAG simulator that this
    closed form does not contain): the printed rows increase with the utilisation and fall with H
    as the closed form does; the closed form's 1-outer-step bandwidths are within a factor 4 of
    the printed ones; and without any overlap modelled the closed form needs at least the printed
    bandwidth for Data-Parallel and un-overlapped Streaming DiLoCo."""
    rows = simulation_rows()
    by = {(r["model"], r["method"], r["H"]): r for r in rows}
    for r in rows:
        assert r["gbit"] == sorted(r["gbit"])
        if r["H"] == 100:
            assert all(a <= b for a, b in zip(r["gbit"], by[(r["model"], r["method"], 30)]["gbit"]))
        if r["method"] == "outer1":
            assert all(a <= b for a, b in zip(r["gbit"], by[(r["model"], "inner1", r["H"])]["gbit"]))
            ours = [U.on_grid(U.required_bandwidth("outer1", PARAMS[r["model"]], r["step"], r["H"], cu, 4.0))
                    for cu in U.CU_TARGETS]
            for a, b in zip(ours, r["gbit"]):
                assert 1 / 4 <= a / b <= 4, (r["model"], r["H"], ours, r["gbit"])
        if r["method"] in ("dp", "streaming"):
            m, H = ("dp", 1) if r["method"] == "dp" else ("diloco", 100)
            ours = [U.required_bandwidth(m, PARAMS[r["model"]], r["step"], H, cu, 16.0) for cu in U.CU_TARGETS]
            assert all(a >= b * 0.99 for a, b in zip(ours, r["gbit"])), (r["model"], r["method"], ours)


def test_table_and_command_line(capsys):
    t = U.table()
    assert len(t) == 3 * 8 and all(len(r["gbit_per_s"]) == 5 for r in t)
    import sys
    argv, sys.argv = sys.argv, ["utilization"]
    try:
        U.main()
    finally:
        sys.argv = argv
    out = capsys.readouterr().out
    assert "outer1" in out and "100B" in out
