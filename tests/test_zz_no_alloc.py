"""The allocation-free loss entry point against the one that takes a workspace.

diloco_sim_quadratic_loss_static keeps its partial sums in a static device array of the library;
it must give the bits of diloco_sim_quadratic_loss on two calls in a row, the second on a smaller
input (the array then still holds the first call's partial sums beyond the second call's reach),
and must not allocate device memory.
"""
import gc

import pytest
import torch

import paper_2502_12996_amd as d
from oracle import diloco_oracle as O
from paper_2502_12996_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _problem(M, n, seed):
    h = W.log_uniform((n,), 1e-3, 1.0, tag="h", seed=seed, device=DEV)
    star = W.normal((n,), 1.0, tag="theta_star", seed=seed, device=DEV)
    theta = W.normal((M, n + 4), 0.5, tag="theta", seed=seed, device=DEV)
    return theta, h, star


def _memory_picture():
    """Device memory as the driver reports it, and torch's own requests to it (the slices of `got`
    that the calls receive are views: they allocate nothing)."""
    stats = torch.cuda.memory_stats()
    return (torch.cuda.mem_get_info()[0], torch.cuda.memory_reserved(), torch.cuda.memory_allocated(),
            stats["allocation.all.allocated"], stats["segment.all.allocated"])


def test_static_loss_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    assert torch.cuda.is_available()
    cases = [(4, (1 << 23) + 5, 11), (3, 70_001, 12)]          # 8192 partial sums, then 69
    assert d.sim_loss_workspace(cases[0][1]) == 8192 and d.sim_loss_workspace(cases[1][1]) < 100
    data = [_problem(*c) for c in cases]
    want = torch.zeros(len(cases), dtype=torch.float64, device=DEV)
    got = torch.full((len(cases),), -1.0, dtype=torch.float64, device=DEV)
    part = torch.empty(8192, dtype=torch.float64, device=DEV)
    for k, ((M, n, _), (theta, h, star)) in enumerate(zip(cases, data)):
        d.sim_quadratic_loss(theta, h, star, part, want[k:k + 1], n=n)
    torch.cuda.synchronize()
    d.sim_quadratic_loss_static(data[1][0], data[1][1], data[1][2], got[1:2], n=cases[1][1])   # first use: set-up
    torch.cuda.synchronize()
    got.fill_(-1.0)
    # Tensors of earlier tests that the collector frees in between would move torch's byte counts:
    # collect them first, keep the collector off meanwhile, and count allocation requests as well.
    gc.collect()
    gc.disable()
    try:
        before = _memory_picture()
        for k, ((M, n, _), (theta, h, star)) in enumerate(zip(cases, data)):                   # large, then small
            d.sim_quadratic_loss_static(theta, h, star, got[k:k + 1], n=n)
        torch.cuda.synchronize()
        after = _memory_picture()
    finally:
        gc.enable()
    assert before == after, "the call changed the device memory in use"
    assert torch.equal(got, want), (got, want)                                                 # same kernels: same bits
    # and against the checker, to the bar of the workspace entry point's own test
    for k, ((M, n, _), (theta, h, star)) in enumerate(zip(cases, data)):
        ref = O.quadratic_loss(O.mean_over_replicas(W.to_f64(theta[:, :n])), W.to_f64(h), W.to_f64(star))
        assert abs(got[k].item() - ref) <= 1e-12 * ref
    # a single vector, and the size limit
    one = torch.zeros(1, dtype=torch.float64, device=DEV)
    two = torch.zeros(1, dtype=torch.float64, device=DEV)
    theta, h, star = data[1]
    d.sim_quadratic_loss_static(theta[0, :1000].contiguous(), h[:1000], star[:1000], one)
    d.sim_quadratic_loss(theta[0, :1000].contiguous(), h[:1000], star[:1000], part, two)
    torch.cuda.synchronize()
    assert torch.equal(one, two)
    rc = d.binding.lib().diloco_sim_quadratic_loss_static(theta.data_ptr(), 1, (1 << 40) + 1, (1 << 40) + 1,
                                                          h.data_ptr(), star.data_ptr(), one.data_ptr(), None)
    assert rc == d.binding.ERR_SHAPE
