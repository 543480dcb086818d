"""Pins of the CPU checker against what the paper and the mathematics fix.

None of these tests re-types the checker's own formulas: they use closed
forms, torch.optim.SGD / torch.optim.AdamW in float64 as black boxes, the
paper's second way of writing the eager combination (Section 2.3: the mean of
the fresh local and all stale non-local outer gradients), reductions the
listings imply (M = 1, identical replicas, stationary outer gradients), and
published generator outputs.
"""
import math
import os

import numpy as np
import pytest
import torch
from scipy import stats

from oracle import diloco_oracle as O

RNG = np.random.default_rng(20250212996)


def rnd(*shape, scale=1.0):
    return RNG.standard_normal(shape) * scale


# ----------------------------------------------------------------- AdamW ---
def test_adamw_constant_gradient_closed_form():
    # constant g != 0 from zero moments: m1_hat = g and m2_hat = g^2 at every t, so
    # theta_t = theta_{t-1} (1 - lr wd) - lr g / (|g| + eps)
    lr, b1, b2, eps, wd = 4e-4, 0.9, 0.95, 1e-8, 0.1
    g = np.array([0.3, -2.0, 1e-3, 7.0])
    th = np.array([0.5, -0.25, 1.0, 0.0])
    m1 = np.zeros(4)
    m2 = np.zeros(4)
    want = th.copy()
    for t in range(1, 40):
        O.adamw_step(th, m1, m2, g, t, lr, b1, b2, eps, wd)
        want = want * (1 - lr * wd) - lr * g / (np.abs(g) + eps)
        np.testing.assert_allclose(th, want, rtol=1e-12, atol=1e-15)


def test_adamw_first_step_is_sign_step():
    lr = 1e-2
    g = np.array([5.0, -1e-4, 3.0])
    th = np.array([1.0, 2.0, -3.0])
    th0 = th.copy()
    O.adamw_step(th, np.zeros(3), np.zeros(3), g, 1, lr, 0.9, 0.999, 1e-12, 0.05)
    np.testing.assert_allclose(th, th0 - lr * (np.sign(g) + 0.05 * th0), rtol=1e-7)


def test_adamw_zero_gradient_no_decay_is_identity():
    th = rnd(5)
    th0 = th.copy()
    O.adamw_step(th, np.zeros(5), np.zeros(5), np.zeros(5), 3, 1e-3, 0.9, 0.95, 1e-8, 0.0)
    np.testing.assert_array_equal(th, th0)


@pytest.mark.parametrize("wd", [0.0, 0.1])
def test_adamw_trajectory_matches_torch_adamw(wd):
    lr, b1, b2, eps = 4e-4, 0.9, 0.95, 1e-8
    n, T = 17, 25
    th0 = rnd(n, scale=0.02)
    p = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    th, m1, m2 = th0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, T + 1):
        g = rnd(n, scale=1e-2)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        O.adamw_step(th, m1, m2, g, t, lr, b1, b2, eps, wd)
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-11, atol=1e-16)
    st = opt.state[p]
    np.testing.assert_allclose(m1, st["exp_avg"].numpy(), rtol=1e-12)
    np.testing.assert_allclose(m2, st["exp_avg_sq"].numpy(), rtol=1e-12)


# -------------------------------------------------------------- Nesterov ---
def test_nesterov_constant_gradient_closed_form():
    eta, mu = 0.7, 0.9
    G = np.array([0.3, -1.5])
    a0 = np.array([1.0, 2.0])
    a, u = a0.copy(), np.zeros(2)
    for k in range(1, 30):
        O.nesterov_step(a, u, G, eta, mu, True)
        uk = G * (1 - mu ** k) / (1 - mu)
        # sum_{j<=k} (G + mu u_j) = G [k + mu/(1-mu) (k - mu (1 - mu^k)/(1-mu))]
        ak = a0 - eta * G * (k + mu / (1 - mu) * (k - mu * (1 - mu ** k) / (1 - mu)))
        np.testing.assert_allclose(u, uk, rtol=1e-12)
        np.testing.assert_allclose(a, ak, rtol=1e-12)


def test_zero_momentum_is_plain_sgd():
    for nesterov in (True, False):
        a, u = np.array([1.0, -2.0]), np.array([0.0, 0.0])
        G = np.array([0.5, 0.25])
        O.nesterov_step(a, u, G, 0.4, 0.0, nesterov)
        np.testing.assert_allclose(a, [1.0 - 0.2, -2.0 - 0.1], rtol=1e-15)


@pytest.mark.parametrize("nesterov", [True, False])
def test_outer_optimizer_matches_torch_sgd(nesterov):
    eta, mu, n = 0.7, 0.9, 11
    a0 = rnd(n)
    p = torch.nn.Parameter(torch.tensor(a0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=eta, momentum=mu, nesterov=nesterov)
    a, u = a0.copy(), np.zeros(n)
    for _ in range(12):
        G = rnd(n, scale=1e-3)
        p.grad = torch.tensor(G, dtype=torch.float64)
        opt.step()
        O.nesterov_step(a, u, G, eta, mu, nesterov)
        np.testing.assert_allclose(a, p.detach().numpy(), rtol=1e-12, atol=1e-16)


def test_velocity_form_equals_lookahead_form_for_constant_lr():
    # Sutskever et al. form with w = -eta u: w <- mu w - eta G ; a <- a + mu w - eta G
    eta, mu, n = 0.4, 0.9, 6
    a, u = rnd(n), np.zeros(n)
    a2, w = a.copy(), np.zeros(n)
    for _ in range(9):
        G = rnd(n)
        O.nesterov_step(a, u, G, eta, mu, True)
        w = mu * w - eta * G
        a2 = a2 + mu * w - eta * G
        np.testing.assert_allclose(a, a2, rtol=1e-11, atol=1e-13)


# ------------------------------------------------- Algorithm 1 (standard) ---
def test_standard_momentum_off_lr_one_gives_replica_average():
    M, n = 5, 9
    a, u = rnd(n), rnd(n)     # any stale velocity is wiped by mu = 0
    theta = rnd(M, n)
    want = theta.mean(axis=0)
    O.outer_standard(theta, a, u, 1.0, 0.0, True)
    np.testing.assert_allclose(a, want, rtol=1e-13, atol=1e-15)
    for m in range(M):
        np.testing.assert_array_equal(theta[m], a)


def test_standard_trajectory_matches_torch_sgd_on_outer_params():
    # outer gradient written as a - mean_m(theta_m): same real number, other route
    M, n, eta, mu = 3, 8, 0.7, 0.9
    a0 = rnd(n, scale=0.02)
    p = torch.nn.Parameter(torch.tensor(a0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=eta, momentum=mu, nesterov=True)
    a, u = a0.copy(), np.zeros(n)
    theta = np.tile(a, (M, 1))
    for _ in range(7):
        theta += rnd(M, n, scale=1e-3)             # stands in for the inner phase
        p.grad = p.detach() - torch.tensor(theta.mean(axis=0))
        ret = O.outer_standard(theta, a, u, eta, mu, True)
        np.testing.assert_allclose(ret, p.grad.numpy(), rtol=1e-9, atol=1e-15)
        opt.step()
        np.testing.assert_allclose(a, p.detach().numpy(), rtol=1e-11, atol=1e-15)
        np.testing.assert_array_equal(theta, np.tile(a, (M, 1)))


# ---------------------------------------------------- Algorithm 3 (eager) ---
@pytest.mark.parametrize("M", [1, 2, 3, 5, 8])
def test_eager_combination_equals_mean_of_fresh_local_and_stale_others(M):
    n = 7
    delta = rnd(M, n)
    P = rnd(M, n)
    D = P.mean(axis=0)          # what the all-reduce of the previous phase delivered
    G = O.eager_combination(delta, P, D)
    for m in range(M):
        others = sum(P[k] for k in range(M) if k != m) if M > 1 else 0.0
        np.testing.assert_allclose(G[m], (delta[m] + others) / M, rtol=1e-12, atol=1e-14)
    # mean over replicas: fresh mean / M + (1 - 1/M) stale mean
    np.testing.assert_allclose(G.mean(axis=0), delta.mean(axis=0) / M + (1 - 1 / M) * D,
                               rtol=1e-12, atol=1e-14)


def test_eager_with_stationary_outer_gradients_feeds_the_stale_mean():
    M, n = 4, 5
    P = rnd(M, n)
    D = rnd(n)
    G = O.eager_combination(P.copy(), P, D)
    np.testing.assert_array_equal(G, np.tile(D, (M, 1)))


def test_single_replica_eager_call_equals_standard_call():
    n = 10
    a1 = rnd(n)
    u1 = rnd(n, scale=1e-3)
    th = a1 - rnd(n, scale=1e-3)
    # standard
    ths, as_, us = th[None].copy(), a1.copy(), u1.copy()
    O.outer_standard(ths, as_, us, 0.7, 0.9, True)
    # eager with M = 1: stored previous mean must be the stored previous local gradient
    P = rnd(1, n, scale=1e-3)
    D = P[0].copy()
    the, ae, ue = th[None].copy(), a1[None].copy(), u1[None].copy()
    O.outer_eager(the, ae, ue, P, D, 0.7, 0.9, True, apply_update=True)
    np.testing.assert_allclose(ae[0], as_, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(ue[0], us, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(the[0], ths[0], rtol=1e-13, atol=1e-16)


@pytest.mark.parametrize("stationary", [False, True])
def test_identical_replicas_stay_identical_and_local_gradient_is_the_mean(stationary):
    """Equal replicas: Delta_m equals the mean, every replica makes the same step, and the
    gradient it feeds OuterOpt is (Delta + (M-1) stale) / M, which is the standard step
    when the outer gradient did not change since the previous phase."""
    M, n, eta, mu = 4, 6, 0.7, 0.9
    a0 = rnd(n)
    th_row = a0 - rnd(n, scale=1e-3)
    Prow = (a0 - th_row) if stationary else rnd(n, scale=1e-3)
    urow = rnd(n, scale=1e-3)
    theta = np.tile(th_row, (M, 1))
    a, u, P = np.tile(a0, (M, 1)), np.tile(urow, (M, 1)), np.tile(Prow, (M, 1))
    D = Prow.copy()
    O.outer_eager(theta, a, u, P, D, eta, mu, True, True)
    p = torch.nn.Parameter(torch.tensor(a0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=eta, momentum=mu, nesterov=True)
    opt.state[p]["momentum_buffer"] = torch.tensor(urow, dtype=torch.float64)
    p.grad = torch.tensor(((a0 - th_row) + (M - 1) * Prow) / M)
    opt.step()
    for m in range(M):
        np.testing.assert_allclose(a[m], p.detach().numpy(), rtol=1e-12, atol=1e-16)
        np.testing.assert_array_equal(a[m], a[0])
        np.testing.assert_array_equal(theta[m], a[m])
        np.testing.assert_allclose(P[m], D, rtol=1e-13)       # Delta_m is the mean
    np.testing.assert_allclose(D, a0 - th_row, rtol=1e-12)
    if stationary:
        ths, as_, us = np.tile(th_row, (M, 1)), a0.copy(), urow.copy()
        O.outer_standard(ths, as_, us, eta, mu, True)
        np.testing.assert_allclose(a[0], as_, rtol=1e-12, atol=1e-16)
        np.testing.assert_allclose(u[0], us, rtol=1e-12, atol=1e-16)


def _torch_replicas(a0, M, eta, mu):
    ps = [torch.nn.Parameter(torch.tensor(a0, dtype=torch.float64)) for _ in range(M)]
    return ps, [torch.optim.SGD([p], lr=eta, momentum=mu, nesterov=True) for p in ps]


@pytest.mark.parametrize("variant", ["eager", "delayed"])
def test_multi_phase_trajectory_by_brute_force(variant):
    """Element-by-element Python re-computation of Algorithms 2 and 3 over several phases:
    per-replica torch SGD instances as OuterOpt, Python lists as the message in flight,
    and the paper's second form of the eager gradient."""
    M, n, eta, mu, phases = 3, 4, 0.7, 0.9, 5
    a0 = rnd(n, scale=0.02)
    ps, opts = _torch_replicas(a0, M, eta, mu)
    theta = np.tile(a0, (M, 1))
    a, u, P, D = np.tile(a0, (M, 1)), np.zeros((M, n)), np.zeros((M, n)), np.zeros(n)
    prev_locals = None          # Delta_m^(t-H) as each replica remembers it
    live = [a0.copy() for _ in range(M)]
    anchors = [a0.copy() for _ in range(M)]
    for k in range(1, phases + 1):
        drift = rnd(M, n, scale=1e-3)
        theta += drift
        for m in range(M):
            live[m] = live[m] + drift[m]
        # ---- brute force
        locals_now = [[anchors[m][i] - live[m][i] for i in range(n)] for m in range(M)]
        if k > 1:
            for m in range(M):
                g = []
                for i in range(n):
                    stale_mean = sum(prev_locals[q][i] for q in range(M)) / M
                    if variant == "eager":
                        g.append((locals_now[m][i]
                                  + sum(prev_locals[q][i] for q in range(M) if q != m)) / M)
                    else:
                        g.append(stale_mean)
                ps[m].grad = torch.tensor(g, dtype=torch.float64)
                opts[m].step()
                anchors[m] = ps[m].detach().numpy().copy()
        else:
            # t = H: no outer step; the replica carries on from where it is
            for m in range(M):
                anchors[m] = live[m].copy()
                with torch.no_grad():
                    ps[m].copy_(torch.tensor(live[m]))
        for m in range(M):
            live[m] = anchors[m].copy()
        prev_locals = locals_now
        # ---- checker
        fn = O.outer_eager if variant == "eager" else O.outer_delayed
        fn(theta, a, u, P, D, eta, mu, True, apply_update=(k > 1))
        for m in range(M):
            np.testing.assert_allclose(a[m], anchors[m], rtol=1e-10, atol=1e-15)
            np.testing.assert_allclose(theta[m], live[m], rtol=1e-10, atol=1e-15)
            np.testing.assert_allclose(P[m], locals_now[m], rtol=1e-10, atol=1e-15)
        np.testing.assert_allclose(D, np.mean(np.array(locals_now), axis=0), rtol=1e-10,
                                   atol=1e-15)
    # replicas really did diverge under eager updates (Section 2.2, first remark)
    if variant == "eager":
        assert np.max(np.abs(a[0] - a[1])) > 0


def test_delayed_is_nesterov_on_the_shifted_mean_sequence():
    M, n, eta, mu = 2, 5, 0.7, 0.9
    a0 = rnd(n, scale=0.02)
    theta = np.tile(a0, (M, 1))
    a, u, P, D = np.tile(a0, (M, 1)), np.zeros((M, n)), np.zeros((M, n)), np.zeros(n)
    means = []
    applied = []
    for k in range(1, 7):
        theta += rnd(M, n, scale=1e-3)
        means.append((a - theta).mean(axis=0))
        a_before = a.copy()
        O.outer_delayed(theta, a, u, P, D, eta, mu, True, apply_update=(k > 1))
        if k > 1:
            applied.append(means[k - 2])
            # replay a hand-rolled optimizer on worker 0 over the shifted sequence
            # one step with the right velocity: rebuild it from the applied history
            vel = np.zeros(n)
            for G in applied[:-1]:
                vel = mu * vel + G
            vel_new = mu * vel + applied[-1]
            want = a_before[0] - eta * (applied[-1] + mu * vel_new)
            np.testing.assert_allclose(a[0], want, rtol=1e-11, atol=1e-15)
        np.testing.assert_allclose(D, means[-1], rtol=1e-12, atol=1e-16)


def test_first_boundary_applies_no_outer_step():
    M, n = 3, 4
    a0 = rnd(n)
    theta = np.tile(a0, (M, 1)) + rnd(M, n, scale=1e-3)
    th_before = theta.copy()
    for fn in (O.outer_eager, O.outer_delayed):
        th = theta.copy()
        a, u, P, D = np.tile(a0, (M, 1)), np.zeros((M, n)), rnd(M, n), rnd(n)
        fn(th, a, u, P, D, 0.7, 0.9, True, apply_update=False)
        np.testing.assert_array_equal(th, th_before)      # replicas untouched
        np.testing.assert_array_equal(a, th_before)       # and they are the next anchors
        np.testing.assert_array_equal(u, 0.0)
        np.testing.assert_allclose(P, a0 - th_before, rtol=1e-13)
        np.testing.assert_allclose(D, (a0 - th_before).mean(axis=0), rtol=1e-12, atol=1e-16)


def test_reset_is_idempotent_and_broadcasts():
    theta = rnd(3, 5)
    a = rnd(5)
    O.reset(theta, a)
    O.reset(theta, a)
    np.testing.assert_array_equal(theta, np.tile(a, (3, 1)))


# -------------------------------------------------- noise and quadratic ---
def test_mix64_matches_published_splitmix64_outputs(golden_dir):
    with open(os.path.join(golden_dir, "splitmix64_seed0.txt")) as f:
        want = [int(l, 16) for l in f if l.strip() and not l.startswith("#")]
    golden = 0x9E3779B97F4A7C15
    got = [int(O.mix64(np.uint64((k * golden) % (1 << 64)))) for k in (1, 2, 3)]
    assert got == want


def test_noise_is_standard_normal_and_streams_are_independent():
    idx = np.arange(200_000)
    z = O.standard_normal(123, 7, 2, idx)
    assert abs(z.mean()) < 0.01 and abs(z.var() - 1.0) < 0.01
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert abs(stats.kurtosis(z)) < 0.05
    # pairs share the radius: z_2j^2 + z_2j+1^2 = -2 ln u1 ~ Exponential(mean 2)
    r2 = z[0::2] ** 2 + z[1::2] ** 2
    assert stats.kstest(r2, "expon", args=(0, 2.0)).pvalue > 1e-3
    # the angle is uniform
    ang = np.arctan2(z[1::2], z[0::2])
    assert stats.kstest((ang + np.pi) / (2 * np.pi), "uniform").pvalue > 1e-3
    for other in (O.standard_normal(123, 8, 2, idx), O.standard_normal(123, 7, 3, idx),
                  O.standard_normal(124, 7, 2, idx)):
        assert abs(np.corrcoef(z, other)[0, 1]) < 0.01
    # a pure function of the coordinates: any slice can be regenerated on its own
    np.testing.assert_array_equal(O.standard_normal(123, 7, 2, idx[1001:1500]), z[1001:1500])
    # serial correlation
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 0.01


def _z_by_hand(seed, t, m, i):
    """z(seed, t, m, i) with Python integers and the math module only, one statement per clause of the
    generator's definition in include/diloco_sim.h (no NumPy, no code shared with the checker)."""
    mask = (1 << 64) - 1
    G = 0x9E3779B97F4A7C15                                    # "the same odd constant"

    def mix64(x):                                             # splitmix64's output function
        x ^= x >> 30
        x = (x * 0xBF58476D1CE4E5B9) & mask
        x ^= x >> 27
        x = (x * 0x94D049BB133111EB) & mask
        x ^= x >> 31
        return x
    key = mix64((mix64((seed + (t + 1) * G) & mask) + (m + 1) * G) & mask)   # key = mix64(mix64(seed + (t+1) G) + (m+1) G)
    j = i // 2                                                # elements 2j and 2j+1 share one word
    x = mix64((key + (j + 1) * G) & mask)                     # x = mix64(key + (j+1) G)
    u1 = ((x >> 40) + 1) / 2 ** 24                            # top 24 bits, in (0, 1]
    u2 = ((x >> 16) & 0xFFFFFF) / 2 ** 24                     # next 24 bits, in [0, 1)
    r = math.sqrt(-2.0 * math.log(u1))
    return r * math.cos(2.0 * math.pi * u2) if i % 2 == 0 else r * math.sin(2.0 * math.pi * u2)


def test_noise_matches_a_hand_computation_of_its_definition():
    """A few coordinates, including the first and an odd index, a large step, a large index and a seed
    that uses all 64 bits, against the definition evaluated with Python integers."""
    cases = [(0, 0, 0, 0), (0, 0, 0, 1), (123, 7, 2, 1001), (0x5EEDD110C0, 2000, 3, (1 << 26) - 1),
             (0xFEDCBA9876543210, 1, 65534, (1 << 33) + 4), (1, 31, 0, 2), (1, 31, 0, 3)]
    for seed, t, m, i in cases:
        got = float(O.standard_normal(seed, t, m, np.array([i]))[0])
        want = _z_by_hand(seed, t, m, i)
        assert abs(got - want) <= 1e-12 * max(1.0, abs(want)), (seed, t, m, i, got, want)
    # both members of a pair come from one word: same radius
    a, b = _z_by_hand(9, 4, 1, 10), _z_by_hand(9, 4, 1, 11)
    pair = O.standard_normal(9, 4, 1, np.array([10, 11]))
    assert abs((pair[0] ** 2 + pair[1] ** 2) - (a * a + b * b)) < 1e-12


def test_noise_radius_and_angle_come_from_disjoint_bits():
    """Radius and angle are recovered from the normals as 24-bit integers (exactly: float64 leaves
    eight decimal digits to spare).  Every one of the 48 bits is balanced and no bit of the radius field
    correlates with a bit of the angle field; fields that overlap, or a field used twice, would give
    correlations of +-1 on the shared bits."""
    n = 1 << 17
    z = O.standard_normal(77, 3, 1, np.arange(2 * n))
    r2 = z[0::2] ** 2 + z[1::2] ** 2
    k1 = np.rint(np.exp(-r2 / 2.0) * 2.0 ** 24).astype(np.int64) - 1              # (x >> 40)
    k2 = np.rint((np.arctan2(z[1::2], z[0::2]) / (2 * np.pi)) % 1.0 * 2.0 ** 24).astype(np.int64) % (1 << 24)
    assert k1.min() >= 0 and k1.max() < (1 << 24) and k2.min() >= 0
    # the recovery is exact: regenerating the normals from the integers gives them back
    r = np.sqrt(-2.0 * np.log((k1 + 1) / 2.0 ** 24))
    np.testing.assert_allclose(r * np.cos(2 * np.pi * k2 / 2.0 ** 24), z[0::2], rtol=0, atol=1e-9)
    b1 = ((k1[:, None] >> np.arange(24)) & 1).astype(np.float64)
    b2 = ((k2[:, None] >> np.arange(24)) & 1).astype(np.float64)
    tol = 5.0 / np.sqrt(n)                                                        # five sigma
    assert np.max(np.abs(b1.mean(axis=0) - 0.5)) < tol and np.max(np.abs(b2.mean(axis=0) - 0.5)) < tol
    c = ((b1 - 0.5).T @ (b2 - 0.5)) / n * 4.0                                     # 24 x 24 bit correlations
    assert np.max(np.abs(c)) < 1.2 * tol * 2, float(np.max(np.abs(c)))
    within1 = ((b1 - 0.5).T @ (b1 - 0.5)) / n * 4.0 - np.eye(24)
    assert np.max(np.abs(within1)) < 1.2 * tol * 2


def test_zero_history_policy_of_the_driver():
    """The driver's alternative first-boundary policy.  With one replica the eager rule under zero
    history feeds Delta_1 itself at every boundary, so the whole run is standard DiLoCo (to rounding);
    under the listing's policy the first phase differs.  With several replicas the first eager step
    feeds Delta_m / M and the first delayed step feeds 0 (the replica returns to its start)."""
    n, H, phases = 24, 4, 5
    r = np.random.default_rng(17)
    h, star = np.exp(r.uniform(np.log(1e-3), 0.0, n)), r.standard_normal(n)
    kw = dict(seed=3, noise_std=0.1, lr=4e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, eta=0.7, mu=0.9)
    std, std_loss = O.run_quadratic("standard", 1, H, phases, h, star, **kw)
    zero, zero_loss = O.run_quadratic("eager", 1, H, phases, h, star, first_boundary="zero_history", **kw)
    lit, lit_loss = O.run_quadratic("eager", 1, H, phases, h, star, **kw)
    # (Delta - P)/1 + D with P = D is Delta up to one rounding of the difference
    np.testing.assert_allclose(zero["a"][0], std["a"], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(zero["u"][0], std["u"], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(zero["theta"][0], std["theta"][0], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(zero_loss, std_loss, rtol=1e-12)
    assert np.max(np.abs(lit["a"][0] - std["a"])) > 1e-6 and abs(lit_loss[0] / std_loss[0] - 1) > 1e-6
    # first boundary with M = 3, by hand from the state after H inner steps
    M = 3
    for variant in ("eager", "delayed"):
        one, _ = O.run_quadratic(variant, M, H, 1, h, star, first_boundary="zero_history", **kw)
        ref, _ = O.run_quadratic(variant, M, H, 1, h, star, **kw)      # listing: a_m = theta_m^(H), nothing applied
        delta = 0.0 - ref["a"]                                         # theta^(0) = 0: Delta_m = 0 - theta_m^(H)
        G = delta / M if variant == "eager" else np.zeros_like(delta)
        np.testing.assert_allclose(one["u"], G, rtol=0, atol=1e-18)    # u = mu * 0 + G
        np.testing.assert_allclose(one["a"], 0.0 - 0.7 * (G + 0.9 * G), rtol=0, atol=1e-18)
        np.testing.assert_array_equal(one["theta"], one["a"])
        np.testing.assert_allclose(one["P"], delta, rtol=0, atol=0)
        np.testing.assert_allclose(one["D"], delta.mean(axis=0), rtol=1e-15)
    with pytest.raises(AssertionError):
        O.run_quadratic("eager", 2, H, 1, h, star, first_boundary="sometimes", **kw)


def test_quadratic_gradient_and_loss_fixed_points():
    n = 33
    h = np.exp(RNG.uniform(np.log(1e-3), 0.0, n))
    star = rnd(n)
    assert O.quadratic_loss(star, h, star) == 0.0
    g = O.quadratic_gradient(star.copy(), h, star, 0.0, 1, 1, 0)
    np.testing.assert_array_equal(g, 0.0)
    # finite-difference check of the gradient against the loss
    th = rnd(n)
    g = O.quadratic_gradient(th, h, star, 0.0, 1, 1, 0)
    for i in (0, 7, 32):
        e = np.zeros(n)
        e[i] = 1e-6
        fd = (O.quadratic_loss(th + e, h, star) - O.quadratic_loss(th - e, h, star)) / 2e-6
        assert abs(fd - g[i]) < 1e-8 * max(1.0, abs(g[i]))
    # the noise term is exactly noise_std * z
    g2 = O.quadratic_gradient(th, h, star, 0.1, 5, 9, 1, index_base=64)
    z = O.standard_normal(5, 9, 1, 64 + np.arange(n))
    np.testing.assert_allclose(g2 - g, 0.1 * z, rtol=1e-9, atol=1e-15)


@pytest.mark.parametrize("variant", ["standard", "eager", "delayed"])
def test_noise_free_quadratic_converges(variant):
    n = 64
    h = np.exp(RNG.uniform(np.log(1e-3), 0.0, n))
    star = rnd(n)
    eta = 0.7 if variant != "delayed" else 0.7 / 4
    _, losses = O.run_quadratic(variant, M=2, H=20, phases=30, h=h, theta_star=star, seed=3,
                                noise_std=0.0, lr=2e-2, beta1=0.9, beta2=0.95, eps=1e-8,
                                weight_decay=0.0, eta=eta, mu=0.5)
    l0 = O.quadratic_loss(np.zeros(n), h, star)
    assert losses[-1] < 1e-3 * l0
    assert np.isfinite(losses).all()


def test_quadratic_run_single_replica_standard_matches_torch_optimizers():
    """Whole driver (inner AdamW x H, outer Nesterov) against torch.optim on one replica."""
    n, H, phases = 12, 5, 4
    lr, b1, b2, eps, eta, mu = 1e-2, 0.9, 0.95, 1e-8, 0.7, 0.9
    h = np.exp(RNG.uniform(np.log(1e-3), 0.0, n))
    star = rnd(n)
    st, losses = O.run_quadratic("standard", 1, H, phases, h, star, seed=11, noise_std=0.1,
                                 lr=lr, beta1=b1, beta2=b2, eps=eps, weight_decay=0.0,
                                 eta=eta, mu=mu)
    p = torch.nn.Parameter(torch.zeros(n, dtype=torch.float64))
    inner = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=0.0)
    outer_p = torch.nn.Parameter(torch.zeros(n, dtype=torch.float64))
    outer = torch.optim.SGD([outer_p], lr=eta, momentum=mu, nesterov=True)
    ht, st_t = torch.tensor(h), torch.tensor(star)
    k = 0
    for t in range(1, H * phases + 1):
        z = torch.tensor(O.standard_normal(11, t, 0, np.arange(n)))
        p.grad = ht * (p.detach() - st_t) + 0.1 * z
        inner.step()
        if t % H == 0:
            outer_p.grad = outer_p.detach() - p.detach()
            outer.step()
            with torch.no_grad():
                p.copy_(outer_p)
            want = 0.5 * float((ht * (outer_p.detach() - st_t) ** 2).sum())
            assert abs(losses[k] - want) <= 1e-10 * max(want, 1e-30)
            k += 1
    np.testing.assert_allclose(st["a"], outer_p.detach().numpy(), rtol=1e-9, atol=1e-14)


def test_eager_run_single_replica_equals_standard_after_first_phase_from_same_state():
    """M = 1: Delta~_1 = Delta_1, so from equal states one eager call is one standard call,
    whatever came before (checked inside a noisy quadratic run)."""
    n, H = 16, 4
    h = np.exp(RNG.uniform(np.log(1e-3), 0.0, n))
    star = rnd(n)
    kw = dict(M=1, H=H, h=h, theta_star=star, seed=5, noise_std=0.1, lr=1e-2, beta1=0.9,
              beta2=0.95, eps=1e-8, weight_decay=0.0, eta=0.7, mu=0.9)
    se, _ = O.run_quadratic("eager", phases=3, **kw)
    # take the eager state, run one more inner phase by hand, then both outer rules
    theta = se["theta"].copy()
    m1, m2 = se["m1"].copy(), se["m2"].copy()
    for t in range(3 * H + 1, 4 * H + 1):
        O.quadratic_inner_step(theta, m1, m2, h, star, t, 5, 0.1, 1e-2, 0.9, 0.95, 1e-8, 0.0)
    te, ae, ue, Pe, De = theta.copy(), se["a"].copy(), se["u"].copy(), se["P"].copy(), se["D"].copy()
    O.outer_eager(te, ae, ue, Pe, De, 0.7, 0.9, True, True)
    ts, as_, us = theta.copy(), se["a"][0].copy(), se["u"][0].copy()
    O.outer_standard(ts, as_, us, 0.7, 0.9, True)
    np.testing.assert_allclose(ae[0], as_, rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(ue[0], us, rtol=1e-12, atol=1e-16)


# ------------------------------------------------ quantised communication ---
def test_bf16_rounding_matches_the_library_conversion():
    x = np.concatenate([rnd(5000, scale=1e-3), rnd(5000), np.array([0.0, -0.0, 1.0, 1.00390625,
                        1.01171875, 3.3895314e38, 1e-40, -1e-40, 2.0 ** -126])]).astype(np.float32)
    want = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(O.round_to_bf16(x).astype(np.float32), want)
    # ties go to even: 1 + 2^-8 is half way between 1 and 1 + 2^-7
    assert O.round_to_bf16(np.float32(1.00390625)) == 1.0
    assert O.round_to_bf16(np.float32(1.01171875)) == 1.015625


def _wide_range_values(count, lo_exp, hi_exp, seed=5):
    r = np.random.default_rng(seed)
    return (r.standard_normal(count) * np.exp2(r.uniform(lo_exp, hi_exp, count))).astype(np.float32)


def test_exmy_value_sets_of_the_four_bit_formats():
    """The sixteen codes of the two 4-bit splits, enumerated by hand from the format definition:
    E2M1 with bias 1 is the published float4 value set; E3M0 has powers of two only, and its
    exponent code 0 holds nothing but zero (no mantissa bit, so no subnormal)."""
    np.testing.assert_array_equal(O.exmy_values(2, 1, 1), [0, 0.5, 1, 1.5, 2, 3, 4, 6])
    np.testing.assert_array_equal(O.exmy_values(3, 0, 3), [0, 0.25, 0.5, 1, 2, 4, 8, 16])
    np.testing.assert_array_equal(O.exmy_values(2, 1, 3), np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6]) / 4)
    # float8 E4M3 with bias 7, every code a number: 2^-9 ... 2^8 * 1.875
    g = O.exmy_values(4, 3, 7)
    assert len(g) == 128 and g[1] == 2.0 ** -9 and g[8] == 2.0 ** -6 and g[-1] == 480.0
    assert np.all(np.diff(g) > 0)


def test_exmy_rounding_worked_cases():
    """Ties go to the even code, overflow saturates, the sign survives, zero stays zero."""
    x = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 7.0, 1e9, -0.3, -5.0, 0.0, 0.2500001, 0.7499999],
                 np.float32)
    want = np.array([0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0, 6.0, 6.0, -0.5, -4.0, 0.0, 0.5, 0.5])
    np.testing.assert_array_equal(O.round_to_exmy(x, 2, 1, 1), want)
    # E3M0: the midpoint of 2^k and 2^(k+1) goes to the even code (1.5 -> 2 = code 4, 3 -> 2, 6 -> 8)
    x = np.array([1.5, 3.0, 6.0, 0.125, 0.1250001, 0.375, 100.0], np.float32)
    np.testing.assert_array_equal(O.round_to_exmy(x, 3, 0, 3), [2.0, 2.0, 8.0, 0.0, 0.25, 0.5, 16.0])


def test_exmy_rounding_is_ieee_half_precision_where_the_two_formats_coincide():
    """E5M10 with bias 15 has the values of IEEE binary16 up to its largest finite one (65504),
    subnormals included; there numpy's float16 conversion is an independent statement of
    round-to-nearest-even."""
    x = np.concatenate([_wide_range_values(400_000, -30, 16), np.float32([0, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25,
                        65504, 2049, 2051, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11])])
    x = x[np.abs(x) <= 65504]
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).astype(np.float64)
    np.testing.assert_array_equal(O.round_to_exmy(x, 5, 10, 15), want)


def test_exmy_rounding_is_bfloat16_where_the_two_formats_coincide():
    """E8M7 with bias 127, against torch's float32 -> bfloat16 conversion (below 2^127, where
    bfloat16 has numbers for every exponent code the format uses)."""
    x = np.concatenate([_wide_range_values(200_000, -140, 126), rnd(1000, scale=1e-3).astype(np.float32)])
    x = x[np.abs(x) < 2.0 ** 127]
    want = torch.tensor(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_to_exmy(x, 8, 7, 127), want)
    np.testing.assert_array_equal(O.round_to_exmy(x, 8, 7, 127), O.round_to_bf16(x))


@pytest.mark.parametrize("fmt", [(2, 1, 11), (3, 0, 12), (4, 3, 16), (5, 2, 24), (3, 4, 12)])
def test_exmy_rounding_is_the_nearest_code_by_brute_force(fmt):
    """Against an exhaustive search over all signed codes, decoded bit field by bit field."""
    E, Mn, bias = fmt
    vals = []
    for code in range(1 << (E + Mn)):
        e, f = code >> Mn, code & ((1 << Mn) - 1)
        vals.append((2.0 ** (1 - bias)) * f / 2 ** Mn if e == 0 else (2.0 ** (e - bias)) * (1 + f / 2 ** Mn))
    x = np.concatenate([rnd(300, scale=1e-3), rnd(100, scale=1e-2), rnd(50, scale=1e-5), [0.0]]).astype(np.float32)
    mids = [(vals[c] + vals[c + 1]) / 2 for c in range(len(vals) - 1)]
    x = np.concatenate([x, np.float32(mids), -np.float32(mids[:5])])
    got = O.round_to_exmy(x, E, Mn, bias)
    for xi, gi in zip(x.astype(np.float64), got):
        best = min(range(len(vals)), key=lambda c: (abs(abs(xi) - vals[c]), c % 2))
        assert gi == np.copysign(vals[best], xi), (xi, gi, vals[best])
    assert np.array_equal(O.round_to_exmy(got.astype(np.float32), E, Mn, bias), got)   # idempotent
    order = np.argsort(x, kind="stable")
    assert np.all(np.diff(got[order]) >= 0)                                         # monotone


@pytest.mark.parametrize("fn", [O.outer_eager, O.outer_delayed])
def test_exmy_communication_stores_what_was_sent(fn):
    M, n = 3, 40
    a0 = rnd(n, scale=0.02).astype(np.float32).astype(np.float64)
    theta = (np.tile(a0, (M, 1)) - rnd(M, n, scale=1e-3)).astype(np.float32).astype(np.float64)
    a, u, P, D = np.tile(a0, (M, 1)), np.zeros((M, n)), np.zeros((M, n)), np.zeros(n)
    fn(theta.copy(), a, u, P, D, 0.7, 0.9, True, apply_update=False, comm=("exmy", 5, 10, 25))
    d32 = (a0[None].astype(np.float32) - theta.astype(np.float32))
    sent = (d32 * np.float32(1024.0)).astype(np.float16).astype(np.float64) / 1024.0   # bias 25 = half scaled by 2^-10
    np.testing.assert_array_equal(P, sent)
    np.testing.assert_allclose(D, sent.mean(axis=0), rtol=1e-14, atol=0)
    assert np.max(np.abs(P - d32)) > 0


@pytest.mark.parametrize("fn", [O.outer_eager, O.outer_delayed])
def test_quantised_communication_keeps_the_stale_share_identity(fn):
    """With bf16 on the wire the stored previous local gradient is what was sent, so the eager
    combination of the NEXT phase is still the mean of the fresh local and the stale non-local
    contributions (Section 2.3), now of the quantised ones; the stored mean is their mean."""
    M, n = 3, 50
    a0 = rnd(n, scale=0.02).astype(np.float32).astype(np.float64)
    theta = (np.tile(a0, (M, 1)) - rnd(M, n, scale=1e-3)).astype(np.float32).astype(np.float64)
    a, u, P, D = np.tile(a0, (M, 1)), np.zeros((M, n)), np.zeros((M, n)), np.zeros(n)
    fn(theta.copy(), a, u, P, D, 0.7, 0.9, True, apply_update=False, comm="bf16")
    sent = torch.tensor((a0[None] - theta).astype(np.float32)).to(torch.bfloat16).double().numpy()
    np.testing.assert_array_equal(P, sent)
    np.testing.assert_allclose(D, sent.mean(axis=0), rtol=1e-14, atol=0)
    assert np.max(np.abs(P - (a0[None] - theta))) > 0           # it really rounded something
    if fn is O.outer_eager:
        fresh = rnd(M, n, scale=1e-3)
        G = O.eager_combination(fresh, P, D)
        for m in range(M):
            others = sum(sent[k] for k in range(M) if k != m)
            np.testing.assert_allclose(G[m], (fresh[m] + others) / M, rtol=1e-10, atol=1e-16)


@pytest.mark.parametrize("comm", ["bf16", ("exmy", 5, 10, 25)])
def test_standard_outer_step_with_quantised_communication_averages_what_was_sent(comm):
    """Momentum off and outer learning rate 1: the new outer parameters are the old ones minus the
    mean of the ROUNDED outer gradients (rounded by an independent library conversion)."""
    M, n = 4, 60
    a0 = rnd(n, scale=0.02).astype(np.float32).astype(np.float64)
    theta = (a0[None] - rnd(M, n, scale=1e-3)).astype(np.float32).astype(np.float64)
    d32 = a0[None].astype(np.float32) - theta.astype(np.float32)
    if comm == "bf16":
        sent = torch.tensor(d32).to(torch.bfloat16).double().numpy()
    else:
        sent = (d32 * np.float32(1024.0)).astype(np.float16).astype(np.float64) / 1024.0
    a, u, th = a0.copy(), np.zeros(n), theta.copy()
    got = O.outer_standard(th, a, u, 1.0, 0.0, True, comm=comm)
    np.testing.assert_allclose(got, sent.mean(axis=0), rtol=1e-14, atol=0)
    np.testing.assert_allclose(a, a0 - sent.mean(axis=0), rtol=1e-14, atol=1e-18)
    np.testing.assert_array_equal(th, np.tile(a, (M, 1)))
    assert np.max(np.abs(sent - d32)) > 0
    # and nothing changes without it
    a2, u2, th2 = a0.copy(), np.zeros(n), theta.copy()
    np.testing.assert_allclose(O.outer_standard(th2, a2, u2, 1.0, 0.0, True), (a0[None] - theta).mean(axis=0),
                               rtol=1e-14, atol=1e-20)


@pytest.mark.parametrize("comm", ["f32", "bf16"])
def test_previous_mean_is_the_mean_of_the_previous_locals_so_it_need_not_be_kept(comm):
    """After every eager boundary the stored mean equals the mean of the stored local outer
    gradients (it is their all-reduce), so a run that never stores it and forms it from them
    walks the same trajectory; checked against the run that stores it, and by hand for one phase."""
    M, n, phases = 3, 40, 6
    rng = np.random.default_rng(21)
    a0 = rng.standard_normal(n) * 0.02
    keep = dict(theta=np.tile(a0, (M, 1)), a=np.tile(a0, (M, 1)), u=np.zeros((M, n)), P=np.zeros((M, n)),
                D=np.zeros(n))
    drop = {k: v.copy() for k, v in keep.items() if k != "D"}
    for k in range(phases):
        step = rng.standard_normal((M, n)) * 1e-3
        for s in (keep, drop):
            s["theta"] = (s["theta"] + step).astype(np.float32).astype(np.float64)
        O.outer_eager(keep["theta"], keep["a"], keep["u"], keep["P"], keep["D"], 0.7, 0.9, True, k > 0, comm=comm)
        O.outer_eager(drop["theta"], drop["a"], drop["u"], drop["P"], None, 0.7, 0.9, True, k > 0, comm=comm)
        np.testing.assert_array_equal(keep["D"], keep["P"].sum(axis=0) / M)
        for name in drop:
            np.testing.assert_array_equal(keep[name], drop[name], err_msg=f"{name} after phase {k}")
    # one phase by hand, with a previous mean that only exists as the mean of P
    P = rng.standard_normal((M, n)) * 1e-3
    a = np.tile(a0, (M, 1)); theta = a - rng.standard_normal((M, n)) * 1e-3; u = np.zeros((M, n))
    delta = a - theta
    want_G = (delta - P) / M + P.mean(axis=0)
    O.outer_eager(theta, a, u, P.copy(), None, 1.0, 0.0, True, True)
    np.testing.assert_allclose(a, a0[None] - want_G, rtol=1e-12, atol=1e-18)


def test_full_precision_communication_is_the_default():
    M, n = 2, 9
    a0 = rnd(n)
    th = np.tile(a0, (M, 1)) - rnd(M, n, scale=1e-3)
    s1 = [th.copy(), np.tile(a0, (M, 1)), rnd(M, n), rnd(M, n), rnd(n)]
    s2 = [x.copy() for x in s1]
    O.outer_eager(*s1, 0.7, 0.9, True, True)
    O.outer_eager(*s2, 0.7, 0.9, True, True, comm="f32")
    for x, y in zip(s1, s2):
        np.testing.assert_array_equal(x, y)


# ------------------------------------------------ two-outer-steps overlap ---
def test_two_step_overlap_by_brute_force_with_full_history():
    """The reading of the 2-outer-steps overlap (no formula in the paper): at boundary b > 2 every
    replica feeds (Delta_m^(b) + sum_{m' != m} Delta_m'^(b-2)) / M.  Recomputed with the complete
    history of outer gradients in Python lists and one torch SGD per replica; the inner phase is
    the noise-free quadratic so both sides can run it."""
    M, n, H, phases = 3, 5, 3, 6
    lr, b1, b2, eps, eta, mu = 2e-2, 0.9, 0.95, 1e-8, 0.7, 0.9
    h = np.exp(RNG.uniform(np.log(1e-3), 0.0, n))
    star = rnd(n)
    st, _ = O.run_quadratic("eager", M, H, phases, h, star, seed=4, noise_std=0.1, lr=lr, beta1=b1,
                            beta2=b2, eps=eps, weight_decay=0.0, eta=eta, mu=mu, overlap=2)
    theta = np.zeros((M, n))
    m1, m2 = np.zeros((M, n)), np.zeros((M, n))
    ps, opts = _torch_replicas(np.zeros(n), M, eta, mu)
    anchors = [np.zeros(n) for _ in range(M)]
    history = []                      # history[b-1][m] = Delta_m at boundary b
    for t in range(1, H * phases + 1):
        O.quadratic_inner_step(theta, m1, m2, h, star, t, 4, 0.1, lr, b1, b2, eps, 0.0)
        if t % H:
            continue
        b = t // H
        now = [anchors[m] - theta[m] for m in range(M)]
        if b > 2:
            old = history[b - 3]
            for m in range(M):
                g = (now[m] + sum(old[q] for q in range(M) if q != m)) / M
                ps[m].grad = torch.tensor(g)
                opts[m].step()
                anchors[m] = ps[m].detach().numpy().copy()
        else:
            for m in range(M):
                anchors[m] = theta[m].copy()
                with torch.no_grad():
                    ps[m].copy_(torch.tensor(theta[m]))
        history.append(now)
        for m in range(M):
            theta[m] = anchors[m]
    np.testing.assert_allclose(st["a"], np.array(anchors), rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(st["theta"], theta, rtol=1e-9, atol=1e-14)
    # the two slots hold the last two generations
    last, before = history[-1], history[-2]
    slot_last = phases % 2
    np.testing.assert_allclose(st["Ps"][slot_last], np.array(last), rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(st["Ps"][1 - slot_last], np.array(before), rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(st["Ds"][slot_last], np.mean(np.array(last), axis=0), rtol=1e-9, atol=1e-14)


def test_overlap_one_is_the_listing():
    n = 6
    h = np.exp(RNG.uniform(np.log(1e-3), 0.0, n))
    star = rnd(n)
    kw = dict(M=2, H=3, phases=4, h=h, theta_star=star, seed=9, noise_std=0.1, lr=1e-2, beta1=0.9,
              beta2=0.95, eps=1e-8, weight_decay=0.0, eta=0.7, mu=0.9)
    s1, l1 = O.run_quadratic("eager", **kw)
    s2, l2 = O.run_quadratic("eager", overlap=1, **kw)
    for k in s1:
        np.testing.assert_array_equal(s1[k], s2[k])
    s3, _ = O.run_quadratic("eager", overlap=2, **kw)
    assert np.max(np.abs(s3["a"] - s1["a"])) > 0


# ------------------------------------------------ frozen outputs of the checker itself ---
def test_checker_outputs_have_not_drifted_from_the_frozen_runs():
    """tests/golden/checker_trajectories.txt was written by tests/golden/make_golden.py from the
    checker alone.  It pins nothing to the paper (the tests above do that); it makes a change to
    the checker's arithmetic visible, so that it is made on purpose and justified."""
    import importlib.util
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    frozen = {}
    for line in open(os.path.join(here, "checker_trajectories.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, *vals = line.split()
        frozen[name] = np.array([float.fromhex(v) for v in vals])
    now = mod.runs()
    assert set(now) == set(frozen)
    for name, want in frozen.items():
        # libm's log / sin / cos may differ in the last place between machines: 1e-13, not bit equality
        np.testing.assert_allclose(now[name], want, rtol=1e-13, atol=1e-300, err_msg=name)
