"""The pins must be able to fail: plausible mistakes are planted in the CPU checker (on the CPU
only), one at a time, and the pin tests are re-run; every planted mistake has to trip at least
one of them."""
import os

import numpy as np
import pytest

from oracle import diloco_oracle as O
from tests import test_oracle_pins as P
from tests import test_streaming as S

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

PINS = [
    P.test_adamw_constant_gradient_closed_form,
    P.test_adamw_first_step_is_sign_step,
    P.test_adamw_zero_gradient_no_decay_is_identity,
    lambda: P.test_adamw_trajectory_matches_torch_adamw(0.0),
    lambda: P.test_adamw_trajectory_matches_torch_adamw(0.1),
    P.test_nesterov_constant_gradient_closed_form,
    P.test_zero_momentum_is_plain_sgd,
    lambda: P.test_outer_optimizer_matches_torch_sgd(True),
    lambda: P.test_outer_optimizer_matches_torch_sgd(False),
    P.test_velocity_form_equals_lookahead_form_for_constant_lr,
    P.test_standard_momentum_off_lr_one_gives_replica_average,
    P.test_standard_trajectory_matches_torch_sgd_on_outer_params,
    lambda: P.test_eager_combination_equals_mean_of_fresh_local_and_stale_others(3),
    lambda: P.test_eager_combination_equals_mean_of_fresh_local_and_stale_others(1),
    P.test_eager_with_stationary_outer_gradients_feeds_the_stale_mean,
    P.test_single_replica_eager_call_equals_standard_call,
    lambda: P.test_identical_replicas_stay_identical_and_local_gradient_is_the_mean(False),
    lambda: P.test_identical_replicas_stay_identical_and_local_gradient_is_the_mean(True),
    lambda: P.test_multi_phase_trajectory_by_brute_force("eager"),
    lambda: P.test_multi_phase_trajectory_by_brute_force("delayed"),
    P.test_delayed_is_nesterov_on_the_shifted_mean_sequence,
    P.test_first_boundary_applies_no_outer_step,
    P.test_reset_is_idempotent_and_broadcasts,
    lambda: P.test_mix64_matches_published_splitmix64_outputs(GOLDEN),
    P.test_noise_is_standard_normal_and_streams_are_independent,
    P.test_noise_matches_a_hand_computation_of_its_definition,
    P.test_noise_radius_and_angle_come_from_disjoint_bits,
    P.test_quadratic_gradient_and_loss_fixed_points,
    lambda: P.test_noise_free_quadratic_converges("eager"),
    P.test_quadratic_run_single_replica_standard_matches_torch_optimizers,
    P.test_bf16_rounding_matches_the_library_conversion,
    P.test_exmy_value_sets_of_the_four_bit_formats,
    P.test_exmy_rounding_worked_cases,
    P.test_exmy_rounding_is_ieee_half_precision_where_the_two_formats_coincide,
    P.test_exmy_rounding_is_bfloat16_where_the_two_formats_coincide,
    lambda: P.test_exmy_rounding_is_the_nearest_code_by_brute_force((2, 1, 11)),
    lambda: P.test_exmy_rounding_is_the_nearest_code_by_brute_force((4, 3, 16)),
    lambda: P.test_exmy_communication_stores_what_was_sent(O.outer_eager),
    lambda: P.test_exmy_communication_stores_what_was_sent(O.outer_delayed),
    lambda: P.test_standard_outer_step_with_quantised_communication_averages_what_was_sent("bf16"),
    lambda: P.test_previous_mean_is_the_mean_of_the_previous_locals_so_it_need_not_be_kept("f32"),
    lambda: P.test_previous_mean_is_the_mean_of_the_previous_locals_so_it_need_not_be_kept("bf16"),
    lambda: P.test_quantised_communication_keeps_the_stale_share_identity(O.outer_eager),
    lambda: P.test_quantised_communication_keeps_the_stale_share_identity(O.outer_delayed),
    S.test_checker_streaming_driver_reduces_to_the_plain_run,
    P.test_zero_history_policy_of_the_driver,
]


def caught():
    for pin in PINS:
        try:
            pin()
        except Exception:           # an assertion, or a crash the mistake provokes
            return True
    return False


def test_the_unmodified_checker_passes_every_pin():
    for pin in PINS:
        pin()


# ---- planted mistakes -----------------------------------------------------------------
def nesterov_wrong_sign(a, u, G, eta, mu, nesterov=True):
    u[...] = mu * u + G
    a[...] = a + eta * (G + mu * u) if nesterov else a + eta * u


def nesterov_stale_velocity(a, u, G, eta, mu, nesterov=True):
    u_old = u.copy()
    u[...] = mu * u + G
    a[...] = a - eta * (G + mu * u_old) if nesterov else a - eta * u


def nesterov_dampened(a, u, G, eta, mu, nesterov=True):
    u[...] = mu * u + (1 - mu) * G
    a[...] = a - eta * (G + mu * u) if nesterov else a - eta * u


def nesterov_ignores_flag(a, u, G, eta, mu, nesterov=True):
    u[...] = mu * u + G
    a[...] = a - eta * (G + mu * u)


def _adam(eps_inside=False, no_bias=False, coupled=False, decay_after=False, beta_swap=False):
    def f(theta, m1, m2, g, t, lr, beta1, beta2, eps, wd):
        if beta_swap:
            beta1, beta2 = beta2, beta1
        gg = g + wd * theta if coupled else g
        m1[...] = beta1 * m1 + (1 - beta1) * gg
        m2[...] = beta2 * m2 + (1 - beta2) * gg * gg
        mh = m1 if no_bias else m1 / (1 - beta1 ** t)
        vh = m2 if no_bias else m2 / (1 - beta2 ** t)
        den = np.sqrt(vh + eps) if eps_inside else np.sqrt(vh) + eps
        if coupled:
            theta[...] = theta - lr * mh / den
        elif decay_after:
            theta[...] = theta - lr * mh / den
            theta[...] = theta - lr * wd * theta
        else:
            theta[...] = theta - lr * (mh / den + wd * theta)
    return f


def eager_no_division(delta, Pp, D):
    return (delta - Pp) + D


def eager_plus_stale(delta, Pp, D):
    return (delta + Pp) / delta.shape[0] + D


def eager_drops_mean(delta, Pp, D):
    return (delta - Pp) / delta.shape[0]


def outer_eager_rotates_first(theta, a, u, Pp, D, eta, mu, nesterov=True, apply_update=True, comm="f32"):
    delta = O.local_outer_gradients(a, theta)
    wire = O.sent_outer_gradients(delta, a, theta, comm)
    Pp[...] = wire
    D[...] = O.mean_over_replicas(wire)
    if apply_update:
        G = O.eager_combination(delta, Pp, D)
        for m in range(theta.shape[0]):
            O.nesterov_step(a[m], u[m], G[m], eta, mu, nesterov)
    else:
        a[...] = theta
    theta[...] = a


def outer_eager_forms_the_mean_from_the_fresh_locals(theta, a, u, Pp, D, eta, mu, nesterov=True, apply_update=True,
                                                     comm="f32"):
    if D is not None:
        return ORIG["outer_eager"](theta, a, u, Pp, D, eta, mu, nesterov, apply_update, comm)
    delta = O.local_outer_gradients(a, theta)
    wire = O.sent_outer_gradients(delta, a, theta, comm)
    if apply_update:
        G = O.eager_combination(delta, Pp, O.mean_over_replicas(wire))
        for m in range(theta.shape[0]):
            O.nesterov_step(a[m], u[m], G[m], eta, mu, nesterov)
    else:
        a[...] = theta
    theta[...] = a
    Pp[...] = wire


def outer_eager_always_applies(theta, a, u, Pp, D, eta, mu, nesterov=True, apply_update=True, comm="f32"):
    return ORIG["outer_eager"](theta, a, u, Pp, D, eta, mu, nesterov, True, comm)


def outer_eager_rounds_local_too(theta, a, u, Pp, D, eta, mu, nesterov=True, apply_update=True, comm="f32"):
    delta = O.local_outer_gradients(a, theta)
    wire = O.sent_outer_gradients(delta, a, theta, comm)
    dbar = O.mean_over_replicas(wire)
    if apply_update:
        G = O.eager_combination(delta, Pp, D)
        for m in range(theta.shape[0]):
            O.nesterov_step(a[m], u[m], G[m], eta, mu, nesterov)
    else:
        a[...] = theta
    theta[...] = a
    Pp[...] = delta          # stores the unrounded gradient although bf16 was sent
    D[...] = dbar


def outer_delayed_uses_fresh_mean(theta, a, u, Pp, D, eta, mu, nesterov=True, apply_update=True, comm="f32"):
    delta = O.local_outer_gradients(a, theta)
    wire = O.sent_outer_gradients(delta, a, theta, comm)
    dbar = O.mean_over_replicas(wire)
    if apply_update:
        for m in range(theta.shape[0]):
            O.nesterov_step(a[m], u[m], dbar, eta, mu, nesterov)
    else:
        a[...] = theta
    theta[...] = a
    Pp[...] = wire
    D[...] = dbar


def mean_forgets_division(delta):
    return delta.sum(axis=0)


def mean_wrong_divisor(delta):
    return delta.sum(axis=0) / max(1, delta.shape[0] - 1)


def local_wrong_sign(a, theta):
    return theta - a


def standard_ignores_wire_format(theta, a, u, eta, mu, nesterov=True, comm="f32"):
    return ORIG["outer_standard"](theta, a, u, eta, mu, nesterov)


def standard_no_reset(theta, a, u, eta, mu, nesterov=True, comm="f32"):
    delta = O.local_outer_gradients(a, theta)
    dbar = O.mean_over_replicas(delta)
    O.nesterov_step(a, u, dbar, eta, mu, nesterov)
    return dbar


def mix64_wrong_shift(x):
    x = np.asarray(x, dtype=np.uint64).copy()
    with np.errstate(over="ignore"):
        x ^= x >> np.uint64(31)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(27)
        x *= np.uint64(0x94D049BB133111EB)
        x ^= x >> np.uint64(31)
    return x


def normal_without_factor_two(seed, t, m, idx):
    return ORIG["standard_normal"](seed, t, m, idx) / np.sqrt(2.0)


def normal_ignores_replica(seed, t, m, idx):
    return ORIG["standard_normal"](seed, t, 0, idx)


def _normal_with_fields(shift1, shift2, t_off=1, m_off=1, j_off=1, swap=False):
    """The generator with its bit fields / counter offsets moved."""
    def f(seed, t, m, idx):
        idx = np.asarray(idx, dtype=np.int64)
        U = np.uint64
        G = U(0x9E3779B97F4A7C15)
        with np.errstate(over="ignore"):
            k0 = ORIG["mix64"](U(seed) + G * U(t + t_off))
            key = ORIG["mix64"](k0 + G * U(m + m_off))
            x = ORIG["mix64"](key + G * ((idx >> 1).astype(U) + U(j_off)))
        f1 = ((x >> U(shift1)) & U(0xFFFFFF)).astype(np.float64)
        f2 = ((x >> U(shift2)) & U(0xFFFFFF)).astype(np.float64)
        if swap:
            f1, f2 = f2, f1
        r = np.sqrt(-2.0 * np.log((f1 + 1.0) / 16777216.0))
        ang = 2.0 * np.pi * f2 / 16777216.0
        return np.where((idx & 1) == 0, r * np.cos(ang), r * np.sin(ang))
    return f


normal_overlapping_fields = _normal_with_fields(40, 28)       # the angle reuses 12 bits of the radius
normal_overlapping_fields.__name__ = "normal_overlapping_fields"
normal_same_field_twice = _normal_with_fields(40, 40)
normal_same_field_twice.__name__ = "normal_same_field_twice"
normal_swapped_fields = _normal_with_fields(40, 16, swap=True)
normal_swapped_fields.__name__ = "normal_swapped_fields"
normal_low_bits = _normal_with_fields(24, 0)                  # bits 0-47 instead of 16-63
normal_low_bits.__name__ = "normal_low_bits"
normal_step_offset = _normal_with_fields(40, 16, t_off=0)     # t instead of t + 1 in the key
normal_step_offset.__name__ = "normal_step_offset"
normal_pair_offset = _normal_with_fields(40, 16, j_off=0)     # j instead of j + 1
normal_pair_offset.__name__ = "normal_pair_offset"


def normal_sine_first(seed, t, m, idx):
    idx = np.asarray(idx, dtype=np.int64)
    return ORIG["standard_normal"](seed, t, m, idx ^ 1)       # sine on the even element, cosine on the odd


def bf16_truncates(x):
    bits = np.asarray(x, dtype=np.float32).view(np.uint32) & np.uint32(0xFFFF0000)
    return bits.view(np.float32).astype(np.float64)


def exmy_without_subnormals(E, Mn, bias):
    g = ORIG["exmy_values"](E, Mn, bias).copy()
    g[1:1 << Mn] = g[1 << Mn] if Mn else g[1:1]       # exponent code 0 flushes to the smallest normal
    return np.sort(g)


def exmy_ieee_top_exponent(E, Mn, bias):
    """Top exponent code reserved, as IEEE formats do: the largest values go missing."""
    g = ORIG["exmy_values"](E, Mn, bias)
    return g[:len(g) - (1 << Mn)]


def exmy_truncates(x, E, Mn, bias):
    grid = O.exmy_values(E, Mn, bias)
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    lo = np.clip(np.searchsorted(grid, np.abs(x), side="right") - 1, 0, len(grid) - 1)
    return np.copysign(grid[lo], x)


def exmy_ties_away(x, E, Mn, bias):
    grid = O.exmy_values(E, Mn, bias)
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    mag = np.abs(x)
    hi = np.clip(np.searchsorted(grid, mag, side="left"), 1, len(grid) - 1)
    out = np.where(grid[hi] - mag <= mag - grid[hi - 1], grid[hi], grid[hi - 1])
    return np.copysign(np.where(mag >= grid[-1], grid[-1], out), x)


def exmy_drops_sign(x, E, Mn, bias):
    return np.abs(ORIG["round_to_exmy"](x, E, Mn, bias))


def exmy_overflow_wraps_to_zero(x, E, Mn, bias):
    out = ORIG["round_to_exmy"](x, E, Mn, bias)
    return np.where(np.abs(np.asarray(x, np.float64)) > O.exmy_values(E, Mn, bias)[-1], 0.0, out)


def sent_ignores_format(delta, a, theta, comm):
    return ORIG["sent_outer_gradients"](delta, a, theta, "bf16" if comm != "f32" else "f32")


def boundary_ignores_offset(t, H, offset=0):
    return t >= 1 and t % H == 0


def quadratic_gradient_without_curvature(theta_m, h, theta_star, noise_std, seed, t, m, index_base=0):
    idx = index_base + np.arange(theta_m.shape[-1], dtype=np.int64)
    return (theta_m - theta_star) + noise_std * O.standard_normal(seed, t, m, idx)


def run_quadratic_ignores_the_policy(*args, first_boundary="listing", **kw):
    return ORIG["run_quadratic"](*args, **kw)


def run_quadratic_always_zero_history(*args, first_boundary="listing", **kw):
    return ORIG["run_quadratic"](*args, first_boundary="zero_history", **kw)


ORIG = {k: getattr(O, k) for k in dir(O) if callable(getattr(O, k)) and not k.startswith("_")}

MUTATIONS = [
    ("nesterov_step", nesterov_wrong_sign), ("nesterov_step", nesterov_stale_velocity),
    ("nesterov_step", nesterov_dampened), ("nesterov_step", nesterov_ignores_flag),
    ("adamw_step", _adam(eps_inside=True)), ("adamw_step", _adam(no_bias=True)),
    ("adamw_step", _adam(coupled=True)), ("adamw_step", _adam(decay_after=True)),
    ("adamw_step", _adam(beta_swap=True)),
    ("eager_combination", eager_no_division), ("eager_combination", eager_plus_stale),
    ("eager_combination", eager_drops_mean),
    ("outer_eager", outer_eager_rotates_first), ("outer_eager", outer_eager_always_applies),
    ("outer_eager", outer_eager_rounds_local_too),
    ("outer_eager", outer_eager_forms_the_mean_from_the_fresh_locals),
    ("outer_delayed", outer_delayed_uses_fresh_mean),
    ("mean_over_replicas", mean_forgets_division), ("mean_over_replicas", mean_wrong_divisor),
    ("local_outer_gradients", local_wrong_sign), ("outer_standard", standard_no_reset),
    ("outer_standard", standard_ignores_wire_format),
    ("mix64", mix64_wrong_shift), ("standard_normal", normal_without_factor_two),
    ("standard_normal", normal_ignores_replica), ("standard_normal", normal_overlapping_fields),
    ("standard_normal", normal_same_field_twice), ("standard_normal", normal_swapped_fields),
    ("standard_normal", normal_low_bits), ("standard_normal", normal_step_offset),
    ("standard_normal", normal_pair_offset), ("standard_normal", normal_sine_first),
    ("round_to_bf16", bf16_truncates),
    ("is_boundary", boundary_ignores_offset),
    ("exmy_values", exmy_without_subnormals), ("exmy_values", exmy_ieee_top_exponent),
    ("round_to_exmy", exmy_truncates), ("round_to_exmy", exmy_ties_away),
    ("round_to_exmy", exmy_drops_sign), ("round_to_exmy", exmy_overflow_wraps_to_zero),
    ("sent_outer_gradients", sent_ignores_format),
    ("quadratic_gradient", quadratic_gradient_without_curvature),
    ("run_quadratic", run_quadratic_ignores_the_policy), ("run_quadratic", run_quadratic_always_zero_history),
]


@pytest.mark.parametrize("name,bad", MUTATIONS, ids=[f"{n}:{f.__name__}:{i}" for i, (n, f) in enumerate(MUTATIONS)])
def test_planted_mistake_is_caught(name, bad, monkeypatch):
    monkeypatch.setattr(O, name, bad)
    assert caught(), f"no pin notices the mistake planted in {name}"
