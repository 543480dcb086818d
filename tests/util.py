"""Shared helpers of the parity tests: the error metric, its tolerances and the operand scales.

Per-call parity is judged element by element against the OPERAND SCALE of each output:

    err = max_i |got_i - want_i| / S_i ,      S_i = sum of the magnitudes of the terms the
                                               algorithm adds up to form output i.

S_i >= |want_i| always, with equality wherever the terms do not cancel, so for those elements
this is the plain relative error.  Where they do cancel (a velocity mu u + G that passes through
zero, a mean of sign-random outer gradients) plain relative error has no bound for ANY float32
evaluation, because the float32 representation error of the inputs alone (mu = 0.9 is not a
float32 number, the mean is stored as float32) is amplified by S_i / |want_i|; the operand scale
is what a forward error analysis of the float32 arithmetic bounds.  The scales below follow the
listings term by term (Algorithm 1 lines 7-10, Algorithm 3 lines 7-12, AdamW as InnerOpt) and
are computed from the checker's float64 inputs only.  Unlike a floor taken from the buffer's own
rms they cannot vanish on a buffer of one element.

Trajectory tests (the checker keeps float64 state over many calls) state their own derived
tolerances and use `rel_err`, the buffer-rms form, which needs a buffer large enough for its rms
to be a population statistic (enforced).
"""
import numpy as np

# fp32 buffers: 1e-6 of the operand scale (a proved bound: at most 14 float32 roundings of
# 2^-24 = 6e-8 each enter any output, see the derivation in the design notes); bf16 buffers:
# 4e-3 (bf16 keeps 8 significant bits: an ulp is 2^-7 relative, round-to-nearest-even costs at most
# half of it, 2^-8 = 3.906e-3; the worst case is met at full size: measured 0.973 of the tolerance).
TOL_F32 = 1e-6
TOL_BF16 = 4e-3

RMS_MIN_ELEMS = 1024


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max_i |got_i - want_i| / (|want_i| + rms(want)): the trajectory metric.  Only for buffers of
    at least RMS_MIN_ELEMS elements: on a handful of elements the rms is no floor at all."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    assert want.size >= RMS_MIN_ELEMS, "the rms floor needs a large buffer: pass operand scales instead"
    assert np.isfinite(got).all(), "non-finite values in the result"
    rms = float(np.sqrt(np.mean(want * want)))
    if rms == 0.0:
        return float(np.max(np.abs(got - want)))
    return float(np.max(np.abs(got - want) / (np.abs(want) + rms)))


def trajectory_tol(steps: int, outer_momentum: float) -> float:
    """Tolerance of a whole run in which the checker keeps float64 state and the library stores float32
    after every call.  Every call contributes an independent rounding error of at most TOL_F32 of its
    scale (the per-call bound); over `steps` calls they add up like a random walk, sqrt(steps), and
    the outer optimizer's momentum hands an error of its input on with gain 1 / (1 - mu).  The step
    size is the BOUND of the per-call error, three to five times the typical one, which is the
    estimate's headroom (measured: 0.24 of it on the 2000-step configuration)."""
    return TOL_F32 * float(np.sqrt(max(1, steps))) / (1.0 - outer_momentum)


def scaled_err(got: np.ndarray, want: np.ndarray, scale: np.ndarray) -> float:
    """max_i |got_i - want_i| / scale_i.  Where the scale is zero every term of the sum is zero and
    the result must be exact."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    scale = np.broadcast_to(np.asarray(scale, dtype=np.float64), want.shape)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    assert np.isfinite(got).all(), "non-finite values in the result"
    assert (scale >= np.abs(want) * (1.0 - 1e-12)).all(), "an operand scale below the result's magnitude"
    diff = np.abs(got - want)
    zero = scale == 0.0
    assert not (diff[zero] != 0.0).any(), "inexact result where every operand is zero"
    return float(np.max(np.where(zero, 0.0, diff / np.where(zero, 1.0, scale))))


def assert_close(got, want, tol, what="", scale=None):
    """Per-call gate: operand-scale metric when `scale` is given, the rms form otherwise."""
    e = rel_err(got, want) if scale is None else scaled_err(got, want, scale)
    assert e <= tol, f"{what}: error {e:.3e} above tolerance {tol:.1e}"
    return e


# ------------------------------------------------------------------ operand scales
def _mean_abs(x):
    return np.mean(np.abs(x), axis=0)


def eager_scales(theta, a, u, P, D, eta, mu, nesterov=True, apply_update=True, variant="eager", sent=None):
    """Operand scales of one eager (Algorithm 3 lines 7-12) or delayed (Algorithm 2 lines 7-11) outer
    step, from the float64 state BEFORE the call.  theta, a, u, P: [M, n]; D: [n] or None (the mean
    is then formed from P).  `sent` is what the replicas put on the wire when it is not Delta_m
    itself (quantised communication).  Returns scales keyed like the state."""
    M = theta.shape[0]
    delta = a - theta                                  # line 7: one rounding of an exact difference
    wire = delta if sent is None else sent
    S = dict(prev_local=np.abs(wire), prev_mean=_mean_abs(wire))
    if not apply_update:                               # t = H: a_m <- theta_m, nothing else moves
        S.update(anchor=np.abs(theta), theta=np.abs(theta), vel=np.abs(u))
        return S
    d_old = np.abs(D) if D is not None else _mean_abs(P)
    if variant == "eager":                             # line 11: (Delta_m - P_m)/M + D
        s_g = (np.abs(delta) + np.abs(P)) / M + d_old
    else:                                              # Algorithm 2 line 11: D itself
        s_g = np.broadcast_to(d_old, theta.shape)
    s_u = mu * np.abs(u) + s_g                         # u <- mu u + G
    s_a = np.abs(a) + eta * ((s_g + mu * s_u) if nesterov else s_u)
    S.update(vel=s_u, anchor=s_a, theta=s_a)
    return S


def standard_scales(theta, a, u, eta, mu, nesterov=True, sent=None):
    """Operand scales of the standard outer step (Algorithm 1 lines 7-10); a, u: [n] shared."""
    wire = (a - theta) if sent is None else sent
    s_g = _mean_abs(wire)
    s_u = mu * np.abs(u) + s_g
    s_a = np.abs(a) + eta * ((s_g + mu * s_u) if nesterov else s_u)
    return dict(mean=s_g, vel=s_u, anchor=s_a, theta=np.broadcast_to(s_a, theta.shape))


def adamw_scales(theta, m1, m2, g, t, lr, beta1, beta2, eps, weight_decay, g_scale=None):
    """Operand scales of one AdamW step (InnerOpt, line 5 of the listings), from the state before.
    g_scale: operand scale of the gradient itself when the call forms it (default: |g|, an input)."""
    sg = np.abs(g) if g_scale is None else g_scale
    s_m1 = beta1 * np.abs(m1) + (1.0 - beta1) * sg
    v = beta2 * np.abs(m2) + (1.0 - beta2) * g * g          # all terms positive: the value itself
    s_m2 = beta2 * np.abs(m2) + (1.0 - beta2) * sg * sg     # = v unless the call forms g with cancellation
    denom = np.sqrt(v / (1.0 - beta2 ** t)) + eps
    # the step m1_hat / (sqrt(m2_hat) + eps) inherits m1's error relative to S_m1 and m2's relative to v
    amp = np.where(v > 0.0, s_m2 / np.where(v > 0.0, v, 1.0), 1.0)
    s_upd = s_m1 / (1.0 - beta1 ** t) / denom * amp
    return dict(m1=s_m1, m2=s_m2, theta=np.abs(theta) + lr * (s_upd + weight_decay * np.abs(theta)))


# ------------------------------------------------------------------ the checker, with its scales
def checked_eager(ref, eta, mu, nesterov=True, apply_update=True, variant="eager", comm="f32", no_mean=False):
    """The checker's eager / delayed outer step in place on the float64 state `ref` (keys theta, anchor,
    vel, prev_local, prev_mean); returns the operand scales of the call, keyed alike."""
    from oracle import diloco_oracle as O
    sent = None
    if comm != "f32":
        sent = O.sent_outer_gradients(ref["anchor"] - ref["theta"], ref["anchor"], ref["theta"], comm)
    D = None if no_mean else ref["prev_mean"]
    S = eager_scales(ref["theta"], ref["anchor"], ref["vel"], ref["prev_local"], D, eta, mu, nesterov,
                     apply_update, variant, sent)
    if variant == "eager":
        O.outer_eager(ref["theta"], ref["anchor"], ref["vel"], ref["prev_local"], D, eta, mu, nesterov,
                      apply_update, comm=comm)
    else:
        assert not no_mean
        O.outer_delayed(ref["theta"], ref["anchor"], ref["vel"], ref["prev_local"], D, eta, mu, nesterov,
                        apply_update, comm=comm)
    return S


def checked_standard(theta, a, u, eta, mu, nesterov=True, comm="f32"):
    """The checker's standard outer step in place; returns (mean, operand scales)."""
    from oracle import diloco_oracle as O
    sent = None if comm == "f32" else O.sent_outer_gradients(a - theta, a, theta, comm)
    S = standard_scales(theta, a, u, eta, mu, nesterov, sent)
    return O.outer_standard(theta, a, u, eta, mu, nesterov, comm=comm), S


def checked_adamw(ref, t, lr, beta1, beta2, eps, weight_decay):
    """The checker's AdamW step in place on ref (keys theta, m1, m2, grad); returns the operand scales."""
    from oracle import diloco_oracle as O
    S = adamw_scales(ref["theta"], ref["m1"], ref["m2"], ref["grad"], t, lr, beta1, beta2, eps, weight_decay)
    O.adamw_step(ref["theta"], ref["m1"], ref["m2"], ref["grad"], t, lr, beta1, beta2, eps, weight_decay)
    return S


def quadratic_scales(theta, m1, m2, h, theta_star, noise_std, seed, t, lr, beta1, beta2, eps, weight_decay,
                     index_base=0):
    """Operand scales of one inner step on the noisy quadratic: AdamW's, with the gradient
    h (theta - theta*) + noise_std z weighed by the magnitudes of its two terms.  theta, m1, m2: [M, n]."""
    from oracle import diloco_oracle as O
    idx = index_base + np.arange(theta.shape[-1], dtype=np.int64)
    g = np.empty_like(theta)
    sg = np.empty_like(theta)
    for m in range(theta.shape[0]):
        z = O.standard_normal(seed, t, m, idx)
        g[m] = h * (theta[m] - theta_star) + noise_std * z
        sg[m] = np.abs(h * (theta[m] - theta_star)) + noise_std * np.abs(z)
    return adamw_scales(theta, m1, m2, g, t, lr, beta1, beta2, eps, weight_decay, g_scale=sg)
