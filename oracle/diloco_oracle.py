"""CPU checker for the DiLoCo optimizer sweep.  TEST INFRASTRUCTURE ONLY.

A plain, slow, single-threaded float64 NumPy statement of what the hot path
computes: the inner AdamW step (InnerOpt of Algorithms 1-3), the standard outer
step (Algorithm 1), the naive delayed outer step (Algorithm 2) and the eager
outer step (Algorithm 3), plus the noisy
quadratic used as a stand-in training problem.  It shares no code with the HIP
library and is imported only by the tests, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing in the product path may call it.

The method is a sequence of arithmetic updates with no independent definition,
so this file follows the algorithms' steps in the paper's order and notation:

    theta_m       live parameters of replica m                     theta[m, :]
    theta_m^(t-H) outer parameters ("anchor") of replica m         a[m, :] or a[:]
    Delta_m^(t)   fresh local outer gradient                       delta[m, :]
    Delta^(t)     its mean over replicas                           delta_bar[:]
    Delta_m^(t-H) previous local outer gradient                    P[m, :]
    Delta^(t-H)   previous averaged outer gradient                 D[:]
    OuterOpt      SGD with Nesterov momentum, velocity             u
    InnerOpt      AdamW, moments                                   m1, m2

Readings where the paper gives no formula (Section 2 names the optimizers
only): AdamW is the decoupled-weight-decay, bias-corrected form with epsilon
added outside the square root; Nesterov momentum is the velocity form
u <- mu u + G, a <- a - eta (G + mu u).  Every function mutates its array
arguments in place and all arrays are float64.

Parity pins (tests/test_oracle_pins.py): closed forms for constant gradients,
torch.optim.SGD / torch.optim.AdamW in float64 as black boxes on whole
trajectories, the paper's equivalent form of the eager combination (Section
2.3: the mean of the fresh local and the stale non-local outer gradients),
M = 1 and identical-worker reductions, the mu = 0, eta = 1 worker average, and
published splitmix64 test vectors plus distribution tests for the noise.
Parity unpinned: run_quadratic(overlap=2) against the paper, which gives no formula for the
2-outer-steps overlap (the function is pinned to the reading stated in its docstring);
round_to_exmy against the paper's float8 / float4 runs, whose formats it does not state (the
rounding is pinned to numpy's float16, torch's bfloat16 and enumerated float4 value sets).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64
U64 = np.uint64


# --------------------------------------------------------------------------
# InnerOpt: AdamW (the inner optimization step of Algorithms 1-3)
# --------------------------------------------------------------------------
def adamw_step(theta, m1, m2, g, t, lr, beta1, beta2, eps, weight_decay):
    """One AdamW step, t >= 1 is the global step count (never reset).

    m1 <- b1 m1 + (1-b1) g ; m2 <- b2 m2 + (1-b2) g^2 ;
    theta <- theta - lr ( m1_hat / (sqrt(m2_hat) + eps) + wd * theta ),
    with m_hat = m / (1 - b^t) and the decay term using theta before the step.
    """
    assert t >= 1
    m1[...] = beta1 * m1 + (1.0 - beta1) * g
    m2[...] = beta2 * m2 + (1.0 - beta2) * (g * g)
    m1_hat = m1 / (1.0 - beta1 ** t)
    m2_hat = m2 / (1.0 - beta2 ** t)
    theta[...] = theta - lr * (m1_hat / (np.sqrt(m2_hat) + eps) + weight_decay * theta)


# --------------------------------------------------------------------------
# OuterOpt: SGD with (Nesterov) momentum (the outer optimization step of Algorithms 1-3)
# --------------------------------------------------------------------------
def nesterov_step(a, u, G, eta, mu, nesterov=True):
    """u <- mu u + G ; a <- a - eta (G + mu u) (Nesterov) or a <- a - eta u (heavy ball)."""
    u[...] = mu * u + G
    if nesterov:
        a[...] = a - eta * (G + mu * u)
    else:
        a[...] = a - eta * u


def local_outer_gradients(a, theta):
    """Local outer gradient: Delta_m = theta_m^(t-H) - theta_m^(t).  `a` is [n] (shared) or [M, n]."""
    return a - theta  # broadcasting covers the shared anchor


def mean_over_replicas(delta):
    """The all-reduce: Delta = (1/M) sum_m Delta_m, summed left to right in m."""
    M = delta.shape[0]
    s = delta[0].copy()
    for m in range(1, M):
        s += delta[m]
    return s / M


# --------------------------------------------------------------------------
# Algorithm 1: standard DiLoCo, one shared set of outer parameters
# --------------------------------------------------------------------------
def outer_standard(theta, a, u, eta, mu, nesterov=True, comm="f32"):
    """theta [M, n]; a, u [n] shared by all replicas.  Returns Delta^(t).  With quantised
    communication (Section 3.2) the mean is taken over what the replicas send."""
    delta = local_outer_gradients(a, theta)          # local outer gradients
    delta_bar = mean_over_replicas(sent_outer_gradients(delta, a, theta, comm))  # blocking all-reduce
    nesterov_step(a, u, delta_bar, eta, mu, nesterov)  # outer optimization on the shared parameters
    theta[...] = a                                    # every replica restarts from the outer params
    return delta_bar


# --------------------------------------------------------------------------
# Quantised communication (Section 3.2): the outer gradient a replica sends is rounded to
# bfloat16, or to a small float of E exponent and Mn mantissa bits (the section names float8
# and float4 in "ExMy" formats from a cited work without fixing E, Mn, the bias or the treatment
# of overflow: reading below; parity with the paper's own runs is unpinned, the rounding itself
# is pinned to IEEE half precision, to bfloat16 and to hand-enumerated float4 grids).
# Rounding is a decision about an integer code, so it is taken in the precision the
# wire format is produced from: the float32 difference of the stored float32 parameters.
# --------------------------------------------------------------------------
def round_to_bf16(x):
    """float32 -> bfloat16 (round to nearest, ties to even) -> back, on an array of finite values."""
    bits = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    bits = (bits + np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).astype(F64)


def exmy_values(E, Mn, bias):
    """All non-negative values of the sign / E exponent bits / Mn mantissa bits format with the
    given exponent bias, indexed by their code c = (e << Mn) | f:
        e = 0:  2^(1-bias) * f / 2^Mn            (zero and the subnormals)
        e >= 1: 2^(e-bias) * (1 + f / 2^Mn)
    Every code is a number: the format has no infinities and no NaNs."""
    assert E >= 1 and Mn >= 0
    c = np.arange(1 << (E + Mn), dtype=np.int64)
    e, f = c >> Mn, c & ((1 << Mn) - 1)
    frac = f.astype(F64) / float(1 << Mn)
    return np.where(e == 0, np.ldexp(frac, 1 - bias), np.ldexp(1.0 + frac, e - bias))


def round_to_exmy(x, E, Mn, bias):
    """Nearest value of the format to each x (finite float32 values), ties to the even code,
    magnitudes beyond the largest value saturate to it; the sign is kept."""
    grid = exmy_values(E, Mn, bias)                   # ascending in the code
    x = np.asarray(x, dtype=np.float32).astype(F64)
    mag = np.abs(x)
    hi = np.clip(np.searchsorted(grid, mag, side="left"), 1, len(grid) - 1)
    lo = hi - 1
    d_lo, d_hi = mag - grid[lo], grid[hi] - mag       # exact: neighbours of a float32 value
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    out = np.where(take_hi, grid[hi], grid[lo])
    out = np.where(mag >= grid[-1], grid[-1], out)
    return np.copysign(out, x)


def sent_outer_gradients(delta, a, theta, comm):
    """What enters the all-reduce: Delta_m, or Delta_m formed in float32 and rounded to the wire
    format: "bf16", or ("exmy", E, Mn, bias)."""
    if comm == "f32":
        return delta
    d32 = (np.asarray(a, np.float32) - np.asarray(theta, np.float32)).astype(np.float32)
    if comm == "bf16":
        return round_to_bf16(d32)
    kind, E, Mn, bias = comm
    assert kind == "exmy"
    return round_to_exmy(d32, E, Mn, bias)


# --------------------------------------------------------------------------
# Algorithm 2: naive delayed outer gradients, per-replica outer parameters
# --------------------------------------------------------------------------
def outer_delayed(theta, a, u, P, D, eta, mu, nesterov=True, apply_update=True, comm="f32"):
    """theta, a, u, P [M, n]; D [n].  apply_update=False is the t = H boundary,
    where the listing applies no outer step: the replica just continues from its
    own parameters, which become its next anchor."""
    delta = local_outer_gradients(a, theta)          # local outer gradients
    wire = sent_outer_gradients(delta, a, theta, comm)
    delta_bar = mean_over_replicas(wire)             # async all-reduce (arrives one phase later)
    if apply_update:                                 # t > H
        for m in range(theta.shape[0]):
            nesterov_step(a[m], u[m], D, eta, mu, nesterov)   # outer step with the received Delta^(t-H)
    else:
        a[...] = theta
    theta[...] = a
    P[...] = wire
    D[...] = delta_bar


# --------------------------------------------------------------------------
# Algorithm 3: eager updates with delayed outer gradients
# --------------------------------------------------------------------------
def eager_combination(delta, P, D):
    """Algorithm 3's mix of fresh local and stale averaged outer gradients:
    Delta~_m = (1/M)(Delta_m^(t) - Delta_m^(t-H)) + Delta^(t-H)."""
    M = delta.shape[0]
    return (delta - P) / M + D


def outer_eager(theta, a, u, P, D, eta, mu, nesterov=True, apply_update=True, comm="f32"):
    """theta, a, u, P [M, n]; D [n].  All Delta~_m are formed from the old P and D
    before either is overwritten.  With quantised communication P holds what the replica
    sent, so that the eager combination removes exactly its own stale share of D, and the fresh local
    Delta_m enters unrounded (the replica has it in full precision).
    D = None: the previous mean is not kept at all.  When all replicas are at hand it is, by its
    definition, the mean of the previous local outer gradients P, and is formed from them."""
    delta = local_outer_gradients(a, theta)          # local outer gradients
    wire = sent_outer_gradients(delta, a, theta, comm)
    delta_bar = mean_over_replicas(wire)             # async all-reduce
    if apply_update:                                 # t > H
        G = eager_combination(delta, P, mean_over_replicas(P) if D is None else D)  # receive Delta^(t-H), combine
        for m in range(theta.shape[0]):
            nesterov_step(a[m], u[m], G[m], eta, mu, nesterov)  # outer optimization per replica
    else:
        a[...] = theta
    theta[...] = a
    P[...] = wire
    if D is not None:
        D[...] = delta_bar


def reset(theta, a):
    """theta_m <- outer parameters (shared [n] or per replica [M, n])."""
    theta[...] = a


# --------------------------------------------------------------------------
# Noisy quadratic stand-in problem: loss 0.5 sum_i h_i (theta_i - theta*_i)^2
# --------------------------------------------------------------------------
_GOLDEN = U64(0x9E3779B97F4A7C15)


def mix64(x):
    """Output function of the splitmix64 generator (Steele, Lea, Flood 2014) on uint64 arrays."""
    x = np.asarray(x, dtype=U64).copy()
    with np.errstate(over="ignore"):
        x ^= x >> U64(30)
        x *= U64(0xBF58476D1CE4E5B9)
        x ^= x >> U64(27)
        x *= U64(0x94D049BB133111EB)
        x ^= x >> U64(31)
    return x


def noise_key(seed, t, m):
    """Stream key of (seed, step t, replica m): two chained splitmix64 outputs."""
    with np.errstate(over="ignore"):
        k0 = mix64(U64(seed) + _GOLDEN * U64(t + 1))
        return mix64(k0 + _GOLDEN * U64(m + 1))


def standard_normal(seed, t, m, idx):
    """z(seed, t, m, i) for int64 indices `idx`: elements 2j and 2j+1 share the 64-bit word
    x_j = splitmix64 output number j of the stream keyed by (seed, t, m);
    u1 = (top 24 bits + 1) / 2^24 in (0, 1], u2 = (next 24 bits) / 2^24 in [0, 1);
    Box-Muller: z_2j = r cos(2 pi u2), z_2j+1 = r sin(2 pi u2), r = sqrt(-2 ln u1)."""
    idx = np.asarray(idx, dtype=np.int64)
    j = (idx >> 1).astype(U64)
    with np.errstate(over="ignore"):
        x = mix64(noise_key(seed, t, m) + _GOLDEN * (j + U64(1)))
    u1 = ((x >> U64(40)).astype(F64) + 1.0) / 16777216.0
    u2 = ((x >> U64(16)) & U64(0xFFFFFF)).astype(F64) / 16777216.0
    r = np.sqrt(-2.0 * np.log(u1))
    ang = 2.0 * np.pi * u2
    return np.where((idx & 1) == 0, r * np.cos(ang), r * np.sin(ang))


def quadratic_gradient(theta_m, h, theta_star, noise_std, seed, t, m, index_base=0):
    """g_m = h (theta_m - theta*) + noise_std z(seed, t, m, i), i = index_base + position."""
    idx = index_base + np.arange(theta_m.shape[-1], dtype=np.int64)
    return h * (theta_m - theta_star) + noise_std * standard_normal(seed, t, m, idx)


def quadratic_loss(theta, h, theta_star):
    """0.5 sum_i h_i (theta_i - theta*_i)^2 for one parameter vector [n]."""
    d = theta - theta_star
    return 0.5 * float(np.sum(h * d * d))


def quadratic_inner_step(theta, m1, m2, h, theta_star, t, seed, noise_std,
                         lr, beta1, beta2, eps, weight_decay, index_base=0):
    """Lines 3-5 on the quadratic: every replica takes one AdamW step on its own noisy gradient."""
    for m in range(theta.shape[0]):
        g = quadratic_gradient(theta[m], h, theta_star, noise_std, seed, t, m, index_base)
        adamw_step(theta[m], m1[m], m2[m], g, t, lr, beta1, beta2, eps, weight_decay)


# --------------------------------------------------------------------------
# Drivers: whole runs of Algorithms 1-3
# --------------------------------------------------------------------------
def stream_offset(H, F, f):
    """Streaming DiLoCo (Section 3: every experiment applies the outer step to fragments of the
    model on different schedules; the stagger itself is not given in the paper): fragment f of
    F has its outer boundaries at the steps t >= 1 with t mod H == floor(f H / F)."""
    return (f * H) // F


def is_boundary(t, H, offset=0):
    return t >= 1 and t % H == offset % H


def run_quadratic(variant, M, H, phases, h, theta_star, seed, noise_std,
                  lr, beta1, beta2, eps, weight_decay, eta, mu, nesterov=True,
                  index_base=0, theta0=None, boundary_offset=0, overlap=1, first_boundary="listing"):
    """T = H * phases steps of Algorithm 1 ("standard"), 2 ("delayed") or 3 ("eager")
    on the noisy quadratic, starting from theta = theta0 (default 0) on every replica.
    Outer boundaries fall on the steps t with t mod H == boundary_offset mod H (the listings
    have boundary_offset = 0); the first one applies no outer step for Algorithms 2 and 3.
    overlap = 2 is the 2-outer-steps overlap of Section 3.2 ("Two-outer-steps overlap"), for
    which the paper gives no formula (PARITY UNPINNED against the paper).  Reading: the
    all-reduce launched at a boundary is consumed two boundaries later, i.e. Algorithms 2 and 3
    with Delta_m^(t-2H), Delta^(t-2H) in place of Delta_m^(t-H), Delta^(t-H) and `if t > 2H`;
    the two generations in flight live in two (P, D) slots used alternately.
    first_boundary: "listing" follows Algorithms 2 and 3 to the letter (`if t > H`: nothing is
    applied at the first boundary, the replica continues from its own parameters); "zero_history"
    is the introduction's wording instead (the local outer gradient is used in an outer step before
    the next phase starts): the outer step is applied at every boundary, the missing history being
    zero (Delta_m^(0) = Delta^(0) = 0, so eager feeds Delta_m / M and delayed feeds 0).  Only under
    zero history does an M = 1 eager run equal the standard run from the first phase on.
    Returns (state dict, losses) with losses[k] the loss after outer boundary k,
    evaluated at the replica mean of the outer parameters."""
    n = h.shape[0]
    theta = np.zeros((M, n), F64) if theta0 is None else np.tile(np.asarray(theta0, F64), (M, 1))
    m1 = np.zeros((M, n), F64)
    m2 = np.zeros((M, n), F64)
    shared = variant == "standard"
    a = theta[0].copy() if shared else theta.copy()
    u = np.zeros_like(a)
    Ps = [np.zeros((M, n), F64) for _ in range(overlap)]
    Ds = [np.zeros(n, F64) for _ in range(overlap)]
    losses = []
    boundaries = 0
    for t in range(1, H * phases + 1):
        quadratic_inner_step(theta, m1, m2, h, theta_star, t, seed, noise_std,
                             lr, beta1, beta2, eps, weight_decay, index_base)
        if is_boundary(t, H, boundary_offset):
            boundaries += 1
            if variant == "standard":
                outer_standard(theta, a, u, eta, mu, nesterov)
                losses.append(quadratic_loss(a, h, theta_star))
            else:
                step = outer_eager if variant == "eager" else outer_delayed
                slot = boundaries % overlap
                assert first_boundary in ("listing", "zero_history")
                step(theta, a, u, Ps[slot], Ds[slot], eta, mu, nesterov,
                     apply_update=(boundaries > overlap or first_boundary == "zero_history"))
                losses.append(quadratic_loss(mean_over_replicas(a), h, theta_star))
    out = dict(theta=theta, a=a, u=u, P=Ps[0], D=Ds[0], m1=m1, m2=m2)
    if overlap > 1:
        out.update(Ps=Ps, Ds=Ds)
    return out, losses


def run_streaming_quadratic(variant, fragments, M, H, phases, h, theta_star, seed, noise_std,
                            lr, beta1, beta2, eps, weight_decay, eta, mu, nesterov=True):
    """The same run with the model cut into fragments [(offset, count), ...] that take their
    outer steps on staggered schedules.  Every update of the path is element-wise, so a
    fragment is simply its own run of the algorithm on its slice with its own boundary offset."""
    F = len(fragments)
    out = []
    for f, (off, cnt) in enumerate(fragments):
        st, _ = run_quadratic(variant, M, H, phases, h[off:off + cnt], theta_star[off:off + cnt],
                              seed, noise_std, lr, beta1, beta2, eps, weight_decay, eta, mu,
                              nesterov, index_base=off, boundary_offset=stream_offset(H, F, f))
        out.append(st)
    return out
