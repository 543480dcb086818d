"""Per-call parity of the HIP library against the CPU checker, through the C ABI.

Every case draws seeded inputs on the CPU, widens them exactly to float64 for the checker,
uploads the same values, runs one library call and compares every output buffer element by
element.  fp32 buffers are held to 1e-6, bf16 buffers to 4e-3 (tests/util.py).
"""
import numpy as np
import pytest
import torch

import paper_2502_12996_amd as d
from oracle import diloco_oracle as O
from paper_2502_12996_amd import workloads as W
from tests import cases
from tests.util import (TOL_BF16, TOL_F32, adamw_scales, assert_close, checked_adamw, checked_eager,
                        checked_standard, quadratic_scales)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
ETA, MU = 0.7, 0.9


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    assert d.version() >= 100
    yield
    torch.cuda.synchronize()


def wl_for(M, n, bf16=False):
    return W.Workload("case", M=M, n=n, theta_dtype="bf16" if bf16 else "f32")


def run_eager_case(M, n, *, bf16=False, variant="eager", apply=True, nesterov=True, pad=0, seed=1,
                   misalign=0):
    """One diloco_outer_eager call against the checker; returns the worst error."""
    wl = wl_for(M, n, bf16)
    stride = n + pad
    st = W.outer_state(wl, n, seed=seed, stride=stride + misalign)
    if misalign:   # shift every buffer by `misalign` elements: still element-aligned, not 16-byte aligned
        st = {k: (v[:, misalign:] if v.dim() == 2 else v) for k, v in st.items()}
    ref = {k: W.to_f64(v[..., :n]) for k, v in st.items()}
    S = checked_eager(ref, ETA, MU, nesterov, apply, variant)
    full = {k: v.to(DEV) for k, v in W.outer_state(wl, n, seed=seed, stride=stride + misalign).items()}
    g = {k: (v[:, misalign:] if (misalign and v.dim() == 2) else v) for k, v in full.items()}
    before = {k: v.clone() for k, v in full.items()}
    d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], n=n,
                  outer_lr=ETA, outer_momentum=MU, nesterov=nesterov,
                  variant=d.EAGER if variant == "eager" else d.DELAYED, apply_update=apply)
    torch.cuda.synchronize()
    worst = 0.0
    for k in ref:
        got = W.to_f64(g[k][..., :n])
        tol = TOL_BF16 if (bf16 and k == "theta") else TOL_F32
        worst = max(worst, assert_close(got, ref[k], tol, f"{variant} M={M} n={n} {k}", scale=S[k]) / tol)
        # columns outside [0, n) of every row (padding, and the skipped leading elements) untouched
        if g[k].dim() == 2 and (pad or misalign):
            assert torch.equal(full[k][:, misalign + n:], before[k][:, misalign + n:]), k
            assert torch.equal(full[k][:, :misalign], before[k][:, :misalign]), k
    # re-seeding: the replica holds exactly its outer parameters (rounded to bf16 if stored so)
    want_theta = g["anchor"][:, :n].to(g["theta"].dtype)
    assert torch.equal(g["theta"][:, :n], want_theta)
    return worst


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 16, 33])
@pytest.mark.parametrize("n", [1, 3, 4, 5, 63, 64, 65, 1000, (1 << 16) + 1])
def test_eager_sizes_and_replica_counts(M, n):
    run_eager_case(M, n)


@pytest.mark.parametrize("variant", ["eager", "delayed"])
@pytest.mark.parametrize("apply", [True, False])
@pytest.mark.parametrize("nesterov", [True, False])
@pytest.mark.parametrize("M", [2, 8, 6])
def test_eager_variants_and_first_boundary(variant, apply, nesterov, M):
    run_eager_case(M, 70_003, variant=variant, apply=apply, nesterov=nesterov, seed=3)


@pytest.mark.parametrize("M", [1, 2, 8, 7])
@pytest.mark.parametrize("variant,apply", [("eager", True), ("delayed", True), ("eager", False)])
def test_eager_bf16_workers(M, variant, apply):
    run_eager_case(M, 50_001, bf16=True, variant=variant, apply=apply, seed=5)


@pytest.mark.parametrize("M", [2, 8, 5, 70])
def test_eager_padded_stride_and_elementwise_path(M):
    run_eager_case(M, 4097, pad=60, seed=9)            # padded rows, still 16-byte aligned
    run_eager_case(M, 4097, pad=2, seed=9)             # stride not a multiple of 4: element-wise path
    run_eager_case(M, 4097, pad=7, misalign=1, seed=9)  # base pointers off by one element
    run_eager_case(M, 1031, pad=7, misalign=1, bf16=True, seed=9)


def test_eager_large_M_paths_agree_bitwise():
    """Register, LDS-staged and element-wise kernels promise the same arithmetic in the same
    order: M = 8 through the register kernel equals M = 8 through the element-wise kernel."""
    n, M = 33_333, 8
    wl = wl_for(M, n)
    a = {k: v.to(DEV) for k, v in W.outer_state(wl, n, seed=11, stride=n + 2).items()}   # odd stride
    b = {k: v.to(DEV) for k, v in W.outer_state(wl, n, seed=11, stride=n + 3).items()}   # multiple of 4
    for s in (a, b):
        d.outer_eager(s["theta"], s["anchor"], s["vel"], s["prev_local"], s["prev_mean"], n=n,
                      outer_lr=ETA, outer_momentum=MU)
    torch.cuda.synchronize()
    for k in a:
        assert torch.equal(a[k][..., :n], b[k][..., :n]), k


@pytest.mark.parametrize("M", [2, 8, 9, 12, 16, 40, 41, 80, 83])
def test_eager_generic_paths_agree_bitwise(M):
    """Replica counts without a register instantiation run the grouped kernel, which stages the
    first 40 (generic_path 1: 80; 2: none) replicas in LDS and reads the others twice; every
    split promises the arithmetic of the register kernel in the same order.  A forced path also
    replaces the register kernel (M = 2, 8), which must not change a bit either."""
    n = 20_003
    out = []
    for path in (0, 1, 2):
        d.tune("generic_path", path)
        try:
            g = _rows(M, n, 71)
            d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"],
                          outer_lr=ETA, outer_momentum=MU)
            torch.cuda.synchronize()
            out.append(g)
        finally:
            d.tune("generic_path", 0)
    for k in out[0]:
        assert torch.equal(out[0][k], out[1][k]), k
        assert torch.equal(out[0][k], out[2][k]), k
    st = W.outer_state(wl_for(M, n), n, seed=71)
    ref = {k: W.to_f64(v) for k, v in st.items()}
    S = checked_eager(ref, ETA, MU)
    for k in ref:
        assert_close(W.to_f64(out[0][k]), ref[k], TOL_F32, f"grouped kernel M={M} {k}", scale=S[k])


@pytest.mark.parametrize("M,n", [(1000, 37), (65535, 5)])
def test_very_many_replicas(M, n):
    """The largest replica count the ABI takes (and one in between): outer steps, AdamW and reset."""
    wl = wl_for(M, n)
    st = W.outer_state(wl, n, seed=89, stride=n + 3)
    ref = {k: W.to_f64(v[..., :n]) for k, v in st.items()}
    S = checked_eager(ref, ETA, MU)
    g = {k: v.to(DEV) for k, v in st.items()}
    d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], n=n,
                  outer_lr=ETA, outer_momentum=MU)
    torch.cuda.synchronize()
    for k in ref:
        assert_close(W.to_f64(g[k][..., :n]), ref[k], TOL_F32, f"eager M={M} {k}", scale=S[k])
    if 3 * M + 1 <= 65535:
        pk = {k: v.to(DEV) for k, v in st.items()}
        state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
        d.pack_state(state, M, n, anchor=pk["anchor"], vel=pk["vel"], prev_local=pk["prev_local"],
                     prev_mean=pk["prev_mean"])
        d.outer_eager_packed(pk["theta"], state, n=n, outer_lr=ETA, outer_momentum=MU)
        d.unpack_state(state, M, n, anchor=pk["anchor"], vel=pk["vel"], prev_local=pk["prev_local"],
                       prev_mean=pk["prev_mean"])
        torch.cuda.synchronize()
        for k in g:
            assert torch.equal(pk[k], g[k]), k
    else:
        big = torch.empty(d.packed_state_elems(M, n), device=DEV)       # 6.4 GB: the size the call names
        with pytest.raises(d.DilocoError) as ei:
            d.pack_state(big, M, n, anchor=g["anchor"])
        assert ei.value.status == d.binding.ERR_SHAPE
        del big
    # standard outer step and reset
    st = W.outer_state(wl, n, seed=97)
    theta, a, u = st["theta"], st["anchor"][0].clone(), st["vel"][0].clone()
    rt, ra, ru = W.to_f64(theta), W.to_f64(a), W.to_f64(u)
    _, S = checked_standard(rt, ra, ru, ETA, MU, True)
    gt, ga, gu = theta.to(DEV), a.to(DEV), u.to(DEV)
    d.outer_sync(gt, ga, gu, outer_lr=ETA, outer_momentum=MU)
    th2 = torch.zeros_like(gt)
    d.reset(th2, ga)
    torch.cuda.synchronize()
    assert_close(W.to_f64(ga), ra, TOL_F32, f"sync anchor M={M}", scale=S["anchor"])
    assert_close(W.to_f64(gu), ru, TOL_F32, f"sync vel M={M}", scale=S["vel"])
    assert torch.equal(gt, ga.expand(M, n)) and torch.equal(th2, gt)
    # AdamW: grid.y = replica
    ad = W.adamw_state(wl, n, seed=101)
    refa = {k: W.to_f64(v) for k, v in ad.items()}
    S = checked_adamw(refa, 3, 4e-4, 0.9, 0.95, 1e-8, 0.1)
    ga = {k: v.to(DEV) for k, v in ad.items()}
    d.inner_adamw(ga["theta"], ga["m1"], ga["m2"], ga["grad"], lr=4e-4, beta1=0.9, beta2=0.95, eps=1e-8,
                  weight_decay=0.1, step=3)
    torch.cuda.synchronize()
    for k in ("theta", "m1", "m2"):
        assert_close(W.to_f64(ga[k]), refa[k], TOL_F32, f"adamw M={M} {k}", scale=S[k])
    with pytest.raises(d.DilocoError) as ei:
        d.outer_sync(torch.zeros((65536, 4), device=DEV), torch.zeros(4, device=DEV), torch.zeros(4, device=DEV),
                     outer_lr=ETA, outer_momentum=MU)
    assert ei.value.status == d.binding.ERR_SHAPE


@pytest.mark.parametrize("K", [1, 2, 4, 5, 8, 9, 16, 17, 33])
def test_stream_rmw_leaves_the_rows_as_they_are(K):
    n = 70_004
    rows = torch.empty((K, n + 8), device=DEV).normal_()
    before = rows.clone()
    d.sim_stream_rmw(rows, n=n)
    d.tune("wg_per_cu", 2)
    d.sim_stream_rmw(rows, n=n)
    d.tune("wg_per_cu", -1)
    torch.cuda.synchronize()
    assert torch.equal(rows, before)
    for bad in (dict(n=n + 1), dict(n=n + 12)):
        with pytest.raises(d.DilocoError):
            d.sim_stream_rmw(rows, **bad)
    if K == 4:
        with pytest.raises(d.DilocoError):
            d.sim_stream_rmw(torch.zeros((3, 64), device=DEV))


@pytest.mark.parametrize("K", [1, 5, 33])
def test_stream_sweep_modes(K):
    """The read-only sweep writes nothing, the write-only sweep fills exactly the first n elements of every row."""
    n = 70_004
    rows = torch.empty((K, n + 8), device=DEV).normal_()
    before = rows.clone()
    d.sim_stream_sweep(rows, d.SWEEP_READ, n=n)
    d.sim_stream_sweep(rows, d.SWEEP_RMW, n=n, launch=(256, 1, 2))
    torch.cuda.synchronize()
    assert torch.equal(rows, before)
    rows[0, 5] = float("nan")          # a NaN among the inputs must not make the read-only sweep write either
    before = rows.clone()
    d.sim_stream_sweep(rows, d.SWEEP_READ, n=n)
    torch.cuda.synchronize()
    assert torch.equal(rows.view(torch.int32), before.view(torch.int32))
    d.sim_stream_sweep(rows, d.SWEEP_WRITE, n=n, fill=2.5)
    torch.cuda.synchronize()
    assert (rows[:, :n] == 2.5).all() and torch.equal(rows[:, n:], before[:, n:])
    with pytest.raises(d.DilocoError) as ei:
        d.sim_stream_sweep(rows, 3, n=n)
    assert ei.value.status == d.binding.ERR_DTYPE


def test_eager_empty_input_is_a_noop():
    wl = wl_for(2, 8)
    g = {k: v.to(DEV) for k, v in W.outer_state(wl, 8, seed=2).items()}
    before = {k: v.clone() for k, v in g.items()}
    d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], n=0,
                  outer_lr=ETA, outer_momentum=MU)
    torch.cuda.synchronize()
    for k in g:
        assert torch.equal(g[k], before[k])


# ------------------------------------------------------------------ standard outer step
@pytest.mark.parametrize("M", [1, 2, 3, 8, 33])
@pytest.mark.parametrize("n", [1, 5, 64, 65, 4099, (1 << 16) + 3])
@pytest.mark.parametrize("bf16", [False, True])
def test_sync_outer_step(M, n, bf16):
    wl = wl_for(M, n, bf16)
    st = W.outer_state(wl, n, seed=13)
    theta, a, u = st["theta"], st["anchor"][0].clone(), st["vel"][0].clone()
    rt, ra, ru = W.to_f64(theta), W.to_f64(a), W.to_f64(u)
    rmean, S = checked_standard(rt, ra, ru, ETA, MU, True)
    gt, ga, gu = theta.to(DEV), a.to(DEV), u.to(DEV)
    gm = torch.empty(n, device=DEV)
    d.outer_sync(gt, ga, gu, mean_out=gm, outer_lr=ETA, outer_momentum=MU)
    torch.cuda.synchronize()
    assert_close(W.to_f64(ga), ra, TOL_F32, "sync anchor", scale=S["anchor"])
    assert_close(W.to_f64(gu), ru, TOL_F32, "sync vel", scale=S["vel"])
    assert_close(W.to_f64(gm), rmean, TOL_F32, "sync mean", scale=S["mean"])
    assert_close(W.to_f64(gt), rt, TOL_BF16 if bf16 else TOL_F32, "sync theta", scale=S["theta"])
    assert torch.equal(gt, ga.to(gt.dtype).expand(M, n))


def test_sync_heavy_ball_misaligned_and_no_mean_out():
    M, n = 3, 2050
    wl = wl_for(M, n)
    st = W.outer_state(wl, n + 1, seed=17)
    theta, a, u = st["theta"][:, 1:], st["anchor"][0, 1:].clone(), st["vel"][0, 1:].clone()
    rt, ra, ru = W.to_f64(theta), W.to_f64(a), W.to_f64(u)
    _, S = checked_standard(rt, ra, ru, 0.4, 0.5, False)
    gfull = st["theta"].to(DEV)
    gt = gfull[:, 1:]
    gab, gub = torch.zeros(n + 1, device=DEV), torch.zeros(n + 1, device=DEV)
    ga, gu = gab[1:], gub[1:]
    ga.copy_(a)
    gu.copy_(u)
    d.outer_sync(gt, ga, gu, n=n, outer_lr=0.4, outer_momentum=0.5, nesterov=False)
    torch.cuda.synchronize()
    assert_close(W.to_f64(ga), ra, TOL_F32, "anchor", scale=S["anchor"])
    assert_close(W.to_f64(gu), ru, TOL_F32, "vel", scale=S["vel"])
    assert_close(W.to_f64(gt), rt, TOL_F32, "theta", scale=S["theta"])
    assert torch.equal(gfull[:, 0].cpu(), st["theta"][:, 0])


def test_sync_momentum_off_lr_one_is_the_replica_average():
    M, n = 8, 10_001
    theta = W.normal((M, n), 0.02, tag="theta", seed=21)
    want = theta.double().mean(dim=0).numpy()
    gt = theta.to(DEV)
    ga = W.normal((n,), 0.02, tag="anchor", seed=21).to(DEV)
    gu = W.normal((n,), 1.0, tag="vel", seed=21).to(DEV)
    d.outer_sync(gt, ga, gu, outer_lr=1.0, outer_momentum=0.0)
    torch.cuda.synchronize()
    a0 = W.to_f64(W.normal((n,), 0.02, tag="anchor", seed=21))
    scale = np.abs(a0) + np.mean(np.abs(a0[None, :] - W.to_f64(theta)), axis=0)
    assert_close(W.to_f64(ga), want, TOL_F32, "replica average", scale=scale)


# ------------------------------------------------------------------ reset
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shared", [True, False])
@pytest.mark.parametrize("n,off", [(1, 0), (4099, 0), (4099, 1), (1 << 16, 0)])
def test_reset(bf16, shared, n, off):
    M = 3
    dt = torch.bfloat16 if bf16 else torch.float32
    a = W.normal((M, n + off), 0.02, tag="anchor", seed=23).to(DEV)
    src = a[0, off:] if shared else a[:, off:]
    base = torch.full((M, n + off + 5), 7.0, dtype=dt, device=DEV)
    th = base[:, off:off + n]
    for _ in range(2):   # idempotent
        d.reset(th, src, n=n)
    torch.cuda.synchronize()
    want = (src.expand(M, n) if shared else src).to(dt)
    assert torch.equal(th, want)
    assert (base[:, off + n:] == 7.0).all() and (base[:, :off] == 7.0).all()


# ------------------------------------------------------------------ inner AdamW
@pytest.mark.parametrize("pdt,gdt", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32"), ("f32", "bf16")])
@pytest.mark.parametrize("M,n,pad,off", [(1, 1, 0, 0), (2, 5, 3, 0), (4, 65, 0, 0), (3, 4099, 5, 1),
                                         (8, (1 << 16) + 2, 2, 0), (2, 1 << 18, 0, 0)])
@pytest.mark.parametrize("step", [1, 31])
def test_inner_adamw(pdt, gdt, M, n, pad, off, step):
    wl = wl_for(M, n, pdt == "bf16")
    gd = torch.bfloat16 if gdt == "bf16" else torch.float32
    st = W.adamw_state(wl, n + off, seed=29, stride=n + off + pad, grad_dtype=gd)
    view = {k: v[:, off:off + n] for k, v in st.items()}
    ref = {k: W.to_f64(v) for k, v in view.items()}
    S = checked_adamw(ref, step, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay)
    full = {k: v.to(DEV) for k, v in st.items()}
    before = {k: v.clone() for k, v in full.items()}
    g = {k: v[:, off:] for k, v in full.items()}
    d.inner_adamw(g["theta"], g["m1"], g["m2"], g["grad"], n=n, lr=wl.lr, beta1=wl.beta1,
                  beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay, step=step)
    torch.cuda.synchronize()
    tol = TOL_BF16 if pdt == "bf16" else TOL_F32
    for k in ("theta", "m1", "m2"):
        assert_close(W.to_f64(g[k][:, :n]), ref[k], tol, f"adamw {k}", scale=S[k])
        assert torch.equal(full[k][:, off + n:], before[k][:, off + n:])
        assert torch.equal(full[k][:, :off], before[k][:, :off])
    assert torch.equal(full["grad"], before["grad"])


def test_inner_adamw_zero_state_first_step_and_zero_gradient():
    M, n = 2, 1003
    th = W.normal((M, n), 0.02, tag="theta", seed=31)
    g = W.normal((M, n), 1e-2, tag="grad", seed=31)
    g[0, :10] = 0.0
    rt, rg = W.to_f64(th), W.to_f64(g)
    r1, r2 = np.zeros((M, n)), np.zeros((M, n))
    S = adamw_scales(rt, r1, r2, rg, 1, 4e-4, 0.9, 0.95, 1e-8, 0.1)
    O.adamw_step(rt, r1, r2, rg, 1, 4e-4, 0.9, 0.95, 1e-8, 0.1)
    gt, gg = th.to(DEV), g.to(DEV)
    g1, g2 = torch.zeros((M, n), device=DEV), torch.zeros((M, n), device=DEV)
    d.inner_adamw(gt, g1, g2, gg, lr=4e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1)
    torch.cuda.synchronize()
    assert_close(W.to_f64(gt), rt, TOL_F32, "theta", scale=S["theta"])
    assert_close(W.to_f64(g1), r1, TOL_F32, "m1", scale=S["m1"])
    assert_close(W.to_f64(g2), r2, TOL_F32, "m2", scale=S["m2"])
    assert np.isfinite(W.to_f64(gt)).all()


# ------------------------------------------------------------------ noisy quadratic
@pytest.mark.parametrize("M,n,base", [(1, 7, 0), (4, 4099, 0), (3, 1 << 14, 1 << 26), (2, 1001, (1 << 33) + 4)])
def test_quadratic_inner_step_and_loss(M, n, base):
    wl = W.WORKLOADS["quadratic"]
    h = W.log_uniform((n,), 1e-3, 1.0, tag="h", seed=37)
    star = W.normal((n,), 1.0, tag="theta_star", seed=37)
    ns = (n + 3) & ~3     # this entry point wants replica rows 16-byte aligned
    th = W.normal((M, ns), 0.5, tag="theta", seed=37)
    m1 = W.normal((M, ns), 0.1, tag="m1", seed=37)
    m2 = W.normal((M, ns), 0.1, tag="m2", seed=37).square_()
    rt, r1, r2 = (W.to_f64(x[:, :n]) for x in (th, m1, m2))
    rh, rs = W.to_f64(h), W.to_f64(star)
    seed, step = 0xC0FFEE, 17
    S = quadratic_scales(rt, r1, r2, rh, rs, wl.noise_std, seed, step, wl.lr, wl.beta1, wl.beta2, wl.eps, 0.0, base)
    O.quadratic_inner_step(rt, r1, r2, rh, rs, step, seed, wl.noise_std, wl.lr, wl.beta1, wl.beta2,
                           wl.eps, 0.0, index_base=base)
    gt, g1, g2, gh, gs = (x.to(DEV) for x in (th, m1, m2, h, star))
    d.sim_quadratic_inner(gt, g1, g2, gh, gs, n=n, noise_std=wl.noise_std, seed=seed, index_base=base,
                          lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=0.0,
                          step=step)
    part = torch.empty(d.sim_loss_workspace(n), dtype=torch.float64, device=DEV)
    out = torch.empty(1, dtype=torch.float64, device=DEV)
    d.sim_quadratic_loss(gt, gh, gs, part, out, n=n)
    torch.cuda.synchronize()
    assert torch.equal(gt[:, n:].cpu(), th[:, n:])
    gt, g1, g2 = gt[:, :n], g1[:, :n], g2[:, :n]
    # the gradient noise goes through fp32 log / sincos: a few 1e-7 relative on z, which AdamW's
    # normalised step turns into the same relative error of the update (lr-sized), far inside 1e-6
    assert_close(W.to_f64(gt), rt, TOL_F32, "theta", scale=S["theta"])
    assert_close(W.to_f64(g1), r1, TOL_F32, "m1", scale=S["m1"])
    assert_close(W.to_f64(g2), r2, TOL_F32, "m2", scale=S["m2"])
    want = O.quadratic_loss(O.mean_over_replicas(W.to_f64(gt)), rh, rs)
    assert abs(out.item() - want) <= 1e-12 * max(want, 1e-300)


@pytest.mark.parametrize("M,n,base,first,steps", [(1, 7, 0, 1, 5), (4, 4099, 0, 1, 50), (3, 1 << 14, 1 << 26, 51, 64),
                                                   (2, 1001, (1 << 33) + 4, 1999, 1), (2, 70_001, 8, 3, 0)])
def test_quadratic_fused_phase_equals_separate_steps_bitwise(M, n, base, first, steps):
    """One pass over `steps` inner steps in registers against the same steps launched one by one
    (which the tests above hold to the checker step by step), and against the checker directly."""
    wl = W.WORKLOADS["quadratic"]
    h = W.log_uniform((n,), 1e-3, 1.0, tag="h", seed=39)
    star = W.normal((n,), 1.0, tag="theta_star", seed=39)
    ns = (n + 3) & ~3
    th = W.normal((M, ns), 0.5, tag="theta", seed=39)
    m1 = W.normal((M, ns), 0.1, tag="m1", seed=39)
    m2 = W.normal((M, ns), 0.1, tag="m2", seed=39).square_()
    kw = dict(n=n, noise_std=wl.noise_std, seed=0xBEEF, index_base=base, lr=wl.lr, beta1=wl.beta1,
              beta2=wl.beta2, eps=wl.eps, weight_decay=0.0)
    a = [x.to(DEV) for x in (th, m1, m2)]
    b = [x.to(DEV) for x in (th, m1, m2)]
    gh, gs = h.to(DEV), star.to(DEV)
    for t in range(first, first + steps):
        d.sim_quadratic_inner(*a, gh, gs, step=t, **kw)
    d.sim_quadratic_phase(*b, gh, gs, step_first=first, steps=steps, **kw)
    torch.cuda.synchronize()
    for x, y, name in zip(a, b, ("theta", "m1", "m2")):
        assert torch.equal(x, y), name
    assert torch.equal(b[0][:, n:].cpu(), th[:, n:])
    if steps and n <= 5000:
        rt, r1, r2 = (W.to_f64(x[:, :n]) for x in (th, m1, m2))
        rh, rs = W.to_f64(h), W.to_f64(star)
        for t in range(first, first + steps):
            if t == first + steps - 1:     # the operand scales of the last step
                S = quadratic_scales(rt, r1, r2, rh, rs, wl.noise_std, 0xBEEF, t, wl.lr, wl.beta1, wl.beta2,
                                     wl.eps, 0.0, base)
            O.quadratic_inner_step(rt, r1, r2, rh, rs, t, 0xBEEF, wl.noise_std, wl.lr, wl.beta1, wl.beta2,
                                   wl.eps, 0.0, index_base=base)
        # per-step differences of a few 1e-7 (fp32 log / sincos in the noise) add up over the steps
        tol = TOL_F32 * max(1, steps) ** 0.5 * 2
        assert_close(W.to_f64(b[0][:, :n]), rt, tol, "theta after the phase", scale=S["theta"])
        assert_close(W.to_f64(b[1][:, :n]), r1, tol, "m1 after the phase", scale=S["m1"])
        assert_close(W.to_f64(b[2][:, :n]), r2, tol, "m2 after the phase", scale=S["m2"])


def test_quadratic_fused_phase_rejects_too_many_steps():
    z = torch.zeros((2, 64), device=DEV)
    v = torch.ones(64, device=DEV)
    with pytest.raises(d.DilocoError) as ei:
        d.sim_quadratic_phase(z, z.clone(), z.clone(), v, v.clone(), noise_std=0.1, seed=1, lr=4e-4, beta1=0.9,
                              beta2=0.95, eps=1e-8, weight_decay=0.0, step_first=1,
                              steps=d.binding.SIM_MAX_FUSED_STEPS + 1)
    assert ei.value.status == d.binding.ERR_SHAPE
    assert not z.any()


# ------------------------------------------------------------------ packed (tile-interleaved) outer state
def _rows(M, n, seed, bf16=False, pad=0):
    return {k: v.to(DEV) for k, v in W.outer_state(wl_for(M, n, bf16), n, seed=seed, stride=n + pad).items()}


@pytest.mark.parametrize("M", [1, 3, 8])
@pytest.mark.parametrize("n,pad", [(1, 0), (8191, 1), (8192, 0), (8193, 3), (3 * 8192 + 5, 2), (70_003, 1)])
def test_pack_unpack_roundtrip_and_layout(M, n, pad):
    g = _rows(M, n, 41, pad=pad)
    state = torch.full((d.packed_state_elems(M, n),), -7.0, device=DEV)
    d.pack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                 prev_mean=g["prev_mean"])
    torch.cuda.synchronize()
    # the documented layout: [tile][a_0..a_{M-1}, D, u_0, P_0, u_1, P_1, ...][STATE_TILE]
    S, T = 3 * M + 1, d.STATE_TILE
    tiles = (n + T - 1) // T
    v = state.view(tiles, S, T).cpu()
    for m in range(M):
        for pos, name in ((m, "anchor"), (M + 1 + 2 * m, "vel"), (M + 2 + 2 * m, "prev_local")):
            rows = g[name][m, :n].cpu()
            got = v[:, pos, :].reshape(-1)[:n]
            assert torch.equal(got, rows), (m, name)
    assert torch.equal(v[:, M, :].reshape(-1)[:n], g["prev_mean"].cpu())
    assert (v.reshape(tiles, S, T)[-1, :, n - (tiles - 1) * T:] == -7.0).all()   # padding untouched
    out = {k: torch.zeros_like(x) for k, x in g.items() if k != "theta"}
    d.unpack_state(state, M, n, anchor=out["anchor"], vel=out["vel"], prev_local=out["prev_local"],
                   prev_mean=out["prev_mean"])
    torch.cuda.synchronize()
    for k in out:
        assert torch.equal(out[k][..., :n], g[k][..., :n]), k
        if out[k].dim() == 2 and pad:
            assert (out[k][:, n:] == 0).all()
    # partial pack: only the anchors, the rest of the state stays
    before = state.clone()
    d.pack_state(state, M, n, anchor=g["vel"])
    torch.cuda.synchronize()
    v2 = state.view(tiles, S, T).cpu()
    assert torch.equal(v2[:, 0, :].reshape(-1)[:n], g["vel"][0, :n].cpu())
    assert torch.equal(v2[:, M, :], before.view(tiles, S, T)[:, M, :].cpu())


@pytest.mark.parametrize("M", [1, 2, 3, 4, 8, 5, 7, 9, 16, 33])
@pytest.mark.parametrize("n", [1, 5, 8191, 8193, 70_003])
@pytest.mark.parametrize("variant,apply", [("eager", True), ("delayed", True), ("eager", False)])
def test_eager_packed_is_bit_identical_to_rows(M, n, variant, apply):
    bf16 = (M + n) % 2 == 0
    rows = _rows(M, n, 43, bf16)
    pk = _rows(M, n, 43, bf16)
    state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
    d.pack_state(state, M, n, anchor=pk["anchor"], vel=pk["vel"], prev_local=pk["prev_local"],
                 prev_mean=pk["prev_mean"])
    var = d.EAGER if variant == "eager" else d.DELAYED
    d.outer_eager(rows["theta"], rows["anchor"], rows["vel"], rows["prev_local"], rows["prev_mean"],
                  outer_lr=ETA, outer_momentum=MU, variant=var, apply_update=apply)
    d.outer_eager_packed(pk["theta"], state, outer_lr=ETA, outer_momentum=MU, variant=var,
                         apply_update=apply)
    d.unpack_state(state, M, n, anchor=pk["anchor"], vel=pk["vel"], prev_local=pk["prev_local"],
                   prev_mean=pk["prev_mean"])
    torch.cuda.synchronize()
    for k in rows:
        assert torch.equal(rows[k], pk[k]), k


def test_eager_packed_against_the_checker_and_elementwise_path():
    M, n = 8, 50_003
    st = W.outer_state(wl_for(M, n), n, seed=47, stride=n + 2)      # odd theta stride: element-wise path
    ref = {k: W.to_f64(v[..., :n]) for k, v in st.items()}
    S = checked_eager(ref, ETA, MU)
    g = {k: v.to(DEV) for k, v in st.items()}
    state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
    d.pack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                 prev_mean=g["prev_mean"])
    d.outer_eager_packed(g["theta"], state, n=n, outer_lr=ETA, outer_momentum=MU)
    d.unpack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                   prev_mean=g["prev_mean"])
    torch.cuda.synchronize()
    for k in ref:
        assert_close(W.to_f64(g[k][..., :n]), ref[k], TOL_F32, f"packed {k}", scale=S[k])


@pytest.mark.parametrize("M", [1, 2, 3, 8, 5, 9, 16, 33, 42])
@pytest.mark.parametrize("n,pad", [(1, 0), (5, 3), (8191, 1), (8193, 0), (70_003, 1), (70_003, 2)])
@pytest.mark.parametrize("flags", ["plain", "delayed", "no_mean+bf16", "fp4"])
def test_eager_pingpong_walks_the_in_place_trajectory_bit_for_bit(M, n, pad, flags):
    """Five boundaries (the first only records, so the velocities must be carried across) through
    diloco_outer_eager_pingpong with two alternating state buffers against the in-place packed
    call: theta after every boundary and the final state, bit for bit.  pad 2 gives theta an odd
    row stride: the element-wise kernel."""
    bf16 = (M + n) % 2 == 1
    var = {"plain": d.EAGER, "delayed": d.DELAYED, "no_mean+bf16": d.EAGER | d.STATE_NO_MEAN | d.COMM_BF16,
           "fp4": d.EAGER | d.COMM_EXMY(2, 1, 11)}[flags]
    runs = []
    for pingpong in (False, True):
        g = _rows(M, n, 127, bf16, pad=pad)
        g["vel"].normal_(0, 1e-3, generator=torch.Generator(device=DEV).manual_seed(5))   # must survive recording
        states = [torch.full((d.packed_state_elems(M, n),), float("nan"), device=DEV) for _ in range(2)]
        d.pack_state(states[0], M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                     prev_mean=g["prev_mean"])
        thetas = []
        cur = 0
        for phase in range(5):
            noise = W.normal((M, n), 1e-3, tag="theta_noise", seed=127, extra=phase, device=DEV)
            g["theta"][:, :n] = (g["theta"][:, :n].float() + noise).to(g["theta"].dtype)
            kw = dict(n=n, outer_lr=ETA, outer_momentum=MU, variant=var, apply_update=phase > 0)
            if pingpong:
                d.outer_eager_pingpong(g["theta"], states[cur], states[1 - cur], **kw)
                cur = 1 - cur
            else:
                d.outer_eager_packed(g["theta"], states[0], **kw)
            thetas.append(g["theta"].clone())
        out = {k: torch.zeros_like(g[k]) for k in ("anchor", "vel", "prev_local", "prev_mean")}
        d.unpack_state(states[cur], M, n, anchor=out["anchor"], vel=out["vel"], prev_local=out["prev_local"],
                       prev_mean=None if "no_mean" in flags else out["prev_mean"])
        torch.cuda.synchronize()
        runs.append((thetas, out))
    for a, b in zip(runs[0][0], runs[1][0]):
        assert torch.equal(a, b)
    for k in runs[0][1]:
        assert torch.equal(runs[0][1][k], runs[1][1][k]), k
        assert torch.isfinite(runs[1][1][k]).all(), k          # every stream of the fresh buffer was written


def test_eager_pingpong_against_the_checker_and_refusals():
    M, n = 8, 50_003
    st = W.outer_state(wl_for(M, n), n, seed=131)
    ref = {k: W.to_f64(v) for k, v in st.items()}
    S = checked_eager(ref, ETA, MU)
    g = {k: v.to(DEV) for k, v in st.items()}
    a, b = (torch.zeros(d.packed_state_elems(M, n), device=DEV) for _ in range(2))
    d.pack_state(a, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"], prev_mean=g["prev_mean"])
    before = a.clone()
    d.outer_eager_pingpong(g["theta"], a, b, outer_lr=ETA, outer_momentum=MU, launch=(256, 1, 2))
    d.unpack_state(b, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"], prev_mean=g["prev_mean"])
    torch.cuda.synchronize()
    assert torch.equal(a, before)                               # the input state is read only
    for k in ref:
        assert_close(W.to_f64(g[k]), ref[k], TOL_F32, f"pingpong {k}", scale=S[k])
    with pytest.raises(d.DilocoError) as ei:
        d.outer_eager_pingpong(g["theta"], a, a, outer_lr=ETA, outer_momentum=MU)
    assert ei.value.status == d.binding.ERR_ALIAS
    with pytest.raises(ValueError):
        d.outer_eager_pingpong(g["theta"], a, b[:-8192], outer_lr=ETA, outer_momentum=MU)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("n,pad", [(5, 0), (8193, 0), (20_001, 1)])
def test_reset_packed(bf16, n, pad):
    M = 3
    g = _rows(M, n, 53, bf16, pad=pad)
    state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
    d.pack_state(state, M, n, anchor=g["anchor"])
    th = torch.full_like(g["theta"], 3.0)
    d.reset_packed(th, state, n=n)
    torch.cuda.synchronize()
    assert torch.equal(th[:, :n], g["anchor"][:, :n].to(th.dtype))
    if pad:
        assert (th[:, n:] == 3.0).all()


# ------------------------------------------------------------------ bf16 on the wire (Section 3.2)
@pytest.mark.parametrize("M", [1, 2, 8, 5, 33])
@pytest.mark.parametrize("variant,apply", [("eager", True), ("delayed", True), ("eager", False)])
@pytest.mark.parametrize("packed", [False, True])
def test_eager_with_bf16_communication(M, variant, apply, packed):
    n = 30_005
    st = W.outer_state(wl_for(M, n), n, seed=59)
    ref = {k: W.to_f64(v) for k, v in st.items()}
    S = checked_eager(ref, ETA, MU, True, apply, variant, comm="bf16")
    g = {k: v.to(DEV) for k, v in st.items()}
    var = (d.EAGER if variant == "eager" else d.DELAYED) | d.COMM_BF16
    if packed:
        state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
        d.pack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                     prev_mean=g["prev_mean"])
        d.outer_eager_packed(g["theta"], state, outer_lr=ETA, outer_momentum=MU, variant=var,
                             apply_update=apply)
        d.unpack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                       prev_mean=g["prev_mean"])
    else:
        d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"],
                      outer_lr=ETA, outer_momentum=MU, variant=var, apply_update=apply)
    torch.cuda.synchronize()
    # what was sent is a bf16 code: bit-exact; everything else to the fp32 tolerance
    assert np.array_equal(W.to_f64(g["prev_local"]), ref["prev_local"])
    bf = g["prev_local"].to(torch.bfloat16).to(torch.float32)
    assert torch.equal(bf, g["prev_local"])
    for k in ref:
        assert_close(W.to_f64(g[k]), ref[k], TOL_F32, f"bf16 comm {variant} {k}", scale=S[k])


# ------------------------------------------------------------------ small floats on the wire (Section 3.2)
EXMY_FORMATS = [(2, 1, 11), (3, 0, 12), (4, 3, 16), (5, 2, 24), (5, 10, 15), (1, 0, 9), (7, 8, 60), (3, 4, -100),
                (2, 10, 117), (4, 3, -112), (6, 0, 30)]


def _rounding_probe(E, Mn, bias):
    """float32 values that exercise the format: every exact tie between neighbouring values (all
    of them for the small formats, 4096 sampled ones otherwise), the values themselves, the
    largest value and beyond, the subnormal range and below it, both signs, zero."""
    grid = O.exmy_values(E, Mn, bias)
    r = np.random.default_rng(E * 1000 + Mn * 10 + bias % 7)
    idx = np.arange(len(grid) - 1) if len(grid) <= 4096 else np.sort(r.choice(len(grid) - 1, 4096, replace=False))
    ties = (grid[idx] + grid[idx + 1]) / 2
    lo, hi = np.log2(grid[1]) - 4, np.log2(grid[-1]) + 2
    wide = r.standard_normal(60_000) * np.exp2(r.uniform(lo, hi, 60_000))
    x = np.concatenate([ties, -ties[::3], np.nextafter(ties.astype(np.float32), np.float32(0)),
                        np.nextafter(ties.astype(np.float32), np.float32(np.inf)), grid[idx], wide,
                        [0.0, grid[-1], -grid[-1], grid[-1] * 1.01, grid[-1] * 4, grid[1] / 2, grid[1] / 4]])
    with np.errstate(over="ignore"):
        x = x.astype(np.float32)
    return x[np.isfinite(x)]


@pytest.mark.parametrize("fmt", EXMY_FORMATS, ids=lambda f: "E%dM%db%d" % f)
@pytest.mark.parametrize("packed", [False, True])
def test_exmy_rounding_is_bit_exact(fmt, packed):
    """theta = 0 and a = x make Delta = x exactly; the recorded previous local gradient is then the
    library's rounding of x, compared bit for bit with the checker's."""
    E, Mn, bias = fmt
    x = _rounding_probe(E, Mn, bias)
    n, M = ((len(x) + 1) // 2) | 1, 2                 # odd n: the scalar tail takes part
    xs = torch.tensor(np.concatenate([x, np.zeros(2 * n - len(x), np.float32)]).reshape(2, n))
    stride = (n + 3) & ~3
    a = torch.zeros((M, stride), device=DEV)
    a[:, :n] = xs.to(DEV)
    theta, vel, P, D = torch.zeros_like(a), torch.zeros_like(a), torch.ones_like(a), torch.ones(n, device=DEV)
    var = d.EAGER | d.COMM_EXMY(E, Mn, bias)
    if packed:
        state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
        d.pack_state(state, M, n, anchor=a, vel=vel, prev_local=P, prev_mean=D)
        d.outer_eager_packed(theta, state, n=n, outer_lr=ETA, outer_momentum=MU, variant=var, apply_update=False)
        d.unpack_state(state, M, n, prev_local=P, prev_mean=D)
    else:
        d.outer_eager(theta, a, vel, P, D, n=n, outer_lr=ETA, outer_momentum=MU, variant=var, apply_update=False)
    torch.cuda.synchronize()
    want = O.round_to_exmy(xs.numpy(), E, Mn, bias)
    got = W.to_f64(P[:, :n])
    bad = np.nonzero(got != want)
    assert bad[0].size == 0, (fmt, xs.numpy()[bad][:5], got[bad][:5], want[bad][:5])
    assert np.array_equal(np.signbit(got), np.signbit(want))
    assert_close(W.to_f64(D), want.mean(axis=0), TOL_F32, f"mean of {fmt}", scale=np.abs(want).mean(axis=0))


@pytest.mark.parametrize("M", [1, 2, 8, 9, 33])
@pytest.mark.parametrize("variant,apply", [("eager", True), ("delayed", True), ("eager", False)])
@pytest.mark.parametrize("packed,misalign", [(False, 0), (True, 0), (False, 1)])
@pytest.mark.parametrize("fmt", [(2, 1, 11), (4, 3, 16)], ids=["fp4", "fp8"])
def test_eager_with_exmy_communication(M, variant, apply, packed, misalign, fmt):
    n = 20_003
    wl = wl_for(M, n)
    cut = (lambda v: v[:, misalign:misalign + n] if v.dim() == 2 else v)
    st = {k: cut(v) for k, v in W.outer_state(wl, n, seed=61, stride=n + 8).items()}
    ref = {k: W.to_f64(v) for k, v in st.items()}
    S = checked_eager(ref, ETA, MU, True, apply, variant, comm=("exmy",) + fmt)
    g = {k: cut(v.to(DEV)) for k, v in W.outer_state(wl, n, seed=61, stride=n + 8).items()}
    var = (d.EAGER if variant == "eager" else d.DELAYED) | d.COMM_EXMY(*fmt)
    if packed:
        state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
        d.pack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                     prev_mean=g["prev_mean"])
        d.outer_eager_packed(g["theta"], state, n=n, outer_lr=ETA, outer_momentum=MU, variant=var,
                             apply_update=apply)
        d.unpack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                       prev_mean=g["prev_mean"])
    else:
        d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], n=n,
                      outer_lr=ETA, outer_momentum=MU, variant=var, apply_update=apply)
    torch.cuda.synchronize()
    assert np.array_equal(W.to_f64(g["prev_local"]), ref["prev_local"])        # codes: bit-exact
    assert len(np.unique(np.abs(ref["prev_local"]))) <= 1 << (fmt[0] + fmt[1])
    for k in ref:
        assert_close(W.to_f64(g[k]), ref[k], TOL_F32, f"exmy {fmt} comm {variant} {k}", scale=S[k])


@pytest.mark.parametrize("M", [1, 3, 8, 12])
@pytest.mark.parametrize("comm", ["bf16", (2, 1, 11), (4, 3, 16)], ids=["bf16", "fp4", "fp8"])
@pytest.mark.parametrize("misalign", [0, 1])
def test_standard_outer_step_with_quantised_communication(M, comm, misalign):
    n = 20_003
    wl = wl_for(M, n)
    st = W.outer_state(wl, n, seed=67, stride=n + 8)
    theta = st["theta"][:, misalign:misalign + n]
    a, u = st["anchor"][0, :n].clone(), st["vel"][0, :n].clone()
    rt, ra, ru = W.to_f64(theta), W.to_f64(a), W.to_f64(u)
    want_mean, S = checked_standard(rt, ra, ru, ETA, MU, True, comm=cases.oracle_comm(comm))
    gt = st["theta"].to(DEV)[:, misalign:misalign + n]
    ga, gu, gm = a.to(DEV), u.to(DEV), torch.zeros(n, device=DEV)
    d.outer_sync(gt, ga, gu, n=n, mean_out=gm, outer_lr=ETA, outer_momentum=MU,
                 comm=d.COMM_BF16 if comm == "bf16" else d.COMM_EXMY(*comm))
    torch.cuda.synchronize()
    assert_close(W.to_f64(gm), want_mean, TOL_F32, "mean of the rounded outer gradients", scale=S["mean"])
    assert_close(W.to_f64(ga), ra, TOL_F32, "anchor", scale=S["anchor"])
    assert_close(W.to_f64(gu), ru, TOL_F32, "vel", scale=S["vel"])
    assert torch.equal(gt, ga.expand(M, n))
    # the mean of M values of a coarse grid sits on the grid refined by 1/M: fp4 has 8 magnitudes
    if comm != "bf16" and comm[0] + comm[1] <= 3:
        q = 2.0 ** (1 - comm[2] - comm[1]) / M
        r = W.to_f64(gm) / q
        assert np.max(np.abs(r - np.rint(r))) < 1e-3
    # comm = 0 is the plain entry point
    p1, p2 = st["theta"].to(DEV), st["theta"].to(DEV)
    a1, a2, u1, u2 = a.to(DEV), a.to(DEV), u.to(DEV), u.to(DEV)
    d.outer_sync(p1, a1, u1, n=n, outer_lr=ETA, outer_momentum=MU)
    d.outer_sync(p2, a2, u2, n=n, outer_lr=ETA, outer_momentum=MU, comm=0)
    torch.cuda.synchronize()
    assert torch.equal(a1, a2) and torch.equal(u1, u2) and torch.equal(p1, p2)
    with pytest.raises(d.DilocoError) as ei:
        d.outer_sync(p1, a1, u1, n=n, outer_lr=ETA, outer_momentum=MU, comm=1)
    assert ei.value.status == d.binding.ERR_DTYPE


# ------------------------------------------------------------------ eager step that does not keep the previous mean
@pytest.mark.parametrize("M", [1, 2, 3, 8, 9, 16, 24, 26, 27, 33, 42])
@pytest.mark.parametrize("layout,misalign,bf16", [("rows", 0, False), ("rows", 1, False), ("packed", 0, False),
                                                   ("packed", 0, True)])
@pytest.mark.parametrize("comm", [0, "bf16"])
def test_eager_without_a_stored_mean_walks_the_same_trajectory_bit_for_bit(M, layout, misalign, bf16, comm):
    """Five boundaries (the first only records) with and without DILOCO_STATE_NO_MEAN: the mean the
    flagged calls form from prev_local is the one the plain calls stored, so every buffer but
    the mean itself must agree exactly; the flagged run never touches its mean buffer."""
    n = 24_579
    wl = wl_for(M, n, bf16)
    cflag = d.COMM_BF16 if comm == "bf16" else 0
    runs = []
    for flag in (0, d.STATE_NO_MEAN):
        st = {k: v.to(DEV) for k, v in W.outer_state(wl, n, seed=103, stride=n + 8).items()}
        g = {k: (v[:, misalign:misalign + n] if v.dim() == 2 else v) for k, v in st.items()}
        g["prev_mean"].fill_(7.0)
        for k in ("prev_local", "vel"):
            st[k].zero_()
        state = None
        if layout == "packed":
            state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
            d.pack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                         prev_mean=g["prev_mean"])
        for phase in range(5):
            noise = W.normal((M, n), 1e-3, tag="theta_noise", seed=103, extra=phase, device=DEV)
            g["theta"].copy_((g["theta"].float() + noise).to(g["theta"].dtype))
            kw = dict(n=n, outer_lr=ETA, outer_momentum=MU, variant=d.EAGER | cflag | flag, apply_update=phase > 0)
            if layout == "packed":
                d.outer_eager_packed(g["theta"], state, **kw)
            else:
                d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], **kw)
        if layout == "packed":
            d.unpack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                           prev_mean=g["prev_mean"])
        torch.cuda.synchronize()
        runs.append(g)
    plain, lean = runs
    for k in ("theta", "anchor", "vel", "prev_local"):
        assert torch.equal(plain[k], lean[k]), k
    assert (lean["prev_mean"] == 7.0).all() and not (plain["prev_mean"] == 7.0).any()


@pytest.mark.parametrize("M", [1, 2, 5, 8, 9, 24, 25, 33, 60])
@pytest.mark.parametrize("packed", [False, True])
def test_eager_without_a_stored_mean_against_the_checker(M, packed):
    n = 20_003
    st = W.outer_state(wl_for(M, n), n, seed=107)
    ref = {k: W.to_f64(v) for k, v in st.items()}
    S = checked_eager(ref, ETA, MU, no_mean=True)
    g = {k: v.to(DEV) for k, v in st.items()}
    g["prev_mean"].fill_(-3.0)          # must not matter
    if packed:
        state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
        d.pack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                     prev_mean=g["prev_mean"])
        d.outer_eager_packed(g["theta"], state, outer_lr=ETA, outer_momentum=MU, variant=d.EAGER | d.STATE_NO_MEAN)
        d.unpack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                       prev_mean=g["prev_mean"])
    else:
        d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], outer_lr=ETA,
                      outer_momentum=MU, variant=d.EAGER | d.STATE_NO_MEAN)
    torch.cuda.synchronize()
    for k in ("theta", "anchor", "vel", "prev_local"):
        assert_close(W.to_f64(g[k]), ref[k], TOL_F32, f"no stored mean M={M} {k}", scale=S[k])
    assert (g["prev_mean"] == -3.0).all()


def test_eager_without_a_stored_mean_is_refused_where_it_cannot_work():
    g = _rows(2, 64, 3)
    with pytest.raises(d.DilocoError) as ei:      # the delayed step reads nothing but the stored mean
        d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], outer_lr=ETA,
                      outer_momentum=MU, variant=d.DELAYED | d.STATE_NO_MEAN)
    assert ei.value.status == d.binding.ERR_DTYPE


@pytest.mark.parametrize("M", [4, 8, 9, 24, 26, 27, 53, 54, 70])
def test_eager_without_a_stored_mean_every_kernel_path_agrees_bitwise(M):
    """The register kernel (M <= 8), the grouped kernel staging all, some (24 with the third LDS slot;
    53 when forced to one workgroup per CU) or none of the replicas, and the element-wise kernel
    form the previous mean from the previous locals in the same order: same bits."""
    n = 12_291
    out = []
    for path, pad in ((0, 0), (1, 0), (2, 0), (0, 2)):       # pad 2: odd stride, element-wise kernel
        g = _rows(M, n, 5, pad=pad)
        g["prev_mean"].fill_(9.0)
        d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], n=n, outer_lr=ETA,
                      outer_momentum=MU, variant=d.EAGER | d.STATE_NO_MEAN, launch=(0, 0, -1, path))
        torch.cuda.synchronize()
        assert (g["prev_mean"] == 9.0).all()
        out.append(g)
    for other in out[1:]:
        for k in ("theta", "anchor", "vel", "prev_local"):
            assert torch.equal(out[0][k][:, :n], other[k][:, :n]), k
    # and the plain call with the mean the flag-less call would have stored
    g = _rows(M, n, 5)
    s = g["prev_local"][0].double()
    for m in range(1, M):
        s += g["prev_local"][m].double()
    g["prev_mean"].copy_((s * (1.0 / M)).float())
    d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], outer_lr=ETA, outer_momentum=MU)
    torch.cuda.synchronize()
    for k in ("theta", "anchor", "vel", "prev_local"):
        assert torch.equal(out[0][k], g[k]), k


@pytest.mark.parametrize("bits", [0x200, 0x800, 0x1000, 1 << 28, 0x100 | 0x200 | (4 << 12) | (3 << 16),
                                  "E0M3b0", "E9M1b0", "E5M11b0", "E8M7b127", "E8M2b100", "E4M3b-120", "E4M3b125", "E2M10b118", "E4M3b-113"])
def test_unknown_variant_bits_are_rejected(bits):
    if isinstance(bits, str):
        E, rest = bits[1:].split("M")
        Mn, bias = rest.split("b")
        bits = d.COMM_EXMY(int(E), int(Mn), int(bias))
    g = _rows(2, 64, 3)
    before = {k: v.clone() for k, v in g.items()}
    for call in ("rows", "packed"):
        with pytest.raises(d.DilocoError) as ei:
            if call == "rows":
                d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"],
                              outer_lr=ETA, outer_momentum=MU, variant=bits)
            else:
                d.outer_eager_packed(g["theta"], torch.zeros(d.packed_state_elems(2, 64), device=DEV),
                                     outer_lr=ETA, outer_momentum=MU, variant=bits)
        assert ei.value.status == d.binding.ERR_DTYPE
    torch.cuda.synchronize()
    for k in g:
        assert torch.equal(g[k], before[k])


# ------------------------------------------------------------------ launch shapes the benchmark may pick
DEFAULT_SHAPE = (0, 0, -1)        # workgroup size and occupancy cap chosen per launch, natural workgroup order


def set_shape(block, xcd, cap):
    d.tune("block", block)
    d.tune("xcd_remap", xcd)
    d.tune("wg_per_cu", cap)


@pytest.fixture
def launch_shape(request):
    set_shape(*request.param)
    yield request.param
    set_shape(*DEFAULT_SHAPE)


@pytest.mark.parametrize("launch_shape", [(64, 0, 0), (64, 1, -1), (128, 1, 0), (256, 0, 0), (256, 1, 0), (512, 0, 0),
                                          (512, 1, 0), (64, 0, 1), (64, 0, 3), (64, 1, 32), (128, 0, 5), (256, 0, 1),
                                          (256, 1, 2), (512, 0, 1), (0, 1, 2), (0, 0, 0)], indirect=True)
def test_every_launch_shape_gives_the_same_bits(launch_shape):
    """Workgroup size, XCD-contiguous workgroup order and the cap on resident workgroups (dynamic
    LDS up to a CU's whole 160 KB) only change who computes what, and when."""
    M, n = 8, 150_003                     # > 32 workgroups at every size, ragged tail
    # eager, rows and packed, against the default shape
    want = _rows(M, n, 73)
    got = _rows(M, n, 73)
    pk = _rows(M, n, 73)
    set_shape(*DEFAULT_SHAPE)
    d.outer_eager(want["theta"], want["anchor"], want["vel"], want["prev_local"], want["prev_mean"],
                  outer_lr=ETA, outer_momentum=MU)
    set_shape(*launch_shape)
    d.outer_eager(got["theta"], got["anchor"], got["vel"], got["prev_local"], got["prev_mean"],
                  outer_lr=ETA, outer_momentum=MU)
    state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
    d.pack_state(state, M, n, anchor=pk["anchor"], vel=pk["vel"], prev_local=pk["prev_local"],
                 prev_mean=pk["prev_mean"])
    d.outer_eager_packed(pk["theta"], state, outer_lr=ETA, outer_momentum=MU)
    d.unpack_state(state, M, n, anchor=pk["anchor"], vel=pk["vel"], prev_local=pk["prev_local"],
                   prev_mean=pk["prev_mean"])
    torch.cuda.synchronize()
    for k in want:
        assert torch.equal(want[k], got[k]), k
        assert torch.equal(want[k], pk[k]), k
    # AdamW, standard outer step, reset, quadratic step: against the checker
    wl = wl_for(3, n)
    ad = W.adamw_state(wl, n, seed=79)
    ref = {k: W.to_f64(v) for k, v in ad.items()}
    S = checked_adamw(ref, 5, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay)
    g = {k: v.to(DEV) for k, v in ad.items()}
    d.inner_adamw(g["theta"], g["m1"], g["m2"], g["grad"], lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2,
                  eps=wl.eps, weight_decay=wl.weight_decay, step=5)
    torch.cuda.synchronize()
    for k in ("theta", "m1", "m2"):
        assert_close(W.to_f64(g[k]), ref[k], TOL_F32, f"adamw {k} at shape {launch_shape}", scale=S[k])
    st = W.outer_state(wl, n, seed=83)
    theta, a, u = st["theta"], st["anchor"][0].clone(), st["vel"][0].clone()
    rt, ra, ru = W.to_f64(theta), W.to_f64(a), W.to_f64(u)
    _, S = checked_standard(rt, ra, ru, ETA, MU, True)
    gt, ga, gu = theta.to(DEV), a.to(DEV), u.to(DEV)
    d.outer_sync(gt, ga, gu, outer_lr=ETA, outer_momentum=MU)
    th2 = torch.zeros_like(gt)
    d.reset(th2, ga)
    torch.cuda.synchronize()
    assert_close(W.to_f64(ga), ra, TOL_F32, "sync anchor", scale=S["anchor"])
    assert_close(W.to_f64(gu), ru, TOL_F32, "sync vel", scale=S["vel"])
    assert torch.equal(gt, ga.expand(3, n)) and torch.equal(th2, gt)


# ------------------------------------------------------------------ seeded sweep over valid argument combinations
EAGER_SWEEP_CHUNKS, STANDARD_SWEEP_CHUNKS = 88, 44


@pytest.mark.parametrize("chunk", range(EAGER_SWEEP_CHUNKS))
def test_seeded_sweep_of_valid_eager_calls_matches_the_checker(chunk):
    """25 argument combinations per chunk, drawn from a fixed seed: replica counts on every kernel
    path, ragged and tiny sizes, both layouts, misaligned rows, bf16 replicas, every wire format,
    with and without the stored mean, first boundary or not, several launch shapes."""
    rng = np.random.default_rng(cases.EAGER_SWEEP_SEED + chunk)
    for _ in range(cases.EAGER_SWEEP_DRAWS):
        c = cases.random_eager_case(rng)
        M, n, mis = c["M"], c["n"], c["misalign"]
        wl = wl_for(M, n, c["bf16"])
        stride = ((n + c["pad"] + mis + 3) & ~3) if c["packed"] else n + c["pad"] + mis
        cut = (lambda v: v[:, mis:mis + n] if v.dim() == 2 else v)
        host = W.outer_state(wl, n, seed=cases.EAGER_STATE_SEED + chunk, stride=stride)
        ref = {k: W.to_f64(cut(v)) for k, v in host.items()}
        S = checked_eager(ref, c["eta"], c["mu"], c["nesterov"], c["apply"], c["variant"],
                          comm=cases.oracle_comm(c["comm"]), no_mean=c["no_mean"])
        full = {k: v.to(DEV) for k, v in host.items()}
        g = {k: cut(v) for k, v in full.items()}
        before_mean = g["prev_mean"].clone()
        flags = (d.EAGER if c["variant"] == "eager" else d.DELAYED) | (d.STATE_NO_MEAN if c["no_mean"] else 0)
        if c["comm"] is not None:
            flags |= d.COMM_BF16 if c["comm"] == "bf16" else d.COMM_EXMY(*c["comm"])
        kw = dict(n=n, outer_lr=c["eta"], outer_momentum=c["mu"], nesterov=c["nesterov"], variant=flags,
                  apply_update=c["apply"])
        set_shape(*c["shape"])
        try:
            if c["packed"]:
                state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
                d.pack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                             prev_mean=g["prev_mean"])
                if (M + n) % 2 == 0:      # half of the packed cases: state read from one buffer, written to another
                    state_out = torch.zeros_like(state)
                    d.outer_eager_pingpong(g["theta"], state, state_out, **kw)
                    state = state_out
                else:
                    d.outer_eager_packed(g["theta"], state, **kw)
                d.unpack_state(state, M, n, anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"],
                               prev_mean=None if c["no_mean"] else g["prev_mean"])
            else:
                d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], **kw)
        finally:
            set_shape(*DEFAULT_SHAPE)
        torch.cuda.synchronize()
        for k in ref:
            if k == "prev_mean" and c["no_mean"]:
                assert torch.equal(g[k], before_mean), c
                continue
            tol = TOL_BF16 if (c["bf16"] and k == "theta") else TOL_F32
            assert_close(W.to_f64(g[k]), ref[k], tol, f"{c} {k}", scale=S[k])
        if c["comm"] is not None:
            assert np.array_equal(W.to_f64(g["prev_local"]), ref["prev_local"]), c


@pytest.mark.parametrize("chunk", range(STANDARD_SWEEP_CHUNKS))
def test_seeded_sweep_of_valid_standard_and_adamw_calls_matches_the_checker(chunk):
    """20 argument combinations per chunk for the standard outer step and the AdamW sweep.  Chunk 27
    holds the one-element draw whose velocity update cancels 2000-fold (tests/test_error_metric.py)."""
    rng = np.random.default_rng(cases.STANDARD_SWEEP_SEED + chunk)
    for _ in range(cases.STANDARD_SWEEP_DRAWS):
        c = cases.random_standard_adamw_case(rng)
        M, n, bf16, mis, pad, comm = c["M"], c["n"], c["bf16"], c["misalign"], c["pad"], c["comm"]
        eta, mu, nest, step = c["eta"], c["mu"], c["nesterov"], c["step"]
        wl = wl_for(M, n, bf16)
        cut = (lambda v: v[:, mis:mis + n])
        host = W.outer_state(wl, n, seed=cases.STANDARD_STATE_SEED + chunk, stride=n + pad + mis)
        a, u = host["anchor"][0, :n].clone(), host["vel"][0, :n].clone()
        rt, ra, ru = W.to_f64(cut(host["theta"])), W.to_f64(a), W.to_f64(u)
        want, S = checked_standard(rt, ra, ru, eta, mu, nest, comm=cases.oracle_comm(comm))
        gt = cut(host["theta"].to(DEV))
        ga, gu, gm = a.to(DEV), u.to(DEV), torch.zeros(n, device=DEV)
        ad = W.adamw_state(wl, n, seed=cases.ADAMW_STATE_SEED + chunk, stride=n + pad + mis,
                           grad_dtype=torch.bfloat16 if c["grad_bf16"] else torch.float32)
        refa = {k: W.to_f64(cut(v)) for k, v in ad.items()}
        Sa = checked_adamw(refa, step, 4e-4, 0.9, 0.95, 1e-8, 0.1)
        gad = {k: cut(v.to(DEV)) for k, v in ad.items()}
        set_shape(*c["shape"])
        try:
            d.outer_sync(gt, ga, gu, n=n, mean_out=gm, outer_lr=eta, outer_momentum=mu, nesterov=nest,
                         comm=None if comm is None else (d.COMM_BF16 if comm == "bf16" else d.COMM_EXMY(*comm)))
            d.inner_adamw(gad["theta"], gad["m1"], gad["m2"], gad["grad"], n=n, lr=4e-4, beta1=0.9, beta2=0.95,
                          eps=1e-8, weight_decay=0.1, step=step)
        finally:
            set_shape(*DEFAULT_SHAPE)
        torch.cuda.synchronize()
        tag = f"M={M} n={n} bf16={bf16} mis={mis} comm={comm} shape={c['shape']}"
        assert_close(W.to_f64(gm), want, TOL_F32, f"standard mean {tag}", scale=S["mean"])
        assert_close(W.to_f64(ga), ra, TOL_F32, f"standard anchor {tag}", scale=S["anchor"])
        assert_close(W.to_f64(gu), ru, TOL_F32, f"standard vel {tag}", scale=S["vel"])
        assert torch.equal(gt, ga.to(gt.dtype).expand(M, n)), tag
        for k in ("theta", "m1", "m2"):
            assert_close(W.to_f64(gad[k]), refa[k], TOL_BF16 if bf16 else TOL_F32, f"adamw {k} {tag} step={step}",
                         scale=Sa[k])


def test_the_one_element_draw_whose_velocity_cancels():
    """Regression case: chunk 27, draw 7 of the sweep above on its own (M = 8, n = 1, heavy ball,
    eta = 1, mu = 0.9): mu u + Delta leaves 1.8e-7 of two terms of 3.4e-4.  The library's value is the
    float32 evaluation of Algorithm 1 line 10 to the bit, and within 1e-6 of the operand scale."""
    c = cases.standard_sweep_case(27, 7)
    assert (c["M"], c["n"], c["eta"], c["mu"], c["nesterov"]) == (8, 1, 1.0, 0.9, False)
    wl = wl_for(c["M"], c["n"])
    host = W.outer_state(wl, 1, seed=cases.STANDARD_STATE_SEED + 27, stride=1 + c["pad"])
    a, u = host["anchor"][0, :1].clone(), host["vel"][0, :1].clone()
    rt, ra, ru = W.to_f64(host["theta"][:, :1]), W.to_f64(a), W.to_f64(u)
    want, S = checked_standard(rt, ra, ru, c["eta"], c["mu"], c["nesterov"])
    gt, ga, gu, gm = host["theta"].to(DEV)[:, :1], a.to(DEV), u.to(DEV), torch.zeros(1, device=DEV)
    d.outer_sync(gt, ga, gu, n=1, mean_out=gm, outer_lr=c["eta"], outer_momentum=c["mu"], nesterov=False)
    torch.cuda.synchronize()
    assert_close(W.to_f64(gu), ru, TOL_F32, "velocity", scale=S["vel"])
    assert_close(W.to_f64(ga), ra, TOL_F32, "outer parameters", scale=S["anchor"])
    assert_close(W.to_f64(gm), want, TOL_F32, "mean", scale=S["mean"])
    # the float32 evaluation, in the library's order: float32 differences, float64 sum rounded once, one fma
    delta = (a.numpy()[None, :] - host["theta"][:, :1].numpy()).astype(np.float32)
    dbar = (np.sum(delta.astype(np.float64), axis=0) / 8).astype(np.float32)
    u32 = (np.float64(np.float32(0.9)) * u.numpy().astype(np.float64) + dbar.astype(np.float64)).astype(np.float32)
    assert np.array_equal(gm.cpu().numpy(), dbar) and np.array_equal(gu.cpu().numpy(), u32)
    # and that value misses 1e-6 of |u| by a wide margin: the cancellation, not the kernel
    assert abs(float(u32[0]) - ru[0]) / abs(ru[0]) > 5e-5


# ------------------------------------------------------------------ non-finite values
def _kind(x):
    """0 finite, 1 NaN, 2 +Inf, 3 -Inf, element by element."""
    x = np.asarray(x, dtype=np.float64)
    return np.where(np.isnan(x), 1, np.where(np.isposinf(x), 2, np.where(np.isneginf(x), 3, 0)))


def _same_kinds_and_close_where_finite(got, want, what):
    kg, kw = _kind(got), _kind(want)
    assert np.array_equal(kg, kw), f"{what}: NaN / Inf pattern {kg.tolist()} against the checker's {kw.tolist()}"
    fin = kw == 0
    np.testing.assert_allclose(np.asarray(got)[fin], np.asarray(want)[fin], rtol=1e-2, atol=1e-6, err_msg=what)


# where the bad values go: inside a vector, first lane, the ragged tail; one index takes +Inf and -Inf
# from two replicas (their sum is NaN)
def _poison(theta, n):
    M = theta.shape[0]
    idx = sorted({0, 5, n // 2, n - 1})
    vals = [float("nan"), float("inf"), float("-inf"), float("inf")]
    for j, (i, v) in enumerate(zip(idx, vals)):
        theta[j % M, i] = v
    if M > 1:
        theta[(len(idx) - 1 + 1) % M, idx[-1]] = float("-inf") if vals[len(idx) - 1] > 0 else float("inf")
    return idx


@pytest.mark.parametrize("M,n,bf16,misalign,packed", [(4, 1027, False, 0, False), (8, 4099, True, 0, True),
                                                      (9, 1027, False, 0, False), (17, 263, False, 0, True),
                                                      (3, 1027, False, 1, False), (1, 70, False, 0, False)])
@pytest.mark.parametrize("variant,apply", [("eager", True), ("delayed", True), ("eager", False)])
def test_non_finite_replica_values_stay_at_their_index(M, n, bf16, misalign, packed, variant, apply):
    """A NaN or an infinity in a replica (a diverged run) must come out as the checker says at that
    index (Nesterov form: same NaN / +Inf / -Inf pattern in every output buffer) and must not change
    a bit at any other index."""
    wl = wl_for(M, n, bf16)
    var = d.EAGER if variant == "eager" else d.DELAYED
    out = []
    for poisoned in (False, True):
        st = W.outer_state(wl, n, seed=91, stride=n + misalign)
        if misalign:
            st = {k: (v[:, misalign:] if v.dim() == 2 else v) for k, v in st.items()}
        idx = _poison(st["theta"], n) if poisoned else None
        ref = {k: W.to_f64(v[..., :n]) for k, v in st.items()}
        with np.errstate(all="ignore"):
            if variant == "eager":
                O.outer_eager(ref["theta"], ref["anchor"], ref["vel"], ref["prev_local"], ref["prev_mean"],
                              ETA, MU, True, apply)
            else:
                O.outer_delayed(ref["theta"], ref["anchor"], ref["vel"], ref["prev_local"], ref["prev_mean"],
                                ETA, MU, True, apply)
        full = {k: v.to(DEV) for k, v in W.outer_state(wl, n, seed=91, stride=n + misalign).items()}
        g = {k: (v[:, misalign:] if (misalign and v.dim() == 2) else v) for k, v in full.items()}
        if poisoned:
            g["theta"][:, :n] = st["theta"][:, :n].to(DEV)
        if packed:
            state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
            names = dict(anchor=g["anchor"], vel=g["vel"], prev_local=g["prev_local"], prev_mean=g["prev_mean"])
            d.pack_state(state, M, n, **names)
            d.outer_eager_packed(g["theta"], state, n=n, outer_lr=ETA, outer_momentum=MU, variant=var,
                                 apply_update=apply)
            d.unpack_state(state, M, n, **names)
        else:
            d.outer_eager(g["theta"], g["anchor"], g["vel"], g["prev_local"], g["prev_mean"], n=n,
                          outer_lr=ETA, outer_momentum=MU, variant=var, apply_update=apply)
        torch.cuda.synchronize()
        out.append(({k: v[..., :n].clone() for k, v in g.items()}, ref, idx))
    (clean, _, _), (bad, ref, idx) = out
    keep = torch.ones(n, dtype=torch.bool, device=DEV)
    keep[idx] = False
    for k in clean:
        assert torch.equal(clean[k][..., keep], bad[k][..., keep]), f"{k}: an index without a bad value changed"
        _same_kinds_and_close_where_finite(W.to_f64(bad[k][..., idx]), ref[k][..., idx], f"{variant} {k}")
    # the test plants something: the new mean holds NaN and infinities in both runs of the checker's pattern
    assert set(_kind(ref["prev_mean"][idx]).tolist()) >= ({1, 3} if M > 1 else {1})


def test_non_finite_values_in_the_standard_step_and_adamw():
    M, n = 5, 1027
    wl = wl_for(M, n)
    # standard outer step: the shared outer parameters take the bad value at that index, every replica with them
    outs = []
    for poisoned in (False, True):
        st = W.outer_state(wl, n, seed=93)
        theta, a, u = st["theta"], st["anchor"][0].clone(), st["vel"][0].clone()
        idx = _poison(theta, n) if poisoned else None
        rt, ra, ru = W.to_f64(theta), W.to_f64(a), W.to_f64(u)
        with np.errstate(all="ignore"):
            rmean = O.outer_standard(rt, ra, ru, ETA, MU, True)
        gt, ga, gu, gm = theta.to(DEV), a.to(DEV), u.to(DEV), torch.empty(n, device=DEV)
        d.outer_sync(gt, ga, gu, mean_out=gm, outer_lr=ETA, outer_momentum=MU)
        torch.cuda.synchronize()
        outs.append((dict(theta=gt, anchor=ga, vel=gu, mean=gm), dict(theta=rt, anchor=ra, vel=ru, mean=rmean), idx))
    (clean, _, _), (bad, ref, idx) = outs
    keep = torch.ones(n, dtype=torch.bool, device=DEV)
    keep[idx] = False
    for k in clean:
        assert torch.equal(clean[k][..., keep], bad[k][..., keep]), k
        _same_kinds_and_close_where_finite(W.to_f64(bad[k][..., idx]), ref[k][..., idx], f"standard {k}")
    assert (_kind(ref["anchor"][idx]) != 0).all()
    # AdamW: a bad gradient value reaches theta_m, m1, m2 of its replica and index only
    outs = []
    for poisoned in (False, True):
        st = W.adamw_state(wl, n, seed=95)
        idx = _poison(st["grad"], n) if poisoned else None
        ref = {k: W.to_f64(v) for k, v in st.items()}
        with np.errstate(all="ignore"):
            O.adamw_step(ref["theta"], ref["m1"], ref["m2"], ref["grad"], 7, wl.lr, wl.beta1, wl.beta2, wl.eps,
                         wl.weight_decay)
        g = {k: v.to(DEV) for k, v in st.items()}
        d.inner_adamw(g["theta"], g["m1"], g["m2"], g["grad"], lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2,
                      eps=wl.eps, weight_decay=wl.weight_decay, step=7)
        torch.cuda.synchronize()
        outs.append((g, ref, idx))
    (clean, _, _), (bad, ref, idx) = outs
    for k in ("theta", "m1", "m2"):
        assert torch.equal(clean[k][..., keep], bad[k][..., keep]), k
        _same_kinds_and_close_where_finite(W.to_f64(bad[k][..., idx]), ref[k][..., idx], f"adamw {k}")
    assert (_kind(ref["theta"][:, idx]) != 0).sum() >= len(idx)


@pytest.mark.parametrize("M,n,stride", [(2, 67, 68), (8, 4099, 4100), (9, 263, 264), (2, 67, 67)])
def test_subnormal_outer_gradients_are_kept_exactly(M, n, stride):
    """Below 2^-126 float32 underflows gradually; the kernels do not flush to zero.  With replicas and
    outer parameters that are even multiples of 2^-149, line 7's differences and line 8's mean (M a
    power of two, or the sum a multiple of M) are exact in float32 and in the checker alike: same bits."""
    rng = np.random.default_rng(97)
    unit = np.float64(2.0) ** -149
    ka = 2 * M * rng.integers(1, 1 << 18, size=(M, n))
    kt = 2 * M * rng.integers(1, 1 << 18, size=(M, n))
    a64, t64 = ka * unit, kt * unit
    ref = dict(theta=t64.copy(), anchor=a64.copy(), vel=np.zeros((M, n)), prev_local=np.zeros((M, n)),
               prev_mean=np.zeros(n))
    O.outer_eager(ref["theta"], ref["anchor"], ref["vel"], ref["prev_local"], ref["prev_mean"], ETA, MU, True, False)
    assert (np.abs(ref["prev_local"]) < 2.0 ** -126).all() and (ref["prev_local"] != 0).any()
    buf = {k: torch.zeros((M, stride), device=DEV) for k in ("theta", "anchor", "vel", "prev_local")}
    buf["theta"][:, :n] = torch.from_numpy(t64.astype(np.float32)).to(DEV)
    buf["anchor"][:, :n] = torch.from_numpy(a64.astype(np.float32)).to(DEV)
    mean = torch.zeros(n, device=DEV)
    d.outer_eager(buf["theta"], buf["anchor"], buf["vel"], buf["prev_local"], mean, n=n, outer_lr=ETA,
                  outer_momentum=MU, apply_update=False)
    torch.cuda.synchronize()
    assert np.array_equal(W.to_f64(buf["prev_local"][:, :n]), ref["prev_local"])
    assert np.array_equal(W.to_f64(mean), ref["prev_mean"])
    assert np.array_equal(W.to_f64(buf["anchor"][:, :n]), ref["anchor"])


# ------------------------------------------------------------------ HIP graph capture
def test_a_captured_step_replays_to_the_same_bits():
    """The entry points only enqueue kernels on the caller's stream (no allocation, no
    synchronisation, no memset), so a step can be captured into a HIP graph.  Three replays, with
    ordinary launches and synchronisations between them, against the same steps launched directly."""
    M, n = 8, 150_003
    wl = wl_for(M, n)

    def fresh():
        st = {k: v.to(DEV) for k, v in W.outer_state(wl, n, seed=113, stride=n + 1).items()}
        ad = {k: v.to(DEV) for k, v in W.adamw_state(wl, n, seed=113, stride=n + 1).items()}
        state = torch.zeros(d.packed_state_elems(M, n), device=DEV)
        d.pack_state(state, M, n, anchor=st["anchor"], vel=st["vel"], prev_local=st["prev_local"],
                     prev_mean=st["prev_mean"])
        return st["theta"], ad["m1"], ad["m2"], ad["grad"], state

    def step(theta, m1, m2, grad, state):
        d.inner_adamw(theta, m1, m2, grad, n=n, lr=4e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=7)
        d.outer_eager_packed(theta, state, n=n, outer_lr=ETA, outer_momentum=MU)
        d.outer_eager_packed(theta, state, n=n, outer_lr=ETA, outer_momentum=MU,
                             variant=d.EAGER | d.STATE_NO_MEAN | d.COMM_BF16)

    direct = fresh()
    for _ in range(3):
        step(*direct)
    torch.cuda.synchronize()

    bufs = fresh()
    warm = fresh()
    step(*warm)                      # first launches (and their one-time LDS grants) outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(*bufs)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 20, device=DEV)
    for k in range(3):
        graph.replay()
        scratch.add_(1.0)            # the program's own eager work between replays
        torch.cuda.synchronize()
    for x, y, name in zip(direct, bufs, ("theta", "m1", "m2", "grad", "state")):
        assert torch.equal(x, y), name
