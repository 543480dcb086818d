"""Boundary tests that need no GPU: the shared library loads, exports every symbol the
headers declare, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2502_12996_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return B.lib()


def declared_functions():
    names = []
    for hdr in ("diloco.h", "diloco_sim.h"):
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(diloco_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported_and_bound(lib):
    names = declared_functions()
    assert {"diloco_inner_adamw", "diloco_outer_sync", "diloco_outer_eager", "diloco_reset"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"
        assert name in B.SIGNATURES, f"{name} has no ctypes signature"
    assert set(B.SIGNATURES) == set(names)


def test_version_and_strerror(lib):
    assert lib.diloco_version() >= 100
    texts = {lib.diloco_strerror(c) for c in range(8)}
    assert len(texts) == 8 and all(texts)
    assert lib.diloco_strerror(1234) == b"unknown status"


# fake, suitably aligned, non-overlapping device addresses: validation never dereferences
P = [0x7000_0000_0000 + k * 0x1000_0000 for k in range(8)]


def eager(lib, theta=P[0], dt=0, M=2, n=64, stride=64, a=P[1], u=P[2], pl=P[3], ss=64, pm=P[4],
          lr=0.7, mu=0.9, nest=1, var=0, apply=1):
    return lib.diloco_outer_eager(theta, dt, M, n, stride, a, u, pl, ss, pm, lr, mu, nest, var, apply, None)


def test_variant_flags_are_validated_before_any_launch(lib):
    assert eager(lib, n=0, var=B.EAGER | B.STATE_NO_MEAN) == B.OK
    assert eager(lib, var=B.DELAYED | B.STATE_NO_MEAN) == B.ERR_DTYPE
    assert eager(lib, M=9, n=0, stride=64, var=B.EAGER | B.STATE_NO_MEAN) == B.OK   # any replica count
    assert eager(lib, var=B.EAGER | B.COMM_BF16 | B.COMM_EXMY(4, 3, 7)) == B.ERR_DTYPE
    assert eager(lib, var=B.EAGER | B.COMM_EXMY(0, 3, 7)) == B.ERR_DTYPE
    assert eager(lib, var=B.EAGER | B.COMM_EXMY(8, 7, 127)) == B.ERR_DTYPE     # below float32's normal range
    assert eager(lib, n=0, var=B.EAGER | B.COMM_EXMY(2, 1, 11) | B.STATE_NO_MEAN) == B.OK
    assert eager(lib, var=0x800) == B.ERR_DTYPE

    def sync(comm, n=64):
        return lib.diloco_outer_sync_comm(P[0], 0, 2, n, 64, P[1], P[2], None, 0.7, 0.9, 1, comm, None)
    assert sync(0, n=0) == B.OK and sync(B.COMM_BF16, n=0) == B.OK and sync(B.COMM_EXMY(4, 3, 16), n=0) == B.OK
    assert sync(1) == B.ERR_DTYPE and sync(B.STATE_NO_MEAN) == B.ERR_DTYPE and sync(B.COMM_EXMY(9, 1, 0)) == B.ERR_DTYPE

    def rmw(K=4, n=64, stride=64, base=P[0]):
        return lib.diloco_sim_stream_rmw(base, K, n, stride, None, None)
    assert rmw(n=0) == B.OK
    assert rmw(K=3) == B.ERR_SHAPE and rmw(n=62) == B.ERR_SHAPE and rmw(stride=32) == B.ERR_SHAPE
    assert rmw(base=None) == B.ERR_NULL and rmw(base=P[0] + 4) == B.ERR_ALIGN and rmw(stride=66) == B.ERR_ALIGN


def test_outer_eager_validation(lib):
    assert eager(lib, n=0) == B.OK                      # empty input: no-op, nothing launched
    assert eager(lib, theta=None) == B.ERR_NULL
    assert eager(lib, pm=None) == B.ERR_NULL
    assert eager(lib, dt=7) == B.ERR_DTYPE
    assert eager(lib, var=2) == B.ERR_DTYPE
    assert eager(lib, M=0) == B.ERR_SHAPE
    assert eager(lib, M=70000) == B.ERR_SHAPE
    assert eager(lib, n=-1) == B.ERR_SHAPE
    assert eager(lib, stride=63) == B.ERR_SHAPE          # rows would overlap
    assert eager(lib, ss=10) == B.ERR_SHAPE
    assert eager(lib, n=1 << 61) == B.ERR_SHAPE
    assert eager(lib, mu=1.0) == B.ERR_HYPER
    assert eager(lib, mu=-0.1) == B.ERR_HYPER
    assert eager(lib, lr=float("nan")) == B.ERR_HYPER
    assert eager(lib, lr=float("inf")) == B.ERR_HYPER
    assert eager(lib, a=P[1] + 2) == B.ERR_ALIGN         # fp32 pointer not 4-byte aligned
    assert eager(lib, theta=P[0] + 1, dt=1) == B.ERR_ALIGN
    assert eager(lib, a=P[0]) == B.ERR_ALIAS             # anchor on top of theta
    assert eager(lib, pm=P[3] + 64) == B.ERR_ALIAS       # prev_mean inside prev_local
    assert eager(lib, u=P[1] + 4 * 100) == B.ERR_ALIAS   # vel overlaps anchor's second row


def test_outer_sync_validation(lib):
    def f(theta=P[0], dt=0, M=2, n=64, stride=64, a=P[1], u=P[2], mo=None, lr=0.7, mu=0.9):
        return lib.diloco_outer_sync(theta, dt, M, n, stride, a, u, mo, lr, mu, 1, None)
    assert f(n=0) == B.OK
    assert f(a=None) == B.ERR_NULL
    assert f(dt=3) == B.ERR_DTYPE
    assert f(M=-1) == B.ERR_SHAPE
    assert f(stride=8) == B.ERR_SHAPE
    assert f(mu=1.5) == B.ERR_HYPER
    assert f(u=P[2] + 1) == B.ERR_ALIGN
    assert f(mo=P[1]) == B.ERR_ALIAS
    assert f(u=P[1] + 16) == B.ERR_ALIAS


def test_inner_adamw_validation(lib):
    def f(th=P[0], m1=P[1], m2=P[2], g=P[3], M=2, n=64, stride=64, pd=0, gd=0, lr=4e-4, b1=0.9,
          b2=0.95, eps=1e-8, wd=0.1, step=1):
        return lib.diloco_inner_adamw(th, m1, m2, g, M, n, stride, pd, gd, lr, b1, b2, eps, wd, step, None)
    assert f(n=0) == B.OK
    assert f(g=None) == B.ERR_NULL
    assert f(pd=2) == B.ERR_DTYPE
    assert f(gd=-1) == B.ERR_DTYPE
    assert f(n=-5) == B.ERR_SHAPE
    assert f(step=0) == B.ERR_HYPER
    assert f(b1=1.0) == B.ERR_HYPER
    assert f(b2=-0.5) == B.ERR_HYPER
    assert f(eps=0.0) == B.ERR_HYPER
    assert f(wd=-1.0) == B.ERR_HYPER
    assert f(lr=float("nan")) == B.ERR_HYPER
    assert f(m1=P[1] + 2) == B.ERR_ALIGN
    assert f(th=P[0] + 2, m1=P[1] + 2, m2=P[2] + 2, pd=1, n=0) == B.OK   # bf16: 2-byte aligned is fine
    assert f(g=P[0]) == B.ERR_ALIAS
    assert f(m2=P[1]) == B.ERR_ALIAS


def test_reset_validation(lib):
    def f(th=P[0], dt=0, M=2, n=64, stride=64, a=P[1], astride=0):
        return lib.diloco_reset(th, dt, M, n, stride, a, astride, None)
    assert f(n=0) == B.OK
    assert f(a=None) == B.ERR_NULL
    assert f(dt=9) == B.ERR_DTYPE
    assert f(astride=5) == B.ERR_SHAPE
    assert f(a=P[0] + 4 * 64) == B.ERR_ALIAS


def test_packed_state_validation(lib):
    tile = int(re.search(r"#define DILOCO_STATE_TILE (\d+)", open(os.path.join(ROOT, "include", "diloco.h")).read()).group(1))
    assert tile == B.STATE_TILE
    assert lib.diloco_packed_state_elems(8, tile + 1) == 2 * 25 * tile
    assert lib.diloco_packed_state_elems(1, 0) == 0
    assert lib.diloco_packed_state_elems(0, 5) == -1
    assert lib.diloco_packed_state_elems(2, -1) == -1

    def f(th=P[0], dt=0, M=2, n=64, stride=64, st=P[1], lr=0.7, mu=0.9, var=0):
        return lib.diloco_outer_eager_packed(th, dt, M, n, stride, st, lr, mu, 1, var, 1, None)
    assert f(n=0) == B.OK
    assert f(st=None) == B.ERR_NULL
    assert f(dt=5) == B.ERR_DTYPE
    assert f(var=3) == B.ERR_DTYPE
    assert f(M=0) == B.ERR_SHAPE
    assert f(stride=3) == B.ERR_SHAPE
    assert f(mu=1.0) == B.ERR_HYPER
    assert f(st=P[1] + 4) == B.ERR_ALIGN          # the packed state must be 16-byte aligned
    assert f(st=P[0] + 16) == B.ERR_ALIAS

    def pp(th=P[0], dt=0, M=2, n=64, stride=64, si=P[1], so=P[2], mu=0.9, var=0):
        return lib.diloco_outer_eager_pingpong(th, dt, M, n, stride, si, so, 0.7, mu, 1, var, 1, None)
    assert pp(n=0) == B.OK
    assert pp(si=None) == B.ERR_NULL and pp(so=None) == B.ERR_NULL and pp(th=None) == B.ERR_NULL
    assert pp(so=P[1]) == B.ERR_ALIAS                      # the same buffer twice: that is the in-place call
    assert pp(so=P[1] + 4 * 8192) == B.ERR_ALIAS           # overlapping state buffers
    assert pp(so=P[0] + 16) == B.ERR_ALIAS and pp(si=P[0] + 16) == B.ERR_ALIAS    # on top of theta
    assert pp(so=P[2] + 4) == B.ERR_ALIGN and pp(si=P[1] + 8) == B.ERR_ALIGN
    assert pp(mu=1.0) == B.ERR_HYPER and pp(var=2) == B.ERR_DTYPE and pp(M=0) == B.ERR_SHAPE
    assert pp(n=0, var=B.EAGER | B.STATE_NO_MEAN | B.COMM_BF16) == B.OK
    assert lib.diloco_outer_eager_pingpong_shaped(P[0], 0, 2, 0, 64, P[1], P[2], 0.7, 0.9, 1, 0, 1, None, None) == B.OK
    assert lib.diloco_outer_eager_pingpong_shaped(P[0], 0, 2, 0, 64, P[1], P[2], 0.7, 0.9, 1, 0, 1, None,
                                                  ctypes.byref(B.Launch(100, 0, 0, 0))) == B.ERR_HYPER
    assert lib.diloco_outer_eager_pingpong_shaped(P[0], 0, 2, 64, 64, P[1], P[1], 0.7, 0.9, 1, 0, 1, None,
                                                  None) == B.ERR_ALIAS

    def o2(th=P[0], M=2, n=64, sp=P[1], sc=P[2], var=0):
        return lib.diloco_outer_eager_overlap2(th, 0, M, n, 64, sp, sc, 0.7, 0.9, 1, var, 1, None)
    assert o2(n=0) == B.OK and o2(n=0, var=B.DELAYED | B.COMM_BF16) == B.OK
    assert o2(sp=None) == B.ERR_NULL and o2(sc=None) == B.ERR_NULL
    assert o2(sc=P[1]) == B.ERR_ALIAS and o2(sc=P[0] + 16) == B.ERR_ALIAS
    assert o2(var=B.EAGER | B.STATE_NO_MEAN) == B.ERR_DTYPE and o2(var=5) == B.ERR_DTYPE
    assert o2(sc=P[2] + 4) == B.ERR_ALIGN and o2(M=0) == B.ERR_SHAPE

    def pk(st=P[0], M=2, n=64, a=P[1], u=P[2], pl=P[3], ss=64, pm=P[4], fn=None):
        return (fn or lib.diloco_pack_state)(st, M, n, a, u, pl, ss, pm, None)
    for fn in (lib.diloco_pack_state, lib.diloco_unpack_state):
        assert pk(n=0, fn=fn) == B.OK
        assert pk(st=None, fn=fn) == B.ERR_NULL
        assert pk(ss=5, fn=fn) == B.ERR_SHAPE
        assert pk(M=30000, ss=64, fn=fn) == B.ERR_SHAPE
        assert pk(st=P[0] + 8, fn=fn) == B.ERR_ALIGN
        assert pk(a=P[1] + 2, fn=fn) == B.ERR_ALIGN
        assert pk(a=P[0], fn=fn) == B.ERR_ALIAS
        assert pk(a=None, u=None, pl=None, pm=None, n=0, fn=fn) == B.OK
    assert lib.diloco_reset_packed(P[0], 0, 2, 0, 64, P[1], None) == B.OK
    assert lib.diloco_reset_packed(P[0], 0, 2, 64, 64, None, None) == B.ERR_NULL
    assert lib.diloco_reset_packed(P[0], 0, 2, 64, 64, P[1] + 4, None) == B.ERR_ALIGN


def test_sim_validation_and_tuning(lib):
    def q(th=P[0], m1=P[1], m2=P[2], M=2, n=64, stride=64, h=P[3], star=P[4], noise=0.1, seed=1,
          base=0, step=1):
        return lib.diloco_sim_quadratic_inner(th, m1, m2, M, n, stride, h, star, noise, seed, base,
                                              4e-4, 0.9, 0.95, 1e-8, 0.0, step, None)
    assert q(n=0) == B.OK
    assert q(h=None) == B.ERR_NULL
    assert q(base=2) == B.ERR_SHAPE
    assert q(noise=-1.0) == B.ERR_HYPER
    assert q(th=P[0] + 4) == B.ERR_ALIGN

    def ph(th=P[0], m1=P[1], m2=P[2], M=2, n=64, stride=64, h=P[3], star=P[4], noise=0.1, base=0, first=1, steps=8):
        return lib.diloco_sim_quadratic_phase(th, m1, m2, M, n, stride, h, star, noise, 1, base,
                                              4e-4, 0.9, 0.95, 1e-8, 0.0, first, steps, None)
    assert ph(n=0) == B.OK and ph(steps=0) == B.OK
    assert ph(m2=None) == B.ERR_NULL
    assert ph(steps=65) == B.ERR_SHAPE and ph(steps=-1) == B.ERR_SHAPE and ph(base=6) == B.ERR_SHAPE
    assert ph(first=0) == B.ERR_HYPER and ph(noise=float("nan")) == B.ERR_HYPER
    assert ph(star=P[4] + 8) == B.ERR_ALIGN and ph(stride=66) == B.ERR_ALIGN
    assert ph(m1=P[0]) == B.ERR_ALIAS
    assert lib.diloco_sim_loss_workspace(0) == 1
    assert lib.diloco_sim_loss_workspace(1 << 26) == 8192
    assert lib.diloco_sim_quadratic_loss(P[0], 2, 64, 64, P[1], P[2], P[3], 0, P[4], None) == B.ERR_SHAPE
    assert lib.diloco_sim_quadratic_loss(P[0], 2, 64, 64, P[1], P[2], None, 1, P[4], None) == B.ERR_NULL
    old = lib.diloco_tune_get(b"block")
    assert lib.diloco_tune(b"block", 128) == B.OK and lib.diloco_tune_get(b"block") == 128
    assert lib.diloco_tune(b"block", 100) == B.ERR_HYPER
    assert lib.diloco_tune(b"block", 2048) == B.ERR_HYPER
    assert lib.diloco_tune(b"nope", 1) == B.ERR_HYPER
    assert lib.diloco_tune(b"block", old) == B.OK
    assert old == 0 and lib.diloco_tune_get(b"wg_per_cu") == -1 and lib.diloco_tune_get(b"xcd_remap") == 0
    assert lib.diloco_tune(b"wg_per_cu", 33) == B.ERR_HYPER and lib.diloco_tune(b"wg_per_cu", -2) == B.ERR_HYPER
    assert lib.diloco_tune(b"wg_per_cu", 4) == B.OK and lib.diloco_tune_get(b"wg_per_cu") == 4
    assert lib.diloco_tune(b"wg_per_cu", -1) == B.OK
    assert lib.diloco_tune_get(b"nope") == -1
    assert lib.diloco_tune(b"generic_path", 3) == B.ERR_HYPER and lib.diloco_tune(b"xcd_remap", 2) == B.ERR_HYPER


def test_static_loss_validation(lib):
    """The allocation-free loss validates like the workspace one, and refuses sizes beyond its limit."""
    def f(th=P[0], M=2, n=64, stride=64, h=P[1], star=P[2], out=P[3]):
        return lib.diloco_sim_quadratic_loss_static(th, M, n, stride, h, star, out, None)
    assert f(th=None) == B.ERR_NULL and f(out=None) == B.ERR_NULL
    assert f(M=0) == B.ERR_SHAPE and f(n=-1) == B.ERR_SHAPE and f(stride=8) == B.ERR_SHAPE
    assert f(M=1, n=(1 << 40) + 1, stride=(1 << 40) + 1) == B.ERR_SHAPE        # beyond the stated maximum
    assert f(h=P[1] + 2) == B.ERR_ALIGN and f(out=P[3] + 4) == B.ERR_ALIGN
    assert f(out=P[0] + 8) == B.ERR_ALIAS


def test_explicit_launch_shapes_are_validated(lib):
    """The *_shaped entry points take the launch shape as an argument: NULL or a valid struct passes
    on to the ordinary validation, a field out of range is refused before anything else."""
    ok, bad = B.Launch(256, 1, 2, 0), [B.Launch(100, 0, -1, 0), B.Launch(0, 2, -1, 0), B.Launch(0, 0, 33, 0),
                                        B.Launch(0, 0, -2, 0), B.Launch(64, 0, 0, 3), B.Launch(1024, 0, 0, 0)]
    calls = {
        "eager": lambda l, n=0: lib.diloco_outer_eager_shaped(P[0], 0, 2, n, 64, P[1], P[2], P[3], 64, P[4], 0.7, 0.9,
                                                            1, 0, 1, None, l),
        "packed": lambda l, n=0: lib.diloco_outer_eager_packed_shaped(P[0], 0, 2, n, 64, P[1], 0.7, 0.9, 1, 0, 1,
                                                                    None, l),
        "sync": lambda l, n=0: lib.diloco_outer_sync_shaped(P[0], 0, 2, n, 64, P[1], P[2], None, 0.7, 0.9, 1, 0,
                                                          None, l),
        "adamw": lambda l, n=0: lib.diloco_inner_adamw_shaped(P[0], P[1], P[2], P[3], 2, n, 64, 0, 0, 4e-4, 0.9, 0.95,
                                                            1e-8, 0.1, 1, None, l),
        "copy": lambda l, n=0: lib.diloco_sim_stream_copy(P[0], P[1], n, None, l),
        "rmw": lambda l, n=0: lib.diloco_sim_stream_rmw(P[0], 4, n, 64, None, l),
    }
    for name, f in calls.items():
        assert f(None) == B.OK, name
        assert f(ctypes.byref(ok)) == B.OK, name
        for b in bad:
            assert f(ctypes.byref(b)) == B.ERR_HYPER, (name, b.block, b.xcd_remap, b.wg_per_cu, b.generic_path)
    # the ordinary validation still runs behind a valid shape
    assert calls["eager"](ctypes.byref(ok), n=-1) == B.ERR_SHAPE
    assert lib.diloco_outer_eager_shaped(P[0], 0, 2, 64, 64, P[0], P[2], P[3], 64, P[4], 0.7, 0.9, 1, 0, 1, None,
                                         ctypes.byref(ok)) == B.ERR_ALIAS
    assert lib.diloco_inner_adamw_shaped(P[0], P[1], P[2], P[3], 2, 64, 64, 0, 0, 4e-4, 1.0, 0.95, 1e-8, 0.1, 1,
                                         None, None) == B.ERR_HYPER
    # binding: tuples of 3 or 4, or a Launch
    assert B._launch(None) is None
    for l in ((64, 1, 2), (64, 1, 2, 1), ok):
        assert B._launch(l) is not None
    with pytest.raises(ValueError):
        B._launch((64, 1))


def test_the_thread_shape_is_thread_local(lib):
    """diloco_tune sets the shape of the calling thread only: two threads that set different
    values each read back their own, a new thread starts from the automatic choice, and the
    main thread's values are untouched throughout."""
    import threading
    assert lib.diloco_tune(b"block", 128) == B.OK and lib.diloco_tune(b"wg_per_cu", 5) == B.OK
    barrier = threading.Barrier(3)
    seen = {}

    def worker(name, block, cap):
        first = (lib.diloco_tune_get(b"block"), lib.diloco_tune_get(b"wg_per_cu"))
        if block is not None:
            assert lib.diloco_tune(b"block", block) == B.OK and lib.diloco_tune(b"wg_per_cu", cap) == B.OK
        barrier.wait()            # every thread has set its values before any reads them back
        seen[name] = (first, (lib.diloco_tune_get(b"block"), lib.diloco_tune_get(b"wg_per_cu")))
        barrier.wait()

    threads = [threading.Thread(target=worker, args=a) for a in (("a", 64, 2), ("b", 512, 16), ("c", None, None))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    try:
        assert seen["a"] == ((0, -1), (64, 2))
        assert seen["b"] == ((0, -1), (512, 16))
        assert seen["c"] == ((0, -1), (0, -1))
        assert (lib.diloco_tune_get(b"block"), lib.diloco_tune_get(b"wg_per_cu")) == (128, 5)
    finally:
        assert lib.diloco_tune(b"block", 0) == B.OK and lib.diloco_tune(b"wg_per_cu", -1) == B.OK


def test_binding_raises_with_status_text(lib):
    with pytest.raises(B.DilocoError) as ei:
        B._check("diloco_outer_eager", eager(lib, a=P[0]))          # anchor on top of theta
    assert ei.value.status == B.ERR_ALIAS and "overlap" in str(ei.value)
    B._check("diloco_outer_eager", eager(lib, n=0))


def test_binding_refuses_what_the_library_cannot_check():
    """The C ABI sees addresses only.  Host tensors, wrong dtypes, short rows, mismatched strides
    and tensors that are not tensors are refused in Python, before any pointer is handed over."""
    import torch
    M, n = 3, 100
    th = torch.zeros((M, n))
    kw = dict(outer_lr=0.7, outer_momentum=0.9)
    # host memory: every entry point refuses, nothing is launched (there is no GPU here anyway)
    with pytest.raises(TypeError, match="GPU memory only"):
        B.outer_eager(th, th.clone(), th.clone(), th.clone(), torch.zeros(n), **kw)
    with pytest.raises(TypeError, match="GPU memory only"):
        B.inner_adamw(th, th.clone(), th.clone(), th.clone(), lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8,
                      weight_decay=0.0, step=1)
    with pytest.raises(TypeError, match="GPU memory only"):
        B.outer_sync(th, torch.zeros(n), torch.zeros(n), **kw)
    with pytest.raises(TypeError, match="GPU memory only"):
        B.reset(th, torch.zeros(n))
    with pytest.raises(TypeError, match="GPU memory only"):
        B.sim_stream_copy(torch.zeros(8), torch.zeros(8))
    with pytest.raises(ValueError):
        B.outer_eager(torch.zeros(n), th, th, th, torch.zeros(n), **kw)          # theta is not [M, n]
    # the checks themselves, on host tensors
    a = B._Args("unit", require_gpu=False)
    assert a.rows(th, "theta", M, n, B._PARAM_DTYPES) == n
    assert a.rows(torch.zeros((M, n + 5))[:, 2:], "view", M, n) == n + 5
    a.vec(torch.zeros(n), "vec", n)
    a.vec(None, "opt", n, optional=True)
    with pytest.raises(TypeError, match="torch tensor"):
        a.rows([[0.0] * n] * M, "theta", M, n)
    with pytest.raises(TypeError, match="float64"):
        a.rows(torch.zeros((M, n), dtype=torch.float64), "anchor", M, n)
    with pytest.raises(TypeError, match="bfloat16"):
        a.rows(torch.zeros((M, n), dtype=torch.bfloat16), "anchor", M, n)           # outer state is fp32
    with pytest.raises(ValueError, match=r"M=3"):
        a.rows(torch.zeros((M + 1, n)), "vel", M, n)
    with pytest.raises(ValueError, match="rows of 100"):
        a.rows(th, "theta", M, n + 1)                                               # n beyond the row
    with pytest.raises(ValueError, match="row stride"):
        a.rows(torch.zeros((M, n + 4)), "vel", M, n, stride=n)
    with pytest.raises(ValueError, match="contiguous rows"):
        a.rows(torch.zeros((n, M)).t(), "theta", M, n)
    with pytest.raises(ValueError, match="holds 99"):
        a.vec(torch.zeros(n - 1), "prev_mean", n)
    with pytest.raises(ValueError, match="contiguous"):
        a.vec(torch.zeros(2 * n)[::2], "prev_mean", n)
    with pytest.raises(TypeError, match="required"):
        a.vec(None, "anchor", n)
    if torch.cuda.is_available() and torch.cuda.device_count() > 1:
        b = B._Args("unit")
        b.vec(torch.zeros(4, device="cuda:0"), "x", 4)
        with pytest.raises(ValueError, match="other arguments on"):
            b.vec(torch.zeros(4, device="cuda:1"), "y", 4)
    # the packed state must hold diloco_packed_state_elems(M, n) floats
    with pytest.raises(ValueError, match="holds 8"):
        B._Args("unit", require_gpu=False).vec(torch.zeros(8), "state", B.packed_state_elems(M, n))


class _NullStream:
    cuda_stream = 0


def test_headers_are_plain_c_and_a_c_program_links_against_the_library(lib, tmp_path):
    """The boundary is a C ABI: both headers must compile as C99 on their own, and a C program
    that includes them must link against the shared library and call it."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler here")
    inc = os.path.join(ROOT, "include")
    for hdr in ("diloco.h", "diloco_sim.h"):
        subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c",
                        os.path.join(inc, hdr)], check=True)
    src = tmp_path / "probe.c"
    src.write_text(
        '#include <stdio.h>\n#include "diloco.h"\n#include "diloco_sim.h"\n'
        "int main(void) {\n"
        "    /* validation only: no launch, no GPU needed */\n"
        "    int rc = diloco_outer_eager(NULL, DILOCO_F32, 2, 64, 64, NULL, NULL, NULL, 64, NULL, 0.7, 0.9, 1,\n"
        "                                DILOCO_EAGER | DILOCO_COMM_EXMY(2, 1, 11) | DILOCO_STATE_NO_MEAN, 1, NULL);\n"
        "    diloco_launch shape = {256, 1, 2, 0};\n"
        "    rc += 100 * diloco_outer_eager_packed_shaped(NULL, DILOCO_F32, 2, 64, 64, NULL, 0.7, 0.9, 1, DILOCO_EAGER, 1, NULL, &shape);\n"
        '    printf("%d %d %s %lld %d\\n", diloco_version(), rc, diloco_strerror(rc),\n'
        "           (long long)diloco_packed_state_elems(8, 8193), DILOCO_SIM_MAX_FUSED_STEPS);\n"
        "    return 0;\n}\n")
    exe = tmp_path / "probe"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe), "-L", libdir,
                    "-l:" + os.path.basename(B.LIB_PATH), "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(maxsplit=2)
    assert int(out[0]) >= 100 and int(out[1]) == 101 * B.ERR_NULL
    assert out[2].strip().endswith(f"{2 * 25 * 8192} 64")
