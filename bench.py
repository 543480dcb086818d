#!/usr/bin/env python3
"""Benchmark of the DiLoCo optimizer sweep on one MI355X.

A step is one pass of the whole hot path over the workload's buffers: one inner AdamW sweep
of all M replicas, then one fused eager outer step (outer gradients, replica mean, eager
combination, Nesterov outer update, re-seeding, state rotation).  All buffers are resident
in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload t550m]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak


def algorithmic_bytes(wl, n):
    """Bytes the method itself must move per launch (each operand read once, written once)."""
    M = wl.M
    ts = 2 if wl.theta_dtype == "bf16" else 4
    # eager outer: theta (ts) + anchor, vel, prev_local (4 each) per replica, prev_mean once; read + write
    outer = 2 * (M * (ts + 12) + 4) * n
    # AdamW: read theta, m1, m2, grad; write theta, m1, m2 (grad has theta's dtype in these workloads)
    inner = 7 * ts * M * n
    return outer, inner


def shape_json(sh):
    if sh is None:
        return "automatic"
    return {"block": sh[0], "xcd_remap": sh[1], "wg_per_cu": sh[2]}


def spread(ms):
    """min / median / max / mean of per-launch times in ms."""
    s = sorted(ms)
    return {"min": s[0], "median": s[len(s) // 2] if len(s) % 2 else 0.5 * (s[len(s) // 2 - 1] + s[len(s) // 2]),
            "max": s[-1], "mean": sum(s) / len(s)}


def outer_bytes_fn(wl, n):
    return algorithmic_bytes(wl, n)[0]


def stored_traffic(workload, layout):
    """HBM bytes per launch of the eager kernel, measured with rocprofv3 --pmc FETCH_SIZE and
    WRITE_SIZE (scaled by a copy kernel of known size) and kept in the committed summary."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_pmc_bench_%s.txt" % workload)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("%s.outer_eager_%s_bytes_per_launch" % (workload, layout)):
                    return int(line.split("=")[1])
    except (OSError, ValueError):
        pass
    return None


def cpu_baseline(wl, sample, min_seconds=10.0, max_reps=16):
    """The CPU checker, as it stands, on `sample` parameter indices of the same workload,
    repeated on fresh copies of the same inputs until about `min_seconds` of checker time."""
    import numpy as np

    from oracle import diloco_oracle as O
    from paper_2502_12996_amd import workloads as W
    st0 = {k: W.to_f64(v) for k, v in W.outer_state(wl, sample, seed=99).items()}
    ad0 = {k: W.to_f64(v) for k, v in W.adamw_state(wl, sample, seed=99).items()}
    inner_s = outer_s = 0.0
    reps = 0
    while reps < max_reps and inner_s + outer_s < min_seconds:
        st = {k: v.copy() for k, v in st0.items()}
        ad = {k: v.copy() for k, v in ad0.items()}
        t0 = time.perf_counter()
        O.adamw_step(ad["theta"], ad["m1"], ad["m2"], ad["grad"], 31, wl.lr, wl.beta1, wl.beta2,
                     wl.eps, wl.weight_decay)
        t1 = time.perf_counter()
        O.outer_eager(st["theta"], st["anchor"], st["vel"], st["prev_local"], st["prev_mean"],
                      wl.outer_lr, wl.outer_momentum, True, True)
        t2 = time.perf_counter()
        inner_s += t1 - t0
        outer_s += t2 - t1
        reps += 1
        assert np.isfinite(st["anchor"]).all()
    # the standard outer step once, outside the headline figure
    th, a, u = st0["theta"].copy(), st0["anchor"][0].copy(), st0["vel"][0].copy()
    t0 = time.perf_counter()
    O.outer_standard(th, a, u, wl.outer_lr, wl.outer_momentum, True)
    standard_s = time.perf_counter() - t0
    cpu_model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return dict(value=reps * sample / (inner_s + outer_s), unit="params/s", cores=1, kind="oracle",
                sample=f"{reps} x {sample} parameter indices x M={wl.M} replicas of {wl.name}: AdamW sweep "
                       f"({inner_s:.2f} s) + eager outer step ({outer_s:.2f} s), float64 NumPy, 1 thread",
                inner_s=inner_s, outer_s=outer_s, outer_params_per_s=reps * sample / outer_s,
                inner_worker_params_per_s=reps * sample * wl.M / inner_s,
                standard_outer_params_per_s=sample / standard_s,
                host_cpus=os.cpu_count(), cpu_model=cpu_model)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="t550m")
    ap.add_argument("--layout", choices=("pingpong", "packed", "rows"), default="packed",
                    help="outer state: library-packed tiles updated in place (default), the same tiles read "
                         "from one buffer and written to a second, or caller rows [M][stride]")
    ap.add_argument("--autotune", type=int, default=1,
                    help="pick workgroup size / XCD mapping per kernel before the warm-up (1) or keep defaults (0)")
    ap.add_argument("--pad", type=int, default=0, help="extra elements between replica rows")
    ap.add_argument("--placement", choices=("classes", "plain"), default="classes",
                    help="where the swept buffers lie in device memory: AdamW's four arrays in one memory class "
                         "and the packed outer state in another (paper_2502_12996_amd/placement.py; falls back to "
                         "plain when that fails), or plain torch allocations")
    ap.add_argument("--cpu-sample", type=int, default=1 << 24,
                    help="parameter indices the CPU checker is timed on (0: skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the M replicas are simulated on it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2502_12996_amd as d
    from paper_2502_12996_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    wl = W.WORKLOADS[args.workload]
    M, n = wl.M, wl.n
    stride = n + args.pad
    bf16 = wl.theta_dtype == "bf16"
    packed = args.layout != "rows"
    pingpong = args.layout == "pingpong"

    # Which physical memory a buffer lies in moves these sweeps by several per cent (two streams read
    # together run 5 % faster inside one memory class than across two): the arrays that one kernel
    # streams together are placed in one class each, before anything else is allocated.
    arena, placed = None, {}
    placement = {"requested": args.placement, "used": False}
    if args.placement == "classes":
        try:
            from paper_2502_12996_amd import placement as PL
            arena = PL.Arena(device=0)
            arena.classify()
            rows_bytes = M * stride * (2 if bf16 else 4)
            groups = [[("theta", rows_bytes), ("m1", rows_bytes), ("m2", rows_bytes), ("grad", rows_bytes)]]
            if packed:
                groups.append([("state", d.packed_state_elems(M, n) * 4)])
            placed = arena.place(groups)
            arena.release_rest()
            placement = {"requested": "classes", "used": True, **arena.summary()}
        except Exception as err:             # no placement on this machine: ordinary allocations
            if arena is not None:
                arena.close()
            arena, placed = None, {}
            placement = {"requested": "classes", "used": False, "reason": repr(err)}

    def adopt(name, t):
        """The generated tensor, moved into the buffer placed for it if there is one."""
        if name not in placed:
            return t
        dst = placed[name].view(t.dtype).view(t.shape)
        dst.copy_(t)
        return dst

    ad = W.adamw_state(wl, n, device=dev, stride=stride,
                       grad_dtype=torch.bfloat16 if bf16 else torch.float32)
    m1, m2, grad = adopt("m1", ad.pop("m1")), adopt("m2", ad.pop("m2")), adopt("grad", ad.pop("grad"))
    del ad                                   # its theta is not used: the replicas' live parameters serve both kernels
    torch.cuda.empty_cache()
    st = W.outer_state(wl, n, device=dev, stride=stride)
    st["theta"] = theta = adopt("theta", st["theta"])
    torch.cuda.empty_cache()
    okw = dict(outer_lr=wl.outer_lr, outer_momentum=wl.outer_momentum)

    def timed(fn, iters):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        ev[0].record()
        for k in range(iters):
            fn()
            ev[k + 1].record()
        torch.cuda.synchronize()
        return sorted(ev[k].elapsed_time(ev[k + 1]) for k in range(iters))

    # Launch shapes travel with each call (the *_shaped entry points): (workgroup size, XCD-contiguous
    # workgroup order, cap on resident workgroups per CU); None, or block 0 and cap -1, leave the
    # choice to the launch itself.  Nothing outside the call holds a shape.
    shape_default = None
    candidates = ([(0, x, -1) for x in (0, 1)]
                  + [(64, x, c) for x in (0, 1) for c in (2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 16)]
                  + [(256, x, c) for x in (0, 1) for c in (0, 1, 2, 3)]
                  + [(b, x, c) for x in (0, 1) for b in (128, 512) for c in (0, 1)])

    def autotune(fn):
        """Fastest of the launch shapes the library offers; fn(shape) launches once.  A first pass
        times every candidate (median of 5); the four best then run in turns, three rounds of three
        launches, and the best median of those nine wins: clocks drift over the seconds a pass takes,
        which a single pass would book to the candidates' places in the list."""
        for _ in range(8):
            fn(candidates[0])                  # steady clocks before the first candidate
        first = []
        for sh in candidates:
            fn(sh)
            first.append((timed(lambda: fn(sh), 5)[2], sh))
        finalists = [sh for _, sh in sorted(first, key=lambda p: p[0])[:4]]
        samples = {sh: [] for sh in finalists}
        for _ in range(3):
            for sh in finalists:
                fn(sh)
                samples[sh] += timed(lambda: fn(sh), 3)
        return min(finalists, key=lambda sh: sorted(samples[sh])[len(samples[sh]) // 2])

    def run_rows(sh=None):
        d.outer_eager(theta, st["anchor"], st["vel"], st["prev_local"], st["prev_mean"], n=n, launch=sh, **okw)

    def run_inner(sh=None, t=31):
        d.inner_adamw(theta, m1, m2, grad, n=n, lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps,
                      weight_decay=wl.weight_decay, step=t, launch=sh)

    shape_rows = autotune(run_rows) if args.autotune else shape_default
    shape_inner = autotune(run_inner) if args.autotune else shape_default

    # the eager step on caller-layout rows, timed on its own (secondary figure)
    run_rows(shape_rows)
    rows_all = timed(lambda: run_rows(shape_rows), max(5, args.steps // 2))
    rows_ms = sum(rows_all) / len(rows_all)

    if packed:
        state = (placed["state"].view(torch.float32) if "state" in placed
                 else torch.empty(d.packed_state_elems(M, n), dtype=torch.float32, device=dev))
        d.pack_state(state, M, n, anchor=st["anchor"], vel=st["vel"], prev_local=st["prev_local"],
                     prev_mean=st["prev_mean"])
        torch.cuda.synchronize()
        for k in ("anchor", "vel", "prev_local", "prev_mean"):
            del st[k]
        torch.cuda.empty_cache()

        def run_in_place(sh=None, **kw):
            d.outer_eager_packed(theta, state, n=n, launch=sh, **okw, **kw)
        shape_in_place = autotune(run_in_place) if args.autotune else shape_default
        # the same step with the state read from one buffer and written to the other (the two swap
        # after every call): timed on its own beside the in-place call, or as the step's kernel
        pair = [state, torch.empty_like(state)]
        flip = [0]

        def run_pingpong(sh=None, **kw):
            d.outer_eager_pingpong(theta, pair[flip[0]], pair[1 - flip[0]], n=n, launch=sh, **okw, **kw)
            flip[0] = 1 - flip[0]
        run_pingpong()        # both buffers hold a full state from here on
        shape_pingpong = autotune(run_pingpong) if args.autotune else shape_default
        if pingpong:
            run_outer, shape_outer = run_pingpong, shape_pingpong
            run_in_place(shape_in_place)
            other_all = timed(lambda: run_in_place(shape_in_place), max(6, args.steps // 2))
        else:
            run_outer, shape_outer = run_in_place, shape_in_place
            run_pingpong(shape_pingpong)
            other_all = timed(lambda: run_pingpong(shape_pingpong), max(6, args.steps // 2))
            state = pair[flip[0]]     # the buffer the last ping-pong call wrote: the current state
    else:
        run_outer, shape_outer = run_rows, shape_rows

    def step(t, ev=None):
        if ev:
            ev[0].record()
        run_inner(shape_inner, t)
        if ev:
            ev[1].record()
        run_outer(shape_outer)
        if ev:
            ev[2].record()

    for w in range(args.warmup):
        step(31 + w)
    torch.cuda.synchronize()
    # events sit on torch's current stream, the stream the library launches on
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(31 + args.warmup + k, events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / args.steps
    inner_all = [e[0].elapsed_time(e[1]) for e in events]
    outer_all = [e[1].elapsed_time(e[2]) for e in events]
    inner_ms = sum(inner_all) / args.steps      # the average launch duration: what the roofline figure uses
    outer_ms = sum(outer_all) / args.steps
    if packed:
        chk = torch.empty((M, 4096), device=dev)
        d.unpack_state(pair[flip[0]] if pingpong else state, M, 4096, anchor=chk)
        assert torch.isfinite(chk).all()
    else:
        assert torch.isfinite(st["anchor"][:, :1024]).all()

    # next rows: the same outer step swept fragment by fragment (Streaming DiLoCo windows, one
    # launch per group of 3 layers) and with bf16 outer gradients on the wire
    extra = {}
    if packed and wl.layers:
        frs = W.fragments(wl.layers, wl.d_model, wl.vocab)

        def run_fragments():
            for off, cnt in frs:
                d.outer_eager_packed(theta[:, off:off + cnt], d.packed_window(state, M, off), n=cnt,
                                     launch=shape_in_place, **okw)
        run_fragments()
        fms = timed(run_fragments, 5)[2]
        extra["outer_step_by_fragments"] = {"fragments": len(frs), "ms": fms,
                                            "GBps": outer_bytes_fn(wl, n) / (fms * 1e-3) / 1e9}

        def run_q():
            run_outer(shape_outer, variant=d.EAGER | d.COMM_BF16)
        run_q()
        qms = timed(run_q, 5)[2]
        extra["outer_step_bf16_comm"] = {"ms": qms, "GBps": outer_bytes_fn(wl, n) / (qms * 1e-3) / 1e9}

        def run_q4():   # float4 (E2M1, range placed at the outer gradients' scale) on the wire
            run_outer(shape_outer, variant=d.EAGER | d.COMM_EXMY(2, 1, 11))
        run_q4()
        q4ms = timed(run_q4, 5)[2]
        extra["outer_step_fp4_comm"] = {"ms": q4ms, "GBps": outer_bytes_fn(wl, n) / (q4ms * 1e-3) / 1e9}

    if packed:
        # the previous mean formed from the previous local outer gradients instead of kept: one
        # stream of 4M+1 less each way, priced at its own bytes
        es_ = 2 if bf16 else 4
        lean_bytes = 2 * (M * es_ + 12 * M) * n

        def run_lean():
            run_outer(shape_outer, variant=d.EAGER | d.STATE_NO_MEAN)
        run_lean()
        lms = timed(run_lean, 7)[3]
        extra["outer_step_no_stored_mean"] = {"ms": lms, "bytes_per_index": lean_bytes // n,
                                              "GBps": lean_bytes / (lms * 1e-3) / 1e9,
                                              "params_per_s": n / (lms * 1e-3)}

    # the standard (Algorithm 1) outer step on the same replicas: shared outer parameters
    es = 2 if bf16 else 4
    sa = W.normal((n,), wl.std_anchor, tag="anchor", device=dev)
    sv = torch.zeros(n, dtype=torch.float32, device=dev)

    def run_sync(sh=None):
        d.outer_sync(theta, sa, sv, launch=sh, **okw)
    shape_sync = autotune(run_sync) if args.autotune else shape_default
    run_sync(shape_sync)
    sms = timed(lambda: run_sync(shape_sync), 7)[3]
    extra["outer_step_standard"] = {"ms": sms, "GBps": (2 * M * es + 16) * n / (sms * 1e-3) / 1e9,
                                    "launch": shape_json(shape_sync)}
    del sa, sv

    # the stand-in training problem (configuration 5's shape): one inner step with the gradient made
    # in the kernel (HBM-bound), and a whole phase of H steps in one pass (vector-ALU-bound)
    ql = W.WORKLOADS["quadratic"]
    qt = torch.zeros((ql.M, ql.n), dtype=torch.float32, device=dev)
    q1, q2 = torch.zeros_like(qt), torch.zeros_like(qt)
    qh = W.log_uniform((ql.n,), 1e-3, 1.0, tag="h", device=dev)
    qs = W.normal((ql.n,), 1.0, tag="theta_star", device=dev)
    qkw = dict(noise_std=ql.noise_std, seed=W.BASE_SEED, lr=ql.lr, beta1=ql.beta1, beta2=ql.beta2, eps=ql.eps,
               weight_decay=ql.weight_decay)
    for t in range(1, 21):      # leave the all-zero start behind
        d.sim_quadratic_inner(qt, q1, q2, qh, qs, step=t, **qkw)
    q_ms = timed(lambda: d.sim_quadratic_inner(qt, q1, q2, qh, qs, step=21, **qkw), 9)[4]
    p_ms = timed(lambda: d.sim_quadratic_phase(qt, q1, q2, qh, qs, step_first=22, steps=ql.H, **qkw), 5)[2]
    extra["quadratic_sim"] = {"M": ql.M, "n": ql.n, "inner_step_ms": q_ms,
                              "inner_step_GBps": (8 + 24 * ql.M) * ql.n / (q_ms * 1e-3) / 1e9,
                              "fused_phase_steps": ql.H, "fused_phase_ms": p_ms,
                              "fused_replica_param_steps_per_s": ql.M * ql.n * ql.H / (p_ms * 1e-3),
                              "fused_speedup_over_single_steps": ql.H * q_ms / p_ms}
    del qt, q1, q2, qh, qs

    # practical ceiling: a plain copy kernel with the same access shape, in its best launch shape
    cbuf = torch.empty(2 * n, dtype=torch.float32, device=dev)
    src, dst = cbuf[:n], cbuf[n:]
    copy_ms = None
    for sh in [(b, x, 0) for b in (64, 256, 512) for x in (0, 1)]:
        for _ in range(3):
            d.sim_stream_copy(dst, src, launch=sh)
        t = timed(lambda: d.sim_stream_copy(dst, src, launch=sh), 10)[5]
        copy_ms = t if copy_ms is None else min(copy_ms, t)
    copy_gbps = 8 * n / (copy_ms * 1e-3) / 1e9
    del cbuf, src, dst

    # ceiling for the eager step's own access pattern: a bare in-place read-modify-write over
    # K = 4M + 1 separated rows (no arithmetic), in its best launch shape
    K = 4 * M + 1
    rmw_gbps, shape_rmw = None, None
    if K in (5, 9, 17, 33):
        nr = min(n & ~3, 1 << 28)
        rbuf = torch.empty((K, nr), dtype=torch.float32, device=dev).normal_(0, 1e-3)
        for sh in [(0, x, -1) for x in (0, 1)] + [(64, x, c) for x in (0, 1) for c in (2, 3, 4, 6, 8)]:
            d.sim_stream_rmw(rbuf, launch=sh)
            t = timed(lambda: d.sim_stream_rmw(rbuf, launch=sh), 5)[2]
            g = 8 * K * nr / (t * 1e-3) / 1e9
            if rmw_gbps is None or g > rmw_gbps:
                rmw_gbps, shape_rmw = g, sh
        del rbuf

    outer_bytes, inner_bytes = algorithmic_bytes(wl, n)
    outer_gbps = outer_bytes / (outer_ms * 1e-3) / 1e9
    inner_gbps = inner_bytes / (inner_ms * 1e-3) / 1e9

    def rates(ms, nbytes):
        """Per-launch time spread with the rate and the fraction of peak each time stands for."""
        sp = spread(ms)
        return {"ms": sp, "GBps": {k: nbytes / (v * 1e-3) / 1e9 for k, v in sp.items()},
                "frac_of_peak": {k: nbytes / (v * 1e-3) / 1e9 / HBM_PEAK_GBPS for k, v in sp.items()}}

    outer_spread, inner_spread, rows_spread = rates(outer_all, outer_bytes), rates(inner_all, inner_bytes), \
        rates(rows_all, outer_bytes)
    result = {
        "metric": "outer-step params/sec and achieved HBM GB/s (% of peak) at M workers",
        # the metric is the outer step's: model parameters through one fused eager outer step per
        # second, from the average duration of the outer kernel inside the timed step loop
        "value": n / (outer_ms * 1e-3),
        "value_is": "N / (average duration of the eager outer-step kernel inside the timed steps)",
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not bf16 else "f32 math, bf16 replica storage",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: M={M} replicas x N={n} params, one AdamW sweep + one "
                               f"fused eager outer step per step",
                   "M": M, "N": n, "theta_dtype": wl.theta_dtype, "stride_pad": args.pad,
                   "outer_state_layout": args.layout, "placement": placement,
                   "launch": {"outer": shape_json(shape_outer), "inner": shape_json(shape_inner)}},
        "whole_step": {"ms": ms_step, "params_per_s": n / (ms_step * 1e-3),
                       "what": "one AdamW sweep + one eager outer step, host clock over the timed steps"},
        "outer_step": {"ms": outer_ms, "params_per_s": n / (outer_ms * 1e-3),
                       "worker_params_per_s": M * n / (outer_ms * 1e-3), "GBps": outer_gbps,
                       "frac_of_peak": outer_gbps / HBM_PEAK_GBPS, "per_step": outer_spread},
        "outer_step_rows_layout": {"ms": rows_ms, "GBps": outer_bytes / (rows_ms * 1e-3) / 1e9,
                                   "frac_of_peak": outer_bytes / (rows_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                   "per_launch": rows_spread, "launch": shape_json(shape_rows)},
        **({("outer_step_packed_in_place" if pingpong else "outer_step_packed_pingpong"):
            dict(rates(other_all, outer_bytes), launch=shape_json(shape_in_place if pingpong else shape_pingpong))}
           if packed else {}),
        "inner_step": {"ms": inner_ms, "worker_params_per_s": M * n / (inner_ms * 1e-3),
                       "GBps": inner_gbps, "frac_of_peak": inner_gbps / HBM_PEAK_GBPS, "per_step": inner_spread},
        **extra,
        "copy_ceiling_GBps": copy_gbps,
        "stream_rmw_ceiling": None if rmw_gbps is None else {"K": K, "GBps": rmw_gbps,
                                                             "launch": shape_json(shape_rmw)},
        "roofline": {"bound": "hbm", "kernel": "outer_eager_reg_kernel<%d, %s, eager, %s>%s" % (
                         M, "bf16" if bf16 else "float", "TiledState" if packed else "RowState",
                         " (state read from one buffer, written to another)" if pingpong else ""),
                     "achieved": outer_gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": outer_gbps / HBM_PEAK_GBPS,
                     "frac_min_median_max": [outer_spread["frac_of_peak"][k] for k in ("max", "median", "min")],
                     "frac_of_copy": outer_gbps / copy_gbps,
                     "frac_of_stream_rmw": None if rmw_gbps is None else outer_gbps / rmw_gbps,
                     "traffic": stored_traffic(wl.name, "packed" if packed else "rows")},
    }
    if result["roofline"]["traffic"]:   # counter bytes over this run's time: the rate the counters imply
        result["roofline"]["traffic_GBps"] = result["roofline"]["traffic"] / (outer_ms * 1e-3) / 1e9
    del st, theta, m1, m2, grad, placed
    if packed:
        del state, pair
    torch.cuda.synchronize()
    if arena is not None:
        arena.close()
    torch.cuda.empty_cache()
    if args.cpu_sample > 0:
        result["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
