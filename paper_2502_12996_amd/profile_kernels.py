"""Launches each streaming kernel of the library a few times on a benchmark workload, and nothing
else: the program to put under `rocprofv3 --pmc ...` or `--kernel-trace --stats`, where the
benchmark's shape search would only add hundreds of launches to every pass.

    python3 -m paper_2502_12996_amd.profile_kernels [--workload t550m] [--reps 3]

Kernels, in launch order (the eager kernel on the packed state appears twice under one name: the
first `reps` launches update the state in place, the next `reps` read one buffer and write another):
    stream_copy_kernel                          plain copy of M*N floats
    stream_sweep_kernel<33|1, 1|2|0>            33 (or 1) separated rows: read only, write only, read-modify-write
    outer_eager_reg_kernel<M, .., RowState>     eager outer step, caller rows
    outer_eager_reg_kernel<M, .., TiledState>   eager outer step, packed state: in place, then ping-pong
    outer_sync_vec_kernel                       standard outer step
    adamw_vec_kernel                            inner AdamW sweep
Prints one line per group with its launch shape and HIP-event time.
"""
from __future__ import annotations

import argparse

import torch

import paper_2502_12996_amd as d
from paper_2502_12996_amd import workloads as W


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="t550m")
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--rows-shape", default="64,0,2")
    ap.add_argument("--packed-shape", default="64,0,3")
    ap.add_argument("--inner-shape", default="0,0,-1")
    args = ap.parse_args()
    shape = lambda s: tuple(int(x) for x in s.split(","))
    dev = "cuda:0"
    wl = W.WORKLOADS[args.workload]
    M, n = wl.M, wl.n
    bf16 = wl.theta_dtype == "bf16"
    okw = dict(outer_lr=wl.outer_lr, outer_momentum=wl.outer_momentum)

    def group(name, fn, nbytes, sh):
        fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.reps + 1)]
        ev[0].record()
        for k in range(args.reps):
            fn()
            ev[k + 1].record()
        torch.cuda.synchronize()
        ms = sorted(ev[k].elapsed_time(ev[k + 1]) for k in range(args.reps))[args.reps // 2]
        print(f"{name:44s} launches {args.reps + 1}  shape {sh}  {ms:8.3f} ms  {nbytes / ms / 1e6:8.1f} GB/s", flush=True)

    # ceilings: copy, and K separated rows read / written / both
    buf = torch.empty(2 * M * n, dtype=torch.float32, device=dev).normal_(0, 1e-3)
    src, dst = buf[:M * n], buf[M * n:]
    group("copy", lambda: d.sim_stream_copy(dst, src, launch=(64, 0, 0)), 8.0 * M * n, (64, 0, 0))
    del buf, src, dst
    K = 4 * M + 1
    for k in sorted({K, 1}, reverse=True):
        if k not in (1, 2, 4, 5, 8, 9, 16, 17, 33):
            continue
        nr = min(n & ~3, 1 << 28) if k > 1 else 1 << 31
        rows = torch.empty((k, nr), dtype=torch.float32, device=dev).normal_(0, 1e-3)
        sh = (64, 0, 3) if k > 1 else (64, 0, 24)
        group(f"K={k} rows read only", lambda: d.sim_stream_sweep(rows, d.SWEEP_READ, launch=sh), 4.0 * k * nr, sh)
        group(f"K={k} rows write only", lambda: d.sim_stream_sweep(rows, d.SWEEP_WRITE, fill=1e-3, launch=sh),
              4.0 * k * nr, sh)
        group(f"K={k} rows read-modify-write", lambda: d.sim_stream_sweep(rows, d.SWEEP_RMW, launch=sh),
              8.0 * k * nr, sh)
        del rows
    torch.cuda.empty_cache()

    st = W.outer_state(wl, n, device=dev)
    theta = st["theta"]
    es = 2 if bf16 else 4
    outer_bytes = 2.0 * (M * (es + 12) + 4) * n
    sh = shape(args.rows_shape)
    group("eager outer step, caller rows", lambda: d.outer_eager(
        theta, st["anchor"], st["vel"], st["prev_local"], st["prev_mean"], launch=sh, **okw), outer_bytes, sh)
    state = torch.empty(d.packed_state_elems(M, n), dtype=torch.float32, device=dev)
    d.pack_state(state, M, n, anchor=st["anchor"], vel=st["vel"], prev_local=st["prev_local"],
                 prev_mean=st["prev_mean"])
    a, u = st["anchor"][0].clone(), st["vel"][0].clone()
    for k in ("anchor", "vel", "prev_local", "prev_mean"):
        del st[k]
    torch.cuda.empty_cache()
    sh = shape(args.packed_shape)
    group("eager outer step, packed state in place", lambda: d.outer_eager_packed(theta, state, launch=sh, **okw),
          outer_bytes, sh)
    pair = [state, torch.empty_like(state)]
    flip = [0]

    def pingpong():
        d.outer_eager_pingpong(theta, pair[flip[0]], pair[1 - flip[0]], launch=sh, **okw)
        flip[0] = 1 - flip[0]
    group("eager outer step, packed state ping-pong", pingpong, outer_bytes, sh)
    del pair, state
    torch.cuda.empty_cache()
    group("standard outer step", lambda: d.outer_sync(theta, a, u, **okw), (2.0 * M * es + 16) * n, "automatic")
    del a, u
    ad = W.adamw_state(wl, n, device=dev, grad_dtype=torch.bfloat16 if bf16 else torch.float32)
    sh = shape(args.inner_shape)
    group("inner AdamW sweep", lambda: d.inner_adamw(
        ad["theta"], ad["m1"], ad["m2"], ad["grad"], lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps,
        weight_decay=wl.weight_decay, step=31, launch=sh), 7.0 * es * M * n, sh)


if __name__ == "__main__":
    main()
