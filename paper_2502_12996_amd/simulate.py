"""End-to-end single-GPU DiLoCo simulation on the noisy quadratic stand-in problem.

The outer loop of Algorithms 1-3 (`for t = 1..T`, `if t mod H == 0`) is host control flow and
lives here; every arithmetic step runs in the library's kernels:

    lines 3-5   diloco_sim_quadratic_inner   (gradient made in registers + AdamW, all replicas)
                diloco_sim_quadratic_phase   (the same for all steps between two boundaries in one
                                              pass; --fused 1)
    lines 7-12  diloco_outer_sync / diloco_outer_eager / diloco_outer_eager_packed /
                diloco_outer_eager_pingpong / diloco_outer_eager_overlap2
    loss        diloco_sim_quadratic_loss    (at the replica mean of the outer parameters)

    python -m paper_2502_12996_amd.simulate            # benchmark configuration 5: 64M params,
                                                       # M=4, H=50, 40 phases, four variants
"""
from __future__ import annotations

import argparse
import json
import time
from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as B
from . import workloads as W


class QuadraticSimulation:
    """M replicas training 0.5 sum_i h_i (theta_i - theta*_i)^2 with AdamW inside and one of the
    three outer rules outside.  variant: "standard" (Algorithm 1), "delayed" (Algorithm 2),
    "eager" (Algorithm 3).  layout (outer state of Algorithms 2/3): "packed" (updated in place),
    "pingpong" (two packed buffers, read one / write the other) or "rows".
    fragments: Streaming-DiLoCo windows [(offset, count), ...] on staggered boundaries.
    overlap: 1 (the listings) or 2 (2-outer-steps overlap: two generations of the previous outer
    gradients, in two row sets or two packed buffers).
    first_boundary: "listing" (Algorithms 2/3: no outer step at a fragment's first boundary) or
    "zero_history" (the outer step is applied from the first boundary on, the history being zero).
    fused: run the inner steps between two outer boundaries as one pass over the buffers
    (bit-identical to the step-by-step run).
    no_mean: eager only, M <= 8: do not keep the previous mean, form it from the previous local
    outer gradients (bit-identical as well)."""

    def __init__(self, M: int, n: int, H: int, variant: str = "eager", *, layout: str = "packed",
                 fragments: Optional[Sequence[Tuple[int, int]]] = None, overlap: int = 1,
                 comm_bf16: bool = False, comm_flags: int = 0, seed: int = W.BASE_SEED, noise_std: float = 0.1,
                 lr: float = 4e-4, beta1: float = 0.9, beta2: float = 0.95, eps: float = 1e-8,
                 weight_decay: float = 0.0, outer_lr: float = 0.7, outer_momentum: float = 0.9,
                 nesterov: bool = True, fused: bool = False, no_mean: bool = False,
                 first_boundary: str = "listing", device: str = "cuda:0"):
        assert variant in ("standard", "delayed", "eager")
        assert layout in ("packed", "pingpong", "rows") and overlap in (1, 2)
        assert first_boundary in ("listing", "zero_history")
        self.M, self.n, self.H, self.variant = M, n, H, variant
        self.shared = variant == "standard"
        self.packed = layout != "rows" and not self.shared
        self.pingpong = layout == "pingpong" and self.packed
        assert not (self.pingpong and (overlap == 2 or fragments)), \
            "ping-pong sweeps the whole model at every boundary, one generation in flight"
        self.zero_history = first_boundary == "zero_history"
        self.fragments = list(fragments) if fragments else [(0, n)]
        self.overlap, self.seed, self.noise_std = overlap, seed, noise_std
        self.adam = dict(lr=lr, beta1=beta1, beta2=beta2, eps=eps, weight_decay=weight_decay)
        self.outer = dict(outer_lr=outer_lr, outer_momentum=outer_momentum, nesterov=nesterov)
        self.flags = ((B.DELAYED if variant == "delayed" else B.EAGER) | (B.COMM_BF16 if comm_bf16 else 0)
                      | comm_flags)      # comm_flags: e.g. binding.COMM_EXMY(2, 1, 11)
        if no_mean:
            assert variant == "eager" and overlap == 1, "only the eager step can do without the stored mean"
            self.flags |= B.STATE_NO_MEAN
        self.fused = fused
        self.t = 0
        f32 = dict(dtype=torch.float32, device=device)
        ns = (n + 3) & ~3                         # replica rows 16-byte aligned
        self.h = W.log_uniform((n,), 1e-3, 1.0, tag="h", seed=seed, device=device)
        self.star = W.normal((n,), 1.0, tag="theta_star", seed=seed, device=device)
        self.theta = torch.zeros((M, ns), **f32)
        self.m1, self.m2 = torch.zeros((M, ns), **f32), torch.zeros((M, ns), **f32)
        if self.shared:
            self.anchor, self.vel = torch.zeros(n, **f32), torch.zeros(n, **f32)
        elif self.packed:
            self.state = torch.zeros(B.packed_state_elems(M, n), **f32)
            if self.pingpong or overlap == 2:             # the second packed buffer
                self.states = [self.state, torch.zeros_like(self.state)]
            self.anchor = torch.zeros((M, ns), **f32)     # scratch for the loss only
        else:
            self.anchor, self.vel = torch.zeros((M, ns), **f32), torch.zeros((M, ns), **f32)
            self.prev_local = [torch.zeros((M, ns), **f32) for _ in range(overlap)]
            self.prev_mean = [torch.zeros(n, **f32) for _ in range(overlap)]
        self._partials = torch.empty(B.sim_loss_workspace(n), dtype=torch.float64, device=device)

    # -- one step of the listings' loop -------------------------------------------------
    def step(self) -> bool:
        """Lines 3-5 for every replica, then the outer step of every fragment whose boundary this
        is.  Returns True if any outer boundary fell on this step."""
        self.t += 1
        B.sim_quadratic_inner(self.theta, self.m1, self.m2, self.h, self.star, n=self.n,
                              noise_std=self.noise_std, seed=self.seed, step=self.t, **self.adam)
        return self._boundaries()

    def advance(self, steps: int) -> bool:
        """`steps` inner steps in as few passes as the library allows, then the outer steps due at
        the step reached.  The caller makes sure no boundary falls strictly inside (run() does)."""
        while steps > 0:
            c = min(steps, B.SIM_MAX_FUSED_STEPS)
            B.sim_quadratic_phase(self.theta, self.m1, self.m2, self.h, self.star, n=self.n,
                                  noise_std=self.noise_std, seed=self.seed, step_first=self.t + 1, steps=c,
                                  **self.adam)
            self.t += c
            steps -= c
        return self._boundaries()

    def _boundaries(self) -> bool:
        t, M, n, H = self.t, self.M, self.n, self.H
        F = len(self.fragments)
        fired = False
        for f, (off, cnt) in enumerate(self.fragments):
            if not B.stream_due(t, H, F, f):
                continue
            fired = True
            b = B.stream_boundary_count(t, H, F, f)
            th = self.theta[:, off:off + cnt]
            if self.shared:
                B.outer_sync(th, self.anchor[off:off + cnt], self.vel[off:off + cnt], n=cnt, **self.outer)
            elif self.packed and self.overlap == 2:
                # the buffer written at this fragment's previous boundary, and the one written before that
                prev, cur = self.states[(b - 1) % 2], self.states[b % 2]
                B.outer_eager_overlap2(th, B.packed_window(prev, M, off), B.packed_window(cur, M, off), n=cnt,
                                       variant=self.flags, apply_update=b > 2 or self.zero_history, **self.outer)
            elif self.pingpong:
                B.outer_eager_pingpong(th, self.states[(b - 1) % 2], self.states[b % 2], n=cnt, variant=self.flags,
                                       apply_update=b > 1 or self.zero_history, **self.outer)
                self.state = self.states[b % 2]
            elif self.packed:
                B.outer_eager_packed(th, B.packed_window(self.state, M, off), n=cnt, variant=self.flags,
                                     apply_update=b > 1 or self.zero_history, **self.outer)
            else:
                slot = b % self.overlap
                B.outer_eager(th, self.anchor[:, off:off + cnt], self.vel[:, off:off + cnt],
                              self.prev_local[slot][:, off:off + cnt], self.prev_mean[slot][off:off + cnt],
                              n=cnt, variant=self.flags, apply_update=b > self.overlap or self.zero_history,
                              **self.outer)
        return fired

    def outer_parameters(self) -> torch.Tensor:
        """[n] (standard) or [M, >= n] (delayed / eager) outer parameters."""
        if self.packed and self.overlap == 2:
            # every fragment's current outer parameters sit in the buffer its last boundary wrote
            F = len(self.fragments)
            for f, (off, cnt) in enumerate(self.fragments):
                b = B.stream_boundary_count(self.t, self.H, F, f)
                B.unpack_state(B.packed_window(self.states[b % 2], self.M, off), self.M, cnt,
                               anchor=self.anchor[:, off:off + cnt])
        elif self.packed:
            B.unpack_state(self.state, self.M, self.n, anchor=self.anchor)
        return self.anchor

    def loss(self, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Loss at the replica mean of the outer parameters, as a device double (no sync)."""
        out = torch.empty(1, dtype=torch.float64, device=self.theta.device) if out is None else out
        B.sim_quadratic_loss(self.outer_parameters(), self.h, self.star, self._partials, out, n=self.n)
        return out

    def run(self, phases: int) -> List[float]:
        """phases * H steps; the loss after every step on which an outer boundary fell."""
        losses = []
        end = self.t + phases * self.H
        while self.t < end:
            if self.fused:
                # up to the next step on which any fragment has a boundary
                F = len(self.fragments)
                nxt = next(t for t in range(self.t + 1, end + 1)
                           if t == end or any(B.stream_due(t, self.H, F, f) for f in range(F)))
                fired = self.advance(nxt - self.t)
            else:
                fired = self.step()
            if fired:
                losses.append(self.loss())
        torch.cuda.synchronize()
        return [float(x.item()) for x in losses]


def main() -> None:
    wl = W.WORKLOADS["quadratic"]
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--n", type=int, default=wl.n)
    ap.add_argument("--M", type=int, default=wl.M)
    ap.add_argument("--H", type=int, default=wl.H)
    ap.add_argument("--phases", type=int, default=wl.phases)
    ap.add_argument("--layout", choices=("packed", "pingpong", "rows"), default="packed")
    ap.add_argument("--fused", type=int, default=0, help="1: inner steps between boundaries in one pass")
    args = ap.parse_args()
    runs = [("standard", 1.0), ("eager", 1.0), ("delayed", 1.0), ("delayed", 0.25)]
    for variant, scale in runs:
        sim = QuadraticSimulation(args.M, args.n, args.H, variant, layout=args.layout,
                                  fused=bool(args.fused), noise_std=wl.noise_std, lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2,
                                  eps=wl.eps, weight_decay=wl.weight_decay,
                                  outer_lr=wl.outer_lr * scale, outer_momentum=wl.outer_momentum)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        losses = sim.run(args.phases)
        dt = time.perf_counter() - t0
        print(json.dumps({"variant": variant, "outer_lr": wl.outer_lr * scale, "M": args.M, "n": args.n,
                          "H": args.H, "phases": args.phases, "fused": args.fused, "seconds": dt,
                          "inner_steps_per_s": args.phases * args.H / dt, "loss": losses}), flush=True)
        del sim
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
