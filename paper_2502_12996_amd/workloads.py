"""Seeded synthetic workloads: shapes, hyper-parameters and input buffers.

This module holds no arithmetic of the method itself.  It only says how large
the flat buffers are, which scalars a run uses, and how the seeded random
inputs are drawn.  Both the CPU checker and the GPU tests take their inputs
from here, so the two sides always see the same numbers.

The paper trains transformer language models with M = 2 replicas (Section 3,
"Experiments"); its datasets and weights are not available, and the optimizer
sweep never looks at the data, so flat buffers with the transformer's tensor
sizes and the value scales of weights / outer gradients stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np
import torch

BASE_SEED = 0x5EEDD110C0

# buffer tags: every buffer draws from its own generator stream
TAGS = {
    "anchor": 1, "delta": 2, "prev_local": 3, "vel": 4, "m1": 5, "m2": 6,
    "grad": 7, "theta_noise": 8, "h": 9, "theta_star": 10, "prev_mean": 11,
    "theta": 12,
}


@dataclass(frozen=True)
class Workload:
    """One of the five benchmark / parity configurations."""
    name: str
    M: int                       # workers (replicas)
    n: int                       # parameters per worker
    layers: int = 0              # transformer shape (0: one flat tensor)
    d_model: int = 0
    vocab: int = 0
    theta_dtype: str = "f32"     # dtype of worker params and AdamW moments
    H: int = 1                   # inner steps per phase
    phases: int = 1
    # inner AdamW
    lr: float = 4e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1
    # outer Nesterov
    outer_lr: float = 0.7
    outer_momentum: float = 0.9
    nesterov: bool = True
    # value scales (standard deviations)
    std_anchor: float = 0.02
    std_delta: float = 1e-3
    std_grad: float = 1e-2
    noise_std: float = 0.1       # quadratic workload only


def transformer_param_count(layers: int, d: int, vocab: int) -> int:
    return layers * 12 * d * d + vocab * d


def tensor_table(layers: int, d: int, vocab: int) -> List[Tuple[str, int, int]]:
    """(name, offset, count) of every tensor of the flat buffer.

    Per layer: four d x d attention matrices and two d x 4d MLP matrices;
    one vocab x d embedding at the end.
    """
    table: List[Tuple[str, int, int]] = []
    off = 0
    for l in range(layers):
        for nm in ("wq", "wk", "wv", "wo"):
            table.append((f"layer{l}.{nm}", off, d * d))
            off += d * d
        for nm in ("w_up", "w_down"):
            table.append((f"layer{l}.{nm}", off, 4 * d * d))
            off += 4 * d * d
    table.append(("embedding", off, vocab * d))
    off += vocab * d
    assert off == transformer_param_count(layers, d, vocab)
    return table


def fragments(layers: int, d: int, vocab: int, layers_per_fragment: int = 3) -> List[Tuple[int, int]]:
    """(offset, count) of the Streaming-DiLoCo fragments of the flat buffer: groups of
    `layers_per_fragment` consecutive layers (the paper's simulations use 3); the embedding,
    which the paper does not place, joins the last group."""
    per_layer = 12 * d * d
    out: List[Tuple[int, int]] = []
    l = 0
    while l < layers:
        k = min(layers_per_fragment, layers - l)
        out.append((l * per_layer, k * per_layer))
        l += k
    off, cnt = out[-1]
    out[-1] = (off, cnt + vocab * d)
    assert out[-1][0] + out[-1][1] == transformer_param_count(layers, d, vocab)
    return out


WORKLOADS: Dict[str, Workload] = {
    # config 1: oracle-in-seconds case, 10 outer phases of noisy workers
    "tiny": Workload("tiny", M=2, n=1 << 20, H=1, phases=10),
    # config 2: H = 30 AdamW steps, then one eager outer step
    "t150m": Workload("t150m", M=4, n=transformer_param_count(12, 768, 32768),
                      layers=12, d_model=768, vocab=32768, H=30, phases=1),
    # config 3: the headline bandwidth case
    "t550m": Workload("t550m", M=8, n=transformer_param_count(24, 1408, 32768),
                      layers=24, d_model=1408, vocab=32768, H=1, phases=1),
    # config 4: bf16 worker buffers, fp32 outer state
    "t2b4_bf16": Workload("t2b4_bf16", M=2, n=transformer_param_count(32, 2432, 32768),
                          layers=32, d_model=2432, vocab=32768, theta_dtype="bf16"),
    # config 5: noisy quadratic, gradient made inside the kernel
    "quadratic": Workload("quadratic", M=4, n=1 << 26, H=50, phases=40,
                          weight_decay=0.0),
}
assert WORKLOADS["t150m"].n == 110_100_480
assert WORKLOADS["t550m"].n == 617_086_976
assert WORKLOADS["t2b4_bf16"].n == 2_350_907_392


def _generator(seed: int, tag: str, extra: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    # distinct 63-bit stream id per (seed, buffer, extra); any injective-ish mix will do
    sid = (seed * 0x9E3779B97F4A7C15 + TAGS[tag] * 0xD1342543DE82EF95
           + (extra + 1) * 0xA0761D6478BD642F) & ((1 << 63) - 1)
    g.manual_seed(sid)
    return g


def normal(shape, std: float, *, tag: str, seed: int = BASE_SEED, extra: int = 0,
           mean: float = 0.0, device="cpu", dtype=torch.float32) -> torch.Tensor:
    """Seeded N(mean, std) draw, made directly on `device` in fp32."""
    g = _generator(seed, tag, extra, device)
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(mean, std, generator=g)
    return t if dtype == torch.float32 else t.to(dtype)


def log_uniform(shape, lo: float, hi: float, *, tag: str, seed: int = BASE_SEED,
                extra: int = 0, device="cpu") -> torch.Tensor:
    """Seeded draw with log(x) uniform on [log lo, log hi]."""
    g = _generator(seed, tag, extra, device)
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.uniform_(float(np.log(lo)), float(np.log(hi)), generator=g)
    return t.exp_()


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a (CPU or GPU) fp32 / bf16 tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy().copy()


def outer_state(wl: Workload, n: int, *, seed: int = BASE_SEED, device="cpu",
                stride: int | None = None) -> Dict[str, torch.Tensor]:
    """Buffers of a mid-training eager outer step (configs 3 and 4).

    anchor ~ N(0, std_anchor), identical on all workers; theta_m = anchor - delta_m
    with delta_m ~ N(0, std_delta); prev_local ~ N(0, std_delta); prev_mean is the
    worker mean of prev_local (taken in fp32 by torch: an input, not a checked
    result); vel ~ N(0, std_delta).  Buffers with a worker axis are [M, stride]
    and only the first n columns are meaningful.
    """
    M = wl.M
    stride = n if stride is None else stride
    th_dtype = torch.bfloat16 if wl.theta_dtype == "bf16" else torch.float32
    a0 = normal((n,), wl.std_anchor, tag="anchor", seed=seed, device=device)
    anchor = torch.zeros((M, stride), dtype=torch.float32, device=device)
    theta = torch.zeros((M, stride), dtype=th_dtype, device=device)
    prev_local = torch.zeros((M, stride), dtype=torch.float32, device=device)
    vel = torch.zeros((M, stride), dtype=torch.float32, device=device)
    for m in range(M):
        anchor[m, :n] = a0
        d = normal((n,), wl.std_delta, tag="delta", seed=seed, extra=m, device=device)
        theta[m, :n] = (a0 - d).to(th_dtype)
        del d
        prev_local[m, :n] = normal((n,), wl.std_delta, tag="prev_local", seed=seed,
                                   extra=m, device=device)
        vel[m, :n] = normal((n,), wl.std_delta, tag="vel", seed=seed, extra=m,
                            device=device)
    prev_mean = prev_local[:, :n].mean(dim=0)
    return dict(theta=theta, anchor=anchor, vel=vel, prev_local=prev_local,
                prev_mean=prev_mean)


def adamw_state(wl: Workload, n: int, *, seed: int = BASE_SEED, device="cpu",
                stride: int | None = None, grad_dtype=torch.float32,
                step_tag: int = 0) -> Dict[str, torch.Tensor]:
    """Buffers of a mid-training inner AdamW step: theta ~ N(0, std_anchor),
    m1 ~ N(0, std_grad), m2 = square of an N(0, std_grad) draw, grad ~ N(0, std_grad)."""
    M = wl.M
    stride = n if stride is None else stride
    dt = torch.bfloat16 if wl.theta_dtype == "bf16" else torch.float32
    out = {k: torch.zeros((M, stride), dtype=dt, device=device) for k in ("theta", "m1", "m2")}
    out["grad"] = torch.zeros((M, stride), dtype=grad_dtype, device=device)
    for m in range(M):
        out["theta"][m, :n] = normal((n,), wl.std_anchor, tag="theta", seed=seed, extra=m,
                                     device=device).to(dt)
        out["m1"][m, :n] = normal((n,), wl.std_grad, tag="m1", seed=seed, extra=m,
                                  device=device).to(dt)
        out["m2"][m, :n] = normal((n,), wl.std_grad, tag="m2", seed=seed, extra=m,
                                  device=device).square_().to(dt)
        out["grad"][m, :n] = normal((n,), wl.std_grad, tag="grad", seed=seed,
                                    extra=m + 1000 * step_tag, device=device).to(grad_dtype)
    return out
