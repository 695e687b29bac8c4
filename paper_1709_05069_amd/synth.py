"""Seeded synthetic worker states (theta_k, grad_k) for the server step.

This module only *generates inputs*; it contains none of the method's
arithmetic and is the one piece shared by the device library's tests, the CPU
oracle's tests and the benchmark.

Workload model (stands in for the paper's Section 3 runs, whose datasets and
network are not available): m workers sit at theta_k = theta0 + N(0, s^2) on a
diagonal quadratic loss J = 0.5 theta^T diag(a) theta - b^T theta and report
grad_k = a * theta_k - b + N(0, noise^2).  theta0, b ~ N(0, 1).  The curvature
a is either log-uniform per element, or block-structured: `blocks` contiguous
equal blocks (the last takes the remainder), one log-uniform scale per block,
times a per-element jitter U(0.5, 2).

Values are computed in fp32 and then stored in the storage dtype (fp32 or
bf16).  Generation is chunked by rows with one generator per chunk, so the
result does not depend on how much device memory is free, and nothing of size
n*m is ever staged on the host.  CPU and GPU generators give different
streams: a test generates once, on one device, and copies.
"""
from dataclasses import dataclass, replace
import math

import torch

CHUNK_ROWS = 1 << 24


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    m: int
    storage: str          # "f32", "bf16" or "f16"
    a_lo: float
    a_hi: float
    blocks: int           # 0: per-element log-uniform curvature
    spread: float         # std of theta_k - theta0
    noise: float          # std of the stochastic-gradient noise
    lam: float
    tau: float
    seed: int = 0

    def scaled(self, n: int) -> "Workload":
        """Same recipe at a different parameter count."""
        return replace(self, n=int(n), name=f"{self.name}@n={int(n)}")


WORKLOADS = {
    "tiny_exact": Workload("tiny_exact", 4096, 4, "f32", 1e-3, 1e2, 0,
                           1e-2, 0.0, 0.01, 1.0),
    "small_mlp": Workload("small_mlp", 1_200_000, 8, "f32", 1e-4, 1e1, 0,
                          1e-3, 1e-2, 0.05, 0.5),
    "resnet50": Workload("resnet50", 25_600_000, 16, "f32", 1e-4, 1e2, 50,
                         1e-3, 1e-3, 0.01, 1.0),
    "gpt2_small": Workload("gpt2_small", 124_000_000, 32, "f32", 1e-4, 1e2,
                           12, 5e-4, 5e-3, 0.01, 1.0),
    "stress_1b_bf16": Workload("stress_1b_bf16", 1_000_000_000, 32, "bf16",
                               1e-4, 1e2, 24, 1e-3, 1e-2, 0.02, 1.0),
}


def torch_dtype(storage: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[storage]


def _block_scales(wl: Workload) -> torch.Tensor:
    g = torch.Generator(device="cpu")
    g.manual_seed(wl.seed * 1_000_003 + 17)
    u = torch.rand(max(wl.blocks, 1), generator=g, dtype=torch.float64)
    lo, hi = math.log(wl.a_lo), math.log(wl.a_hi)
    return torch.exp(lo + (hi - lo) * u).to(torch.float32)


def make_worker_states(wl: Workload, device="cpu", chunk_rows: int = CHUNK_ROWS):
    """Returns (thetas, grads): two (m, n) tensors of wl's storage dtype on
    `device`; worker k's vector is the contiguous row [k]."""
    device = torch.device(device)
    dt = torch_dtype(wl.storage)
    thetas = torch.empty((wl.m, wl.n), dtype=dt, device=device)
    grads = torch.empty((wl.m, wl.n), dtype=dt, device=device)
    scales = _block_scales(wl).to(device)
    bs = max(wl.n // wl.blocks, 1) if wl.blocks else 0
    lo, hi = math.log(wl.a_lo), math.log(wl.a_hi)

    for ci, r0 in enumerate(range(0, wl.n, chunk_rows)):
        rows = min(chunk_rows, wl.n - r0)
        g = torch.Generator(device=device)
        g.manual_seed(wl.seed * 1_000_003 + 1000 + ci)

        def rnd(*shape):
            return torch.rand(*shape, generator=g, device=device,
                              dtype=torch.float32)

        def nrm(*shape):
            return torch.randn(*shape, generator=g, device=device,
                               dtype=torch.float32)

        if wl.blocks:
            idx = torch.arange(r0, r0 + rows, device=device) // bs
            idx.clamp_(max=wl.blocks - 1)
            a = scales[idx] * (0.5 + 1.5 * rnd(rows))
        else:
            a = torch.exp(lo + (hi - lo) * rnd(rows))
        b = nrm(rows)
        theta0 = nrm(rows)
        for k in range(wl.m):
            # the worker's parameters are what it stores; its gradient is
            # evaluated there
            th = (theta0 + wl.spread * nrm(rows)).to(dt)
            gr = a * th.to(torch.float32) - b
            if wl.noise > 0.0:
                gr = gr + wl.noise * nrm(rows)
            thetas[k, r0:r0 + rows] = th
            grads[k, r0:r0 + rows] = gr.to(dt)
    return thetas, grads


def to_numpy_stored(t: torch.Tensor):
    """Host copy of the *stored* values for the oracle: fp32 stays fp32, bf16
    is handed over as its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
