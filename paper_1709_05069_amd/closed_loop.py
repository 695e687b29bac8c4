"""Closed-loop demonstration on a synthetic quadratic: m simulated workers and
a server that either averages (distributed SGD) or takes the quasi-Newton step
of Section 2 through the HIP library.

It stands in for the paper's Section 3 experiment (DistNewton-m against SGD on
MNIST / CIFAR-10), whose datasets and network are not available here.  Loss:
J(theta) = 0.5 theta^T diag(a) theta - b^T theta, with a few stiff coordinates
(a_i in 10..20) among many flat ones (a_i in 1e-3..5e-2).  Plain averaging is
stable only for tau < 2/a_max ~ 0.1 and then crawls along the flat coordinates;
the quasi-Newton server inverts the curvature on the few directions its secant
pairs resolve and can take tau = 1 on the rest.  With fewer workers than stiff
directions (m - 1 < stiff) it diverges, as the paper reports for too few
workers.  One synchronous iteration, as in the paper's
Section 1: every worker reads theta, takes one local stochastic-gradient step,
and writes its updated parameters together with the gradient evaluated there;
the server combines the m pairs.

The workers are simulated with torch ops (they are the training loop around
the server, not part of it); the server step is qn_update.

  python -m paper_1709_05069_amd.closed_loop [--n 100000] [--iters 40] [--stiff 4]
"""
import argparse
import math

import torch

from . import qn


def make_problem(n, stiff, device, seed=0):
    """Diagonal quadratic with `stiff` coordinates of curvature 10..20 and the
    rest log-uniform in [1e-3, 5e-2]; minimiser theta* ~ N(0, 1), start
    theta* + N(0, 1).  Returns (a, b, theta0, theta_star)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    lo, hi = math.log(1e-3), math.log(5e-2)
    a = torch.exp(lo + (hi - lo) * torch.rand(n, generator=g, dtype=torch.float64))
    idx = torch.randperm(n, generator=g)[:stiff]
    a[idx] = 10.0 + 10.0 * torch.rand(stiff, generator=g, dtype=torch.float64)
    star = torch.randn(n, generator=g, dtype=torch.float64)
    theta0 = star + torch.randn(n, generator=g, dtype=torch.float64)
    f32 = lambda t: t.to(torch.float32).to(device)
    return f32(a), f32(a * star), f32(theta0), f32(star)


def excess_loss(a, theta, star):
    """J(theta) - J(theta*) = 0.5 (theta - theta*)^T diag(a) (theta - theta*)."""
    d = theta.double() - star.double()
    return float((0.5 * a.double() * d * d).sum().item())


def worker_round(a, b, theta, m, eta, step_noise, grad_noise, gen):
    """Each of the m workers: one local stochastic-gradient step from theta
    (minibatch noise of std step_noise), then the gradient at its new parameters
    (residual noise grad_noise).  Returns (thetas, grads), (m, n)."""
    n = theta.numel()
    g0 = a * theta - b
    thetas = theta[None, :] - eta * (g0[None, :] + step_noise * torch.randn(
        (m, n), generator=gen, device=theta.device, dtype=torch.float32))
    grads = a[None, :] * thetas - b[None, :] + grad_noise * torch.randn(
        (m, n), generator=gen, device=theta.device, dtype=torch.float32)
    return thetas.contiguous(), grads.contiguous()


def run(n=100_000, m=16, iters=40, server="qn", tau=1.0, lam=0.1, eta=2e-3,
        step_noise=0.5, grad_noise=1e-5, stiff=4, device="cuda:0", seed=0,
        on_step=None):
    """Returns the excess losses J(theta_t) - J(theta*) for t = 0..iters and
    the list of selected j (empty for the SGD server)."""
    a, b, theta, star = make_problem(n, stiff, device, seed)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed + 1)
    hist = [excess_loss(a, theta, star)]
    js = []
    for it in range(iters):
        thetas, grads = worker_round(a, b, theta, m, eta, step_noise, grad_noise, gen)
        if server == "qn":
            theta, j = qn.qn_update(thetas, grads, tau, lam)
            js.append(int(j.item()))
            if on_step is not None:
                on_step(it, thetas, grads, theta, js[-1])
        elif server in ("qn_sigma1", "qn_secant"):
            # the same step with tau capped at 1 / sigma_max (Section 3, closing discussion)
            mode = qn.BOUND_SIGMA1 if server == "qn_sigma1" else qn.BOUND_SECANT
            theta, j, _ = qn.qn_update_bounded(thetas, grads, tau, lam, mode)
            js.append(int(j.item()))
        elif server == "sgd":
            theta = thetas.mean(0) - tau * grads.mean(0)
        else:
            raise ValueError(server)
        hist.append(excess_loss(a, theta, star))
        if not math.isfinite(hist[-1]):
            break
    return hist, js


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=100_000)
    ap.add_argument("--iters", type=int, default=40)
    ap.add_argument("--stiff", type=int, default=4)
    args = ap.parse_args()
    kw = dict(n=args.n, iters=args.iters, stiff=args.stiff)
    cols = {}
    for m in (4, 8, 16):
        cols[f"DistNewton-{m} tau=1"], js = run(server="qn", m=m, tau=1.0, **kw)
        print(f"DistNewton-{m}: selected j per iteration: {js}")
    # plain averaging with tau = 1 diverges on the stiff coordinates, so SGD is
    # also run at about the largest stable step, just under 2 / a_max
    cols["SGD tau=1"], _ = run(server="sgd", m=16, tau=1.0, **kw)
    cols["SGD tau=0.095"], _ = run(server="sgd", m=16, tau=0.095, **kw)
    names = list(cols)
    print(f"{'iter':>5} " + " ".join(f"{c:>21}" for c in names))
    for t in range(0, args.iters + 1, max(args.iters // 10, 1)):
        row = [cols[c][t] if t < len(cols[c]) else float("nan") for c in names]
        print(f"{t:5d} " + " ".join(f"{v:21.4e}" for v in row))


if __name__ == "__main__":
    main()
