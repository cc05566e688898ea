"""PowerSGD against PowerSGD+ on a distributed least-squares problem, driven through the library
(Section 3, Claim 1 and Figure 1: PowerSGD can fail to converge where PowerSGD+ does; Algorithm 2; Eq. (7c)).

    f_i(X) = 1/(2 rows) ||A_i X - B_i||_F^2,  f = mean_i f_i,  X in R^{256 x 128}, N = 16 workers.

The paper does not give the set-up of its figure.  This one lifts the stochastic gradient of the paper's 2 x 2 example
(Eq. (10b)) to the least-squares problem:  g^(i) = grad f + xi^(i) (sigma u v^T - grad f),  xi^(i) = +-1 with equal
probability and +1 on every worker at step 0, u the leading eigenvector of mean_i A_i^T A_i and v the right singular
vector of X_0 - X* with the smallest singular value.  The mean over the workers is an unbiased estimate of grad f.
The first step's gradient is then sigma u v^T on every worker, PowerSGD's projection Q starts along v, and what the
true gradient has outside that direction is only ever seen through the error feedback.

Every step is the library's: psgd_compress (PowerSGD: every step; PowerSGD+: psgd_compress_refresh when t is a
multiple of tau) and psgd_decompress_msgd on the factors it left in the workspace.  torch computes the gradient
of the least-squares problem (the model's side of a training step) and holds the buffers.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np

from . import psgd, synth


def run(problem: synth.LeastSquares, tau: Optional[int], steps: int, record_every: int = 100) -> List[float]:
    """Gradient norms ||grad f(X_t)||_F at t = 0, record_every, ..., and after the last step.  tau = None: PowerSGD."""
    import torch
    dev = "cuda"
    n = len(problem.a)
    rows = problem.a[0].shape[0]
    a = [torch.from_numpy(x).to(dev) for x in problem.a]
    b = [torch.from_numpy(x).to(dev) for x in problem.b]
    h = sum(x.T @ x for x in a) / (n * rows)
    c = sum(x.T @ y for x, y in zip(a, b)) / (n * rows)
    lam, vec = torch.linalg.eigh(h.double())
    u = vec[:, -1:].float()
    x = torch.zeros_like(c)
    v = torch.linalg.svd((x - torch.from_numpy(problem.x_star).to(dev)).double())[2][-1:].T.float()
    noise_term = (problem.sigma * (u @ v.T)).contiguous()
    eta = problem.eta_scale * (1.0 - problem.mu) / float(lam[-1])
    d, k = x.shape
    comp = psgd.Compressor([(d, k, problem.r, psgd.PSGD_F32)], n)
    gen = torch.Generator(device=dev)
    gen.manual_seed(4321)
    q = [torch.randn((k, problem.r), generator=gen, device=dev)]
    p = [torch.zeros((d, problem.r), device=dev)]
    e = [torch.zeros_like(x)]
    mom = [torch.zeros_like(x)]
    xs = [x]
    minus = torch.empty_like(x)
    hist = []
    for t in range(steps):
        grad = h @ xs[0] - c
        if t % record_every == 0:
            hist.append(float(torch.linalg.norm(grad)))
        # xi = +1: sigma u v^T;  xi = -1: 2 grad f - sigma u v^T
        torch.sub(2.0 * grad, noise_term, out=minus)
        g = [[noise_term if problem.xi[t, i] > 0 else minus for i in range(n)]]
        if tau is not None and t % tau == 0:
            comp.compress_refresh(g, e, q, p)
        else:
            comp.compress(g, e, q, p)
        comp.decompress_msgd(None, None, mom, xs, problem.mu, eta)
    hist.append(float(torch.linalg.norm(h @ xs[0] - c)))
    torch.cuda.synchronize()
    return hist
