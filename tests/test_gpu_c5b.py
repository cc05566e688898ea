"""Config 5b: PowerSGD against PowerSGD+ on the least-squares problem, every compressor and optimizer step through
the library (Section 3, Claim 1 / Figure 1; Algorithm 2; Eq. (7c)).  The figure's set-up is not in the paper, so the
curves cannot be pinned: this is a demonstration, and what is asserted is the direction of the gap, and that the first
stretch of both runs agrees with the oracle run on the same problem and the same random signs."""
import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2509_11254_amd import demo_least_squares, synth

pytestmark = pytest.mark.gpu


def _oracle_run(problem, tau, steps, record_every):
    n = len(problem.a)
    a = [x.astype(np.float64) for x in problem.a]
    b = [x.astype(np.float64) for x in problem.b]
    rows = a[0].shape[0]
    h = sum(x.T @ x for x in a) / (n * rows)
    c = sum(x.T @ y for x, y in zip(a, b)) / (n * rows)
    lam, vec = np.linalg.eigh(h)
    u = vec[:, -1:]
    x = np.zeros_like(c)
    v = np.linalg.svd(x - problem.x_star.astype(np.float64))[2][-1:].T
    noise_term = problem.sigma * (u @ v.T)
    eta = problem.eta_scale * (1.0 - problem.mu) / lam[-1]
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4321)
    q = torch.randn((c.shape[1], problem.r), generator=gen, device="cuda").cpu().numpy().astype(np.float64)
    e = [np.zeros_like(c) for _ in range(n)]
    mom = np.zeros_like(c)
    hist = []
    for t in range(steps):
        grad = h @ x - c
        if t % record_every == 0:
            hist.append(float(np.linalg.norm(grad)))
        g = [grad + xi * (noise_term - grad) for xi in problem.xi[t]]
        out = orc.compress_step(t, tau, problem.r, q, g, e)
        q, e = out.comp.q, out.e_next
        x, mom = orc.msgd_update(x, mom, out.comp.delta_hat, eta, problem.mu)
    hist.append(float(np.linalg.norm(h @ x - c)))
    return hist


def test_least_squares_powersgd_plus_converges_where_powersgd_does_not():
    problem = synth.least_squares_problem(steps=2000)
    plain = demo_least_squares.run(problem, None, 2000, record_every=200)
    plus = demo_least_squares.run(problem, problem.tau, 2000, record_every=200)
    print("PowerSGD ", ["%.3g" % v for v in plain])
    print("PowerSGD+", ["%.3g" % v for v in plus])
    assert np.all(np.isfinite(plain)) and np.all(np.isfinite(plus))
    # PowerSGD+ has come down by orders of magnitude (to the floor its gradient noise sets); PowerSGD has not moved
    # towards the solution at all
    assert plus[-1] <= 0.05 * plus[0], plus
    assert plain[-1] >= 0.5 * plain[0], plain
    assert plain[-1] >= 20.0 * plus[-1], (plain[-1], plus[-1])


@pytest.mark.parametrize("tau", [None, 10])
def test_least_squares_first_stretch_against_the_oracle(tau):
    """Same problem, same signs, same Q_{-1}: over the first steps (before rounding differences have had time to
    grow along the unstable directions) the gradient norms agree closely, later within the run's own scatter."""
    problem = synth.least_squares_problem(steps=300)
    gpu = demo_least_squares.run(problem, tau, 300, record_every=10)
    ref = _oracle_run(problem, tau, 300, 10)
    print("tau", tau, "gpu", ["%.4g" % v for v in gpu[:6]], "...", "%.4g" % gpu[-1])
    print("tau", tau, "ref", ["%.4g" % v for v in ref[:6]], "...", "%.4g" % ref[-1])
    # (PowerSGD+: the matrix of the refresh at t = 0 has rank one -- every worker's gradient is sigma u v^T there --, so
    # three of its four leading singular vectors are arbitrary and the two sides' runs differ by what they picked)
    tol = 1e-3 if tau is None else 5e-2
    for k in range(4):                                   # t = 0, 10, 20, 30
        assert abs(gpu[k] - ref[k]) <= tol * ref[k], (k, gpu[k], ref[k])
    assert 0.2 * ref[-1] <= gpu[-1] <= 5.0 * ref[-1], (gpu[-1], ref[-1])
