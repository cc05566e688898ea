"""Pins for the CPU oracle: values the paper prints, closed forms, invariants, brute force.

None of these tests re-types the oracle's own formula with the same routines: brute-force
checks use explicit scalar loops, closed forms come from the paper's Appendix A and Lemmas 1-2,
and library cross-checks call LAPACK's QR (the oracle's QR is hand-written Gram-Schmidt).
"""
import itertools
import math

import numpy as np
import pytest

from conftest import read_golden
from oracle import psgd_oracle as orc
from paper_2509_11254_amd import synth


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- QR (Section 2, QR decomposition)
def test_qr_hand_example_gram_schmidt():
    gold = read_golden("gram_schmidt_3x2.txt")
    a = np.array(gold["a"]).reshape(3, 2)
    q = orc.qr_thin(a)
    np.testing.assert_allclose(q, np.array(gold["q"]).reshape(3, 2), atol=1e-15)
    r = q.T @ a
    np.testing.assert_allclose(r, np.array(gold["r"]).reshape(2, 2), atol=1e-15)


@pytest.mark.parametrize("rows,r,seed", [(7, 3, 0), (64, 8, 1), (300, 33, 2), (5, 5, 3)])
def test_qr_matches_lapack_up_to_sign_and_contract(rows, r, seed):
    a = rng(seed).standard_normal((rows, r))
    q = orc.qr_thin(a)
    np.testing.assert_allclose(q.T @ q, np.eye(r), atol=1e-13)          # Q^T Q = I_r
    rmat = q.T @ a
    assert np.all(np.diag(rmat) > 0)                                    # positive diagonal
    np.testing.assert_allclose(np.tril(rmat, -1), 0, atol=1e-12)        # upper triangular
    np.testing.assert_allclose(q @ rmat, a, atol=1e-12)                 # A = Q R
    ql, rl = np.linalg.qr(a)
    ql = ql * np.sign(np.diag(rl))[None, :]
    np.testing.assert_allclose(q, ql, atol=1e-12)


def test_qr_ill_conditioned_columns_stay_orthonormal():
    g = rng(5)
    u = synth.haar_orthonormal(200, 6, 11)
    a = (u * (10.0 ** (-0.7 * np.arange(6)))[None, :]) @ g.standard_normal((6, 6))    # cond ~ 3e3
    q = orc.qr_thin(a)
    np.testing.assert_allclose(q.T @ q, np.eye(6), atol=1e-12)


def test_qr_invariant_under_right_upper_triangular_factor():
    """QR(A T) = QR(A) for upper-triangular T with positive diagonal."""
    g = rng(7)
    a = g.standard_normal((40, 5))
    t = np.triu(g.standard_normal((5, 5)))
    t[np.diag_indices(5)] = np.abs(np.diag(t)) + 0.5
    np.testing.assert_allclose(orc.qr_thin(a @ t), orc.qr_thin(a), atol=1e-12)


def test_qr_rank_deficient_column_is_zeroed():
    g = rng(9)
    a = g.standard_normal((30, 3))
    a[:, 1] = 2.0 * a[:, 0]
    q = orc.qr_thin(a)
    assert np.all(q[:, 1] == 0)
    np.testing.assert_allclose(np.linalg.norm(q[:, [0, 2]], axis=0), 1.0, atol=1e-13)
    assert abs(q[:, 0] @ q[:, 2]) < 1e-13
    z = orc.qr_thin(np.zeros((4, 2)))
    assert np.all(z == 0)


# ---------------------------------------------------------------- SSP-Comp by brute force
def _brute_ssp(q_prev, deltas):
    """Algorithm 1, SSP-Comp with scalar loops only (tiny sizes)."""
    n_w = len(deltas)
    m, n = len(deltas[0]), len(deltas[0][0])
    r = len(q_prev[0])
    p = [[0.0] * r for _ in range(m)]
    for w in range(n_w):
        for i in range(m):
            for c in range(r):
                s = 0.0
                for k in range(n):
                    s += deltas[w][i][k] * q_prev[k][c]
                p[i][c] += s / n_w
    # Gram-Schmidt column by column (second sweep for safety)
    pt = [[p[i][c] for c in range(r)] for i in range(m)]
    for c in range(r):
        for _ in range(2):
            for j in range(c):
                dot = sum(pt[i][j] * pt[i][c] for i in range(m))
                for i in range(m):
                    pt[i][c] -= dot * pt[i][j]
        nrm = math.sqrt(sum(pt[i][c] ** 2 for i in range(m)))
        for i in range(m):
            pt[i][c] /= nrm
    q = [[0.0] * r for _ in range(n)]
    for w in range(n_w):
        for k in range(n):
            for c in range(r):
                s = 0.0
                for i in range(m):
                    s += deltas[w][i][k] * pt[i][c]
                q[k][c] += s / n_w
    e = []
    for w in range(n_w):
        ew = [[0.0] * n for _ in range(m)]
        for i in range(m):
            for k in range(n):
                rec = 0.0
                for c in range(r):
                    qi = sum(deltas[w][ii][k] * pt[ii][c] for ii in range(m))
                    rec += pt[i][c] * qi
                ew[i][k] = deltas[w][i][k] - rec
        e.append(ew)
    return np.array(pt), np.array(q), [np.array(x) for x in e]


@pytest.mark.parametrize("m,n,r,n_w,seed", [(4, 3, 1, 1, 0), (6, 4, 2, 3, 1), (8, 8, 3, 2, 2), (5, 2, 2, 4, 3)])
def test_ssp_step_matches_brute_force(m, n, r, n_w, seed):
    g = rng(seed)
    grads = [g.standard_normal((m, n)) for _ in range(n_w)]
    errs = [0.3 * g.standard_normal((m, n)) for _ in range(n_w)]
    q_prev = g.standard_normal((n, r))
    out = orc.compress_step(1, None, r, q_prev, grads, errs)
    deltas = [(grads[w] + errs[w]).tolist() for w in range(n_w)]
    pt, q, e = _brute_ssp(q_prev.tolist(), deltas)
    np.testing.assert_allclose(out.comp.p_tilde, pt, atol=1e-12)
    np.testing.assert_allclose(out.comp.q, q, atol=1e-12)
    for w in range(n_w):
        np.testing.assert_allclose(out.e_next[w], e[w], atol=1e-12)


# ---------------------------------------------------------------- Appendix A worked example (t = 0)
def test_worked_example_first_step_values():
    gold = read_golden("appendix_a_worked_example.txt")
    sigma = gold["sigma"][0]
    q_init = np.array(gold["q_init"]).reshape(2, 1)
    for n_w in (1, 2, 5):
        x0 = np.array([[0.3, -0.4], [0.1, 0.9]])
        grads = [orc.counter_stochastic_grad(x0, +1.0, sigma) for _ in range(n_w)]
        np.testing.assert_allclose(grads[0].ravel(), gold["delta0"], atol=1e-15)
        errs = [np.zeros((2, 2)) for _ in range(n_w)]
        out = orc.compress_step(0, None, 1, q_init, grads, errs)
        np.testing.assert_allclose((out.delta_mean @ q_init).ravel(), gold["p0"], atol=1e-14)
        np.testing.assert_allclose(out.comp.p_tilde.ravel(), gold["p_tilde0"], atol=1e-14)
        np.testing.assert_allclose(out.comp.q.ravel(), gold["q0"], atol=1e-13)
        np.testing.assert_allclose(out.comp.delta_hat.ravel(), gold["delta_hat0"], atol=1e-13)
        for w in range(n_w):
            np.testing.assert_allclose(out.e_next[w].ravel(), gold["e1"], atol=1e-13)
        _x1, m0 = orc.msgd_update(x0, np.zeros((2, 2)), out.comp.delta_hat, 0.1, 0.9)
        np.testing.assert_allclose(m0.ravel(), gold["m0"], atol=1e-13)


def test_counterexample_constants_and_identities():
    gold = read_golden("appendix_a_worked_example.txt")
    a, b, c = orc.A_MAT, orc.B_MAT, orc.C_VEC
    np.testing.assert_array_equal(a.ravel(), gold["A"])
    np.testing.assert_array_equal(b.ravel(), gold["B"])
    np.testing.assert_allclose(c.ravel(), gold["C"], atol=1e-16)
    np.testing.assert_allclose(c @ c.T @ b, b, atol=1e-15)
    np.testing.assert_allclose(c @ c.T @ a, 0, atol=1e-15)
    np.testing.assert_allclose(b @ c, 2 * c, atol=1e-15)
    np.testing.assert_allclose(b.T @ c, 2 * c, atol=1e-15)
    np.testing.assert_allclose(a @ c, 0, atol=1e-15)
    np.testing.assert_allclose(a.T @ c, 0, atol=1e-15)


def test_psi_and_gradient_against_finite_differences():
    # psi is x^2 inside [-1, 1] and 2|x| - 1 outside; both branches give 1 (slope 2) at |x| = 1.
    assert orc.psi(0.5) == 0.25 and orc.psi(-3.0) == 5.0 and orc.psi(1.0) == 1.0
    assert orc.dpsi(0.25) == 0.5 and orc.dpsi(-7.0) == -2.0 and orc.dpsi(1.0) == 2.0
    g = rng(3)
    for _ in range(20):
        x = g.standard_normal((2, 2)) * 1.5
        an = orc.counter_grad(x)
        fd = np.zeros((2, 2))
        h = 1e-6
        for i, j in itertools.product(range(2), range(2)):
            xp, xm = x.copy(), x.copy()
            xp[i, j] += h
            xm[i, j] -= h
            fd[i, j] = (orc.counter_f(xp) - orc.counter_f(xm)) / (2 * h)
        np.testing.assert_allclose(an, fd, atol=1e-5)
        # unbiased stochastic gradient: mean over xi = +-1 is grad f
        mean = 0.5 * (orc.counter_stochastic_grad(x, 1.0, 2.5) + orc.counter_stochastic_grad(x, -1.0, 2.5))
        np.testing.assert_allclose(mean, an, atol=1e-14)


# ---------------------------------------------------------------- invariants of one compress step
def _random_step(m, n, r, n_w, seed, t=1, tau=None):
    g = rng(seed)
    grads = [g.standard_normal((m, n)) for _ in range(n_w)]
    errs = [0.5 * g.standard_normal((m, n)) for _ in range(n_w)]
    q_prev = g.standard_normal((n, r))
    return orc.compress_step(t, tau, r, q_prev, grads, errs), grads, errs, q_prev


@pytest.mark.parametrize("t,tau", [(1, None), (3, 5), (0, 5), (10, 5)])
def test_step_invariants(t, tau):
    m, n, r, n_w = 40, 24, 5, 3
    out, grads, errs, _ = _random_step(m, n, r, n_w, 17, t, tau)
    assert out.refreshed == (tau is not None and t % tau == 0)
    pt, q = out.comp.p_tilde, out.comp.q
    dbar = out.delta_mean
    np.testing.assert_allclose(dbar, sum(grads) / n_w + sum(errs) / n_w, atol=1e-13)
    np.testing.assert_allclose(pt.T @ pt, np.eye(r), atol=1e-13)                      # semi-orthogonal
    np.testing.assert_allclose(out.comp.delta_hat, pt @ pt.T @ dbar, atol=1e-12)      # Eq. (9)
    e_bar = out.e_mean
    np.testing.assert_allclose(e_bar, dbar - out.comp.delta_hat, atol=1e-12)          # linearity (App. B)
    np.testing.assert_allclose(pt.T @ e_bar, 0, atol=1e-12)
    lhs = np.sum(e_bar ** 2) + np.sum(out.comp.delta_hat ** 2)                        # Eq. (4)
    assert abs(lhs - np.sum(dbar ** 2)) < 1e-10 * np.sum(dbar ** 2)
    for w in range(n_w):                                                              # per-worker form
        np.testing.assert_allclose(out.comp.delta_hat_i[w], pt @ pt.T @ out.deltas[w], atol=1e-12)
        np.testing.assert_allclose(out.e_next[w], out.deltas[w] - out.comp.delta_hat_i[w], atol=1e-13)


def test_ssp_exact_rank_r_matrix_is_recovered():
    m, n, r = 50, 30, 4
    g = rng(23)
    mat = g.standard_normal((m, r)) @ g.standard_normal((r, n))
    out = orc.compress_step(1, None, r, g.standard_normal((n, r)), [mat], [np.zeros((m, n))])
    assert np.linalg.norm(out.e_next[0]) < 1e-12 * np.linalg.norm(mat)
    np.testing.assert_allclose(out.comp.delta_hat, mat, atol=1e-12)


def test_transposed_operand_would_be_caught():
    """P uses Delta Q and Q uses Delta^T P~: shapes m x r and n x r with m != n."""
    out, _, _, _ = _random_step(12, 7, 2, 2, 5)
    assert out.comp.p_tilde.shape == (12, 2) and out.comp.q.shape == (7, 2)
    np.testing.assert_allclose(out.comp.q, out.delta_mean.T @ out.comp.p_tilde, atol=1e-13)


# ---------------------------------------------------------------- SVD-Comp (Definition 3, Lemma 2)
def test_svd_comp_prescribed_svd():
    m, n, r = 60, 40, 6
    sigma = 2.0 ** -np.arange(12)
    mat, u, v = synth.prescribed_svd_matrix(m, n, sigma, seed=3)
    mat = mat.astype(np.float64)
    out = orc.svd_comp([mat], r)
    assert orc.sin_theta_max(u[:, :r], out.p_tilde) < 1e-6        # fp32-rounded input: not exact
    np.testing.assert_allclose(out.sigma[:12], sigma, rtol=1e-5)
    # Q = V_r Sigma_r up to the sign of each column
    signs = np.sign(np.sum(out.p_tilde * u[:, :r], axis=0))
    np.testing.assert_allclose(out.q * signs[None, :], v[:, :r] * sigma[None, :r], atol=1e-6)


def test_svd_comp_eckart_young_equality_and_bound():
    m, n, r, n_w = 48, 32, 5, 3
    g = rng(31)
    deltas = [g.standard_normal((m, n)) for _ in range(n_w)]
    out = orc.svd_comp(deltas, r)
    dbar = sum(deltas) / n_w
    err = np.sum((dbar - out.delta_hat) ** 2)
    # independent route to the singular values: eigenvalues of the n x n Gram matrix
    lam = np.sort(np.linalg.eigvalsh(dbar.T @ dbar))[::-1]
    assert abs(err - np.sum(lam[r:])) < 1e-10 * np.sum(lam)
    assert err <= (1 - r / n) * np.sum(dbar ** 2) + 1e-12                              # Eq. (6)
    # no other r-dimensional projector does better (spot check with random ones and with SSP)
    for s in range(5):
        p = synth.haar_orthonormal(m, r, 77, s)
        assert np.sum((dbar - p @ p.T @ dbar) ** 2) >= err - 1e-12
    ssp = orc.ssp_comp(g.standard_normal((n, r)), deltas)
    assert np.sum((dbar - ssp.delta_hat) ** 2) >= err - 1e-12


def test_svd_comp_2x2_closed_form():
    """alpha A + beta B has singular values 2|alpha|, 2|beta| with left vectors (1,-1)/sqrt2, (1,1)/sqrt2."""
    for alpha, beta in [(0.7, 0.2), (-0.1, 0.9), (2.0, -0.5)]:
        mat = alpha * orc.A_MAT + beta * orc.B_MAT
        out = orc.svd_comp([mat], 1)
        np.testing.assert_allclose(out.sigma, sorted([2 * abs(alpha), 2 * abs(beta)], reverse=True), atol=1e-14)
        lead = np.array([1.0, -1.0]) / np.sqrt(2) if abs(alpha) > abs(beta) else np.array([1.0, 1.0]) / np.sqrt(2)
        assert abs(abs(out.p_tilde[:, 0] @ lead) - 1) < 1e-14


def test_svd_comp_exact_rank_r_gives_zero_error():
    m, n, r = 33, 21, 3
    g = rng(41)
    mat = g.standard_normal((m, r)) @ g.standard_normal((r, n))
    out = orc.compress_step(0, 4, r, np.zeros((n, r)), [mat], [np.zeros((m, n))])
    assert out.refreshed
    assert np.linalg.norm(out.e_next[0]) < 1e-12 * np.linalg.norm(mat)


def test_refresh_step_ignores_previous_q_and_replaces_ssp():
    m, n, r = 20, 12, 2
    g = rng(43)
    grads = [g.standard_normal((m, n)) for _ in range(2)]
    errs = [g.standard_normal((m, n)) for _ in range(2)]
    o1 = orc.compress_step(10, 5, r, g.standard_normal((n, r)), grads, errs)
    o2 = orc.compress_step(10, 5, r, g.standard_normal((n, r)), grads, errs)
    np.testing.assert_array_equal(o1.comp.delta_hat, o2.comp.delta_hat)
    o3 = orc.compress_step(11, 5, r, g.standard_normal((n, r)), grads, errs)
    assert not o3.refreshed


# ---------------------------------------------------------------- Eq. (8): K-step power iteration
def test_power_iteration_converges_at_predicted_rate():
    m, n, r = 80, 50, 3
    sigma = np.array([1.0, 0.9, 0.8, 0.4, 0.2, 0.1, 0.05])
    mat, u, _ = synth.prescribed_svd_matrix(m, n, sigma, seed=9)
    mat = mat.astype(np.float64)
    q0 = rng(1).standard_normal((n, r))
    angles = []
    for k in (1, 2, 4, 8, 16):
        pt, q = orc.power_iteration(mat, q0, k)
        angles.append(orc.sin_theta_max(u[:, :r], pt))
        np.testing.assert_allclose(q, mat.T @ pt, atol=1e-13)
    assert all(a2 < a1 for a1, a2 in zip(angles, angles[1:]))
    # one more iteration multiplies tan(theta) by (sigma_{r+1}/sigma_r)^2 = 0.25 asymptotically
    p8, _ = orc.power_iteration(mat, q0, 8)
    p9, _ = orc.power_iteration(mat, q0, 9)
    ratio = orc.sin_theta_max(u[:, :r], p9) / orc.sin_theta_max(u[:, :r], p8)
    assert 0.2 < ratio < 0.3
    assert angles[-1] < 1e-6


# ---------------------------------------------------------------- Theorem 1 / Claim 1 and PowerSGD+
# In exact arithmetic the invariants of Claim 1 hold for every t.  In floating point a one-ulp
# asymmetry between the two components of P_t is multiplied by about (x_t / beta_t)^2 per step
# (x_t = mean coefficient of A in Delta_t, which grows by about psi' per step because it is
# never transmitted; beta_t = sigma * mean(xi_t)), so the lock-in is only observable while
# x_t < |beta_t| plus the few steps rounding noise needs to grow to O(1).  The tests therefore
# use a large sigma and a horizon inside that window.
def _span_coeff(mat, basis):
    return float(np.sum(mat * basis) / np.sum(basis * basis))


def _signs(shape, seed):
    return np.where(rng(seed).random(shape) < 0.5, -1.0, 1.0)


# odd N: the mean of the xi never vanishes, so P_t is never the zero matrix (a case Claim 1 skips)
@pytest.mark.parametrize("mu,n_w", [(0.0, 3), (0.9, 5)])
def test_powersgd_locks_in_when_first_noise_is_all_plus_one(mu, n_w):
    steps, sigma = 16, 400.0          # x_t <= 4 t = 64 < sigma / n_w = 80
    xi = _signs((steps, n_w), 5)
    xi[0, :] = 1.0
    x0 = np.array([[0.9, -0.3], [0.2, 0.4]])        # a - b - c + d = 1.4 -> psi' = 2
    tr = orc.run_counterexample(x0, np.array([[0.3], [1.1]]), xi, sigma, eta=0.05, mu=mu, tau=None)
    d0 = x0[0, 0] - x0[0, 1] - x0[1, 0] + x0[1, 1]
    tol = 1e-9
    for t in range(steps):
        x = tr.x[t]
        assert abs((x[0, 0] - x[0, 1] - x[1, 0] + x[1, 1]) - d0) < tol            # gradient never changes
        assert abs(tr.grad_norm_sq[t] - 4 * orc.dpsi(d0) ** 2) < tol
        np.testing.assert_allclose(np.abs(tr.p_tilde[t]), orc.C_VEC, atol=tol)     # P~_t = C
        qv = tr.q[t]
        assert abs(qv[0, 0] - qv[1, 0]) < tol * np.linalg.norm(qv)                # Q_t in span(C)
        mm = tr.mom[t]
        np.testing.assert_allclose(mm, _span_coeff(mm, orc.B_MAT) * orc.B_MAT, atol=tol * sigma)
        for e in tr.e_next[t]:
            np.testing.assert_allclose(e, _span_coeff(e, orc.A_MAT) * orc.A_MAT, atol=tol * sigma)
        dx = tr.x[t + 1] - x0
        np.testing.assert_allclose(dx, _span_coeff(dx, orc.B_MAT) * orc.B_MAT, atol=tol * sigma)
    # the residual that is never transmitted keeps growing along A (this is what breaks convergence)
    assert abs(_span_coeff(tr.e_next[-1][0], orc.A_MAT)) > abs(_span_coeff(tr.e_next[2][0], orc.A_MAT))


def test_powersgd_lower_bound_monte_carlo():
    """E ||grad f(X_t)||^2 >= psi'(a-b-c+d)^2 / 2^(N-2) (Theorem 1), checked at a fixed t over seeds."""
    n_w, steps, sigma = 3, 12, 400.0
    x0 = np.array([[0.9, -0.3], [0.2, 0.4]])
    d0 = 1.4
    eps0 = orc.dpsi(d0) ** 2 / 2 ** (n_w - 2)
    finals, stuck = [], 0
    n_seeds = 64
    for seed in range(n_seeds):
        xi = _signs((steps, n_w), 100 + seed)
        q0 = rng(200 + seed).standard_normal((2, 1))
        v = orc.run_counterexample(x0, q0, xi, sigma, 0.02, 0.5, None).grad_norm_sq[-1]
        finals.append(v)
        if np.all(xi[0] == 1.0):
            stuck += 1
            assert abs(v - 4 * orc.dpsi(d0) ** 2) < 1e-8      # an all-plus start never moves the gradient
    assert stuck >= 3                                          # expected n_seeds / 2^N = 8
    assert np.mean(finals) >= eps0                             # the bound itself (probability-weighted)


def test_powersgd_plus_converges_on_the_counterexample():
    """With a periodic SVD refresh the gradient is driven to a small noise ball on every seed,
    including the seeds whose first noise draw is all plus (the start that locks PowerSGD in)."""
    n_w, steps, sigma = 3, 400, 1.0
    x0 = np.array([[0.9, -0.3], [0.2, 0.4]])
    g0 = 4 * orc.dpsi(1.4) ** 2
    worst = 0.0
    for seed in range(24):
        xi = _signs((steps, n_w), 300 + seed)
        if seed % 3 == 0:
            xi[0, :] = 1.0
        q0 = rng(400 + seed).standard_normal((2, 1))
        tr = orc.run_counterexample(x0, q0, xi, sigma, 0.02, 0.5, 5)
        worst = max(worst, float(np.mean(tr.grad_norm_sq[-50:])))
    assert worst < 0.05 * g0


# ---------------------------------------------------------------- aggregated vs per-worker error feedback
def test_mean_error_trajectory_equals_single_aggregated_buffer():
    wl = synth.config1(seed=7)
    spec = wl.layers[0]
    sig = synth.signal_matrix(spec, wl, 0)
    n_w, r = wl.n_workers, wl.r
    e_w = [np.zeros((spec.rows, spec.cols)) for _ in range(n_w)]
    e_agg = [np.zeros((spec.rows, spec.cols))]
    q_w = q_a = synth.initial_q(spec.n, r, wl.seed).astype(np.float64)
    for t in range(7):
        grads = [synth.gradient_as_f64(synth.worker_gradient(spec, wl, 0, w, t, sig)) for w in range(n_w)]
        ow = orc.compress_step(t, wl.tau, r, q_w, grads, e_w)
        oa = orc.compress_step(t, wl.tau, r, q_a, [sum(grads) / n_w], e_agg)
        np.testing.assert_allclose(ow.e_mean, oa.e_next[0], atol=1e-12)
        np.testing.assert_allclose(ow.comp.delta_hat, oa.comp.delta_hat, atol=1e-12)
        e_w, e_agg, q_w, q_a = ow.e_next, oa.e_next, ow.comp.q, oa.comp.q


# ------------------------------------------------------------------ Adam / AdamW on the compressed update
def test_adam_first_step_and_constant_gradient_closed_form():
    """From zero moments the bias-corrected moments of step 1 are g and g^2, so the step is
    -eta g / (|g| + eps); with the same g at every step the bias corrections cancel the (1 - beta^t) factors
    exactly and every step is that same step."""
    rng = np.random.default_rng(3)
    g = rng.standard_normal((5, 3))
    x0 = rng.standard_normal((5, 3))
    eta, eps = 0.01, 1e-8
    x, m1, m2 = x0, np.zeros_like(g), np.zeros_like(g)
    for t in range(1, 8):
        x, m1, m2 = orc.adam_update(x, m1, m2, g, t, eta, 0.9, 0.999, eps)
        np.testing.assert_allclose(x, x0 - t * eta * g / (np.abs(g) + eps), rtol=0, atol=1e-14)
    np.testing.assert_allclose(m1, (1 - 0.9 ** 7) * g, atol=1e-15)
    np.testing.assert_allclose(m2, (1 - 0.999 ** 7) * g * g, atol=1e-15)


def test_adam_two_steps_by_hand():
    """g_1 = 1, g_2 = -1, beta = (0.9, 0.999), eps = 0: m = 0.1 then -0.01, v = 0.001 then 0.001999;
    at step 2 m^ = -0.01 / 0.19 and v^ = 0.001999 / (1 - 0.998001) = 1, so x_2 = x_1 + eta / 19."""
    x, m1, m2 = np.array([2.0]), np.zeros(1), np.zeros(1)
    x, m1, m2 = orc.adam_update(x, m1, m2, np.array([1.0]), 1, 0.5, 0.9, 0.999, 0.0)
    assert x[0] == pytest.approx(1.5, abs=1e-15) and m1[0] == pytest.approx(0.1) and m2[0] == pytest.approx(0.001)
    x, m1, m2 = orc.adam_update(x, m1, m2, np.array([-1.0]), 2, 0.5, 0.9, 0.999, 0.0)
    assert m1[0] == pytest.approx(-0.01, abs=1e-15) and m2[0] == pytest.approx(0.001999, abs=1e-15)
    assert x[0] == pytest.approx(1.5 + 0.5 / 19.0, abs=1e-13)


def test_adam_scale_invariance_and_decoupled_weight_decay():
    rng = np.random.default_rng(4)
    gs = [rng.standard_normal((4, 4)) for _ in range(5)]
    x0 = rng.standard_normal((4, 4))
    def run(scale, wd):
        x, m1, m2 = x0, np.zeros((4, 4)), np.zeros((4, 4))
        for t, g in enumerate(gs, 1):
            x, m1, m2 = orc.adam_update(x, m1, m2, scale * g, t, 0.02, 0.8, 0.95, 0.0, wd)
        return x
    # with eps = 0 the step does not see the scale of the gradients
    np.testing.assert_allclose(run(1.0, 0.0), run(37.5, 0.0), atol=1e-13)
    # zero gradient (eps > 0 so that 0 / (0 + eps) = 0): only the decay acts, x_t = (1 - eta lambda)^t x_0,
    # and it does not enter the moments
    x, m1, m2 = x0, np.zeros((4, 4)), np.zeros((4, 4))
    for t in range(1, 4):
        x, m1, m2 = orc.adam_update(x, m1, m2, np.zeros((4, 4)), t, 0.02, 0.9, 0.999, 1e-8, 0.1)
    np.testing.assert_allclose(x, (1 - 0.02 * 0.1) ** 3 * x0, atol=1e-15)
    assert not m1.any() and not m2.any()


# ---------------------------------------------------------------------------------------------------
# Eq. (7c) over two steps, by hand: m_t = mu m_{t-1} + Delta_hat_t, X_{t+1} = X_t - eta m_t.
# ---------------------------------------------------------------------------------------------------
def test_msgd_update_two_steps_by_hand():
    # scalar: Delta_hat = 1, then -1; mu = 0.5, eta = 0.1  ->  m = 1, -0.5;  x = x0 - 0.1, x0 - 0.1 + 0.05
    x0 = np.array([[2.0]])
    x1, m1 = orc.msgd_update(x0, np.zeros((1, 1)), np.array([[1.0]]), 0.1, 0.5)
    assert m1[0, 0] == 1.0 and abs(x1[0, 0] - 1.9) < 1e-15
    x2, m2 = orc.msgd_update(x1, m1, np.array([[-1.0]]), 0.1, 0.5)
    assert m2[0, 0] == -0.5 and abs(x2[0, 0] - 1.95) < 1e-15          # (stepping with Delta_hat instead of m_t gives 2.0)
    # a matrix, two steps, mu = 0.9, eta = 0.25: entries worked out one by one
    d1 = np.array([[1.0, -2.0], [0.5, 4.0]])
    d2 = np.array([[-3.0, 1.0], [2.0, 0.0]])
    xa = np.array([[1.0, 1.0], [1.0, 1.0]])
    xb, ma = orc.msgd_update(xa, np.zeros((2, 2)), d1, 0.25, 0.9)
    xc, mb = orc.msgd_update(xb, ma, d2, 0.25, 0.9)
    np.testing.assert_allclose(mb, [[0.9 - 3.0, -1.8 + 1.0], [0.45 + 2.0, 3.6]], atol=1e-15)
    np.testing.assert_allclose(xc, [[1 - 0.25 + 0.525, 1 + 0.5 + 0.2], [1 - 0.125 - 0.6125, 1 - 1.0 - 0.9]], atol=1e-15)


# ---------------------------------------------------------------------------------------------------
# svd_comp_large (the iteration used where a dense SVD is too slow) against svd_comp (the definition).
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("m,n,r,gap", [(300, 200, 20, True), (256, 128, 4, False), (160, 160, 33, True)])
def test_svd_comp_large_matches_the_definition(m, n, r, gap):
    rng = np.random.default_rng([m, n, r])
    u, _ = np.linalg.qr(rng.standard_normal((m, min(m, n))))
    v, _ = np.linalg.qr(rng.standard_normal((n, min(m, n))))
    k = min(m, n)
    s = np.concatenate([np.linspace(2.0, 1.0, r), (0.6 if gap else 0.97) * 0.95 ** np.arange(k - r)])
    mats = [(u * s) @ v.T + 1e-3 * rng.standard_normal((m, n)) for _ in range(3)]
    ref = orc.svd_comp(mats, r)
    out, resid = orc.svd_comp_large(mats, r, oversample=48, iters=400)
    assert resid <= 1e-10                                      # its own certificate
    np.testing.assert_allclose(out.sigma, ref.sigma[:r], rtol=1e-10)
    assert orc.sin_theta_max(ref.p_tilde, out.p_tilde) <= 1e-8
    np.testing.assert_allclose(out.delta_hat, ref.delta_hat, atol=1e-8)
    for a, b in zip(out.delta_hat_i, ref.delta_hat_i):
        np.testing.assert_allclose(a, b, atol=1e-8)


# ---------------------------------------------------------------------------------------------------
# range_finder_comp (reading of the "lighter contractive compressor" the paper allows in place of SVD-Comp).
# ---------------------------------------------------------------------------------------------------
def test_range_finder_two_by_two_by_hand():
    # M = diag(3, 1), Omega = (1, 1)^T, r = 1: Y = (3, 1), Z = (3, 1)/sqrt(10), Delta_hat = Z Z^T M
    out = orc.range_finder_comp([np.diag([3.0, 1.0])], 1, np.array([[1.0], [1.0]]))
    np.testing.assert_allclose(np.abs(out.p_tilde.ravel()), np.array([3.0, 1.0]) / np.sqrt(10.0), atol=1e-15)
    np.testing.assert_allclose(out.delta_hat, np.array([[27.0, 3.0], [9.0, 1.0]]) / 10.0, atol=1e-14)
    np.testing.assert_allclose(np.abs(out.q.ravel()), np.array([9.0, 1.0]) / np.sqrt(10.0), atol=1e-14)


def test_range_finder_is_exact_within_the_block_and_bounded_by_eckart_young():
    rng = np.random.default_rng(5)
    m, n, r, b = 120, 80, 6, 10
    # rank 9 <= b: the sketch spans the range, the result is SVD-Comp's
    low = rng.standard_normal((m, 9)) @ rng.standard_normal((9, n))
    mats = [low + 0.0 * rng.standard_normal((m, n)) for _ in range(2)]
    om = rng.standard_normal((n, b))
    out, ref = orc.range_finder_comp(mats, r, om), orc.svd_comp(mats, r)
    assert orc.sin_theta_max(ref.p_tilde, out.p_tilde) <= 1e-9
    np.testing.assert_allclose(out.delta_hat, ref.delta_hat, atol=1e-9)
    np.testing.assert_allclose(out.sigma[:9], ref.sigma[:9], rtol=1e-9)
    # full rank: a projector (Pythagoras, Eq. (4)), never better than the optimum (Eq. (6)), contractive
    mats = [rng.standard_normal((m, n)) * (0.9 ** np.arange(n))[None, :] for _ in range(3)]
    mean = orc.worker_mean(mats)
    out, ref = orc.range_finder_comp(mats, r, om), orc.svd_comp(mats, r)
    p = out.p_tilde
    np.testing.assert_allclose(p.T @ p, np.eye(r), atol=1e-13)
    np.testing.assert_allclose(out.delta_hat, p @ (p.T @ mean), atol=1e-12)
    np.testing.assert_allclose(out.q, mean.T @ p, atol=1e-12)
    err2 = np.linalg.norm(mean - out.delta_hat) ** 2
    assert abs(err2 + np.linalg.norm(out.delta_hat) ** 2 - np.linalg.norm(mean) ** 2) <= 1e-10 * np.linalg.norm(mean) ** 2
    assert float(np.sum(ref.sigma[r:] ** 2)) * (1 - 1e-12) <= err2 <= np.linalg.norm(mean) ** 2
    # per-worker reconstructions average to the global one (linearity, Appendix B notations)
    np.testing.assert_allclose(orc.worker_mean(out.delta_hat_i), out.delta_hat, atol=1e-12)
    # a square non-singular Omega spans everything: SVD-Comp again
    out = orc.range_finder_comp(mats, r, rng.standard_normal((n, n)))
    assert orc.sin_theta_max(ref.p_tilde, out.p_tilde) <= 1e-8


def _mix32_scalar(x):
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x7FEB352D) & 0xFFFFFFFF
    x ^= x >> 15
    x = (x * 0x846CA68B) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def test_counter_uniform_against_a_scalar_loop():
    seed, layer = 0x5EED5EED, 3
    got = orc.counter_uniform(seed, layer, 5, 7)
    h0 = _mix32_scalar(seed ^ _mix32_scalar(layer * 0x9E3779B9 + 0x85EBCA6B))
    for i in range(5):
        for c in range(7):
            h = _mix32_scalar(h0 ^ _mix32_scalar(i + 0x632BE5AB) ^ _mix32_scalar(c * 0xC2B2AE35 + 0x27D4EB2F))
            assert got[i, c] == (h >> 8) * (2.0 / 16777216.0) - 1.0
    big = orc.counter_uniform(1, 0, 400, 300)
    assert -1.0 <= big.min() and big.max() < 1.0 and abs(big.mean()) < 0.01 and abs(big.var() - 1.0 / 3.0) < 0.01
    assert not np.array_equal(big, orc.counter_uniform(2, 0, 400, 300))
