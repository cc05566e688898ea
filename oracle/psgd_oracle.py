"""CPU oracle for the PowerSGD / PowerSGD+ compressor  --  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy transcription of what the method computes, written from the paper
(arXiv 2509.11254) so that a reader can check each function against the cited passage by eye.
It is independent of the GPU library: it shares no code, tables, constants or helpers with it
and must never be imported by the product path; only the tests, the smoke check and the
benchmark's CPU-baseline leg use it.

What is written out here and what is a library step:
  * matrix products are NumPy `@` (a library primitive used as a step);
  * the economic QR (Section 2, "QR decomposition") is written out as classical Gram-Schmidt
    applied twice per column, which yields the Q-factor whose R has a positive diagonal;
  * the SVD of SVD-Comp (Definition 3, Algorithm 1) is `numpy.linalg.svd`, i.e. the plain
    definition "first r left singular vectors", not an iteration towards it (`svd_comp_large`, for
    matrices a dense SVD is too slow for in a test, is an fp64 iteration that returns its own
    certificate and is pinned against `svd_comp`);
  * `range_finder_comp` is this build's reading of the "lighter contractive compressor" the paper
    allows in place of SVD-Comp without printing one (randomized range finder).

Every input is widened exactly to fp64; nothing is blocked, fused or reordered relative to
Algorithm 1 / Algorithm 2.  The literal per-worker form (one error buffer e^(i) per worker) is
kept; the GPU library keeps only their mean, which is the same for every global quantity by the
linearity noted at the start of Appendix B.

Readings taken where the paper is silent (also listed in the design notes):
  * sign convention of QR: R_ii > 0;
  * a column of P whose part orthogonal to the previous columns is at most `rank_tol` times
    its own norm (or which is exactly zero) yields a zero column of P~ (parity unpinned: the
    paper's QR is undefined there);
  * mod(t, tau) = 0 selects SVD-Comp *instead of* SSP-Comp, and t = 0 is such a step;
  * the derivative of psi in Appendix A is evaluated at x11 - x12 - x21 + x22 (the argument of
    psi itself; one printed line has the signs permuted).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

RANK_TOL = 1e-5


# ----------------------------------------------------------------------------------------
# Section 2, "QR decomposition": A (n x r, n >= r) = Q R, return Q only, Q^T Q = I_r.
# ----------------------------------------------------------------------------------------
def qr_thin(a: np.ndarray, rank_tol: float = RANK_TOL) -> np.ndarray:
    """Q-factor of the economic QR with positive diagonal of R.

    Column k of Q is column k of A minus its projections on the earlier columns of Q,
    normalised.  The projection is done twice so that the result is orthonormal to fp64
    rounding even when the columns of A are nearly dependent.
    """
    a = np.asarray(a, dtype=np.float64)
    rows, r = a.shape
    q = np.zeros((rows, r), dtype=np.float64)
    for k in range(r):
        v = a[:, k].copy()
        norm0 = np.linalg.norm(v)
        for _ in range(2):
            for j in range(k):
                v -= (q[:, j] @ v) * q[:, j]
        nv = np.linalg.norm(v)
        if norm0 == 0.0 or nv <= rank_tol * norm0:
            q[:, k] = 0.0
        else:
            q[:, k] = v / nv
    return q


# ----------------------------------------------------------------------------------------
# Eq. (7a): Delta^(i) = g^(i) + e^(i)
# ----------------------------------------------------------------------------------------
def ef_accumulate(g: Sequence[np.ndarray], e: Sequence[np.ndarray]) -> List[np.ndarray]:
    return [np.asarray(gi, dtype=np.float64) + np.asarray(ei, dtype=np.float64) for gi, ei in zip(g, e)]


def worker_mean(xs: Sequence[np.ndarray]) -> np.ndarray:
    """All-Reduce Mean of Algorithm 1."""
    acc = np.zeros_like(np.asarray(xs[0], dtype=np.float64))
    for x in xs:
        acc = acc + x
    return acc / len(xs)


@dataclass
class CompOut:
    q: np.ndarray                    # Q_t            (n x r)
    p_tilde: np.ndarray              # P~_t           (m x r)
    delta_hat_i: List[np.ndarray]    # P~ (Q^(i))^T   per worker (m x n)
    delta_hat: np.ndarray            # P~ Q^T         (m x n)
    sigma: Optional[np.ndarray] = None   # singular values (SVD-Comp only)


# ----------------------------------------------------------------------------------------
# Algorithm 1, function SSP-Comp
# ----------------------------------------------------------------------------------------
def ssp_comp(q_prev: np.ndarray, deltas: Sequence[np.ndarray], rank_tol: float = RANK_TOL) -> CompOut:
    q_prev = np.asarray(q_prev, dtype=np.float64)
    p_i = [d @ q_prev for d in deltas]                 # P^(i) <- Delta^(i) Q
    p = worker_mean(p_i)                               # P <- mean
    p_tilde = qr_thin(p, rank_tol)                     # P~ <- QR(P)
    q_i = [d.T @ p_tilde for d in deltas]              # Q^(i) <- Delta^(i)^T P~
    q = worker_mean(q_i)                               # Q <- mean
    return CompOut(q, p_tilde, [p_tilde @ qi.T for qi in q_i], p_tilde @ q.T)


# ----------------------------------------------------------------------------------------
# Algorithm 1, function SVD-Comp (Definition 3: P~ = U[:, :r])
# ----------------------------------------------------------------------------------------
def svd_comp(deltas: Sequence[np.ndarray], r: int) -> CompOut:
    delta = worker_mean(deltas)                        # Delta <- mean (full matrix)
    u, s, _vt = np.linalg.svd(delta, full_matrices=False)
    p_tilde = u[:, :r]                                 # P~ <- U[:, :r]
    q_i = [d.T @ p_tilde for d in deltas]
    q = worker_mean(q_i)
    return CompOut(q, p_tilde, [p_tilde @ qi.T for qi in q_i], p_tilde @ q.T, sigma=s)


# ----------------------------------------------------------------------------------------
# SVD-Comp on matrices too large for a dense SVD in a test (4096^2 takes seconds, 8192^2 minutes).
# Definition 3 fixes the result, not an algorithm: the top-r left singular subspace.  This routine reaches it by
# fp64 block subspace iteration with generous oversampling and Rayleigh-Ritz, and returns a certificate with it:
# the residuals ||M^T u_k - s_k v_k|| and ||M v_k - s_k u_k|| of the r leading triplets, relative to s_1.  A caller
# asserts the certificate; `tests/test_oracle_pins.py` checks the routine against `svd_comp` on sizes where both run.
# ----------------------------------------------------------------------------------------
def svd_comp_large(deltas: Sequence[np.ndarray], r: int, oversample: int = 64, iters: int = 40,
                   tol: float = 1e-11, seed: int = 0) -> Tuple[CompOut, float]:
    delta = worker_mean(deltas)
    m, n = delta.shape
    b = min(n, r + oversample)
    y = np.random.default_rng(seed).standard_normal((n, b))
    resid = np.inf
    for _ in range(iters):
        z, _ = np.linalg.qr(delta @ y)                 # orthonormal basis of M Y
        y = delta.T @ z                                # Y = M^T Z
        w, s, vt = np.linalg.svd(y.T, full_matrices=False)     # Z^T M = W S V^T  (b x n)
        u = z @ w[:, :r]                               # Ritz vectors: leading left singular vectors
        v = vt[:r].T
        resid = max(float(np.linalg.norm(delta.T @ u - v * s[:r])), float(np.linalg.norm(delta @ v - u * s[:r]))) / s[0]
        if resid <= tol:
            break
    p_tilde = u
    q_i = [d.T @ p_tilde for d in deltas]
    q = worker_mean(q_i)
    return CompOut(q, p_tilde, [p_tilde @ qi.T for qi in q_i], p_tilde @ q.T, sigma=s[:r]), resid


# ----------------------------------------------------------------------------------------
# A lighter contractive compressor in place of SVD-Comp (the remark after Theorem 2 and the last row of Table 1
# allow any contractive compressor there and name random projection and an approximate top-r; the paper prints no
# algorithm for them).  Reading: the randomized range finder --
#   sketch  Y = M Omega  (Omega: n x b random, b >= r);  Z = orthonormal basis of Y;  B = Z^T M  (b x n);
#   B = W S V^T (small SVD);  P~ = Z W[:, :r];  then Q = M^T P~ and the residual as in SVD-Comp.
# P~ P~^T is an orthogonal projector, so the compressor is contractive (||M - P~P~^T M|| <= ||M||), and it is exact
# when rank(M) <= b.  Omega is an input: the GPU draws it from a counter-based generator (`counter_uniform` below is
# the same generator written in NumPy), so both sides can be given the same one.
# ----------------------------------------------------------------------------------------
def range_finder_comp(deltas: Sequence[np.ndarray], r: int, omega: np.ndarray) -> CompOut:
    delta = worker_mean(deltas)
    z = qr_thin(delta @ np.asarray(omega, dtype=np.float64))
    b_mat = z.T @ delta
    w, s, _vt = np.linalg.svd(b_mat, full_matrices=False)
    p_tilde = z @ w[:, :r]
    q_i = [d.T @ p_tilde for d in deltas]
    q = worker_mean(q_i)
    return CompOut(q, p_tilde, [p_tilde @ qi.T for qi in q_i], p_tilde @ q.T, sigma=s)


def _mix32(x: np.ndarray) -> np.ndarray:
    """32-bit integer finaliser (xor-shift-multiply, two rounds), on uint32 arrays with wrap-around."""
    x = x.astype(np.uint64)
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x7FEB352D)) & np.uint64(0xFFFFFFFF)
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x846CA68B)) & np.uint64(0xFFFFFFFF)
    x ^= x >> np.uint64(16)
    return x


def counter_uniform(seed: int, layer: int, rows: int, cols: int) -> np.ndarray:
    """rows x cols matrix of uniform numbers in [-1, 1) with 24 random bits each, a pure function of
    (seed, layer, row, column): entry = (h >> 8) * 2^-23 - 1 with
    h = mix(mix(seed ^ mix(layer * 0x9E3779B9 + 0x85EBCA6B)) ^ mix(row + 0x632BE5AB) ^ mix(column * 0xC2B2AE35 + 0x27D4EB2F)).
    The library's random start block of the refresh is drawn by the same rule on the device."""
    m32 = np.uint64(0xFFFFFFFF)
    lay = _mix32(np.array([(layer * 0x9E3779B9 + 0x85EBCA6B) & 0xFFFFFFFF], dtype=np.uint64))
    h0 = _mix32(np.uint64(seed & 0xFFFFFFFF) ^ lay)
    ri = _mix32((np.arange(rows, dtype=np.uint64) + np.uint64(0x632BE5AB)) & m32)
    ci = _mix32((np.arange(cols, dtype=np.uint64) * np.uint64(0xC2B2AE35) + np.uint64(0x27D4EB2F)) & m32)
    h = _mix32(h0 ^ ri[:, None] ^ ci[None, :])
    return (h >> np.uint64(8)).astype(np.float64) * (2.0 / 16777216.0) - 1.0


# ----------------------------------------------------------------------------------------
# Eq. (8): K-step power iteration on one matrix (K = 1 is Eq. (9), the SSP compressor)
# ----------------------------------------------------------------------------------------
def power_iteration(delta: np.ndarray, q_init: np.ndarray, k_steps: int) -> Tuple[np.ndarray, np.ndarray]:
    delta = np.asarray(delta, dtype=np.float64)
    q = np.asarray(q_init, dtype=np.float64)
    p_tilde = None
    for _ in range(k_steps):
        p_tilde = qr_thin(delta @ q)
        q = delta.T @ p_tilde
    return p_tilde, q


def decompress(p_tilde: np.ndarray, q: np.ndarray) -> np.ndarray:
    """Delta_hat = P~ Q^T (return value of both functions of Algorithm 1)."""
    return np.asarray(p_tilde, dtype=np.float64) @ np.asarray(q, dtype=np.float64).T


# ----------------------------------------------------------------------------------------
# Algorithm 2: one iteration of PowerSGD (tau = None) / PowerSGD+ (tau >= 1), compressor part.
# ----------------------------------------------------------------------------------------
@dataclass
class StepOut:
    comp: CompOut
    deltas: List[np.ndarray]
    e_next: List[np.ndarray]         # e^(i)_{t+1} = Delta^(i) - Delta_hat^(i)
    refreshed: bool

    @property
    def e_mean(self) -> np.ndarray:
        return worker_mean(self.e_next)

    @property
    def delta_mean(self) -> np.ndarray:
        return worker_mean(self.deltas)


def is_refresh_step(t: int, tau: Optional[int]) -> bool:
    return tau is not None and t % tau == 0


def compress_step(t: int, tau: Optional[int], r: int, q_prev: np.ndarray,
                  g: Sequence[np.ndarray], e: Sequence[np.ndarray], rank_tol: float = RANK_TOL) -> StepOut:
    deltas = ef_accumulate(g, e)
    if is_refresh_step(t, tau):
        comp = svd_comp(deltas, r)
        refreshed = True
    else:
        comp = ssp_comp(q_prev, deltas, rank_tol)
        refreshed = False
    e_next = [d - dh for d, dh in zip(deltas, comp.delta_hat_i)]
    return StepOut(comp, deltas, e_next, refreshed)


# ----------------------------------------------------------------------------------------
# Eq. (7c): momentum SGD on the compressed update
# ----------------------------------------------------------------------------------------
def msgd_update(x: np.ndarray, mom: np.ndarray, delta_hat: np.ndarray, eta: float, mu: float):
    mom = mu * mom + delta_hat
    return x - eta * mom, mom


# ----------------------------------------------------------------------------------------
# Adam as the base optimizer (Section 3, Claim 1 and Figure 1 name it next to MSGD; the pre-training runs of
# Section 5 / Appendix C use Adam and the fine-tuning runs AdamW with betas (0.9, 0.999)).  The paper does not
# print the update; this is the published one (Kingma & Ba, Algorithm 1) applied to the compressed update
# Delta_hat in place of the gradient, with the decoupled weight decay of AdamW (Loshchilov & Hutter,
# Algorithm 2 with schedule multiplier 1); weight_decay = 0 is plain Adam.  `step` counts from 1.
# ----------------------------------------------------------------------------------------
def adam_update(x: np.ndarray, m1: np.ndarray, m2: np.ndarray, delta_hat: np.ndarray, step: int, eta: float,
                beta1: float, beta2: float, eps: float, weight_decay: float = 0.0):
    m1 = beta1 * m1 + (1.0 - beta1) * delta_hat
    m2 = beta2 * m2 + (1.0 - beta2) * delta_hat * delta_hat
    m1_hat = m1 / (1.0 - beta1 ** step)
    m2_hat = m2 / (1.0 - beta2 ** step)
    x = x - eta * (m1_hat / (np.sqrt(m2_hat) + eps) + weight_decay * x)
    return x, m1, m2


# ----------------------------------------------------------------------------------------
# Section 3 / Appendix A: the 2x2 problem on which PowerSGD stalls.
# ----------------------------------------------------------------------------------------
A_MAT = np.array([[1.0, -1.0], [-1.0, 1.0]])
B_MAT = np.array([[1.0, 1.0], [1.0, 1.0]])
C_VEC = np.array([[np.sqrt(2.0) / 2.0], [np.sqrt(2.0) / 2.0]])
D_VEC = np.array([[1.0], [-1.0]])


def psi(x: float) -> float:
    return x * x if abs(x) <= 1.0 else 2.0 * abs(x) - 1.0


def dpsi(x: float) -> float:
    return 2.0 * x if abs(x) <= 1.0 else 2.0 * np.sign(x)


def counter_f(x: np.ndarray) -> float:
    """f_i(X) = psi(D^T X D), the same on every node (Eq. 10a)."""
    return psi(float((D_VEC.T @ x @ D_VEC)[0, 0]))


def counter_grad(x: np.ndarray) -> np.ndarray:
    """grad f(X) = psi'(x11 - x12 - x21 + x22) * A."""
    return dpsi(float((D_VEC.T @ x @ D_VEC)[0, 0])) * A_MAT


def counter_stochastic_grad(x: np.ndarray, xi: float, sigma: float) -> np.ndarray:
    """Eq. (10b): grad f + xi (sigma B - grad f), xi in {-1, +1}."""
    gf = counter_grad(x)
    return gf + xi * (sigma * B_MAT - gf)


@dataclass
class Trajectory:
    x: List[np.ndarray] = field(default_factory=list)
    grad_norm_sq: List[float] = field(default_factory=list)
    p_tilde: List[np.ndarray] = field(default_factory=list)
    q: List[np.ndarray] = field(default_factory=list)
    e_next: List[List[np.ndarray]] = field(default_factory=list)
    mom: List[np.ndarray] = field(default_factory=list)


def run_counterexample(x0: np.ndarray, q_init: np.ndarray, xi: np.ndarray, sigma: float, eta: float,
                       mu: float, tau: Optional[int], r: int = 1) -> Trajectory:
    """Algorithm 2 with MSGD on the 2x2 problem.  xi has shape (T, N); tau=None is PowerSGD."""
    steps, n_workers = xi.shape
    x = np.asarray(x0, dtype=np.float64).copy()
    mom = np.zeros_like(x)
    e = [np.zeros_like(x) for _ in range(n_workers)]
    q = np.asarray(q_init, dtype=np.float64).copy()
    tr = Trajectory()
    for t in range(steps):
        tr.x.append(x.copy())
        tr.grad_norm_sq.append(float(np.sum(counter_grad(x) ** 2)))
        g = [counter_stochastic_grad(x, float(xi[t, i]), sigma) for i in range(n_workers)]
        out = compress_step(t, tau, r, q, g, e)
        q, e = out.comp.q, out.e_next
        x, mom = msgd_update(x, mom, out.comp.delta_hat, eta, mu)
        tr.p_tilde.append(out.comp.p_tilde)
        tr.q.append(q.copy())
        tr.e_next.append([ei.copy() for ei in e])
        tr.mom.append(mom.copy())
    tr.x.append(x.copy())
    tr.grad_norm_sq.append(float(np.sum(counter_grad(x) ** 2)))
    return tr


# ----------------------------------------------------------------------------------------
# Comparison helpers used by the parity tests (not part of the method).
# ----------------------------------------------------------------------------------------
def sin_theta_max(basis_ref: np.ndarray, basis: np.ndarray) -> float:
    """Largest sine of the principal angles between range(basis) and range(basis_ref).

    Both arguments must have orthonormal columns; equals ||(I - Pref Pref^T) P||_2.
    """
    ref = np.asarray(basis_ref, dtype=np.float64)
    b = np.asarray(basis, dtype=np.float64)
    resid = b - ref @ (ref.T @ b)
    return float(np.linalg.norm(resid, 2))


def rel_fro(x: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    num = np.linalg.norm(np.asarray(x, dtype=np.float64) - ref)
    return float(num / den) if den > 0 else float(num)
