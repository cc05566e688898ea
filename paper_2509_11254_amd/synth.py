"""Seeded synthetic gradient sets shaped like the workloads the compressor is measured on.

This module only *draws inputs*: random orthonormal factors, prescribed spectra, Gaussian
noise, bf16 rounding of the generated values.  It holds none of the compressor's arithmetic
(no error feedback, no power iteration, no orthonormalisation of the method's iterates, no
reconstruction) and is the one piece of code that both the CPU oracle's tests and the GPU
tests may share.  Everything is a pure function of the integer seed and of the
(layer, worker, step) coordinates, so any sub-sample of a workload can be regenerated alone.

The paper trains RoBERTa-Base on GLUE and LLaMA-60M/130M on C4 (Section 5); neither the
data nor the models are available here, so per-worker stochastic gradients are replaced by
"shared low-rank signal + fresh iid noise per worker and per step", which is the slowly
varying leading subspace regime that single-step power iteration assumes (Section 3,
paragraph on non-convergence).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32 = "f32"
BF16 = "bf16"


def _rng(seed: int, *coords: int) -> np.random.Generator:
    """Counter-style generator: one independent stream per coordinate tuple."""
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), *map(int, coords)])))


def haar_orthonormal(rows: int, cols: int, seed: int, *coords: int) -> np.ndarray:
    """rows x cols matrix with orthonormal columns, Haar distributed (fp64)."""
    g = _rng(seed, *coords).standard_normal((rows, cols))
    q, r = np.linalg.qr(g)
    return q * np.sign(np.diag(r))[None, :]


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


@dataclass
class LayerSpec:
    """One matrix variable as it is stored: `rows x cols`, row-major.

    The logical matrix of the paper has m >= n (Section 1).  When rows < cols the stored
    buffer is the transpose of the logical matrix (`transposed` is True), m = cols, n = rows.
    """

    rows: int
    cols: int
    name: str = ""

    @property
    def transposed(self) -> bool:
        return self.rows < self.cols

    @property
    def m(self) -> int:
        return max(self.rows, self.cols)

    @property
    def n(self) -> int:
        return min(self.rows, self.cols)


@dataclass
class Workload:
    name: str
    layers: List[LayerSpec]
    r: int
    n_workers: int
    grad_dtype: str
    signal_rank: int
    spectrum: np.ndarray          # singular values of the shared signal, descending
    noise_std: Optional[float]    # per-entry std of each worker's noise, or None
    noise_rel: Optional[float]    # ... or noise Frobenius norm as a fraction of the signal's
    tau: int
    steps: int
    seed: int = 1234
    notes: str = ""

    def describe(self) -> dict:
        return {
            "workload": self.name,
            "layers": len(self.layers),
            "elements": int(sum(l.rows * l.cols for l in self.layers)),
            "r": self.r,
            "n_workers": self.n_workers,
            "grad_dtype": self.grad_dtype,
            "signal_rank": self.signal_rank,
            "spectrum": "%.4g..%.4g" % (self.spectrum[0], self.spectrum[-1]),
            "noise_std": self.noise_std,
            "noise_rel": self.noise_rel,
            "tau": self.tau,
            "seed": self.seed,
        }


def signal_factors(spec: LayerSpec, wl: Workload, layer: int) -> Tuple[np.ndarray, np.ndarray]:
    """Fixed-in-time orthonormal factors (U: rows x k, V: cols x k) of the shared signal."""
    k = wl.signal_rank
    u = haar_orthonormal(spec.rows, k, wl.seed, 101, layer)
    v = haar_orthonormal(spec.cols, k, wl.seed, 202, layer)
    return u, v


def signal_matrix(spec: LayerSpec, wl: Workload, layer: int) -> np.ndarray:
    u, v = signal_factors(spec, wl, layer)
    return (u * wl.spectrum[None, :]) @ v.T


def noise_sigma(spec: LayerSpec, wl: Workload) -> float:
    """Per-entry noise std of one worker's gradient."""
    if wl.noise_std is not None:
        return float(wl.noise_std)
    sig_fro = float(np.sqrt(np.sum(wl.spectrum ** 2)))
    return float(wl.noise_rel) * sig_fro / np.sqrt(spec.rows * spec.cols)


def worker_gradient(spec: LayerSpec, wl: Workload, layer: int, worker: int, step: int,
                    signal: Optional[np.ndarray] = None) -> np.ndarray:
    """Gradient of one worker at one step, in the storage dtype.

    Returns fp32 values for F32 workloads and uint16 bf16 bit patterns for BF16 ones.
    """
    if signal is None:
        signal = signal_matrix(spec, wl, layer)
    noise = _rng(wl.seed, 303, layer, worker, step).standard_normal((spec.rows, spec.cols), dtype=np.float32)
    g = (signal + noise_sigma(spec, wl) * noise).astype(np.float32)
    if wl.grad_dtype == BF16:
        return round_to_bf16(g)
    return g


def gradient_as_f64(g: np.ndarray) -> np.ndarray:
    """Exact widening of a stored gradient (fp32 values or bf16 bit patterns) to fp64."""
    if g.dtype == np.uint16:
        return bf16_bits_to_f32(g).astype(np.float64)
    return g.astype(np.float64)


def initial_q(n: int, r: int, seed: int, layer: int = 0) -> np.ndarray:
    """Q_{-1}: iid N(0,1), identical on every worker (Algorithm 2 leaves it unspecified)."""
    return _rng(seed, 404, layer).standard_normal((n, r)).astype(np.float32)


def prescribed_svd_matrix(m: int, n: int, sigma: Sequence[float], seed: int,
                          noise_std: float = 0.0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """M = U diag(sigma) V^T (+ noise) with known Haar factors; returns (M fp32, U, V)."""
    sigma = np.asarray(sigma, dtype=np.float64)
    k = sigma.shape[0]
    u = haar_orthonormal(m, k, seed, 505)
    v = haar_orthonormal(n, k, seed, 606)
    mat = (u * sigma[None, :]) @ v.T
    if noise_std > 0:
        mat = mat + noise_std * _rng(seed, 707).standard_normal((m, n))
    return mat.astype(np.float32), u, v


# --------------------------------------------------------------------------------------
# The five benchmark configurations.  Unstated details (index range of the spectra, decay
# rates of configs 3-5) are fixed here and repeated in the design notes.
# --------------------------------------------------------------------------------------

def config1(seed: int = 1234) -> Workload:
    return Workload("c1_256x128_f32_r4_n4", [LayerSpec(256, 128, "x")], r=4, n_workers=4,
                    grad_dtype=F32, signal_rank=8, spectrum=2.0 ** -np.arange(1, 9),
                    noise_std=0.01, noise_rel=None, tau=5, steps=20, seed=seed)


def config2(seed: int = 1234) -> Workload:
    return Workload("c2_4096x4096_f32_r8_n8", [LayerSpec(4096, 4096, "x")], r=8, n_workers=8,
                    grad_dtype=F32, signal_rank=32, spectrum=0.8 ** np.arange(32),
                    noise_std=1e-3, noise_rel=None, tau=10, steps=50, seed=seed)


def _llama_layers(n_blocks: int, hidden: int, inter: int) -> List[LayerSpec]:
    out = []
    for b in range(n_blocks):
        for nm in ("q", "k", "v", "o"):
            out.append(LayerSpec(hidden, hidden, f"b{b}.{nm}"))
        out.append(LayerSpec(inter, hidden, f"b{b}.gate"))
        out.append(LayerSpec(inter, hidden, f"b{b}.up"))
        out.append(LayerSpec(hidden, inter, f"b{b}.down"))
    return out


def config3(seed: int = 1234) -> Workload:
    return Workload("c3_1b_layers_bf16_r32_n4", _llama_layers(22, 2048, 5632), r=32, n_workers=4,
                    grad_dtype=BF16, signal_rank=64, spectrum=0.9 ** np.arange(64),
                    noise_std=None, noise_rel=0.01, tau=100, steps=1, seed=seed)


def config4(seed: int = 1234) -> Workload:
    layers = []
    for b in range(32):
        for nm in ("q", "k", "v", "o"):
            layers.append(LayerSpec(4096, 4096, f"b{b}.{nm}"))
        for nm in ("gate", "up", "down"):
            layers.append(LayerSpec(11008, 4096, f"b{b}.{nm}"))
    return Workload("c4_7b_layers_bf16_r64_n1", layers, r=64, n_workers=1,
                    grad_dtype=BF16, signal_rank=64, spectrum=0.9 ** np.arange(64),
                    noise_std=None, noise_rel=0.01, tau=100, steps=1, seed=seed)


def config5a(dtype: str = F32, seed: int = 1234) -> Workload:
    return Workload(f"c5a_8192x8192_{dtype}_r128_refresh", [LayerSpec(8192, 8192, "x")], r=128,
                    n_workers=1, grad_dtype=dtype, signal_rank=256, spectrum=0.95 ** np.arange(256),
                    noise_std=None, noise_rel=0.01, tau=1, steps=1, seed=seed)


def scaled_down(wl: Workload, rows: int, cols: int, n_layers: int = 1) -> Workload:
    """Same recipe on smaller matrices (parity cases the CPU oracle finishes in seconds)."""
    k = min(wl.signal_rank, min(rows, cols))
    return Workload(wl.name + f"_small{rows}x{cols}", [LayerSpec(rows, cols, f"s{i}") for i in range(n_layers)],
                    r=min(wl.r, min(rows, cols)), n_workers=wl.n_workers, grad_dtype=wl.grad_dtype,
                    signal_rank=k, spectrum=wl.spectrum[:k], noise_std=wl.noise_std, noise_rel=wl.noise_rel,
                    tau=wl.tau, steps=wl.steps, seed=wl.seed)


def device_gradients(wl, n_sets, torch, no_qr=False):
    """Same recipe as worker_gradient (shared low-rank signal + fresh iid noise per worker), drawn on the device
    with torch's generator (passed in: this module does not import torch): the full-size batches of the benchmark
    and of the parity tests that sample layers of them.  Returns (sets[s][l][w], E[l] zeros, Q[l], P[l], OUT[l])."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.seed)
    gdt = torch.bfloat16 if wl.grad_dtype == BF16 else torch.float32
    spectrum = torch.tensor(wl.spectrum, dtype=torch.float32, device="cuda")
    sets = [[] for _ in range(n_sets)]
    E, Q, P, OUT = [], [], [], []
    for l, spec in enumerate(wl.layers):
        k = wl.signal_rank
        u = torch.randn((spec.rows, k), generator=gen, device="cuda")
        v = torch.randn((spec.cols, k), generator=gen, device="cuda")
        if no_qr:
            u, v = u / spec.rows ** 0.5, v / spec.cols ** 0.5
        else:
            u, v = torch.linalg.qr(u)[0], torch.linalg.qr(v)[0]
        signal = (u * spectrum[None, :]) @ v.T
        sigma = noise_sigma(spec, wl)
        for s in range(n_sets):
            per_worker = []
            for w in range(wl.n_workers):
                g = signal + sigma * torch.randn((spec.rows, spec.cols), generator=gen, device="cuda")
                per_worker.append(g.to(gdt).contiguous())
            sets[s].append(per_worker)
        del signal, u, v
        E.append(torch.zeros((spec.rows, spec.cols), dtype=torch.float32, device="cuda"))
        Q.append(torch.randn((spec.n, wl.r), generator=gen, device="cuda"))
        P.append(torch.zeros((spec.m, wl.r), dtype=torch.float32, device="cuda"))
        OUT.append(torch.empty((spec.rows, spec.cols), dtype=torch.float32, device="cuda"))
    return sets, E, Q, P, OUT


# ----------------------------------------------------------------------------------------------------------------
# Config 5b: the least-squares problem behind the PowerSGD / PowerSGD+ comparison of Section 3 (Figure 1).  The paper
# gives none of its parameters; the ones here are this build's (listed in the design notes).  Only the data of the
# problem and the random signs of the stochastic gradient are made here; the gradient itself, the compressor and the
# optimizer are the caller's.
# ----------------------------------------------------------------------------------------------------------------
@dataclass
class LeastSquares:
    a: List[np.ndarray]          # A_i, N x (rows x d), fp32
    b: List[np.ndarray]          # B_i = A_i X* + noise, N x (rows x k), fp32
    x_star: np.ndarray           # d x k
    xi: np.ndarray               # steps x N signs in {-1, +1}; step 0 is all +1
    r: int = 4
    tau: int = 10
    mu: float = 0.9
    sigma: float = 50.0          # size of the rank-one term of the stochastic gradient
    eta_scale: float = 0.03      # eta = eta_scale (1 - mu) / lambda_max(mean_i A_i^T A_i / rows)


def least_squares_problem(steps: int = 2000, n_workers: int = 16, rows: int = 512, d: int = 256, k: int = 128,
                          noise: float = 0.1, seed: int = 1234) -> LeastSquares:
    g = _rng(seed, 55)
    a = [g.standard_normal((rows, d)).astype(np.float32) for _ in range(n_workers)]
    x_star = g.standard_normal((d, k)).astype(np.float32)
    b = [(ai.astype(np.float64) @ x_star + noise * g.standard_normal((rows, k))).astype(np.float32) for ai in a]
    xi = g.choice(np.array([-1.0, 1.0]), size=(steps, n_workers))
    xi[0, :] = 1.0
    return LeastSquares(a, b, x_star, xi)
