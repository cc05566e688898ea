"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times: the whole batch of config 3
(154 matrices) and of config 4 (224 matrices) in one psgd_compress / psgd_decompress each, inputs drawn on the device
by the same generator bench.py uses, and the outputs of a sample of layers -- one of every distinct shape, the
transposed one, the first and the last of the batch -- compared with the oracle, which computes those layers one by
one from the inputs read back before the step.
"""
import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2509_11254_amd import psgd, synth
from gpu_harness import back, logical, torch_mod

pytestmark = pytest.mark.gpu


def _sample_layers(wl):
    seen, sample = set(), []
    for l, spec in enumerate(wl.layers):
        if (spec.rows, spec.cols) not in seen:
            seen.add((spec.rows, spec.cols))
            sample.append(l)
    if len(wl.layers) - 1 not in sample:
        sample.append(len(wl.layers) - 1)
    return sample


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_full_batch_step_sampled_layers(name):
    torch = torch_mod()
    wl = {"c3": synth.config3, "c4": synth.config4}[name]()
    gd = psgd.PSGD_BF16 if wl.grad_dtype == synth.BF16 else psgd.PSGD_F32
    comp = psgd.Compressor([(s.rows, s.cols, wl.r, gd) for s in wl.layers], wl.n_workers)
    sets, E, Q, P, OUT = synth.device_gradients(wl, 1, torch)
    G = sets[0]
    comp.compress(G, E, Q, P)                       # step 1: leaves a non-trivial E and the Q of a run
    torch.cuda.synchronize()
    sample = _sample_layers(wl)
    before = {l: (back(E[l]), back(Q[l])) for l in sample}
    comp.compress(G, E, Q, P)                       # step 2, the one compared
    comp.decompress(P, Q, OUT)
    torch.cuda.synchronize()
    worst = {}
    for l in sample:
        spec = wl.layers[l]
        g = [logical(back(x), spec.rows, spec.cols) for x in G[l]]
        e0, q0 = before[l]
        e = [logical(e0, spec.rows, spec.cols)] * wl.n_workers
        ref = orc.compress_step(1, None, wl.r, q0, g, e)
        p_gpu, q_gpu = back(P[l]), back(Q[l])
        errs = {"P": orc.rel_fro(p_gpu, ref.comp.p_tilde), "Q": orc.rel_fro(q_gpu, ref.comp.q),
                "E": orc.rel_fro(logical(back(E[l]), spec.rows, spec.cols), ref.e_mean),
                "D": orc.rel_fro(logical(back(OUT[l]), spec.rows, spec.cols), ref.comp.delta_hat)}
        assert float(np.abs(p_gpu.T @ p_gpu - np.eye(wl.r)).max()) < 2e-5, l
        for k, v in errs.items():
            assert v <= 2e-2, (name, l, spec, k, errs)            # bf16 gradients: the bf16 bar
            worst[k] = max(worst.get(k, 0.0), v)
    print(name, "layers", sample, worst)


def _error_after_lazy_step(torch, wl, l, E, P, Q):
    """E_1 of a layer after a deferred-residual step, from what the step left on the device: the error buffer holds
    M_1 and the residual is owed, E_1 = M_1 - P~_1 Q_1^T (Algorithm 2, error update), formed here in fp64."""
    spec = wl.layers[l]
    m1 = logical(back(E[l]), spec.rows, spec.cols)
    return m1 - back(P[l]) @ back(Q[l]).T


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_full_batch_deferred_residual_step_sampled_layers(name):
    """The configuration bench.py times by default: the whole batch with lazy_residual (and q_resident), i.e. the
    forming pass that applies the residual of the step before on the way in, launched through the XCD table.  Step 1
    leaves M_1 and the factors; step 2 is compared: M_2 as found in the buffer, P~_2, Q_2, then E_2 after the flush
    and the reconstruction from the workspace's factors."""
    torch = torch_mod()
    wl = {"c3": synth.config3, "c4": synth.config4}[name]()
    gd = psgd.PSGD_BF16 if wl.grad_dtype == synth.BF16 else psgd.PSGD_F32
    comp = psgd.Compressor([(s.rows, s.cols, wl.r, gd) for s in wl.layers], wl.n_workers, lazy_residual=True,
                           q_resident=True)
    sets, E, Q, P, OUT = synth.device_gradients(wl, 1, torch)
    G = sets[0]
    comp.compress(G, E, Q, P)
    torch.cuda.synchronize()
    sample = _sample_layers(wl)
    before = {l: (_error_after_lazy_step(torch, wl, l, E, P, Q), back(Q[l])) for l in sample}
    comp.compress(G, E, Q, P)                       # step 2, the one compared
    torch.cuda.synchronize()
    m_found = {l: logical(back(E[l]), wl.layers[l].rows, wl.layers[l].cols) for l in sample}
    comp.flush_residual(E)
    comp.decompress(None, None, OUT)
    torch.cuda.synchronize()
    worst = {}
    for l in sample:
        spec = wl.layers[l]
        g = [logical(back(x), spec.rows, spec.cols) for x in G[l]]
        e1, q1 = before[l]
        ref = orc.compress_step(1, None, wl.r, q1, g, [e1] * wl.n_workers)
        m_ref = orc.worker_mean(g) + e1
        p_gpu, q_gpu = back(P[l]), back(Q[l])
        errs = {"M": orc.rel_fro(m_found[l], m_ref), "P": orc.rel_fro(p_gpu, ref.comp.p_tilde),
                "Q": orc.rel_fro(q_gpu, ref.comp.q),
                "E": orc.rel_fro(logical(back(E[l]), spec.rows, spec.cols), ref.e_mean),
                "D": orc.rel_fro(logical(back(OUT[l]), spec.rows, spec.cols), ref.comp.delta_hat)}
        assert float(np.abs(p_gpu.T @ p_gpu - np.eye(wl.r)).max()) < 2e-5, l
        for k, v in errs.items():
            assert v <= 2e-2, (name, l, spec, k, errs)            # bf16 gradients: the bf16 bar
            worst[k] = max(worst.get(k, 0.0), v)
    print(name, "deferred, layers", sample, worst)


def test_full_batch_refresh_config4_sampled_layers():
    """SVD-Comp on the whole batch of config 4 (block width 80: the forming pass, the column-mode product and the
    128-row row product at width 96, gated launches through the XCD table) after one error-feedback step.  The cut of
    this workload has no gap (sigma_64 of the signal is at the level of the noise), so the subspace is not unique and
    the checks are the ones that hold for any of its valid answers: P~ orthonormal, Q = M^T P~, E = M - P~ Q^T, and
    Lemma 2's equality ||E||^2 = sum_{i > r} sigma_i^2 to 1e-4 ||M||^2, with the singular values from the eigenvalues
    of M^T M in fp64.  One layer of each distinct shape."""
    torch = torch_mod()
    wl = synth.config4()
    comp = psgd.Compressor([(s.rows, s.cols, wl.r, psgd.PSGD_BF16) for s in wl.layers], wl.n_workers,
                           lazy_residual=True, q_resident=True)
    sets, E, Q, P, OUT = synth.device_gradients(wl, 1, torch)
    G = sets[0]
    comp.compress(G, E, Q, P)
    torch.cuda.synchronize()
    sample = _sample_layers(wl)[:2]
    e1 = {l: _error_after_lazy_step(torch, wl, l, E, P, Q) for l in sample}
    comp.compress_refresh(G, E, Q, P)               # settles the owed residual, then SVD-Comp of M_2 = G + E_1
    comp.flush_residual(E)                          # (nothing owed after a refresh step: a no-op or the residual)
    torch.cuda.synchronize()
    for l in sample:
        spec = wl.layers[l]
        m = logical(back(G[l][0]), spec.rows, spec.cols) + e1[l]
        p_gpu, q_gpu = back(P[l]), back(Q[l])
        e_gpu = logical(back(E[l]), spec.rows, spec.cols)
        lam = np.linalg.eigvalsh(m.T @ m)[::-1]
        total = float(np.sum(lam))
        errs = {"orth": float(np.abs(p_gpu.T @ p_gpu - np.eye(wl.r)).max()),
                "Q": orc.rel_fro(q_gpu, m.T @ p_gpu),
                "E": orc.rel_fro(e_gpu, m - p_gpu @ q_gpu.T),
                "tail": abs(float(np.sum(e_gpu ** 2)) - float(np.sum(lam[wl.r:]))) / total}
        print("c4 refresh layer", l, spec, errs, flush=True)
        assert errs["orth"] < 2e-5 and errs["Q"] <= 2e-2 and errs["E"] <= 2e-2 and errs["tail"] <= 1e-4, (l, errs)
