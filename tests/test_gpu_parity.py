"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle, element by element.

Tolerances (relative Frobenius error against the oracle's value): 1e-4 for fp32 gradients, 2e-2 for
bf16 gradients; refreshed subspaces within sin(theta_max) <= 1e-4.  E is compared against
||E_oracle||_F (not ||M||_F).
"""
import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2509_11254_amd import psgd, synth
from gpu_harness import Case, back, logical, oracle_inputs, to_dev_f32, torch_mod, to_dev_grad

pytestmark = pytest.mark.gpu

TOL = {synth.F32: 1e-4, synth.BF16: 2e-2}


def _workload_inputs(wl, step=0, err_scale=0.3, seed_off=0):
    grads, errs, qs = [], [], []
    for l, spec in enumerate(wl.layers):
        sig = synth.signal_matrix(spec, wl, l)
        grads.append([synth.worker_gradient(spec, wl, l, w, step, sig) for w in range(wl.n_workers)])
        rng = np.random.default_rng([wl.seed, 909, l, seed_off])
        errs.append((err_scale * synth.noise_sigma(spec, wl) * rng.standard_normal((spec.rows, spec.cols))).astype(np.float32))
        qs.append(synth.initial_q(spec.n, wl.r, wl.seed, l))
    return grads, errs, qs


def _check_step(case, wl, grads, errs, qs, refresh, tol, check_pq=True):
    worst = {}
    for l, spec in enumerate(wl.layers):
        g, e = oracle_inputs(grads[l], errs[l], spec.rows, spec.cols, wl.n_workers)
        out = orc.compress_step(0 if refresh else 1, 1 if refresh else None, wl.r, qs[l].astype(np.float64), g, e)
        p_gpu, q_gpu, e_gpu = case.outputs(l)
        e_gpu = logical(e_gpu, spec.rows, spec.cols)
        assert np.all(np.isfinite(p_gpu)) and np.all(np.isfinite(q_gpu)) and np.all(np.isfinite(e_gpu))
        errs_l = {"E": orc.rel_fro(e_gpu, out.e_mean)}
        if refresh:
            errs_l["sin"] = orc.sin_theta_max(out.comp.p_tilde, p_gpu)
            errs_l["dhat"] = orc.rel_fro(p_gpu @ q_gpu.T, out.comp.delta_hat)
        elif check_pq:
            errs_l["P"] = orc.rel_fro(p_gpu, out.comp.p_tilde)
            errs_l["Q"] = orc.rel_fro(q_gpu, out.comp.q)
        errs_l["orth"] = float(np.abs(p_gpu.T @ p_gpu - np.eye(wl.r)).max())
        for k, v in errs_l.items():
            worst[k] = max(worst.get(k, 0.0), v)
        assert errs_l["orth"] < 2e-5, (l, errs_l)
        for k in ("E", "P", "Q", "dhat"):
            if k in errs_l:
                assert errs_l[k] <= tol, (spec, k, errs_l)
        if "sin" in errs_l:
            assert errs_l["sin"] <= 1e-4, (spec, errs_l)
    return worst


def _run_case(wl, refresh=False, lds=None, **opts):
    grads, errs, qs = _workload_inputs(wl)
    case = Case([(s.rows, s.cols) for s in wl.layers], wl.r, wl.n_workers, wl.grad_dtype, lds=lds, **opts)
    case.upload(grads, errs, qs)
    case.compress(refresh=refresh)
    return _check_step(case, wl, grads, errs, qs, refresh, TOL[wl.grad_dtype])


# ------------------------------------------------------------------ single SSP step, many shapes
def test_ssp_step_config1():
    w = _run_case(synth.config1())
    print("config1 ssp", w)


@pytest.mark.parametrize("rows,cols,ld", [(333, 203, 208), (130, 129, 136), (64, 8, 8), (1000, 40, 40), (129, 600, 600)])
def test_ssp_step_ragged_shapes(rows, cols, ld):
    wl = synth.scaled_down(synth.config2(), rows, cols)
    wl.r = min(8, min(rows, cols) // 2)      # r = n would make E exactly zero (nothing to compare relatively)
    print(rows, cols, _run_case(wl, lds=[ld]))


def test_ssp_step_bf16_r32_four_workers():
    wl = synth.scaled_down(synth.config3(), 640, 384)
    print(_run_case(wl))


def test_ssp_step_transposed_storage_bf16():
    wl = synth.scaled_down(synth.config3(), 384, 1024)
    print(_run_case(wl))


def test_ssp_step_r64_single_worker_bf16():
    wl = synth.scaled_down(synth.config4(), 1100, 512)
    print(_run_case(wl))


def test_ssp_step_r128():
    """r = 128 on a slowly decaying spectrum (0.95^k).  Q_{t-1} comes from one earlier oracle step, as it
    does in a run (Algorithm 2 starts with a refresh, so Q is never a random matrix); the columns of
    P = M Q_{t-1} are then close to orthogonal and the step is well conditioned."""
    wl = synth.scaled_down(synth.config5a(), 768, 512)
    grads, errs, qs = _workload_inputs(wl)
    spec = wl.layers[0]
    g0 = [synth.gradient_as_f64(synth.worker_gradient(spec, wl, 0, w, 7)) for w in range(wl.n_workers)]
    warm = orc.compress_step(0, 1, wl.r, qs[0].astype(np.float64), g0, [np.zeros((spec.rows, spec.cols))] * wl.n_workers)
    qs = [warm.comp.q.astype(np.float32)]
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype)
    case.upload(grads, errs, qs)
    case.compress()
    print(_check_step(case, wl, grads, errs, qs, False, 1e-4))


@pytest.mark.parametrize("precision,tol", [(0, 1e-4), (2, 5e-3)])
def test_ssp_step_r128_random_q_ill_conditioned(precision, tol):
    """Same matrix from a random Q: cond(P) ~ sigma_1/sigma_128 ~ 700, and the Q-factor of P moves by cond(P) times
    the relative error of P.  With the default three operand planes of fp32 gradients (24 mantissa bits) the fp32
    bar of 1e-4 holds; with two planes (precision = 2: 2^-17 per operand) the bound is cond(P) * 2^-17 ~ 5e-3 on
    P~ (E is less sensitive).  The invariants hold tightly either way."""
    wl = synth.scaled_down(synth.config5a(), 768, 512)
    grads, errs, qs = _workload_inputs(wl)
    case = Case([(768, 512)], wl.r, wl.n_workers, wl.grad_dtype, precision=precision)
    case.upload(grads, errs, qs)
    case.compress()
    w = _check_step(case, wl, grads, errs, qs, False, tol)
    print(precision, w)
    p, q, e = case.outputs(0)
    mat = orc.worker_mean(oracle_inputs(grads[0], errs[0], 768, 512, wl.n_workers)[0]) + errs[0].astype(np.float64)
    assert np.linalg.norm(e - (mat - p @ (p.T @ mat))) <= 2e-5 * np.linalg.norm(mat)     # E = (I - P~P~^T) M
    assert np.linalg.norm(q - mat.T @ p) <= 2e-5 * np.linalg.norm(mat)                   # Q = M^T P~


def test_ssp_step_batched_mixed_layers():
    base = synth.config3()
    wl = synth.scaled_down(base, 256, 256)
    wl.layers = [synth.LayerSpec(256, 256, "a"), synth.LayerSpec(704, 256, "b"), synth.LayerSpec(256, 704, "c"),
                 synth.LayerSpec(256, 256, "d"), synth.LayerSpec(200, 136, "e")]
    print(_run_case(wl))


@pytest.mark.parametrize("m_policy", [1, 2])
@pytest.mark.parametrize("which", ["f32_n4", "bf16_n1", "bf16_n3_transposed", "batched"])
def test_ssp_step_m_stored_or_formed_again(which, m_policy):
    """M = mean G + E between the passes of an SSP step: stored over E by the first pass (policy 1) or
    formed again from G and E by every pass (policy 2).  Same result."""
    if which == "f32_n4":
        wl = synth.scaled_down(synth.config1(), 333, 203)
        lds = [208]
    elif which == "bf16_n1":
        wl = synth.scaled_down(synth.config4(), 700, 384)
        lds = None
    elif which == "bf16_n3_transposed":
        wl = synth.scaled_down(synth.config3(), 384, 1024)
        wl.n_workers = 3
        lds = None
    else:
        wl = synth.scaled_down(synth.config4(), 256, 256)
        wl.layers = [synth.LayerSpec(256, 256, "a"), synth.LayerSpec(704, 256, "b"), synth.LayerSpec(256, 704, "c"),
                     synth.LayerSpec(200, 136, "e")]
        lds = None
    print(which, m_policy, _run_case(wl, lds=lds, m_policy=m_policy))


# ------------------------------------------------------------------ trajectory, teacher-forced (config 1)
def test_config1_trajectory_teacher_forced():
    wl = synth.config1()
    spec = wl.layers[0]
    sig = synth.signal_matrix(spec, wl, 0)
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype)
    e_w = [np.zeros((spec.rows, spec.cols)) for _ in range(wl.n_workers)]
    q = synth.initial_q(spec.n, wl.r, wl.seed).astype(np.float64)
    worst = {}
    for t in range(wl.steps):
        grads = [synth.worker_gradient(spec, wl, 0, w, t, sig) for w in range(wl.n_workers)]
        refresh = orc.is_refresh_step(t, wl.tau)
        out = orc.compress_step(t, wl.tau, wl.r, q, [synth.gradient_as_f64(g) for g in grads], e_w)
        # teacher forcing: the GPU gets the oracle's E_t (mean of the per-worker buffers) and Q_{t-1}
        e_mean = orc.worker_mean(e_w).astype(np.float32)
        case.upload([grads], [e_mean], [q.astype(np.float32)])
        case.compress(refresh=refresh)
        p_gpu, q_gpu, e_gpu = case.outputs(0)
        ref_e = orc.compress_step(t, wl.tau, wl.r, q.astype(np.float32).astype(np.float64),
                                  [synth.gradient_as_f64(g) for g in grads], [e_mean.astype(np.float64)] * wl.n_workers)
        errs = {"E": orc.rel_fro(e_gpu, ref_e.e_mean)}
        if refresh:
            # the r = 4 cut of this workload lies inside the noise bulk (sigma_4 ~ sigma_5): the
            # subspace itself is ill-conditioned, so compare what is well-posed: the captured energy
            s = ref_e.comp.sigma
            tail = float(np.sum(s[wl.r:] ** 2))
            errs["tail"] = abs(float(np.sum(e_gpu ** 2)) - tail) / float(np.sum(s ** 2))
            assert errs["tail"] <= 1e-4, (t, errs)
        else:
            errs["P"] = orc.rel_fro(p_gpu, ref_e.comp.p_tilde)
            errs["Q"] = orc.rel_fro(q_gpu, ref_e.comp.q)
            assert max(errs.values()) <= 1e-4, (t, errs)
        for k, v in errs.items():
            worst[k] = max(worst.get(k, 0.0), v)
        e_w, q = out.e_next, out.comp.q
    print("config1 trajectory worst", worst)


# ------------------------------------------------------------------ refresh (SVD-Comp)
def test_refresh_prescribed_svd():
    torch = torch_mod()
    m, n, r = 1536, 640, 16
    sigma = np.concatenate([np.linspace(2.0, 1.0, r), 0.5 * 0.9 ** np.arange(48)])
    mat, u, v = synth.prescribed_svd_matrix(m, n, sigma, seed=11, noise_std=1e-6)
    comp = psgd.Compressor([(m, n, r, psgd.PSGD_F32)], 1)
    M = to_dev_f32(mat)
    P = torch.empty((m, r), device="cuda")
    Q = torch.empty((n, r), device="cuda")
    S = torch.empty((r,), device="cuda")
    comp.refresh(0, M, P, Q, S)
    torch.cuda.synchronize()
    out = orc.svd_comp([mat.astype(np.float64)], r)
    p_gpu, q_gpu = back(P), back(Q)
    assert orc.sin_theta_max(out.p_tilde, p_gpu) <= 1e-4
    assert orc.sin_theta_max(u[:, :r], p_gpu) <= 1e-3            # the prescribed factors (noise perturbs them)
    np.testing.assert_allclose(back(S), out.sigma[:r], rtol=1e-4)
    assert orc.rel_fro(p_gpu @ q_gpu.T, out.delta_hat) <= 1e-4
    assert np.abs(p_gpu.T @ p_gpu - np.eye(r)).max() < 2e-5
    # columns are the Ritz vectors in order: Q = V_r Sigma_r up to sign
    signs = np.sign(np.sum(p_gpu * out.p_tilde, axis=0))
    assert orc.rel_fro(q_gpu * signs[None, :], out.q) <= 1e-3
    st = comp.status(0)
    assert st.rank_deficient == 0
    assert st.sigma_max == pytest.approx(out.sigma[0], rel=1e-4)
    assert st.sigma_r == pytest.approx(out.sigma[r - 1], rel=1e-4)
    # the first refresh ran the maximum (16) and left the count its spectrum needs: block width 24,
    # (sigma_24 / sigma_16)^2 ~ 0.057 per iteration -> ceil(log 1e-5 / log 0.057) + 1 = 6
    assert 4 <= st.refresh_iters_next <= 7
    P.fill_(float("nan")); Q.fill_(float("nan"))
    comp.refresh(0, M, P, Q, S)                      # second refresh: fewer iterations, same bar
    torch.cuda.synchronize()
    assert orc.sin_theta_max(out.p_tilde, back(P)) <= 1e-4
    assert orc.rel_fro(back(P) @ back(Q).T, out.delta_hat) <= 1e-4


def test_refresh_step_config2_shape_small_and_transposed():
    wl = synth.scaled_down(synth.config2(), 768, 512)
    print(_run_case(wl, refresh=True))
    wl = synth.scaled_down(synth.config2(), 512, 768)
    print(_run_case(wl, refresh=True))


def test_refresh_exact_rank_r_gives_zero_error():
    torch = torch_mod()
    m, n, r = 512, 256, 8
    mat, _, _ = synth.prescribed_svd_matrix(m, n, np.linspace(3, 1, r), seed=5)
    case = Case([(m, n)], r, 1, synth.F32)
    case.upload([[mat]], [np.zeros((m, n), np.float32)], [synth.initial_q(n, r, 1)])
    case.compress(refresh=True)
    _, _, e = case.outputs(0)
    assert np.linalg.norm(e) <= 2e-5 * np.linalg.norm(mat)
    case.upload([[mat]], [np.zeros((m, n), np.float32)], [synth.initial_q(n, r, 1)])
    case.compress(refresh=False)
    _, _, e = case.outputs(0)
    assert np.linalg.norm(e) <= 2e-5 * np.linalg.norm(mat)


# ------------------------------------------------------------------ decompress
@pytest.mark.parametrize("rows,cols", [(640, 384), (200, 328)])
def test_decompress_matches_outer_product(rows, cols):
    torch = torch_mod()
    r = 12
    m, n = max(rows, cols), min(rows, cols)
    rng = np.random.default_rng(3)
    p = rng.standard_normal((m, r)).astype(np.float32)
    q = rng.standard_normal((n, r)).astype(np.float32)
    comp = psgd.Compressor([(rows, cols, r, psgd.PSGD_F32)], 1)
    P, Q = to_dev_f32(p), to_dev_f32(q)
    ref = logical(orc.decompress(p, q), rows, cols)       # stored orientation
    out32 = torch.full((rows, cols), float("nan"), device="cuda")
    comp.decompress([P], [Q], [out32], psgd.PSGD_F32)
    out16 = torch.full((rows, cols), float("nan"), device="cuda", dtype=torch.bfloat16)
    comp.decompress([P], [Q], [out16], psgd.PSGD_BF16)
    torch.cuda.synchronize()
    assert orc.rel_fro(back(out32), ref) <= 1e-5
    assert orc.rel_fro(back(out16), ref) <= 4e-3          # bf16 rounding of the output (2^-9 per element)


# ------------------------------------------------------------------ degenerate inputs
def test_rank_deficient_projection_is_flagged_and_projector_stays_valid():
    m, n, r = 384, 256, 4
    mat, _, _ = synth.prescribed_svd_matrix(m, n, [2.0, 1.0], seed=9)      # rank 2 < r
    case = Case([(m, n)], r, 1, synth.F32)
    case.upload([[mat]], [np.zeros((m, n), np.float32)], [synth.initial_q(n, r, 2)])
    case.compress()
    p, q, e = case.outputs(0)
    st = case.comp.status(0)
    assert st.rank_deficient == 2
    assert np.all(p[:, 2:] == 0)
    np.testing.assert_allclose(p[:, :2].T @ p[:, :2], np.eye(2), atol=2e-5)
    assert np.linalg.norm(e - (mat - p @ (p.T @ mat))) <= 1e-4 * np.linalg.norm(mat)
    assert np.linalg.norm(e) <= 2e-5 * np.linalg.norm(mat)


def test_zero_gradient_gives_zero_outputs():
    m, n, r = 256, 128, 4
    case = Case([(m, n)], r, 2, synth.F32)
    z = np.zeros((m, n), np.float32)
    case.upload([[z, z]], [z], [synth.initial_q(n, r, 3)])
    case.compress()
    p, q, e = case.outputs(0)
    assert np.all(p == 0) and np.all(q == 0) and np.all(e == 0)
    assert case.comp.status(0).rank_deficient == r


def test_abi_rejects_misaligned_pointers():
    torch = torch_mod()
    case = Case([(256, 128)], 4, 1, synth.F32)
    buf = torch.zeros(256 * 128 + 4, device="cuda")
    g = buf[1:1 + 256 * 128].view(256, 128)          # 4-byte aligned only
    e = torch.zeros((256, 128), device="cuda")
    q = torch.zeros((128, 4), device="cuda")
    p = torch.zeros((256, 4), device="cuda")
    with pytest.raises(psgd.PsgdError) as ei:
        case.comp.compress([[g]], [e], [q], [p])
    assert ei.value.code == psgd.PSGD_E_ALIGN


# ------------------------------------------------------------------ full-size layer shapes of configs 3 and 4
@pytest.mark.parametrize("cfg,rows,cols", [("c3", 2048, 2048), ("c3", 5632, 2048), ("c3", 2048, 5632),
                                           ("c4", 4096, 4096), ("c4", 11008, 4096)])
def test_llm_layer_shapes_full_size_ssp_step(cfg, rows, cols):
    """One matrix of each distinct shape of the 1B-style (bf16, r = 32, N = 4) and 7B-shaped
    (bf16, r = 64, N = 1) layer sets, at full size, against the oracle element by element."""
    base = synth.config3() if cfg == "c3" else synth.config4()
    wl = synth.scaled_down(base, rows, cols)
    print(cfg, rows, cols, _run_case(wl))


# ------------------------------------------------------------------ full size (config 2), bench launch configuration
def test_config2_full_size_ssp_step():
    wl = synth.config2()
    spec = wl.layers[0]
    grads, errs, qs = _workload_inputs(wl, err_scale=1.0)
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype)
    case.upload(grads, errs, qs)
    case.compress()
    w = _check_step(case, wl, grads, errs, qs, False, 1e-4)
    print("config2 full", w)


def test_config2_full_size_refresh_step():
    """SVD-Comp step at config 2's size and worker count, against the oracle's SVD of the 4096 x 4096 mean."""
    wl = synth.config2()
    spec = wl.layers[0]
    grads, errs, qs = _workload_inputs(wl, err_scale=1.0)
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype)
    case.upload(grads, errs, qs)
    case.compress(refresh=True)
    print("config2 full refresh", _check_step(case, wl, grads, errs, qs, True, 1e-4))


def test_config2_full_size_refresh_schedule_adaptive_count():
    """Error-feedback schedule at config 2's size with a refresh at t = 0, 2, 4 and SSP steps in between, the
    library keeping its own E and Q.  The later refreshes run the iteration count the layer chose from its own
    Ritz values (fewer than the budget of 16); each is compared with the oracle's SVD-Comp of the same
    M = mean G_t + E_t, E_t read back from the device before the step."""
    wl = synth.config2()
    spec = wl.layers[0]
    sig = synth.signal_matrix(spec, wl, 0)
    grads, errs, qs = _workload_inputs(wl, err_scale=0.3)
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype)
    case.upload(grads, errs, qs)
    worst = 0.0
    for t in range(5):
        if t > 0:
            grads = [[synth.worker_gradient(spec, wl, 0, w, t, sig) for w in range(wl.n_workers)]]
            case.G = [[to_dev_grad(g, case.lds[0]) for g in grads[0]]]
        refresh = t % 2 == 0
        if refresh and t > 0:
            e_before = back(case.E[0], spec.cols)
            k_used = case.comp.status(0).refresh_iters_next
            assert 2 <= k_used < 16, k_used
        case.compress(refresh=refresh)
        if refresh and t > 0:
            g, e = oracle_inputs(grads[0], e_before, spec.rows, spec.cols, wl.n_workers)
            out = orc.compress_step(0, 1, wl.r, back(case.Q[0]), g, e)
            p_gpu, q_gpu, e_gpu = case.outputs(0)
            sn = orc.sin_theta_max(out.comp.p_tilde, p_gpu)
            worst = max(worst, sn)
            assert sn <= 1e-4, (t, k_used, sn)
            assert orc.rel_fro(p_gpu @ q_gpu.T, out.comp.delta_hat) <= 1e-4
            assert orc.rel_fro(e_gpu, out.e_mean) <= 1e-4
    print("config2 refresh schedule, worst sin", worst)


def test_refresh_step_bf16_gradients():
    """SVD-Comp with bf16 gradients (four workers, r = 32, normal and transposed storage): the oracle sees the
    same bf16 values, so the subspace bar is the same 1e-4; E and Delta_hat are held to the bf16 bar."""
    for rows, cols in ((640, 384), (384, 1024)):
        wl = synth.scaled_down(synth.config3(), rows, cols)
        print(rows, cols, _run_case(wl, refresh=True))


def test_config5_full_size_refresh_known_factors():
    """8192 x 8192 fp32, r = 128 (config 5's refresh at full size).  The matrix is built from prescribed
    factors, M = U diag(s) V^T with a gap after s_128, so the answer is known without an SVD of this size:
    span(P~) = span(U[:, :128]), sigma = s[:128], and E = M - P~ P~^T M has squared norm sum_{k>128} s_k^2
    (Eq. (6))."""
    torch = torch_mod()
    m = n = 8192
    r = 128
    sigma = np.concatenate([np.linspace(2.0, 1.0, r), 0.6 * 0.97 ** np.arange(128)])
    mat, u, v = synth.prescribed_svd_matrix(m, n, sigma, seed=21)
    comp = psgd.Compressor([(m, n, r, psgd.PSGD_F32)], 1)
    M = to_dev_f32(mat)
    P = torch.empty((m, r), device="cuda")
    Q = torch.empty((n, r), device="cuda")
    S = torch.empty((r,), device="cuda")
    comp.refresh(0, M, P, Q, S)
    torch.cuda.synchronize()
    p_gpu, q_gpu = back(P), back(Q)
    assert np.abs(p_gpu.T @ p_gpu - np.eye(r)).max() < 2e-5
    assert orc.sin_theta_max(u[:, :r], p_gpu) <= 1e-4
    np.testing.assert_allclose(back(S), sigma[:r], rtol=1e-4)
    # Q = M^T P~ and the residual norm, from the factors (fp64): M^T P~ = V diag(s) (U^T P~)
    utp = u.T @ p_gpu
    q_ref = (v * sigma[None, :]) @ utp
    assert orc.rel_fro(q_gpu, q_ref) <= 1e-4
    res2 = float(np.sum(sigma ** 2) - np.sum((sigma[:, None] * utp) ** 2))      # ||M||^2 - ||P~^T M||^2
    assert abs(res2 - float(np.sum(sigma[r:] ** 2))) <= 1e-4 * float(np.sum(sigma[r:] ** 2))
    assert comp.status(0).rank_deficient == 0


def test_widest_block_r150():
    """r = 150: the subspace iteration's block is 192 wide, the widest the library plans for (six MFMA column
    blocks, the unblocked fall-back of the factorisation, the largest Rayleigh-Ritz problem), and the SSP step
    runs at 160 packed columns."""
    torch = torch_mod()
    m, n, r = 1024, 640, 150
    sigma = np.concatenate([np.linspace(2.0, 1.0, r), 0.5 * 0.97 ** np.arange(100)])
    mat, u, v = synth.prescribed_svd_matrix(m, n, sigma, seed=31)
    comp = psgd.Compressor([(m, n, r, psgd.PSGD_F32)], 1)
    M = to_dev_f32(mat)
    P = torch.empty((m, r), device="cuda")
    Q = torch.empty((n, r), device="cuda")
    S = torch.empty((r,), device="cuda")
    comp.refresh(0, M, P, Q, S)
    torch.cuda.synchronize()
    p_gpu, q_gpu = back(P), back(Q)
    assert np.abs(p_gpu.T @ p_gpu - np.eye(r)).max() < 2e-5
    assert orc.sin_theta_max(u[:, :r], p_gpu) <= 1e-4
    np.testing.assert_allclose(back(S), sigma[:r], rtol=1e-4)
    assert orc.rel_fro(q_gpu, mat.astype(np.float64).T @ p_gpu) <= 1e-4
    # one SSP step from the refreshed Q against the oracle
    case = Case([(m, n)], r, 1, synth.F32)
    case.upload([[mat]], [np.zeros((m, n), np.float32)], [q_gpu.astype(np.float32)])
    case.compress()
    out = orc.compress_step(1, None, r, q_gpu.astype(np.float32).astype(np.float64), [mat.astype(np.float64)],
                            [np.zeros((m, n))])
    p2, q2, e2 = case.outputs(0)
    assert orc.rel_fro(p2, out.comp.p_tilde) <= 1e-4 and orc.rel_fro(q2, out.comp.q) <= 1e-4
    assert orc.rel_fro(e2, out.e_mean) <= 1e-4


@pytest.mark.parametrize("r", [1, 2, 3, 5, 13, 16, 20, 24, 40, 70, 84, 100, 128, 150])
def test_rank_sweep_ssp_and_refresh(r):
    """Every width path of the thin kernels: odd and tiny ranks (the register factorisation at compiled widths
    4, 8, 12, 16, non-vectorised thin rows), the LDS path, the blocked one with a ragged last block; refresh block
    widths 88, 112, 128, 160 and 192 take the Jacobi kernel through one to five 2 x 2 blocks per thread."""
    m, n = 640, 384
    sigma = np.concatenate([np.linspace(2.0, 1.0, r), 0.4 * 0.9 ** np.arange(40)])
    mat, u, v = synth.prescribed_svd_matrix(m, n, sigma, seed=100 + r, noise_std=1e-6)
    q0 = synth.initial_q(n, r, 77)
    g = [mat.astype(np.float64)]
    e = [np.zeros((m, n))]
    for refresh in (False, True):
        case = Case([(m, n)], r, 1, synth.F32)
        case.upload([[mat]], [np.zeros((m, n), np.float32)], [q0])
        case.compress(refresh=refresh)
        out = orc.compress_step(0 if refresh else 1, 1 if refresh else None, r, q0.astype(np.float64), g, e)
        p_gpu, q_gpu, e_gpu = case.outputs(0)
        assert np.abs(p_gpu.T @ p_gpu - np.eye(r)).max() < 2e-5
        assert orc.rel_fro(e_gpu, out.e_mean) <= 1e-4, (r, refresh)
        if refresh:
            assert orc.sin_theta_max(out.comp.p_tilde, p_gpu) <= 1e-4, (r, refresh)
            assert orc.rel_fro(p_gpu @ q_gpu.T, out.comp.delta_hat) <= 1e-4
        else:
            assert orc.rel_fro(p_gpu, out.comp.p_tilde) <= 1e-4 and orc.rel_fro(q_gpu, out.comp.q) <= 1e-4, (r, refresh)


# ------------------------------------------------------------------ decompress fused with the momentum update
@pytest.mark.parametrize("rows,cols,dtype", [(640, 384, synth.F32), (200, 328, synth.F32), (1000, 264, synth.BF16)])
def test_decompress_msgd_matches_eq_7c(rows, cols, dtype):
    """m <- mu m + P~ Q^T, X <- X - eta m (Eq. (7c)) against the oracle's update applied to the oracle's
    Delta_hat, over two steps so that the momentum term is exercised (normal, transposed and ragged storage)."""
    torch = torch_mod()
    r, mu, eta = 12, 0.9, 0.05
    m, n = max(rows, cols), min(rows, cols)
    rng = np.random.default_rng(17)
    case = Case([(rows, cols)], r, 1, dtype)
    x_ref = rng.standard_normal((rows, cols))
    mom_ref = np.zeros((rows, cols))
    X = [to_dev_f32(x_ref.astype(np.float32))]
    MOM = [to_dev_f32(mom_ref.astype(np.float32))]
    x_ref = x_ref.astype(np.float32).astype(np.float64)
    for step in range(2):
        p = np.linalg.qr(rng.standard_normal((m, r)))[0].astype(np.float32)
        q = rng.standard_normal((n, r)).astype(np.float32)
        P, Q = [to_dev_f32(p)], [to_dev_f32(q)]
        case.comp.decompress_msgd(P, Q, MOM, X, mu, eta)
        torch.cuda.synchronize()
        dhat = orc.decompress(p.astype(np.float64), q.astype(np.float64))          # logical m x n
        dhat = dhat.T if rows < cols else dhat                                     # storage orientation
        x_ref, mom_ref = orc.msgd_update(x_ref, mom_ref, dhat, eta, mu)
        assert orc.rel_fro(back(MOM[0], cols), mom_ref) <= 1e-5, step
        assert orc.rel_fro(back(X[0], cols), x_ref) <= 1e-5, step


# ------------------------------------------------------------------ decompress fused with Adam / AdamW
@pytest.mark.parametrize("rows,cols,dtype,r,wd", [(640, 384, synth.F32, 12, 0.0), (200, 328, synth.F32, 12, 0.05),
                                                  (1000, 264, synth.BF16, 40, 0.01), (384, 512, synth.BF16, 64, 0.0)])
def test_decompress_adam_matches_published_update(rows, cols, dtype, r, wd):
    """Adam moments and weights from Delta_hat = P~ Q^T over three steps (bias corrections of steps 1..3, both
    moments carried over), against the oracle's update applied to the oracle's Delta_hat.  The step itself,
    X_t - X_{t-1}, is compared as well: relative to X it would pass even if it were wrong by a factor."""
    torch = torch_mod()
    eta, b1, b2, eps = 0.01, 0.9, 0.999, 1e-8
    m, n = max(rows, cols), min(rows, cols)
    rng = np.random.default_rng(23)
    case = Case([(rows, cols)], r, 1, dtype)
    x_ref = rng.standard_normal((rows, cols)).astype(np.float32).astype(np.float64)
    m1_ref, m2_ref = np.zeros((rows, cols)), np.zeros((rows, cols))
    X, M1, M2 = [to_dev_f32(x_ref.astype(np.float32))], [to_dev_f32(m1_ref.astype(np.float32))], [to_dev_f32(m2_ref.astype(np.float32))]
    posed = np.ones((rows, cols), dtype=bool)
    for step in range(1, 4):
        p = np.linalg.qr(rng.standard_normal((m, r)))[0].astype(np.float32)
        q = (rng.standard_normal((n, r)) * 0.9 ** np.arange(r)).astype(np.float32)
        P, Q = [to_dev_f32(p)], [to_dev_f32(q)]
        x_before = back(X[0], cols)
        case.comp.decompress_adam(P, Q, M1, M2, X, step, eta, b1, b2, eps, wd)
        torch.cuda.synchronize()
        dhat = orc.decompress(p.astype(np.float64), q.astype(np.float64))          # logical m x n
        dhat = dhat.T if rows < cols else dhat                                     # storage orientation
        x_new, m1_ref, m2_ref = orc.adam_update(x_ref, m1_ref, m2_ref, dhat, step, eta, b1, b2, eps, wd)
        assert orc.rel_fro(back(M1[0], cols), m1_ref) <= 1e-5, step
        assert orc.rel_fro(back(M2[0], cols), m2_ref) <= 3e-5, step      # D.D carries twice D's relative error
        # Adam's step m^ / (sqrt(v^) + eps) is sign(D) at step 1 and stays discontinuous wherever the D's seen so
        # far vanish together: an entry of D smaller than D's own error bar (split-bf16 operands, 2^-16 of
        # |P~||Q| with two planes) has no well-defined step.  Those few entries are only held to Adam's bound
        # on a step; all others are compared.
        posed &= np.abs(dhat) > 1e-3 * np.sqrt(np.mean(dhat * dhat))
        assert posed.mean() > 0.99
        x_gpu = back(X[0], cols)
        assert np.linalg.norm((x_gpu - x_new)[posed]) <= 1e-6 * np.linalg.norm(x_new[posed]), step
        # fp32 weights: the step is known to about ulp(X) / |step| ~ 6e-8 / 1e-2 per entry
        assert np.linalg.norm(((x_gpu - x_before) - (x_new - x_ref))[posed]) <= 1e-4 * np.linalg.norm((x_new - x_ref)[posed]), step
        assert np.abs(x_gpu - x_new).max() <= 10 * eta * step
        x_ref = x_new


def test_decompress_adam_batched_and_rejected_arguments():
    """All layers of a mixed batch in one call; the argument checks of the entry point."""
    torch = torch_mod()
    shapes = [(256, 256), (704, 256), (256, 704), (200, 136)]
    r = 32
    rng = np.random.default_rng(29)
    case = Case(shapes, r, 1, synth.BF16)
    P, Q, X, M1, M2, refs = [], [], [], [], [], []
    for rows, cols in shapes:
        m, n = max(rows, cols), min(rows, cols)
        p = np.linalg.qr(rng.standard_normal((m, r)))[0].astype(np.float32)
        q = rng.standard_normal((n, r)).astype(np.float32)
        x = rng.standard_normal((rows, cols)).astype(np.float32)
        m1 = (0.1 * rng.standard_normal((rows, cols))).astype(np.float32)
        # second moment bounded away from zero: where it and D both vanish the step m^ / sqrt(v^) is ill-conditioned
        m2 = (0.01 + 0.1 * rng.standard_normal((rows, cols)) ** 2).astype(np.float32)
        P.append(to_dev_f32(p)); Q.append(to_dev_f32(q)); X.append(to_dev_f32(x)); M1.append(to_dev_f32(m1)); M2.append(to_dev_f32(m2))
        dhat = orc.decompress(p.astype(np.float64), q.astype(np.float64))
        dhat = dhat.T if rows < cols else dhat
        refs.append(orc.adam_update(x.astype(np.float64), m1.astype(np.float64), m2.astype(np.float64), dhat, 7, 0.003,
                                    0.9, 0.95, 1e-6, 0.1))
    case.comp.decompress_adam(P, Q, M1, M2, X, 7, 0.003, 0.9, 0.95, 1e-6, 0.1)
    torch.cuda.synchronize()
    for l, (rows, cols) in enumerate(shapes):
        x_ref, m1_ref, m2_ref = refs[l]
        assert orc.rel_fro(back(M1[l], cols), m1_ref) <= 1e-5, l
        assert orc.rel_fro(back(M2[l], cols), m2_ref) <= 3e-5, l
        assert orc.rel_fro(back(X[l], cols), x_ref) <= 1e-6, l
    for bad in (dict(step=0), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=-1.0), dict(eta=float("nan"))):
        args = dict(step=1, eta=0.01, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)
        args.update(bad)
        with pytest.raises(psgd.PsgdError):
            case.comp.decompress_adam(P, Q, M1, M2, X, **args)


# ------------------------------------------------------------------ K-step power iteration (Eq. (8))
@pytest.mark.parametrize("k_steps,m_policy", [(2, 0), (3, 0), (2, 2)])
def test_k_step_power_iteration(k_steps, m_policy):
    """psgd_options.power_iters = K: P~_k = QR(M Q_{k-1}), Q_k = M^T P~_k, K times, then E = M - P~ Q^T."""
    wl = synth.scaled_down(synth.config1(), 640, 384)
    wl.r = 8
    grads, errs, qs = _workload_inputs(wl)
    spec = wl.layers[0]
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype, power_iters=k_steps, m_policy=m_policy)
    case.upload(grads, errs, qs)
    case.compress()
    g, e = oracle_inputs(grads[0], errs[0], spec.rows, spec.cols, wl.n_workers)
    mat = orc.worker_mean([gi + ei for gi, ei in zip(g, e)])
    p_ref, q_ref = orc.power_iteration(mat, qs[0].astype(np.float64), k_steps)
    p_gpu, q_gpu, e_gpu = case.outputs(0)
    assert orc.rel_fro(p_gpu, p_ref) <= 1e-4 and orc.rel_fro(q_gpu, q_ref) <= 1e-4
    assert orc.rel_fro(e_gpu, mat - p_ref @ q_ref.T) <= 1e-4
    # more steps never capture less (the projection onto span(P~_k) is the one of a power step)
    if k_steps > 1:
        p1, q1 = orc.power_iteration(mat, qs[0].astype(np.float64), 1)
        assert np.linalg.norm(e_gpu) <= np.linalg.norm(mat - p1 @ q1.T) * (1 + 1e-6)


def test_rotating_gradient_buffers_more_than_table_slots():
    """The library keeps the last few gradient pointer tables on the device; six distinct buffer sets visited
    twice in turn (more sets than slots, so tables are evicted and re-uploaded) must all give their own result."""
    torch = torch_mod()
    wl = synth.scaled_down(synth.config1(), 256, 128)
    spec = wl.layers[0]
    sig = synth.signal_matrix(spec, wl, 0)
    sets = [[synth.worker_gradient(spec, wl, 0, w, 100 + s, sig) for w in range(wl.n_workers)] for s in range(6)]
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype)
    dev_sets = [[to_dev_grad(g, spec.cols) for g in gs] for gs in sets]
    q0 = synth.initial_q(spec.n, wl.r, wl.seed, 0)
    e0 = np.zeros((spec.rows, spec.cols), np.float32)
    for visit in range(2):
        for s in range(6):
            case.upload([sets[s]], [e0], [q0])
            case.G = [dev_sets[s]]                       # a different set of device buffers every call
            case.compress()
            g, e = oracle_inputs(sets[s], e0, spec.rows, spec.cols, wl.n_workers)
            out = orc.compress_step(1, None, wl.r, q0.astype(np.float64), g, e)
            p_gpu, q_gpu, e_gpu = case.outputs(0)
            assert orc.rel_fro(e_gpu, out.e_mean) <= 1e-4 and orc.rel_fro(q_gpu, out.comp.q) <= 1e-4, (visit, s)


def test_refresh_as_randomized_range_finder():
    """refresh_iters = 1 with a random start is the randomized range finder (sketch Y = M Omega, orthonormalise,
    project, small SVD): one pass captures the range of a matrix whose rank is within the block width exactly,
    and on a decaying spectrum it is within a small factor of the optimal rank-r error (Eq. (6))."""
    torch = torch_mod()
    m, n, r = 768, 512, 8
    mat, _, _ = synth.prescribed_svd_matrix(m, n, np.linspace(3, 1, 12), seed=9)      # rank 12 <= block width 16
    case = Case([(m, n)], r, 1, synth.F32, refresh_iters=1, refresh_warm_start=False)
    case.upload([[mat]], [np.zeros((m, n), np.float32)], [synth.initial_q(n, r, 1)])
    case.compress(refresh=True)
    p, q, e = case.outputs(0)
    out = orc.svd_comp([mat.astype(np.float64)], r)
    assert orc.sin_theta_max(out.p_tilde, p) <= 1e-4               # exact: the sketch spans the whole range
    assert orc.rel_fro(e, mat.astype(np.float64) - out.delta_hat) <= 1e-4
    sigma = 0.85 ** np.arange(64)
    mat, _, _ = synth.prescribed_svd_matrix(m, n, sigma, seed=10)
    case.upload([[mat]], [np.zeros((m, n), np.float32)], [synth.initial_q(n, r, 1)])
    case.compress(refresh=True)
    _, _, e = case.outputs(0)
    opt = float(np.sum(sigma[r:] ** 2))
    assert opt * (1 - 1e-6) <= float(np.sum(e ** 2)) <= 1.5 * opt      # never below the optimum, close above it


def test_range_finder_result_against_the_oracle():
    """The same compressor result against result: the oracle's randomized range finder is given the Omega the
    library draws (same counter-based generator, seed and layer), so P~ (as a subspace), Delta_hat, Q and E must agree
    to the usual bars -- with oversampling (block 16 for r = 8), normal and transposed storage, two layers."""
    seed = 0x1234ABCD
    shapes = [(640, 384), (256, 520)]
    r, nw = 8, 2
    wl = synth.scaled_down(synth.config2(), 640, 384)
    wl.layers = [synth.LayerSpec(rw, cl, "l%d" % i) for i, (rw, cl) in enumerate(shapes)]
    wl.r = r
    wl.n_workers = nw
    grads, errs, qs = _workload_inputs(wl, err_scale=1.0)
    case = Case(shapes, r, nw, synth.F32, refresh_iters=1, refresh_warm_start=False, seed=seed)
    case.upload(grads, errs, qs)
    case.compress(refresh=True)
    for l, (rows, cols) in enumerate(shapes):
        g, e = oracle_inputs(grads[l], errs[l], rows, cols, nw)
        deltas = orc.ef_accumulate(g, e)
        omega = orc.counter_uniform(seed, l, min(rows, cols), 16)
        ref = orc.range_finder_comp(deltas, r, omega)
        p_gpu, q_gpu, e_gpu = case.outputs(l)
        e_gpu = logical(e_gpu, rows, cols)
        assert np.abs(p_gpu.T @ p_gpu - np.eye(r)).max() < 2e-5
        assert orc.sin_theta_max(ref.p_tilde, p_gpu) <= 1e-4, l
        assert orc.rel_fro(p_gpu @ q_gpu.T, ref.delta_hat) <= 1e-4, l
        assert orc.rel_fro(e_gpu, orc.worker_mean(deltas) - ref.delta_hat) <= 1e-4, l
        # the Ritz vectors come in the order of the small SVD: column by column up to sign where the values are apart
        sg = ref.sigma
        for k in range(r):
            if min(abs(sg[k] - sg[j]) for j in range(len(sg)) if j != k) > 1e-3 * sg[0]:
                c = float(ref.p_tilde[:, k] @ p_gpu[:, k])
                assert abs(abs(c) - 1.0) <= 1e-4, (l, k, c)


def test_config5_bf16_full_size_refresh_step():
    """Config 5's other half: 8192 x 8192 bf16 gradient, r = 128, one SVD-Comp step through psgd_compress_refresh
    (forming pass from bf16, two operand planes, block width 160).  The gradient is a matrix with prescribed factors and
    a gap after sigma_128, rounded to bf16; the oracle works on those bf16 values (svd_comp_large: a dense SVD of this
    size takes minutes) and asserts its own certificate."""
    torch = torch_mod()
    m = n = 8192
    r = 128
    sigma = np.concatenate([np.linspace(2.0, 1.0, r), 0.6 * 0.97 ** np.arange(128)])
    mat, _, _ = synth.prescribed_svd_matrix(m, n, sigma, seed=23)
    bits = synth.round_to_bf16(mat)
    del mat
    g64 = synth.gradient_as_f64(bits)
    ref, resid = orc.svd_comp_large([g64], r, oversample=64)
    assert resid <= 1e-9, resid
    comp = psgd.Compressor([(m, n, r, psgd.PSGD_BF16)], 1)
    G = [[to_dev_grad(bits)]]
    E = [torch.zeros((m, n), device="cuda")]
    Q = [to_dev_f32(synth.initial_q(n, r, 5))]
    P = [torch.empty((m, r), device="cuda")]
    comp.compress_refresh(G, E, Q, P)
    torch.cuda.synchronize()
    p_gpu, q_gpu = back(P[0]), back(Q[0])
    assert np.abs(p_gpu.T @ p_gpu - np.eye(r)).max() < 2e-5
    sn = orc.sin_theta_max(ref.p_tilde, p_gpu)
    assert sn <= 1e-4, sn
    assert orc.rel_fro(q_gpu, g64.T @ p_gpu) <= 1e-4                      # Q = M^T P~ for the P~ it returned
    d_gpu = p_gpu @ q_gpu.T
    err_d = orc.rel_fro(d_gpu, ref.delta_hat)
    e_ref = g64 - ref.delta_hat
    err_e = orc.rel_fro(back(E[0]), e_ref)
    print("config 5 bf16 refresh: sin", sn, "Delta_hat", err_d, "E", err_e)
    assert err_d <= 2e-2 and err_e <= 2e-2
    st = comp.status(0)
    assert st.rank_deficient == 0 and abs(st.sigma_max - ref.sigma[0]) <= 1e-3 * ref.sigma[0]


# ------------------------------------------------------------------ single-worker variants of the forming passes
@pytest.mark.parametrize("rows,cols,dtype,r", [(520, 328, synth.F32, 8), (328, 520, synth.F32, 8), (333, 203, synth.BF16, 40),
                                               (264, 1000, synth.BF16, 64), (640, 512, synth.F32, 128)])
def test_single_worker_forming_passes(rows, cols, dtype, r):
    """N = 1 selects kernels compiled without the loop over further gradient buffers (row and column mode, both
    operand precisions): one SSP step and one SVD-Comp step against the oracle."""
    base = synth.config4() if dtype == synth.BF16 else synth.config2()
    wl = synth.scaled_down(base, rows, cols)
    wl.n_workers = 1
    wl.r = r
    lds = [(cols + 7) // 8 * 8]
    print("ssp", _run_case(wl, lds=lds))
    if r <= 40:      # at these small shapes a wider cut lies inside the noise bulk: no gap, no subspace to compare
        print("refresh", _run_case(wl, refresh=True, lds=lds))
