"""GPU parity of the deferred residual (psgd_options.lazy_residual = 1): free-running trajectories of
psgd_compress against the fp64 oracle's own trajectory of Algorithm 2.

With the option on, psgd_compress leaves M_t in the E buffers of the layers stored with rows >= cols and the next
forming pass applies E_{t+1} = M_t - P~_t Q_t^T (Algorithm 2, error update) on the way; psgd_flush_residual
materialises it.  Every step's P~ and Q, M_t as found in the E buffer before the flush, and E after it are compared.
"""
import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2509_11254_amd import psgd, synth
from gpu_harness import Case, back, logical, to_dev_grad, torch_mod

pytestmark = pytest.mark.gpu

TOL = {synth.F32: 1e-4, synth.BF16: 2e-2}


def _layers_inputs(wl, step):
    out = []
    for l, spec in enumerate(wl.layers):
        sig = synth.signal_matrix(spec, wl, l)
        out.append([synth.worker_gradient(spec, wl, l, w, step, sig) for w in range(wl.n_workers)])
    return out


def _trajectory(wl, steps, lds=None, refresh_at=(), check_m=True, **opts):
    """Free-running: the GPU keeps its own E and Q from step to step, and so does the oracle."""
    torch = torch_mod()
    tol = TOL[wl.grad_dtype]
    case = Case([(s.rows, s.cols) for s in wl.layers], wl.r, wl.n_workers, wl.grad_dtype, lds=lds,
                lazy_residual=True, **opts)
    nl = len(wl.layers)
    rng = np.random.default_rng([wl.seed, 4242])
    errs0 = [(0.3 * synth.noise_sigma(s, wl) * rng.standard_normal((s.rows, s.cols))).astype(np.float32) for s in wl.layers]
    qs0 = [synth.initial_q(s.n, wl.r, wl.seed, l) for l, s in enumerate(wl.layers)]
    grads = _layers_inputs(wl, 0)
    case.upload(grads, errs0, qs0)
    # oracle state per layer: per-worker error buffers (all equal to E_0) and Q
    e_w = [[logical(np.asarray(errs0[l], np.float64), s.rows, s.cols) for _ in range(wl.n_workers)]
           for l, s in enumerate(wl.layers)]
    q_or = [q.astype(np.float64) for q in qs0]
    worst = {}
    for t in range(steps):
        if t > 0:
            grads = _layers_inputs(wl, t)
            case.G = [[to_dev_grad(g, case.lds[l]) for g in grads[l]] for l in range(nl)]
        refresh = t in refresh_at
        case.compress(refresh=refresh)
        for l, spec in enumerate(wl.layers):
            g = [logical(synth.gradient_as_f64(gw), spec.rows, spec.cols) for gw in grads[l]]
            out = orc.compress_step(0 if refresh else 1, 1 if refresh else None, wl.r, q_or[l], g, e_w[l])
            p_gpu, q_gpu, s_gpu = case.outputs(l)
            s_gpu = logical(s_gpu, spec.rows, spec.cols)
            errs = {}
            if refresh:
                errs["sin"] = orc.sin_theta_max(out.comp.p_tilde, p_gpu)
                errs["dhat"] = orc.rel_fro(p_gpu @ q_gpu.T, out.comp.delta_hat)
                assert errs["sin"] <= 1e-4, (t, l, errs)
            else:
                errs["P"] = orc.rel_fro(p_gpu, out.comp.p_tilde)
                errs["Q"] = orc.rel_fro(q_gpu, out.comp.q)
            # layers stored with rows < cols defer too when no rank exceeds 32 (column-mode forming pass)
            deferred = (spec.rows >= spec.cols or wl.r <= 32) and not refresh
            if deferred and check_m:
                # what the option documents: the buffer holds M_t = mean_i (G^(i) + e^(i)) until the flush
                m_t = orc.worker_mean([gi + ei for gi, ei in zip(g, e_w[l])])
                errs["M"] = orc.rel_fro(s_gpu, m_t)
            elif not deferred:
                errs["E"] = orc.rel_fro(s_gpu, out.e_mean)
            for k, v in errs.items():
                worst[k] = max(worst.get(k, 0.0), v)
                if k != "sin":
                    assert v <= tol, (t, l, spec, k, errs)
            e_w[l], q_or[l] = out.e_next, out.comp.q
            if refresh:
                # Definition 3 fixes the subspace, not the signs of the Ritz vectors: the oracle carries on from
                # the library's Q and E of this step
                q_or[l] = q_gpu
                e_w[l] = [s_gpu.copy() for _ in range(wl.n_workers)]
    case.comp.flush_residual(case.E)
    torch.cuda.synchronize()
    for l, spec in enumerate(wl.layers):
        e_gpu = logical(case.outputs(l)[2], spec.rows, spec.cols)
        err = orc.rel_fro(e_gpu, orc.worker_mean(e_w[l]))
        worst["E_flushed"] = max(worst.get("E_flushed", 0.0), err)
        assert err <= tol, (l, spec, err)
    return worst


@pytest.mark.parametrize("which", ["f32_n4_ragged_r4", "bf16_n1_r64", "bf16_n4_r32", "f32_n2_r128", "f32_r40"])
@pytest.mark.parametrize("q_resident", [False, True], ids=["q_packed", "q_resident"])
def test_deferred_residual_trajectory(which, q_resident):
    """q_resident: the caller's promise not to write the Q buffers between calls, with which the forming pass takes the
    kept Q from the product's own operand fragments instead of reading the kept copies (another kernel variant)."""
    lds = None
    if which == "f32_n4_ragged_r4":
        wl = synth.scaled_down(synth.config1(), 333, 203)
        lds = [208]
    elif which == "bf16_n1_r64":
        wl = synth.scaled_down(synth.config4(), 700, 384)
    elif which == "bf16_n4_r32":
        wl = synth.scaled_down(synth.config3(), 640, 256)
    elif which == "f32_n2_r128":
        wl = synth.scaled_down(synth.config5a(), 640, 512)
        wl.n_workers = 2
    else:
        wl = synth.scaled_down(synth.config2(), 520, 328)
        wl.r = 40
    print(which, _trajectory(wl, 4, lds=lds, q_resident=q_resident))


@pytest.mark.parametrize("r", [32, 40, 5])
def test_deferred_residual_batched_with_transposed_layers(r):
    """Layers stored with rows < cols defer their residual only up to rank 32 (column-mode forming pass) and take it
    at once above; one batch holds both kinds of storage, ragged shapes included."""
    wl = synth.scaled_down(synth.config3(), 256, 256)
    wl.r = r
    wl.layers = [synth.LayerSpec(256, 256, "a"), synth.LayerSpec(704, 256, "b"), synth.LayerSpec(256, 704, "c"),
                 synth.LayerSpec(200, 136, "e"), synth.LayerSpec(136, 333, "f")]
    print(r, _trajectory(wl, 3, lds=[256, 256, 704, 136, 336]))


def test_deferred_residual_transposed_full_size():
    """The 2048 x 5632 layer of the 1B-style set (stored with rows < cols, rank 32, 4 workers), two free-running steps."""
    wl = synth.scaled_down(synth.config3(), 2048, 5632)
    print(_trajectory(wl, 2))


def test_deferred_residual_with_refresh_steps_in_between():
    """psgd_compress_refresh settles what is owed before it forms M, and leaves nothing owed."""
    wl = synth.scaled_down(synth.config2(), 512, 384)
    print(_trajectory(wl, 5, refresh_at=(0, 3)))


def test_deferred_residual_with_two_power_steps():
    wl = synth.scaled_down(synth.config1(), 640, 384)
    wl.r = 8
    torch = torch_mod()
    spec = wl.layers[0]
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype, lazy_residual=True, power_iters=2)
    e = np.zeros((spec.rows, spec.cols), np.float32)
    q = synth.initial_q(spec.n, wl.r, wl.seed, 0)
    e_or = np.zeros((spec.rows, spec.cols))
    q_or = q.astype(np.float64)
    for t in range(3):
        grads = _layers_inputs(wl, t)
        if t == 0:
            case.upload(grads, [e], [q])
        else:
            case.G = [[to_dev_grad(g, spec.cols) for g in grads[0]]]
        case.compress()
        mat = orc.worker_mean([synth.gradient_as_f64(g) for g in grads[0]]) + e_or
        p_ref, q_ref = orc.power_iteration(mat, q_or, 2)
        p_gpu, q_gpu, _ = case.outputs(0)
        assert orc.rel_fro(p_gpu, p_ref) <= 1e-4 and orc.rel_fro(q_gpu, q_ref) <= 1e-4, t
        e_or, q_or = mat - p_ref @ q_ref.T, q_ref
    case.comp.flush_residual(case.E)
    torch.cuda.synchronize()
    assert orc.rel_fro(case.outputs(0)[2], e_or) <= 1e-4


def test_flush_without_anything_owed_is_a_no_op():
    wl = synth.scaled_down(synth.config1(), 256, 128)
    spec = wl.layers[0]
    torch = torch_mod()
    for lazy in (False, True):
        case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype, lazy_residual=lazy)
        grads = _layers_inputs(wl, 0)
        e0 = np.zeros((spec.rows, spec.cols), np.float32)
        case.upload(grads, [e0], [synth.initial_q(spec.n, wl.r, wl.seed, 0)])
        case.comp.flush_residual(case.E)                 # nothing has run yet
        case.compress()
        case.comp.flush_residual(case.E)
        torch.cuda.synchronize()
        first = back(case.E[0]).copy()
        case.comp.flush_residual(case.E)                 # settled already: must not subtract twice
        torch.cuda.synchronize()
        assert np.array_equal(first, back(case.E[0]))
        g = [synth.gradient_as_f64(gw) for gw in grads[0]]
        out = orc.compress_step(1, None, wl.r, synth.initial_q(spec.n, wl.r, wl.seed, 0).astype(np.float64), g,
                                [e0.astype(np.float64)] * wl.n_workers)
        assert orc.rel_fro(first, out.e_mean) <= 1e-4


def test_lazy_option_rejects_unsupported_combinations():
    with pytest.raises(psgd.PsgdError):
        psgd.Compressor([(256, 128, 4, psgd.PSGD_F32)], 1, lazy_residual=True, m_policy=2, allocate=False)
    with pytest.raises(psgd.PsgdError):
        psgd.Compressor([(512, 512, 150, psgd.PSGD_F32)], 1, lazy_residual=True, allocate=False)


@pytest.mark.parametrize("cfg,rows,cols", [("c4", 4096, 4096), ("c4", 11008, 4096), ("c3", 5632, 2048)])
@pytest.mark.parametrize("q_resident", [False, True], ids=["q_packed", "q_resident"])
def test_deferred_residual_full_size_llm_shapes(cfg, rows, cols, q_resident):
    """Two free-running steps at the full size of a benchmark layer, so that the second forming pass applies the
    first step's residual across many row blocks and rotated chunk walks, in the benchmark's launch configuration."""
    base = synth.config3() if cfg == "c3" else synth.config4()
    wl = synth.scaled_down(base, rows, cols)
    print(cfg, rows, cols, _trajectory(wl, 2, q_resident=q_resident))


@pytest.mark.parametrize("rows,cols,dtype,r", [(328, 520, synth.F32, 8), (264, 1000, synth.BF16, 32), (1000, 264, synth.F32, 96)])
@pytest.mark.parametrize("q_resident", [False, True], ids=["q_packed", "q_resident"])
def test_deferred_residual_single_worker(rows, cols, dtype, r, q_resident):
    """N = 1 with the deferred residual: the single-worker forming kernels in row and column mode."""
    base = synth.config4() if dtype == synth.BF16 else synth.config2()
    wl = synth.scaled_down(base, rows, cols)
    wl.n_workers = 1
    wl.r = r
    print(_trajectory(wl, 3, q_resident=q_resident))


def test_flush_on_another_workspace_is_rejected():
    """The owed operands live in the workspace of the compress call: settling them from another one is an error."""
    import ctypes as C
    torch = torch_mod()
    wl = synth.scaled_down(synth.config1(), 256, 128)
    spec = wl.layers[0]
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype, lazy_residual=True)
    grads = _layers_inputs(wl, 0)
    case.upload(grads, [np.zeros((spec.rows, spec.cols), np.float32)], [synth.initial_q(spec.n, wl.r, wl.seed, 0)])
    case.compress()
    other = torch.empty(case.comp.workspace_bytes + 256, dtype=torch.uint8, device="cuda")
    other_ptr = (other.data_ptr() + 255) // 256 * 256
    te = (C.c_void_p * 1)(case.E[0].data_ptr())
    rc = case.comp.lib.psgd_flush_residual(case.comp.ctx, other_ptr, 0, te)
    assert rc == psgd.PSGD_E_INVALID_ARG
    case.comp.flush_residual(case.E)                      # the right one still settles it
    torch.cuda.synchronize()
    g = [synth.gradient_as_f64(gw) for gw in grads[0]]
    out = orc.compress_step(1, None, wl.r, synth.initial_q(spec.n, wl.r, wl.seed, 0).astype(np.float64), g,
                            [np.zeros((spec.rows, spec.cols))] * wl.n_workers)
    assert orc.rel_fro(back(case.E[0]), out.e_mean) <= 1e-4


def test_compress_on_another_workspace_while_a_residual_is_owed_is_rejected():
    """The same for the two compress calls: they would subtract the kept operands of a workspace that has none, so
    they are refused before anything is uploaded or enqueued, and the step goes on in the right workspace."""
    import ctypes as C
    torch = torch_mod()
    wl = synth.scaled_down(synth.config1(), 256, 128)
    spec = wl.layers[0]
    case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype, lazy_residual=True)
    grads = _layers_inputs(wl, 0)
    q0 = synth.initial_q(spec.n, wl.r, wl.seed, 0)
    case.upload(grads, [np.zeros((spec.rows, spec.cols), np.float32)], [q0])
    case.compress()                                       # leaves M_0 in E, the residual owed
    other = torch.empty(case.comp.workspace_bytes + 256, dtype=torch.uint8, device="cuda")
    other_ptr = (other.data_ptr() + 255) // 256 * 256
    vp = C.c_void_p
    tg = (vp * wl.n_workers)(*[g.data_ptr() for g in case.G[0]])
    te, tq, tp = (vp * 1)(case.E[0].data_ptr()), (vp * 1)(case.Q[0].data_ptr()), (vp * 1)(case.P[0].data_ptr())
    e_before, q_before = back(case.E[0]), back(case.Q[0])
    for fn in (case.comp.lib.psgd_compress, case.comp.lib.psgd_compress_refresh):
        assert fn(case.comp.ctx, other_ptr, 0, tg, te, tq, tp) == psgd.PSGD_E_INVALID_ARG
    torch.cuda.synchronize()
    assert np.array_equal(e_before, back(case.E[0])) and np.array_equal(q_before, back(case.Q[0]))   # nothing ran
    # the run continues in its own workspace: step 1 of the oracle's trajectory
    case.compress()
    case.comp.flush_residual(case.E)
    torch.cuda.synchronize()
    g = [synth.gradient_as_f64(gw) for gw in grads[0]]
    o0 = orc.compress_step(1, None, wl.r, q0.astype(np.float64), g, [np.zeros((spec.rows, spec.cols))] * wl.n_workers)
    o1 = orc.compress_step(1, None, wl.r, o0.comp.q, g, o0.e_next)
    assert orc.rel_fro(back(case.E[0]), o1.e_mean) <= 1e-4
    assert orc.rel_fro(back(case.P[0]), o1.comp.p_tilde) <= 1e-4


@pytest.mark.parametrize("rows,cols,ld,r,dtype,n_workers", [
    (257, 129, 136, 17, synth.F32, 2), (1000, 264, 264, 33, synth.BF16, 1), (333, 100, 104, 40, synth.F32, 1),
    (2049, 260, 264, 65, synth.BF16, 2), (515, 36, 40, 5, synth.BF16, 3), (1200, 520, 520, 72, synth.F32, 1),
    (900, 300, 304, 96, synth.BF16, 1), (641, 257, 264, 48, synth.F32, 4)])
@pytest.mark.parametrize("q_resident", [False, True], ids=["q_packed", "q_resident"])
def test_deferred_residual_odd_shapes_and_ranks(rows, cols, ld, r, dtype, n_workers, q_resident):
    """Shapes that are multiples of nothing (rows not of 8, columns not of 4, a leading dimension beyond the columns) at
    ranks on both sides of every width class of the kernels (16, 32, 64, 80, 96): three free-running steps with the
    deferred residual, every step's P~, Q and M and the flushed E against the oracle."""
    base = synth.config4() if dtype == synth.BF16 else synth.config2()
    wl = synth.scaled_down(base, rows, cols)
    wl.r = r
    wl.n_workers = n_workers
    print((rows, cols, ld, r, dtype, n_workers), _trajectory(wl, 3, lds=[ld], q_resident=q_resident))
