"""GPU parity of the two halves of psgd_compress (psgd_compress_project, psgd_compress_finish) that a data-parallel
job runs on every worker, with the exchange of P and Q between and after them.

Here the workers are N contexts (n_workers = 1 each, own workspace, own error buffer e^(i)) on the one GPU, run one
after the other; the two all-reduce-means of Algorithm 1 (P after the projection, Q after the back-projection) are
torch means over the workers' buffers -- plumbing that stands in for the collective.  The oracle runs the literal
per-worker form of Algorithm 1 / Algorithm 2, so every worker's e^(i)_{t+1} is compared, not only their mean.
"""
import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2509_11254_amd import psgd, synth
from gpu_harness import Case, back, logical, to_dev_f32, to_dev_grad, torch_mod

pytestmark = pytest.mark.gpu

TOL = {synth.F32: 1e-4, synth.BF16: 2e-2}


def _worker_inputs(wl, seed):
    """Per layer and worker: gradient (stored dtype) and a distinct error buffer e^(i); per layer Q_{t-1}."""
    grads, errs, qs = [], [], []
    for l, spec in enumerate(wl.layers):
        sig = synth.signal_matrix(spec, wl, l)
        grads.append([synth.worker_gradient(spec, wl, l, w, 0, sig) for w in range(wl.n_workers)])
        rng = np.random.default_rng([wl.seed, seed, l])
        errs.append([(0.3 * synth.noise_sigma(spec, wl) * rng.standard_normal((spec.rows, spec.cols))).astype(np.float32)
                     for _ in range(wl.n_workers)])
        qs.append(synth.initial_q(spec.n, wl.r, wl.seed, l))
    return grads, errs, qs


def _data_parallel_step(wl, grads, errs, qs):
    """Returns per layer (P~, Q_t, [e^(i)]) from N single-worker contexts and two device-side means."""
    torch = torch_mod()
    nl, nw = len(wl.layers), wl.n_workers
    shapes = [(s.rows, s.cols) for s in wl.layers]
    workers = []
    for i in range(nw):
        c = Case(shapes, wl.r, 1, wl.grad_dtype)
        c.upload([[grads[l][i]] for l in range(nl)], [errs[l][i] for l in range(nl)], qs)
        workers.append(c)
    for c in workers:
        c.comp.compress_project(c.G, c.E, c.Q, c.P)
    torch.cuda.synchronize()
    for l in range(nl):                                     # all-reduce-mean of P
        mean_p = torch.stack([c.P[l] for c in workers]).mean(dim=0)
        for c in workers:
            c.P[l].copy_(mean_p)
    for c in workers:
        c.comp.compress_finish(c.E, c.Q, c.P)
    torch.cuda.synchronize()
    out = []
    for l in range(nl):
        q_t = torch.stack([c.Q[l] for c in workers]).mean(dim=0)          # all-reduce-mean of Q
        for c in workers[1:]:
            assert torch.equal(c.P[l], workers[0].P[l])                   # every worker holds the same P~
        out.append((back(workers[0].P[l]), back(q_t), [back(c.E[l], shapes[l][1]) for c in workers]))
    return out


@pytest.mark.parametrize("which", ["f32_n3", "bf16_n4_transposed", "bf16_r64_n2", "batched_n2"])
def test_data_parallel_step_matches_per_worker_oracle(which):
    if which == "f32_n3":
        wl = synth.scaled_down(synth.config2(), 640, 384); wl.n_workers = 3
    elif which == "bf16_n4_transposed":
        wl = synth.scaled_down(synth.config3(), 384, 1024)
    elif which == "bf16_r64_n2":
        wl = synth.scaled_down(synth.config4(), 1100, 512); wl.n_workers = 2
    else:
        wl = synth.scaled_down(synth.config3(), 256, 256); wl.n_workers = 2
        wl.layers = [synth.LayerSpec(256, 256, "a"), synth.LayerSpec(704, 256, "b"), synth.LayerSpec(256, 704, "c"),
                     synth.LayerSpec(200, 136, "e")]
    tol = TOL[wl.grad_dtype]
    grads, errs, qs = _worker_inputs(wl, 31)
    got = _data_parallel_step(wl, grads, errs, qs)
    worst = {}
    for l, spec in enumerate(wl.layers):
        g = [logical(synth.gradient_as_f64(gw), spec.rows, spec.cols) for gw in grads[l]]
        e = [logical(np.asarray(ew, np.float64), spec.rows, spec.cols) for ew in errs[l]]
        ref = orc.compress_step(1, None, wl.r, qs[l].astype(np.float64), g, e)
        p_gpu, q_gpu, e_gpu = got[l]
        errs_l = {"P": orc.rel_fro(p_gpu, ref.comp.p_tilde), "Q": orc.rel_fro(q_gpu, ref.comp.q),
                  "orth": float(np.abs(p_gpu.T @ p_gpu - np.eye(wl.r)).max())}
        for i in range(wl.n_workers):
            errs_l["e%d" % i] = orc.rel_fro(logical(e_gpu[i], spec.rows, spec.cols), ref.e_next[i])
        assert errs_l.pop("orth") < 2e-5, (l, errs_l)
        for k, v in errs_l.items():
            assert v <= tol, (which, l, k, errs_l)
            worst[k[0]] = max(worst.get(k[0], 0.0), v)
    print(which, worst)


def test_one_worker_halves_equal_the_whole_step():
    """project followed by finish on one worker with all N gradients is psgd_compress."""
    wl = synth.scaled_down(synth.config1(), 333, 203)
    spec = wl.layers[0]
    grads, errs, qs = _worker_inputs(wl, 5)
    e0 = [errs[0][0]]
    whole = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype, lds=[208])
    whole.upload(grads, e0, qs)
    whole.compress()
    halves = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype, lds=[208])
    halves.upload(grads, e0, qs)
    halves.comp.compress_project(halves.G, halves.E, halves.Q, halves.P)
    halves.comp.compress_finish(halves.E, halves.Q, halves.P)
    torch_mod().cuda.synchronize()
    for a, b in zip(whole.outputs(0), halves.outputs(0)):
        assert orc.rel_fro(b, a) <= 2e-6


def test_halves_rejected_with_options_they_do_not_support():
    wl = synth.scaled_down(synth.config1(), 256, 128)
    spec = wl.layers[0]
    grads, errs, qs = _worker_inputs(wl, 6)
    for opts in (dict(lazy_residual=True), dict(m_policy=2), dict(power_iters=2)):
        case = Case([(spec.rows, spec.cols)], wl.r, wl.n_workers, wl.grad_dtype, **opts)
        case.upload(grads, [errs[0][0]], qs)
        with pytest.raises(psgd.PsgdError):
            case.comp.compress_project(case.G, case.E, case.Q, case.P)
        with pytest.raises(psgd.PsgdError):
            case.comp.compress_finish(case.E, case.Q, case.P)


def test_data_parallel_refresh_step_from_the_same_entry_points():
    """The SVD-Comp step of a data-parallel job (Algorithm 1: the averaged Delta is decomposed, then every node
    projects its own Delta^(i)): project stores M^(i), the mean of the M^(i) stands in for the full-gradient
    all-reduce, psgd_refresh gives P~ = U_r of it, and finish (whose QR leaves an orthonormal P~ as it is) gives
    every worker its Q^(i) and e^(i)."""
    torch = torch_mod()
    wl = synth.scaled_down(synth.config2(), 768, 512)
    wl.n_workers = 3
    spec = wl.layers[0]
    grads, errs, qs = _worker_inputs(wl, 41)
    workers = []
    for i in range(wl.n_workers):
        c = Case([(spec.rows, spec.cols)], wl.r, 1, wl.grad_dtype)
        c.upload([[grads[0][i]]], [errs[0][i]], qs)
        c.comp.compress_project(c.G, c.E, c.Q, c.P)
        workers.append(c)
    torch.cuda.synchronize()
    m_bar = torch.stack([c.E[0] for c in workers]).mean(dim=0).contiguous()
    w0 = workers[0]
    q_tmp = torch.empty_like(w0.Q[0])
    w0.comp.refresh(0, m_bar, w0.P[0], q_tmp)
    torch.cuda.synchronize()
    for c in workers[1:]:
        c.P[0].copy_(w0.P[0])
    for c in workers:
        c.comp.compress_finish(c.E, c.Q, c.P)
    torch.cuda.synchronize()
    g = [synth.gradient_as_f64(gw) for gw in grads[0]]
    e = [np.asarray(ew, np.float64) for ew in errs[0]]
    ref = orc.compress_step(0, 1, wl.r, qs[0].astype(np.float64), g, e)
    p_gpu = back(w0.P[0])
    assert orc.sin_theta_max(ref.comp.p_tilde, p_gpu) <= 1e-4
    assert np.abs(p_gpu.T @ p_gpu - np.eye(wl.r)).max() < 2e-5
    q_t = back(torch.stack([c.Q[0] for c in workers]).mean(dim=0))
    assert orc.rel_fro(p_gpu @ q_t.T, ref.comp.delta_hat) <= 1e-4
    for i, c in enumerate(workers):
        assert orc.rel_fro(back(c.E[0], spec.cols), ref.e_next[i]) <= 1e-4, i


def test_halves_on_degenerate_inputs():
    """Zero gradient and zero error: the supplied P is zero, every column is flagged, all outputs are zero.  A
    rank-deficient P (rank 2 < r) keeps a valid projector, as in the whole step."""
    torch = torch_mod()
    m, n, r = 256, 128, 4
    z = np.zeros((m, n), np.float32)
    case = Case([(m, n)], r, 1, synth.F32)
    case.upload([[z]], [z], [synth.initial_q(n, r, 3)])
    case.comp.compress_project(case.G, case.E, case.Q, case.P)
    case.comp.compress_finish(case.E, case.Q, case.P)
    torch.cuda.synchronize()
    p, q, e = case.outputs(0)
    assert np.all(p == 0) and np.all(q == 0) and np.all(e == 0)
    assert case.comp.status(0).rank_deficient == r
    m, n = 384, 256
    mat, _, _ = synth.prescribed_svd_matrix(m, n, [2.0, 1.0], seed=9)
    case = Case([(m, n)], r, 1, synth.F32)
    case.upload([[mat]], [np.zeros((m, n), np.float32)], [synth.initial_q(n, r, 2)])
    case.comp.compress_project(case.G, case.E, case.Q, case.P)
    case.comp.compress_finish(case.E, case.Q, case.P)
    torch.cuda.synchronize()
    p, q, e = case.outputs(0)
    assert case.comp.status(0).rank_deficient == 2
    assert np.all(p[:, 2:] == 0)
    np.testing.assert_allclose(p[:, :2].T @ p[:, :2], np.eye(2), atol=2e-5)
    assert np.linalg.norm(e - (mat - p @ (p.T @ mat))) <= 1e-4 * np.linalg.norm(mat)


@pytest.mark.parametrize("opts,r", [({}, 32), (dict(lazy_residual=True), 32), (dict(lazy_residual=True), 48)],
                         ids=["plain", "deferred_r32", "deferred_r48"])
def test_decompress_from_the_factors_of_the_last_compress_call(opts, r):
    """P = Q = NULL in the decompress-type calls: the operand copies the last compress call left in the workspace.
    Same bits as with the factors passed explicitly; refused when some other call wrote the copies last.
    With the deferred residual the layers that defer hold those copies in another order (all three layers at rank 32,
    the two stored with rows >= cols at rank 48)."""
    torch = torch_mod()
    wl = synth.scaled_down(synth.config3(), 256, 256)
    wl.r = r
    wl.layers = [synth.LayerSpec(256, 256, "a"), synth.LayerSpec(704, 256, "b"), synth.LayerSpec(256, 704, "c")]
    grads, errs, qs = _worker_inputs(wl, 51)
    case = Case([(s.rows, s.cols) for s in wl.layers], wl.r, wl.n_workers, wl.grad_dtype, **opts)
    case.upload(grads, [errs[l][0] for l in range(3)], qs)
    out_a = [torch.zeros_like(e) for e in case.E]
    out_b = [torch.zeros_like(e) for e in case.E]
    with pytest.raises(psgd.PsgdError):
        case.comp.decompress(None, None, out_a)                 # nothing compressed on this workspace yet
    for refresh in (False, True):
        case.compress(refresh=refresh)
        case.comp.decompress(None, None, out_a)
        case.comp.decompress(case.P, case.Q, out_b)
        torch.cuda.synchronize()
        for a, b in zip(out_a, out_b):
            assert torch.equal(a, b), refresh
        with pytest.raises(psgd.PsgdError):
            case.comp.decompress(None, None, out_a)             # the explicit call above re-packed the copies
    # the fused optimizer passes take the same convention
    case.compress()
    mom_a, x_a = [torch.zeros_like(e) for e in case.E], [torch.ones_like(e) for e in case.E]
    mom_b, x_b = [torch.zeros_like(e) for e in case.E], [torch.ones_like(e) for e in case.E]
    case.comp.decompress_msgd(None, None, mom_a, x_a, 0.9, 0.1)
    case.comp.decompress_msgd(case.P, case.Q, mom_b, x_b, 0.9, 0.1)
    torch.cuda.synchronize()
    for a, b in zip(x_a + mom_a, x_b + mom_b):
        assert torch.equal(a, b)
    case.compress()
    m1_a, m2_a = [torch.zeros_like(e) for e in case.E], [torch.zeros_like(e) for e in case.E]
    m1_b, m2_b = [torch.zeros_like(e) for e in case.E], [torch.zeros_like(e) for e in case.E]
    case.comp.decompress_adam(None, None, m1_a, m2_a, x_a, 1, 0.01)
    case.comp.decompress_adam(case.P, case.Q, m1_b, m2_b, x_b, 1, 0.01)
    torch.cuda.synchronize()
    for a, b in zip(x_a + m1_a + m2_a, x_b + m1_b + m2_b):
        assert torch.equal(a, b)


@pytest.mark.parametrize("lazy", [False, True])
def test_q_resident_gives_the_same_steps(lazy):
    """psgd_options.q_resident: Q_{t-1} taken from the operand copies of the previous call instead of packing the Q
    buffers again.  Same bits as the default over a schedule with refresh steps, the fused decompress in between
    (NULL factors: the copies stay), and an explicit decompress (which re-packs: the next step packs Q again).
    With the deferred residual the promise also lets the forming pass take the kept Q from those copies, which adds
    the terms of the owed residual in another order: the same numbers up to fp32 rounding of that sum, not the same
    bits; what is compared there is what the factors stand for, P~ Q^T, and E."""
    torch = torch_mod()
    wl = synth.scaled_down(synth.config3(), 256, 256)
    wl.layers = [synth.LayerSpec(256, 256, "a"), synth.LayerSpec(704, 256, "b"), synth.LayerSpec(256, 704, "c")]
    shapes = [(s.rows, s.cols) for s in wl.layers]
    grads0, errs, qs = _worker_inputs(wl, 61)
    a = Case(shapes, wl.r, wl.n_workers, wl.grad_dtype, lazy_residual=lazy)
    b = Case(shapes, wl.r, wl.n_workers, wl.grad_dtype, lazy_residual=lazy, q_resident=True)
    for c in (a, b):
        c.upload(grads0, [errs[l][0] for l in range(3)], qs)
        c.OUT = [torch.zeros_like(e) for e in c.E]

    def same(x, y, t):
        if not lazy:
            return torch.equal(x, y)
        # (rounding-level where the two first differ; a free-running run then drifts apart in the directions the rank
        # cuts through noise: a tenth per cent after seven steps.  Parity of either variant is the oracle's business,
        # tests/test_gpu_lazy.py.)
        return float((x - y).norm()) <= (1e-5 if t <= 2 else 5e-3) * float(y.norm())

    for t in range(7):
        for c in (a, b):
            if t > 0:
                sig = [synth.signal_matrix(s, wl, l) for l, s in enumerate(wl.layers)]
                for l, s in enumerate(wl.layers):
                    for w in range(wl.n_workers):
                        c.G[l][w].copy_(to_dev_grad(synth.worker_gradient(s, wl, l, w, t, sig[l]), c.lds[l]))
            c.compress(refresh=(t in (0, 3)))
            if t == 4:
                c.comp.decompress(c.P, c.Q, c.OUT)       # explicit factors: re-packs the copies
            else:
                c.comp.decompress(None, None, c.OUT)
        torch.cuda.synchronize()
        for l in range(3):
            for x, y in ((a.OUT[l], b.OUT[l]),) if lazy else ((a.P[l], b.P[l]), (a.Q[l], b.Q[l]), (a.OUT[l], b.OUT[l])):
                assert same(x, y, t), (t, l)
    if lazy:
        a.comp.flush_residual(a.E); b.comp.flush_residual(b.E)
        torch.cuda.synchronize()
    for l in range(3):
        assert same(a.E[l], b.E[l], 7)


def test_workspace_reset_after_the_workspace_was_overwritten():
    """A workspace whose contents were lost: psgd_workspace_reset makes the next call treat it as new (tables
    uploaded, per-layer state cleared, operands packed), and the steps go on as those of an undisturbed twin."""
    torch = torch_mod()
    wl = synth.scaled_down(synth.config3(), 640, 384)
    grads, errs, qs = _worker_inputs(wl, 71)
    a = Case([(640, 384)], wl.r, wl.n_workers, wl.grad_dtype, q_resident=True)
    b = Case([(640, 384)], wl.r, wl.n_workers, wl.grad_dtype, q_resident=True)
    for c in (a, b):
        c.upload(grads, [errs[0][0]], qs)
        c.compress()
    b.comp.workspace.fill_(0xA5)                                # everything the library kept there is gone
    b.comp.workspace_reset()
    out = [torch.zeros_like(b.E[0])]
    with pytest.raises(psgd.PsgdError):
        b.comp.decompress(None, None, out)                      # no factors known in this workspace any more
    for c in (a, b):
        c.compress()
    torch.cuda.synchronize()
    assert torch.equal(a.P[0], b.P[0]) and torch.equal(a.Q[0], b.Q[0]) and torch.equal(a.E[0], b.E[0])
