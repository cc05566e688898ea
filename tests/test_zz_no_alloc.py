"""psgd_compress_static (the entry point that allocates nothing: its workspace is a static device array inside the
library) against psgd_compress on the same inputs, through the C ABI.  Two calls in a row on the shared buffer, the
second with a smaller input and another context; same kernels, same launch plan, so the outputs must agree bit for bit.
"""
import numpy as np
import pytest

from paper_2509_11254_amd import psgd, synth

pytestmark = pytest.mark.gpu


def _inputs(rows, cols, r, n_workers, seed):
    import torch
    wl = synth.scaled_down(synth.config2(seed), rows, cols)
    spec = wl.layers[0]
    sig = synth.signal_matrix(spec, wl, 0)
    G = [[torch.from_numpy(synth.worker_gradient(spec, wl, 0, w, 0, sig)).cuda() for w in range(n_workers)]]
    rng = np.random.default_rng(seed)
    E = [torch.from_numpy((1e-3 * rng.standard_normal((rows, cols))).astype(np.float32)).cuda()]
    Q = [torch.from_numpy(synth.initial_q(min(rows, cols), r, seed)).cuda()]
    P = [torch.full((max(rows, cols), r), float("nan"), device="cuda")]
    return G, E, Q, P


def _both(rows, cols, r, n_workers, seed, steps=2):
    """Runs `steps` SSP steps through each entry point; returns the two (P, Q, E) triples."""
    import torch
    layers = [(rows, cols, r, psgd.PSGD_F32)]
    out = []
    for static in (False, True):
        comp = psgd.Compressor(layers, n_workers, allocate=not static)
        G, E, Q, P = _inputs(rows, cols, r, n_workers, seed)
        for _ in range(steps):
            (comp.compress_static if static else comp.compress)(G, E, Q, P)
        torch.cuda.synchronize()
        out.append((P[0].cpu().numpy(), Q[0].cpu().numpy(), E[0].cpu().numpy()))
        del comp
    return out


def test_static_workspace_two_calls_second_smaller():
    # config 2's shape (35.7 MiB of workspace, under the 64 MiB of the built-in buffer), then a smaller, ragged one
    for rows, cols, r, nw, seed in ((4096, 4096, 8, 2, 11), (1000, 520, 8, 2, 12)):
        (p0, q0, e0), (p1, q1, e1) = _both(rows, cols, r, nw, seed)
        assert np.isfinite(p1).all() and np.isfinite(q1).all() and np.isfinite(e1).all()
        assert np.array_equal(p0, p1), (rows, cols, float(np.abs(p0 - p1).max()))
        assert np.array_equal(q0, q1), (rows, cols, float(np.abs(q0 - q1).max()))
        assert np.array_equal(e0, e1), (rows, cols, float(np.abs(e0 - e1).max()))


def test_static_workspace_contexts_alternate():
    """Two contexts take turns on the shared buffer: each finds the other's contents and must start over cleanly."""
    import torch
    shapes = ((768, 512, 8, 2, 21), (1000, 520, 4, 1, 22))
    ref = [_both(*s, steps=2)[0] for s in shapes]
    comps = [psgd.Compressor([(s[0], s[1], s[2], psgd.PSGD_F32)], s[3], allocate=False) for s in shapes]
    data = [_inputs(*s) for s in shapes]
    for _ in range(2):
        for comp, (G, E, Q, P) in zip(comps, data):
            comp.compress_static(G, E, Q, P)
    torch.cuda.synchronize()
    for (p0, q0, e0), (G, E, Q, P) in zip(ref, data):
        assert np.array_equal(p0, P[0].cpu().numpy())
        assert np.array_equal(q0, Q[0].cpu().numpy())
        assert np.array_equal(e0, E[0].cpu().numpy())


def test_static_workspace_rejects_large_context():
    import torch
    comp = psgd.Compressor([(8192, 8192, 128, psgd.PSGD_F32)], 1, allocate=False)
    assert comp.workspace_bytes > psgd.STATIC_WORKSPACE_BYTES
    x = torch.zeros(8, device="cuda")
    with pytest.raises(psgd.PsgdError) as err:
        comp.compress_static([[x]], [x], [x], [x])
    assert err.value.code == psgd.PSGD_E_TOO_LARGE
