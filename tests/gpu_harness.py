"""Helpers shared by the GPU parity tests: move seeded NumPy inputs to the device, run one
call of the library through its binding, bring the outputs back as fp64 NumPy arrays."""
from __future__ import annotations

import numpy as np

from paper_2509_11254_amd import psgd, synth


def torch_mod():
    import torch
    return torch


def to_dev_grad(g: np.ndarray, ld: int | None = None):
    """fp32 values or bf16 bit patterns -> device tensor of the storage dtype (optionally padded to ld)."""
    torch = torch_mod()
    rows, cols = g.shape
    if g.dtype == np.uint16:
        t = torch.from_numpy(g.view(np.int16).copy()).view(torch.bfloat16)
    else:
        t = torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32))
    if ld is not None and ld != cols:
        buf = torch.full((rows, ld), float("nan"), dtype=t.dtype)
        buf[:, :cols] = t
        t = buf
    return t.cuda()


def to_dev_f32(x: np.ndarray, ld: int | None = None):
    torch = torch_mod()
    x = np.ascontiguousarray(x, dtype=np.float32)
    t = torch.from_numpy(x)
    if ld is not None and x.ndim == 2 and ld != x.shape[1]:
        buf = torch.full((x.shape[0], ld), float("nan"), dtype=torch.float32)
        buf[:, : x.shape[1]] = t
        t = buf
    return t.cuda()


def back(t, cols: int | None = None) -> np.ndarray:
    a = t.detach().float().cpu().numpy().astype(np.float64)
    return a if cols is None else a[:, :cols]


class Case:
    """One compressor instance over a list of stored matrices with per-layer inputs on the device."""

    def __init__(self, shapes, r, n_workers, dtype, lds=None, **opts):
        self.shapes = list(shapes)
        self.r = r if isinstance(r, (list, tuple)) else [r] * len(self.shapes)
        self.n_workers = n_workers
        self.dtype = dtype
        self.lds = list(lds) if lds is not None else [c for (_, c) in self.shapes]
        gd = psgd.PSGD_BF16 if dtype == synth.BF16 else psgd.PSGD_F32
        layers = [(rw, cl, self.r[i], gd, self.lds[i]) for i, (rw, cl) in enumerate(self.shapes)]
        self.comp = psgd.Compressor(layers, n_workers, **opts)

    def upload(self, grads, errs, qs):
        """grads[l][w]: stored-dtype arrays, errs[l]: fp32 (rows x cols), qs[l]: fp32 (n x r)."""
        torch = torch_mod()
        self.G = [[to_dev_grad(g, self.lds[l]) for g in grads[l]] for l in range(len(self.shapes))]
        self.E = [to_dev_f32(errs[l], self.lds[l]) for l in range(len(self.shapes))]
        self.Q = [to_dev_f32(qs[l]) for l in range(len(self.shapes))]
        self.P = []
        for l, (rw, cl) in enumerate(self.shapes):
            self.P.append(torch.full((max(rw, cl), self.r[l]), float("nan"), dtype=torch.float32, device="cuda"))

    def compress(self, refresh=False):
        torch = torch_mod()
        (self.comp.compress_refresh if refresh else self.comp.compress)(self.G, self.E, self.Q, self.P)
        torch.cuda.synchronize()

    def outputs(self, l):
        """(P~ m x r, Q n x r, E rows x cols) as fp64; E in the stored orientation."""
        return back(self.P[l]), back(self.Q[l]), back(self.E[l], self.shapes[l][1])


def logical(x: np.ndarray, rows: int, cols: int) -> np.ndarray:
    """Stored (rows x cols) -> logical (m x n) matrix with m >= n."""
    return x.T if rows < cols else x


def oracle_inputs(grads_l, err_l, rows, cols, n_workers):
    """Per-worker fp64 logical gradients and error buffers for the oracle (e^(i) = E for every i,
    which has mean E: by linearity every global output is the same as with any other split)."""
    g = [logical(synth.gradient_as_f64(gw), rows, cols) for gw in grads_l]
    e = [logical(np.asarray(err_l, dtype=np.float64), rows, cols) for _ in range(n_workers)]
    return g, e
