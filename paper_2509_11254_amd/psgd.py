"""Thin ctypes binding over libpsgd.so (the C ABI of include/psgd.h).

Argument marshalling only: every step of the compressor runs in the library's HIP kernels.
PyTorch provides device memory (tensors whose data_ptr() is handed over) and the stream.
There is no CPU or PyTorch fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpsgd.so")

PSGD_F32, PSGD_BF16 = 0, 1
PSGD_OK = 0
PSGD_E_INVALID_ARG, PSGD_E_SHAPE, PSGD_E_ALIGN, PSGD_E_HIP, PSGD_E_NOMEM, PSGD_E_CAPTURE = -1, -2, -3, -4, -5, -6
PSGD_E_TOO_LARGE = -7
STATIC_WORKSPACE_BYTES = 64 * 1024 * 1024

EXPORTS = [
    "psgd_init", "psgd_workspace_bytes", "psgd_workspace_reset", "psgd_compress", "psgd_compress_static", "psgd_compress_refresh", "psgd_flush_residual", "psgd_refresh",
    "psgd_decompress", "psgd_decompress_msgd", "psgd_decompress_adam", "psgd_compress_project", "psgd_compress_finish", "psgd_status", "psgd_algorithmic_bytes", "psgd_kernel_bytes", "psgd_copy_bytes",
    "psgd_last_hip_error",
    "psgd_strerror", "psgd_destroy", "psgd_profile_enable", "psgd_profile_select", "psgd_profile_read",
]
PROF_TAGS = ("sweep1", "sweep2", "residual")


class LayerDesc(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64), ("r", C.c_int32),
                ("grad_dtype", C.c_int32)]


class Options(C.Structure):
    _fields_ = [("refresh_iters", C.c_int32), ("refresh_oversample", C.c_int32),
                ("refresh_warm_start", C.c_int32), ("seed", C.c_uint32), ("rank_tol", C.c_float),
                ("precision", C.c_int32), ("m_policy", C.c_int32), ("power_iters", C.c_int32),
                ("lazy_residual", C.c_int32), ("q_resident", C.c_int32)]


class LayerStatus(C.Structure):
    _fields_ = [("rank_deficient", C.c_int32), ("refresh_iters_next", C.c_int32), ("sigma_max", C.c_float),
                ("sigma_r", C.c_float), ("refresh_iters_no_gap", C.c_int32)]


class PsgdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"psgd error {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Load libpsgd.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2509_11254_amd.build` "
            "(hipcc, gfx950). The compressor has no CPU fallback.")
    # PyTorch owns the device memory and the streams handed to the library, so both must talk to
    # the same HIP runtime instance: import torch first, then libpsgd.so binds to the runtime
    # (libamdhip64.so.7) that torch has already loaded instead of opening a second one.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, pp = C.c_void_p, C.POINTER(C.c_void_p)
    lib.psgd_init.argtypes = [pp, C.c_int, C.POINTER(LayerDesc), C.c_int, C.POINTER(Options)]
    lib.psgd_init.restype = C.c_int
    lib.psgd_workspace_bytes.argtypes = [vp]
    lib.psgd_workspace_bytes.restype = C.c_size_t
    lib.psgd_workspace_reset.argtypes = [vp]
    lib.psgd_workspace_reset.restype = C.c_int
    for name in ("psgd_compress", "psgd_compress_refresh", "psgd_compress_project"):
        fn = getattr(lib, name)
        fn.argtypes = [vp, vp, vp, pp, pp, pp, pp]
        fn.restype = C.c_int
    lib.psgd_compress_static.argtypes = [vp, vp, pp, pp, pp, pp]
    lib.psgd_compress_static.restype = C.c_int
    lib.psgd_compress_finish.argtypes = [vp, vp, vp, pp, pp, pp]
    lib.psgd_compress_finish.restype = C.c_int
    lib.psgd_flush_residual.argtypes = [vp, vp, vp, pp]
    lib.psgd_flush_residual.restype = C.c_int
    lib.psgd_refresh.argtypes = [vp, vp, vp, C.c_int, vp, vp, vp, vp]
    lib.psgd_refresh.restype = C.c_int
    lib.psgd_decompress.argtypes = [vp, vp, vp, pp, pp, pp, C.c_int]
    lib.psgd_decompress.restype = C.c_int
    lib.psgd_decompress_msgd.argtypes = [vp, vp, vp, pp, pp, pp, pp, C.c_float, C.c_float]
    lib.psgd_decompress_msgd.restype = C.c_int
    lib.psgd_decompress_adam.argtypes = [vp, vp, vp, pp, pp, pp, pp, pp, C.c_int, C.c_float, C.c_float, C.c_float,
                                         C.c_float, C.c_float]
    lib.psgd_decompress_adam.restype = C.c_int
    lib.psgd_status.argtypes = [vp, vp, vp, C.c_int, C.POINTER(LayerStatus)]
    lib.psgd_status.restype = C.c_int
    lib.psgd_algorithmic_bytes.argtypes = [vp]
    lib.psgd_algorithmic_bytes.restype = C.c_double
    lib.psgd_kernel_bytes.argtypes = [vp, C.c_int]
    lib.psgd_kernel_bytes.restype = C.c_double
    lib.psgd_copy_bytes.argtypes = [vp, vp, vp, C.c_size_t]
    lib.psgd_copy_bytes.restype = C.c_int
    lib.psgd_last_hip_error.argtypes = [vp]
    lib.psgd_last_hip_error.restype = C.c_int
    lib.psgd_strerror.argtypes = [C.c_int]
    lib.psgd_strerror.restype = C.c_char_p
    lib.psgd_profile_enable.argtypes = [vp, C.c_int]
    lib.psgd_profile_enable.restype = C.c_int
    lib.psgd_profile_select.argtypes = [vp, C.c_int]
    lib.psgd_profile_select.restype = C.c_int
    lib.psgd_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int), C.c_int]
    lib.psgd_profile_read.restype = C.c_int
    lib.psgd_destroy.argtypes = [vp]
    lib.psgd_destroy.restype = None
    _lib = lib
    return lib


def _check(lib, ctx, rc: int):
    if rc != PSGD_OK:
        msg = lib.psgd_strerror(rc).decode()
        if rc == PSGD_E_HIP and ctx:
            msg += f" (hipError {lib.psgd_last_hip_error(ctx)})"
        raise PsgdError(rc, msg)


def _ptr_table(tensors: Sequence) -> C.Array:
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def _opt_table(tensors):
    """Pointer table, or a null pointer for None (where the ABI gives NULL a meaning)."""
    return _ptr_table(tensors) if tensors is not None else None


def _stream_handle(stream) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


class Compressor:
    """psgd_init + a torch-allocated workspace; methods mirror the C entry points one to one.

    layers: sequence of (rows, cols, r, grad_dtype) or (rows, cols, r, grad_dtype, ld).
    """

    def __init__(self, layers: Sequence[Sequence[int]], n_workers: int, *, refresh_iters: int = 0,
                 refresh_oversample: int = -1, refresh_warm_start: bool = True, seed: int = 0x5EED5EED,
                 rank_tol: float = 0.0, precision: int = 0, m_policy: int = 0, power_iters: int = 0,
                 lazy_residual: bool = False, q_resident: bool = False, device: str = "cuda:0",
                 allocate: bool = True):
        self.lib = load_library()
        self.n_layers = len(layers)
        self.n_workers = int(n_workers)
        descs = (LayerDesc * max(1, self.n_layers))()
        for i, l in enumerate(layers):
            descs[i].rows, descs[i].cols, descs[i].r, descs[i].grad_dtype = int(l[0]), int(l[1]), int(l[2]), int(l[3])
            descs[i].ld = int(l[4]) if len(l) > 4 else 0
        opt = Options(int(refresh_iters), int(refresh_oversample), 1 if refresh_warm_start else 0,
                      int(seed) & 0xFFFFFFFF, float(rank_tol), int(precision), int(m_policy), int(power_iters),
                      1 if lazy_residual else 0, 1 if q_resident else 0)
        self.ctx = C.c_void_p()
        rc = self.lib.psgd_init(C.byref(self.ctx), self.n_layers, descs, self.n_workers, C.byref(opt))
        _check(self.lib, None, rc)
        self.layers = [tuple(l) for l in layers]
        self.workspace_bytes = int(self.lib.psgd_workspace_bytes(self.ctx))
        self.workspace = None
        if allocate:
            import torch
            self.workspace = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=device)
            self._ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
        self._keep = None

    def __del__(self):
        try:
            if getattr(self, "ctx", None) is not None and self.ctx:
                self.lib.psgd_destroy(self.ctx)
                self.ctx = None
        except Exception:
            pass

    @property
    def algorithmic_bytes(self) -> float:
        return float(self.lib.psgd_algorithmic_bytes(self.ctx))

    def kernel_bytes(self, tag: str) -> float:
        """Algorithmic bytes of one launch of the streaming kernel `tag` (one of PROF_TAGS) over all layers."""
        return float(self.lib.psgd_kernel_bytes(self.ctx, PROF_TAGS.index(tag)))

    def _tables(self, G, E, Q, P):
        flat_g = [g for per_layer in G for g in per_layer] if G and isinstance(G[0], (list, tuple)) else list(G)
        tabs = (_ptr_table(flat_g), _ptr_table(E), _ptr_table(Q), _ptr_table(P))
        self._keep = tabs
        return tabs

    def compress(self, G, E, Q, P, stream=None) -> None:
        """psgd_compress: G[l][i] gradients, E[l] error buffers (in place), Q[l] in/out, P[l] out."""
        tg, te, tq, tp = self._tables(G, E, Q, P)
        _check(self.lib, self.ctx, self.lib.psgd_compress(self.ctx, self._ws_ptr, _stream_handle(stream), tg, te, tq, tp))

    def compress_static(self, G, E, Q, P, stream=None) -> None:
        """psgd_compress_static: psgd_compress in the library's built-in workspace (allocates nothing)."""
        tg, te, tq, tp = self._tables(G, E, Q, P)
        _check(self.lib, self.ctx, self.lib.psgd_compress_static(self.ctx, _stream_handle(stream), tg, te, tq, tp))

    def compress_refresh(self, G, E, Q, P, stream=None) -> None:
        tg, te, tq, tp = self._tables(G, E, Q, P)
        _check(self.lib, self.ctx,
               self.lib.psgd_compress_refresh(self.ctx, self._ws_ptr, _stream_handle(stream), tg, te, tq, tp))

    def compress_project(self, G, E, Q, P, stream=None) -> None:
        """psgd_compress_project: E[l] <- M = G[l] + E[l]; P[l] <- M Q[l] (first half of a data-parallel step)."""
        tg, te, tq, tp = self._tables(G, E, Q, P)
        _check(self.lib, self.ctx,
               self.lib.psgd_compress_project(self.ctx, self._ws_ptr, _stream_handle(stream), tg, te, tq, tp))

    def compress_finish(self, E, Q, P, stream=None) -> None:
        """psgd_compress_finish: P[l] <- QR(P[l]) (the averaged P); Q[l] <- M^T P~; E[l] <- M - P~ Q[l]^T."""
        te, tq, tp = _ptr_table(E), _ptr_table(Q), _ptr_table(P)
        self._keep = (te, tq, tp)
        _check(self.lib, self.ctx,
               self.lib.psgd_compress_finish(self.ctx, self._ws_ptr, _stream_handle(stream), te, tq, tp))

    def workspace_reset(self) -> None:
        """psgd_workspace_reset: treat the workspace as new (its contents were lost or recycled)."""
        _check(self.lib, self.ctx, self.lib.psgd_workspace_reset(self.ctx))

    def flush_residual(self, E, stream=None) -> None:
        """psgd_flush_residual: settle the residual a lazy_residual compress step left owed (E[l] <- E_{t+1})."""
        te = _ptr_table(E)
        self._keep = (te,)
        _check(self.lib, self.ctx, self.lib.psgd_flush_residual(self.ctx, self._ws_ptr, _stream_handle(stream), te))

    def refresh(self, layer: int, M, P, Q, sigma=None, stream=None) -> None:
        _check(self.lib, self.ctx,
               self.lib.psgd_refresh(self.ctx, self._ws_ptr, _stream_handle(stream), int(layer), M.data_ptr(),
                                     P.data_ptr(), Q.data_ptr(), sigma.data_ptr() if sigma is not None else None))

    def decompress(self, P, Q, out, out_dtype: int = PSGD_F32, stream=None) -> None:
        """psgd_decompress: out[l] <- P[l] Q[l]^T; P = Q = None: the factors of the last compress call."""
        tp, tq, to = _opt_table(P), _opt_table(Q), _ptr_table(out)
        self._keep = (tp, tq, to)
        _check(self.lib, self.ctx,
               self.lib.psgd_decompress(self.ctx, self._ws_ptr, _stream_handle(stream), tp, tq, to, int(out_dtype)))

    def decompress_msgd(self, P, Q, mom, X, mu: float, eta: float, stream=None) -> None:
        """psgd_decompress_msgd: mom[l] <- mu mom[l] + P[l] Q[l]^T, X[l] <- X[l] - eta mom[l] (in place)."""
        tp, tq, tm, tx = _opt_table(P), _opt_table(Q), _ptr_table(mom), _ptr_table(X)
        self._keep = (tp, tq, tm, tx)
        _check(self.lib, self.ctx,
               self.lib.psgd_decompress_msgd(self.ctx, self._ws_ptr, _stream_handle(stream), tp, tq, tm, tx,
                                             C.c_float(mu), C.c_float(eta)))

    def decompress_adam(self, P, Q, m1, m2, X, step: int, eta: float, beta1: float = 0.9, beta2: float = 0.999,
                        eps: float = 1e-8, weight_decay: float = 0.0, stream=None) -> None:
        """psgd_decompress_adam: Adam / AdamW moments m1[l], m2[l] and weights X[l] from P[l] Q[l]^T (in place)."""
        tp, tq, t1, t2, tx = _opt_table(P), _opt_table(Q), _ptr_table(m1), _ptr_table(m2), _ptr_table(X)
        self._keep = (tp, tq, t1, t2, tx)
        _check(self.lib, self.ctx,
               self.lib.psgd_decompress_adam(self.ctx, self._ws_ptr, _stream_handle(stream), tp, tq, t1, t2, tx,
                                             int(step), C.c_float(eta), C.c_float(beta1), C.c_float(beta2),
                                             C.c_float(eps), C.c_float(weight_decay)))

    def profile_enable(self, max_records: int) -> None:
        _check(self.lib, self.ctx, self.lib.psgd_profile_enable(self.ctx, int(max_records)))

    def profile_select(self, tags: Sequence[str]) -> None:
        """Time only the launches with these tags (each timed launch costs two event records on the stream)."""
        mask = 0
        for t in tags:
            mask |= 1 << PROF_TAGS.index(t)
        _check(self.lib, self.ctx, self.lib.psgd_profile_select(self.ctx, mask))

    def profile_read(self) -> dict:
        """{tag: (total_ms, count)} of the event pairs recorded since the last read."""
        n = len(PROF_TAGS)
        ms, cnt = (C.c_double * n)(), (C.c_int * n)()
        _check(self.lib, self.ctx, self.lib.psgd_profile_read(self.ctx, ms, cnt, n))
        return {PROF_TAGS[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}

    def status(self, layer: int, stream=None) -> LayerStatus:
        st = LayerStatus()
        _check(self.lib, self.ctx,
               self.lib.psgd_status(self.ctx, self._ws_ptr, _stream_handle(stream), int(layer), C.byref(st)))
        return st


def copy_bytes(dst, src, n_bytes: int, stream=None) -> None:
    lib = load_library()
    rc = lib.psgd_copy_bytes(_stream_handle(stream), dst.data_ptr(), src.data_ptr(), int(n_bytes))
    _check(lib, None, rc)
