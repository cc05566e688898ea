"""Host-side checks of the C ABI that need no GPU: exported symbols, argument validation, planning."""
import ctypes as C
import os
import re

import pytest

from paper_2509_11254_amd import psgd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return psgd.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "psgd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(psgd_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(psgd.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def _init(lib, layers, n_workers=1, opt=None):
    descs = (psgd.LayerDesc * max(1, len(layers)))()
    for i, l in enumerate(layers):
        descs[i].rows, descs[i].cols, descs[i].ld, descs[i].r, descs[i].grad_dtype = l
    ctx = C.c_void_p()
    rc = lib.psgd_init(C.byref(ctx), len(layers), descs, n_workers, opt)
    return rc, ctx


def test_init_rejects_bad_arguments(lib):
    ok = (256, 128, 0, 4, psgd.PSGD_F32)
    rc, ctx = _init(lib, [ok])
    assert rc == psgd.PSGD_OK and ctx
    lib.psgd_destroy(ctx)
    assert _init(lib, [ok], n_workers=0)[0] == psgd.PSGD_E_INVALID_ARG
    assert _init(lib, [])[0] == psgd.PSGD_E_INVALID_ARG
    assert lib.psgd_init(None, 1, None, 1, None) == psgd.PSGD_E_INVALID_ARG
    assert _init(lib, [(256, 128, 0, 0, psgd.PSGD_F32)])[0] == psgd.PSGD_E_SHAPE       # r < 1
    assert _init(lib, [(256, 128, 0, 129, psgd.PSGD_F32)])[0] == psgd.PSGD_E_SHAPE     # r > n
    assert _init(lib, [(128, 256, 0, 129, psgd.PSGD_F32)])[0] == psgd.PSGD_E_SHAPE     # r > n (transposed)
    assert _init(lib, [(0, 128, 0, 4, psgd.PSGD_F32)])[0] == psgd.PSGD_E_SHAPE         # empty matrix
    assert _init(lib, [(256, 128, 0, 4, 7)])[0] == psgd.PSGD_E_INVALID_ARG             # dtype
    assert _init(lib, [(256, 128, 120, 4, psgd.PSGD_F32)])[0] == psgd.PSGD_E_ALIGN     # ld < cols
    assert _init(lib, [(256, 130, 0, 4, psgd.PSGD_F32)])[0] == psgd.PSGD_E_ALIGN       # ld = cols not multiple of 8
    assert _init(lib, [(256, 130, 136, 4, psgd.PSGD_F32)])[0] == psgd.PSGD_OK          # padded ld is fine
    assert _init(lib, [(4096, 4096, 0, 190, psgd.PSGD_F32)])[0] == psgd.PSGD_E_SHAPE   # block wider than supported
    # leading dimensions beyond what the kernels' 32-bit lane offsets cover (127 rows * ld * 4 bytes < 2^32)
    assert _init(lib, [(256, 128, (1 << 23) + 8, 4, psgd.PSGD_F32)])[0] == psgd.PSGD_E_SHAPE
    assert _init(lib, [(256, 128, 1 << 23, 4, psgd.PSGD_F32)])[0] == psgd.PSGD_OK
    # the refresh's iteration budget has eight bits in the launches' gate word
    for iters, want in ((255, psgd.PSGD_OK), (256, psgd.PSGD_E_INVALID_ARG), (-1, psgd.PSGD_E_INVALID_ARG)):
        opt = psgd.Options(iters, -1, 1, 1, 0.0, 0, 0, 0, 0, 0)
        rc, ctx = _init(lib, [ok], opt=C.byref(opt))
        assert rc == want, iters
        if rc == psgd.PSGD_OK:
            lib.psgd_destroy(ctx)
    for code in (0, -1, -2, -3, -4, -5, -6, -7, -99):
        assert lib.psgd_strerror(code)


def test_compute_calls_reject_null_without_touching_a_gpu(lib):
    rc, ctx = _init(lib, [(256, 128, 0, 4, psgd.PSGD_F32)])
    assert rc == 0
    assert lib.psgd_compress(ctx, None, None, None, None, None, None) == psgd.PSGD_E_INVALID_ARG
    assert lib.psgd_compress_static(ctx, None, None, None, None, None) == psgd.PSGD_E_INVALID_ARG
    assert lib.psgd_compress_refresh(ctx, None, None, None, None, None, None) == psgd.PSGD_E_INVALID_ARG
    assert lib.psgd_refresh(ctx, None, None, 0, None, None, None, None) == psgd.PSGD_E_INVALID_ARG
    assert lib.psgd_decompress(ctx, None, None, None, None, None, 0) == psgd.PSGD_E_INVALID_ARG
    assert lib.psgd_status(ctx, None, None, 0, None) == psgd.PSGD_E_INVALID_ARG
    assert lib.psgd_copy_bytes(None, None, None, 16) == psgd.PSGD_E_INVALID_ARG
    lib.psgd_destroy(ctx)


def test_workspace_and_algorithmic_bytes(lib):
    rc, ctx = _init(lib, [(4096, 4096, 0, 8, psgd.PSGD_F32)], n_workers=8)
    assert rc == 0
    ws = lib.psgd_workspace_bytes(ctx)
    assert 0 < ws < 1 << 30
    # 8 fp32 gradients + E read, M written and read, E written: 48 bytes per element (+ thin matrices)
    elems = 4096 * 4096
    thin = 16 * (4096 + 4096) * 8
    assert lib.psgd_algorithmic_bytes(ctx) == pytest.approx(elems * 48 + thin)
    lib.psgd_destroy(ctx)
    # one bf16 gradient: forming M twice (2*2 + 12 = 16 bytes) beats storing it (2 + 16)
    rc, ctx = _init(lib, [(11008, 4096, 0, 64, psgd.PSGD_BF16)], n_workers=1)
    assert rc == 0
    assert lib.psgd_algorithmic_bytes(ctx) == pytest.approx(11008 * 4096 * 16 + 16 * (11008 + 4096) * 64)
    lib.psgd_destroy(ctx)
    rc1, c1 = _init(lib, [(512, 512, 0, 8, 0)])
    rc2, c2 = _init(lib, [(512, 512, 0, 8, 0)] * 3)
    assert lib.psgd_workspace_bytes(c2) > lib.psgd_workspace_bytes(c1)
    lib.psgd_destroy(c1)
    lib.psgd_destroy(c2)


def test_struct_layouts_match_the_header(tmp_path):
    """The ctypes mirrors of the ABI structs against the C compiler's view of include/psgd.h: sizes and the offset
    of every field, and the error codes the binding names."""
    import subprocess
    fields = {"psgd_layer_desc": [f[0] for f in psgd.LayerDesc._fields_],
              "psgd_options": [f[0] for f in psgd.Options._fields_],
              "psgd_layer_status": [f[0] for f in psgd.LayerStatus._fields_]}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "psgd.h"', 'int main(void) {']
    for s, fs in fields.items():
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (s, s))
        for f in fs:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (s, f, s, f))
    lines.append('printf("codes %d %d %d %d %d %d %d\\n", PSGD_E_INVALID_ARG, PSGD_E_SHAPE, PSGD_E_ALIGN, PSGD_E_HIP, '
                 'PSGD_E_NOMEM, PSGD_E_CAPTURE, PSGD_E_TOO_LARGE);')
    lines.append('printf("static_ws %u\\n", (unsigned)PSGD_STATIC_WORKSPACE_BYTES);')
    lines += ['return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = dict(l.split(" ", 1) for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    mirrors = {"psgd_layer_desc": psgd.LayerDesc, "psgd_options": psgd.Options, "psgd_layer_status": psgd.LayerStatus}
    for s, cls in mirrors.items():
        assert int(out[s]) == C.sizeof(cls), s
        for f in fields[s]:
            assert int(out["%s.%s" % (s, f)]) == getattr(cls, f).offset, (s, f)
    assert [int(x) for x in out["codes"].split()] == [psgd.PSGD_E_INVALID_ARG, psgd.PSGD_E_SHAPE, psgd.PSGD_E_ALIGN,
                                                      psgd.PSGD_E_HIP, psgd.PSGD_E_NOMEM, psgd.PSGD_E_CAPTURE,
                                                      psgd.PSGD_E_TOO_LARGE]
    assert int(out["static_ws"]) == psgd.STATIC_WORKSPACE_BYTES
