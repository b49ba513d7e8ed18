"""CPU-side checks of the boundary: the library builds/loads and exports every symbol the headers declare;
host-side validation rejects bad arguments before anything touches a device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2407_09722_amd import binding as mb
    if not os.path.exists(mb.LIB_PATH):
        from paper_2407_09722_amd import build
        build.build()
    return mb.lib()


def _declared():
    names = set()
    for h in ("mtad.h", "mtad_kernels.h"):
        src = open(os.path.join(ROOT, "include", h)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(mtad_[a-z_0-9]+)\s*\(", src))
    return names


def test_every_declared_symbol_is_exported(lib):
    from paper_2407_09722_amd import binding as mb
    decl = _declared()
    assert decl == set(mb.EXPORTS)
    for name in decl:
        assert getattr(lib, name) is not None


def test_strerror_and_host_validation(lib):
    from paper_2407_09722_amd import binding as mb
    assert lib.mtad_strerror(0) == b"ok"
    assert lib.mtad_strerror(mb.MTAD_ESHAPE) == b"unsupported shape"
    good = dict(n_layers=2, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, d_ffn=352, vocab=1024, dtype=1)

    def model(**kw):
        d = dict(good, **kw)
        return mb.mtad_model(d["n_layers"], d["d_model"], d["n_heads"], d["n_kv_heads"], d["head_dim"], d["d_ffn"], d["vocab"],
                             d["dtype"], 1e-5, 10000.0, None)

    def create(cfg, t, d):
        h = C.c_void_p()
        st = lib.mtad_create(C.byref(h), C.byref(cfg), C.byref(t), C.byref(d))
        if st == 0:
            assert lib.mtad_workspace_bytes(h) > 0
            lib.mtad_destroy(h)
        return st

    cfg = mb.mtad_config(1, 4, 4, mb.MTAD_MODE_MMTAD, 64, 512)
    assert create(cfg, model(), model()) == mb.MTAD_OK
    assert create(mb.mtad_config(1, 4, 9, 1, 64, 512), model(), model()) == mb.MTAD_ESHAPE       # beam > 8
    assert create(mb.mtad_config(1, 16, 4, 1, 64, 512), model(), model()) == mb.MTAD_ESHAPE      # 65 rows
    assert create(mb.mtad_config(1, 4, 4, 7, 64, 512), model(), model()) == mb.MTAD_EINVAL       # bad mode
    assert create(cfg, model(head_dim=96), model()) == mb.MTAD_ESHAPE
    assert create(cfg, model(d_ffn=344), model()) == mb.MTAD_ESHAPE                              # bf16 K % 32
    assert create(cfg, model(dtype=0, d_ffn=344), model(dtype=0, d_ffn=344)) == mb.MTAD_OK
    assert create(cfg, model(vocab=1040), model()) == mb.MTAD_ESHAPE                             # vocab mismatch
    assert create(mb.mtad_config(8, 4, 4, 1, 64, 512), model(), model()) == mb.MTAD_ESHAPE       # > 256 rows in a pass
    # hot calls validate before launching: null context / null buffers
    assert lib.mtad_k_gemm(None, 1, None, None, None, 5, 64, 64, 64, 0, None) == mb.MTAD_EINVAL
    assert lib.mtad_k_gemm(None, 1, C.c_void_p(256), C.c_void_p(256), C.c_void_p(256), 5, 60, 64, 64, 0, None) == mb.MTAD_ESHAPE
    assert lib.mtad_k_gemm_x(None, 1, C.c_void_p(256), C.c_void_p(256), C.c_void_p(256), 5, 64, 64, 64, 0, 7, None) == mb.MTAD_EINVAL    # no such order
    assert lib.mtad_k_gemm_x(None, 0, C.c_void_p(256), C.c_void_p(256), C.c_void_p(256), 5, 64, 64, 64, 0, 1, None) == mb.MTAD_EINVAL    # float32 has planes only
    assert lib.mtad_bind_workspace(None, None, 0) == mb.MTAD_EINVAL
