"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad shapes before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moda.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moda_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def L():
    from paper_2603_15619_amd import binding as libmoda

    if not os.path.exists(libmoda.LIB_PATH):
        from paper_2603_15619_amd.build import build_libmoda

        build_libmoda()
    return libmoda.lib()


def test_header_functions_are_exported(L):
    names = declared_functions()
    assert {"moda_attn_fwd", "moda_attn_bwd", "moda_attn_bwd_workspace_bytes",
            "moda_status_string", "moda_version"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_binding_lists_every_export():
    from paper_2603_15619_amd import binding as libmoda

    assert sorted(libmoda.EXPORTS) == declared_functions()


def test_status_strings_and_version(L):
    from paper_2603_15619_amd import binding as libmoda

    assert L.moda_version() >= 100
    seen = {libmoda.status_string(c) for c in range(7)}
    assert len(seen) == 7 and "ok" in seen


def test_shape_errors_without_gpu(L):
    from paper_2603_15619_amd.binding import MODAShape

    def fwd(shape, ptr=0x1000):
        p = ctypes.c_void_p(ptr)
        return L.moda_attn_fwd(p, p, p, p, p, p, p, ctypes.byref(shape), None)

    ok = dict(B=1, Hq=2, Hk=2, T=16, d=128, depth_alloc=2, depth_count=2, causal=1, scale=0.0, dtype=1)
    assert L.moda_attn_fwd(None, None, None, None, None, None, None, None, None) == 1  # NULL shape
    assert fwd(MODAShape(**dict(ok, d=96))) == 3          # unsupported head dim
    assert fwd(MODAShape(**dict(ok, dtype=7))) == 3       # unsupported dtype
    assert fwd(MODAShape(**dict(ok, Hq=3))) == 2          # Hq % Hk != 0
    assert fwd(MODAShape(**dict(ok, depth_count=3))) == 2  # more slots than allocated
    assert fwd(MODAShape(**dict(ok, T=-1))) == 2
    assert fwd(MODAShape(**dict(ok, causal=2))) == 2
    assert fwd(MODAShape(**ok), ptr=0x1008) == 4          # misaligned pointer
    assert L.moda_attn_fwd(None, None, None, None, None, None, None,
                           ctypes.byref(MODAShape(**ok)), None) == 1  # NULL tensors
    assert fwd(MODAShape(**dict(ok, B=0))) == 0           # empty problem: nothing launched
    assert fwd(MODAShape(**dict(ok, T=0))) == 0
