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


def test_new_entry_points_reject_bad_arguments_without_gpu(L):
    """moda_depth_append, moda_attn_decode and moda_attn_bwd validate everything on the host
    before any kernel is launched."""
    from paper_2603_15619_amd.binding import MODAShape

    ok = dict(B=1, Hq=4, Hk=2, T=16, d=128, depth_alloc=3, depth_count=2, causal=1, scale=0.0, dtype=1)
    p, bad = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)

    def append(shape, slot, a=p):
        return L.moda_depth_append(a, p, p, p, slot, ctypes.byref(shape), None)

    assert append(MODAShape(**ok), 3) == 2                 # slot >= depth_alloc
    assert append(MODAShape(**ok), -1) == 2
    assert append(MODAShape(**ok), 0, a=None) == 1
    assert append(MODAShape(**ok), 0, a=bad) == 4
    assert append(MODAShape(**dict(ok, T=0)), 0) == 0      # empty: nothing launched
    assert append(MODAShape(**dict(ok, depth_alloc=0, depth_count=0)), 0) == 2

    def decode(shape, kv_alloc, ws=p, ws_bytes=1 << 30, q=p):
        return L.moda_attn_decode(q, p, p, p, p, p, p, kv_alloc, ws, ws_bytes, ctypes.byref(shape), None)

    need = L.moda_attn_decode_workspace_bytes(ctypes.byref(MODAShape(**ok)))
    assert need > 0
    assert decode(MODAShape(**ok), 15) == 2                # cache shorter than the attended length
    assert decode(MODAShape(**dict(ok, T=0)), 16) == 2     # the new token's own key is always attended
    assert decode(MODAShape(**dict(ok, dtype=0)), 16) == 3  # bf16 only
    assert decode(MODAShape(**ok), 16, ws=None) == 6
    assert decode(MODAShape(**ok), 16, ws_bytes=need - 1) == 6
    assert decode(MODAShape(**ok), 16, q=None) == 1
    assert decode(MODAShape(**ok), 16, q=bad) == 4
    assert decode(MODAShape(**dict(ok, B=0)), 16) == 0

    def bwd(shape, ws_bytes=1 << 30):
        return L.moda_attn_bwd(*([p] * 14), ws_bytes, ctypes.byref(shape), None)

    assert bwd(MODAShape(**dict(ok, Hq=256, Hk=2))) == 3   # more than 64 query heads per key/value head
    assert bwd(MODAShape(**dict(ok, dtype=0))) == 3
    assert bwd(MODAShape(**ok), ws_bytes=8) == 6
    assert L.moda_kernels_per_call(ctypes.byref(MODAShape(**ok)), 1) == 3               # up to 4 heads per group: the depth-slot gradients run inside dK/dV
    assert L.moda_kernels_per_call(ctypes.byref(MODAShape(**dict(ok, Hq=16))), 1) == 4  # 8 heads per group: a kernel of their own
    assert L.moda_kernels_per_call(ctypes.byref(MODAShape(**dict(ok, Hq=40))), 1) == 4  # 20 heads per group: likewise
    assert L.moda_kernels_per_call(ctypes.byref(MODAShape(**dict(ok, Hq=2))), 1) == 3
    assert L.moda_kernels_per_call(ctypes.byref(MODAShape(**ok)), 0) == 1


def test_size_limits_without_gpu(L):
    """One (batch, head) slab of a SEQUENCE tensor must stay below 4 GiB (32-bit byte offsets
    inside a slab); the depth tensors have no such limit (64-bit tile bases), only a cap on the
    slots per position; the decoding step addresses its caches with 64-bit pointers."""
    from paper_2603_15619_amd.binding import MODAFwdTuning, MODAShape

    p = ctypes.c_void_p(0x1000)
    base = dict(B=1, Hq=1, Hk=1, d=128, depth_count=1, causal=1, scale=0.0, dtype=1)

    def fwd_status(T, depth_alloc):
        s = MODAShape(T=T, depth_alloc=depth_alloc, **base)
        # NULL output pointer: a shape that passes validation stops at the pointer check
        return L.moda_attn_fwd(p, p, p, p, p, None, p, ctypes.byref(s), None)

    assert fwd_status(65536, 256) == 1          # 4 GiB of depth slots per head: accepted (then NULL output)
    assert fwd_status(131072, 8192) == 1
    assert fwd_status(65536, 8193) == 3         # more slots per position than the cap
    assert fwd_status((1 << 24) - 1, 1) == 1    # T * 128 * 2 bytes just below 4 GiB
    assert fwd_status(1 << 24, 1) == 3          # exactly 4 GiB: unsupported

    s = MODAShape(T=1 << 20, depth_alloc=256, **base)
    assert L.moda_attn_decode(p, p, p, p, p, None, p, 1 << 25, p, 1 << 30, ctypes.byref(s), None) == 1

    ok = MODAShape(B=1, Hq=4, Hk=2, T=16, d=128, depth_alloc=0, depth_count=0, causal=1, scale=0.0, dtype=1)

    def tuned(**kw):
        return L.moda_attn_fwd_tuned(p, p, p, None, None, None, p, ctypes.byref(ok), ctypes.byref(MODAFwdTuning(**kw)),
                                     None)

    assert tuned(waves=8, heads_per_tile=2, head_group=1) == 1   # accepted (then NULL output)
    assert tuned(waves=5) == 2 and tuned(heads_per_tile=4) == 2 and tuned(head_group=-2) == 2
