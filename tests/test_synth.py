"""The seeded input generator (paper_2603_15619_amd/synth.py, libmoda_synth.so): the library
loads and exports its entry point (CPU); on the GPU its values are reproducible, differ between
tensors and seeds, and are distributed like N(0,1) rounded to the requested type."""
import ctypes
import os

import numpy as np
import pytest
import torch

from paper_2603_15619_amd import synth


def test_generator_library_loads_and_exports():
    if not os.path.exists(synth._SYNTH_LIB_PATH):
        from paper_2603_15619_amd.build import build_synth

        build_synth()
    L = ctypes.CDLL(synth._SYNTH_LIB_PATH)
    assert hasattr(L, "moda_synth_normal")
    # bad arguments are rejected on the host, nothing is launched
    L.moda_synth_normal.argtypes = [ctypes.c_void_p, ctypes.c_ulonglong, ctypes.c_ulonglong, ctypes.c_uint,
                                    ctypes.c_int, ctypes.c_void_p]
    assert L.moda_synth_normal(None, 16, 0, 0, 1, None) == 1
    assert L.moda_synth_normal(ctypes.c_void_p(0x1000), 16, 0, 0, 7, None) == 1
    assert L.moda_synth_normal(None, 0, 0, 0, 1, None) == 0


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_generator_values(dtype):
    a = synth.make_inputs(2, 4, 2, 1001, 64, 3, dtype=dtype, seed=5, device="cuda", with_dO=True)
    b = synth.make_inputs(2, 4, 2, 1001, 64, 3, dtype=dtype, seed=5, device="cuda", with_dO=True)
    c = synth.make_inputs(2, 4, 2, 1001, 64, 3, dtype=dtype, seed=6, device="cuda", with_dO=True)
    for k in a:
        assert torch.equal(a[k], b[k]), k                 # reproducible
        assert not torch.equal(a[k], c[k]), k             # the seed matters
    assert not torch.equal(a["Q"], a["dO"]) and not torch.equal(a["Kseq"], a["Vseq"])  # so does the tensor
    x = synth.to_f64(a["Kdepth"]).ravel()
    n = x.size
    assert abs(x.mean()) < 5 / np.sqrt(n) and abs(x.var() - 1.0) < 0.02
    assert abs((x ** 3).mean()) < 0.05 and abs((x ** 4).mean() - 3.0) < 0.1
    # neighbouring elements (the two outputs of one Box-Muller pair, and successive pairs) are uncorrelated
    assert abs(np.mean(x[:-1] * x[1:])) < 5 / np.sqrt(n)
    assert abs(np.mean(x[:-2] * x[2:])) < 5 / np.sqrt(n)
    # odd lengths: the last element is written, nothing beyond it
    t = torch.full((7,), 9.0, dtype=torch.float32, device="cuda")
    u = synth._randn((5,), torch.float32, 1, 0, "cuda")
    assert u.shape == (5,) and torch.isfinite(u).all() and (t == 9.0).all()
