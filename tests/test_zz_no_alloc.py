"""GPU test of moda_attn_decode_noalloc (through the C ABI): the entry point that allocates
nothing gives the results of moda_attn_decode, on two calls in a row that share the library's
scratch array, the second on a smaller input (so that stale partial results of the first call lie
beyond what the second one writes)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import moda_ref as R
from paper_2603_15619_amd import synth

pytestmark = pytest.mark.gpu


def _inputs(B, Hq, Hk, T, d, L, seed):
    inp = synth.make_inputs(B, Hq, Hk, T, d, 0, dtype="bf16", seed=seed, device="cuda")
    one = synth.make_inputs(B, Hq, Hk, 1, d, L, dtype="bf16", seed=seed + 1, device="cuda")
    return (one["Q"][:, :, 0].contiguous(), inp["Kseq"], inp["Vseq"], one["Kdepth"][:, :, 0].contiguous(),
            one["Vdepth"][:, :, 0].contiguous())


def test_noalloc_matches_workspace_entry_point_twice():
    from paper_2603_15619_amd import MODAError, lib, moda_attn_decode

    assert lib().moda_attn_decode_noalloc_max_bytes() == 8 << 20
    f = synth.to_f64
    # first a large call (many slices per head), then a smaller one
    for (B, Hq, Hk, T, d, L, seed) in ((4, 16, 4, 40000, 128, 15, 950), (2, 8, 2, 3000, 64, 6, 960)):
        print("noalloc case", dict(B=B, Hq=Hq, Hk=Hk, T=T, d=d, L=L), flush=True)
        Q, Kc, Vc, Kd, Vd = _inputs(B, Hq, Hk, T, d, L, seed)
        O_ref, L_ref = moda_attn_decode(Q, Kc, Vc, Kd, Vd)
        O = torch.full_like(Q, float("nan"))
        LSE = torch.full((B, Hq), float("nan"), dtype=torch.float32, device="cuda")
        moda_attn_decode(Q, Kc, Vc, Kd, Vd, out=O, lse=LSE, noalloc=True)
        torch.cuda.synchronize()
        # the same kernels on the same inputs: identical bits
        assert torch.equal(O, O_ref) and torch.equal(LSE, L_ref)
        # and the operator's definition, to the forward's tolerance
        rows = np.array([T - 1], dtype=np.int32)
        Oo, Lo = R.fwd_rows(f(Q)[:, :, None], f(Kc), f(Vc), f(Kd)[:, :, None], f(Vd)[:, :, None], rows, depth_count=L)
        assert np.abs(f(O) - Oo[:, :, 0]).max() <= 2e-2 and np.abs(f(LSE) - Lo[:, :, 0]).max() <= 1e-3
    # a shape whose partial results do not fit the library's array is rejected, nothing launched
    B, Hq, Hk, T, d = 8, 64, 1, 65536, 128
    s = lib().moda_attn_decode_workspace_bytes
    from paper_2603_15619_amd.binding import MODAShape
    shape = MODAShape(B, Hq, Hk, T, d, 0, 0, 1, 0.0, 1)
    assert s(ctypes.byref(shape)) > 8 << 20
    p = ctypes.c_void_p(0x1000)
    assert lib().moda_attn_decode_noalloc(p, p, p, None, None, p, p, T, ctypes.byref(shape), None) == 6
