"""GPU parity: the depth stream's write step (moda_depth_append, through the C ABI) against
plain array indexing, bit for bit; and a stack of layers that reads the stream with the
attention kernel while it is being filled (depth_alloc > depth_count)."""
import numpy as np
import pytest
import torch

from oracle import moda_ref as R
from paper_2603_15619_amd import synth

pytestmark = pytest.mark.gpu


def bits(t):
    """Raw element bits of a tensor as a numpy integer array (bf16 -> uint16, fp32 -> uint32)."""
    it = torch.int16 if t.dtype == torch.bfloat16 else torch.int32
    return t.detach().contiguous().view(it).cpu().numpy()


@pytest.mark.parametrize("dtype,B,Hk,T,d,La,slot", [("bf16", 2, 3, 333, 128, 5, 2), ("bf16", 1, 2, 1000, 64, 16, 15),
                                                     ("f32", 2, 2, 130, 64, 3, 0), ("bf16", 1, 1, 1, 128, 1, 0),
                                                     ("f32", 1, 2, 77, 128, 4, 3)])
def test_append_bit_exact(dtype, B, Hk, T, d, La, slot):
    from paper_2603_15619_amd import moda_depth_append

    print("append case", dict(dtype=dtype, B=B, Hk=Hk, T=T, d=d, La=La, slot=slot), flush=True)
    inp = synth.make_inputs(B, Hk, Hk, T, d, La, dtype=dtype, seed=600 + T, device="cuda")
    K, V, Kd, Vd = inp["Kseq"], inp["Vseq"], inp["Kdepth"], inp["Vdepth"]
    ek, ev = R.depth_append(bits(Kd), bits(Vd), bits(K), bits(V), slot)
    moda_depth_append(K, V, Kd, Vd, slot)
    torch.cuda.synchronize()
    assert np.array_equal(bits(Kd), ek) and np.array_equal(bits(Vd), ev)


def test_append_rejects_bad_arguments_and_empty():
    from paper_2603_15619_amd import MODAError, moda_depth_append

    inp = synth.make_inputs(1, 2, 2, 16, 64, 3, dtype="bf16", seed=1, device="cuda")
    with pytest.raises(MODAError):
        moda_depth_append(inp["Kseq"], inp["Vseq"], inp["Kdepth"], inp["Vdepth"], 3)
    with pytest.raises(MODAError):
        moda_depth_append(inp["Kseq"], inp["Vseq"], inp["Kdepth"], inp["Vdepth"], -1)
    e = torch.empty(0, 2, 16, 64, dtype=torch.bfloat16, device="cuda")
    ed = torch.empty(0, 2, 16, 3, 64, dtype=torch.bfloat16, device="cuda")
    moda_depth_append(e, e, ed, ed, 1)


def test_layer_stack_reads_the_stream_it_fills():
    """Six layers share one cache allocated for six writers: layer l attends the l slots
    written so far (depth_count = l < depth_alloc), then appends its own K / V.  Every layer's
    output is checked against the fp64 checker fed with the explicitly stacked history."""
    from paper_2603_15619_amd import moda_attn_fwd, moda_depth_append

    B, Hq, Hk, T, d, NL = 1, 4, 2, 300, 128, 6
    Kd = torch.full((B, Hk, T, NL, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    Vd = torch.full_like(Kd, float("nan"))
    hist_k, hist_v = [], []
    for l in range(NL):
        inp = synth.make_inputs(B, Hq, Hk, T, d, 0, dtype="bf16", seed=700 + l, device="cuda")
        O, LSE = moda_attn_fwd(inp["Q"], inp["Kseq"], inp["Vseq"], Kd, Vd, depth_count=l)
        torch.cuda.synchronize()
        kd = np.stack(hist_k, axis=3) if l else None
        vd = np.stack(hist_v, axis=3) if l else None
        Oref, Lref = R.fwd(synth.to_f64(inp["Q"]), synth.to_f64(inp["Kseq"]), synth.to_f64(inp["Vseq"]), kd, vd,
                           depth_count=l)
        eo = np.abs(synth.to_f64(O) - Oref).max()
        el = np.abs(synth.to_f64(LSE) - Lref).max()
        print("   layer %d: max|dO| = %.3e   max|dLSE| = %.3e" % (l, eo, el), flush=True)
        assert eo <= 2e-2 and el <= 1e-3  # the forward's bf16 tolerances
        moda_depth_append(inp["Kseq"], inp["Vseq"], Kd, Vd, l)
        hist_k.append(synth.to_f64(inp["Kseq"]))
        hist_v.append(synth.to_f64(inp["Vseq"]))
    torch.cuda.synchronize()
    assert np.array_equal(synth.to_f64(Kd), np.stack(hist_k, axis=3))
