"""GPU parity on inputs whose LOGITS are structured (synth.make_structured_inputs), through the C
ABI against the fp64 CPU oracle: forward, backward and decoding step.

Algorithm 1 raises its running maximum whenever a block brings a larger score (m' = max(m, max S))
and scales what it has accumulated by 2^(m - m').  With iid N(0,1) inputs that only happens on the
first blocks of a row.  Here the logits rise along the sequence, so that every key tile of every
row raises the maximum; or they sit a bounded amount above the first tile's, so that a kernel
which raises its maximum lazily accumulates weights far above 1; or one depth slot towers over
the row; or the depth slots vanish next to the sequence keys; or the softmax scale is far above
1/sqrt(d).  Both workgroup geometries of the bf16 forward kernel and both head dimensions are
covered; the shapes give every kernel workgroups that take their depth slots before the key loop
and workgroups that take them after it.  Tolerances: the forward's (2e-2 on O, 1e-3 on LSE) and
the backward's (tests/test_bwd_parity.py).
"""
import numpy as np
import pytest
import torch

from oracle import moda_ref as R
from paper_2603_15619_amd import synth

from test_bwd_parity import NAMES, compare, run_gpu as run_bwd_gpu
from test_fwd_parity import check_full as check_fwd_full, check_sampled as check_fwd_sampled

pytestmark = pytest.mark.gpu

KINDS = [("rising", dict(slope=0.15)), ("rising", dict(slope=0.05)), ("plateau", dict(excess_log2=6.5)),
         ("plateau", dict(excess_log2=7.8)), ("depth_dominant", {}), ("seq_dominant", {})]


def structured(kind, kw, B, Hq, Hk, T, d, L, seed, scale=None, with_dO=False, depth_alloc=None):
    return synth.make_structured_inputs(kind, B, Hq, Hk, T, d, L, seed=seed, device="cuda", scale=scale,
                                        with_dO=with_dO, depth_alloc=depth_alloc, **kw)


@pytest.mark.parametrize("waves", [4, 8])
@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("kind,kw", KINDS)
def test_fwd_structured(kind, kw, d, waves):
    B, Hq, Hk, T, L = 2, 4, 2, 1500, 5
    inp = structured(kind, kw, B, Hq, Hk, T, d, L, seed=700 + d + waves)
    check_fwd_full(B, Hq, Hk, T, d, L, "bf16", 0, tuning=dict(waves=waves), inp=inp)


@pytest.mark.parametrize("d,scale", [(128, 1.0), (64, 0.75)])
def test_fwd_large_scale(d, scale):
    """iid N(0,1) inputs with a softmax scale far above 1/sqrt(d): logits of standard deviation
    ~sqrt(d) * scale, one or two keys carry each row, so |O| reaches the largest |V| (about 5 among
    a million N(0,1) values) instead of the ~0.1 of the task's configurations.  The task's 2e-2 is
    stated for those; here the bound is what bf16 arithmetic guarantees for values of that size:
    weights rounded to bf16 (relative 2^-8, at most 2^-8 max|V| on the weighted sum) plus the
    output's own rounding (2^-8 |O|), i.e. 2 * 2^-8 * max|V| (3.9e-2 at 5); the measured error
    is about 2e-2."""
    B, Hq, Hk, T, L, seed = 2, 4, 2, 1300, 7, 720 + d
    inp = synth.make_inputs(B, Hq, Hk, T, d, L, dtype="bf16", seed=seed, device="cuda")
    vmax = max(inp["Vseq"].abs().max().item(), inp["Vdepth"].abs().max().item())
    check_fwd_full(B, Hq, Hk, T, d, L, "bf16", seed, scale=scale, inp=inp, tol_o=2 * 2.0 ** -8 * vmax)


@pytest.mark.parametrize("kind,kw", [("rising", dict(slope=0.15)), ("plateau", dict(excess_log2=7.0))])
def test_fwd_structured_grouped_heads_per_tile(kind, kw):
    """Eight query heads of a group in one tile (the paper's kernel-benchmark geometry, d = 64)."""
    B, Hq, Hk, T, d, L = 1, 16, 2, 900, 64, 9
    inp = structured(kind, kw, B, Hq, Hk, T, d, L, seed=730)
    check_fwd_full(B, Hq, Hk, T, d, L, "bf16", 0, inp=inp)


def test_fwd_rising_long_sequence_sampled():
    """Rising logits at the length of the 1.5B-model-shaped configuration (T = 4096, 16 heads):
    64 key tiles per row, the maximum raised on every one of them."""
    B, H, T, d, L = 2, 16, 4096, 128, 15
    inp = structured("rising", dict(slope=0.1), B, H, H, T, d, L, seed=740)
    check_fwd_sampled(B, H, H, T, d, L, "bf16", 740, n_random=16, inp=inp)


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("kind,kw", KINDS)
def test_bwd_structured(kind, kw, d):
    B, Hq, Hk, T, L = 1, 4, 2, 700, 5
    inp = structured(kind, kw, B, Hq, Hk, T, d, L, seed=750 + d, with_dO=True)
    print("bwd structured", kind, kw, dict(B=B, Hq=Hq, Hk=Hk, T=T, d=d, L=L), flush=True)
    grads = run_bwd_gpu(inp, L)
    args = [synth.to_f64(inp[k]) for k in ("Q", "Kseq", "Vseq", "Kdepth", "Vdepth", "dO")]
    ref = R.bwd(*args, depth_count=L)
    noise = R.bwd_noise(*args, depth_count=L)
    for name, g, r, n in zip(NAMES, grads, ref, noise):
        compare(name, g, r, n)


def test_bwd_structured_no_groups_and_large_scale():
    """One query head per key/value head (the depth-slot gradients then run inside the dK/dV
    kernel) on rising logits, and iid inputs with scale = 1."""
    B, H, T, d, L = 2, 2, 600, 128, 7
    for kind, kw, scale in (("rising", dict(slope=0.15), None), ("depth_dominant", {}, None)):
        inp = structured(kind, kw, B, H, H, T, d, L, seed=760, with_dO=True)
        grads = run_bwd_gpu(inp, L)
        args = [synth.to_f64(inp[k]) for k in ("Q", "Kseq", "Vseq", "Kdepth", "Vdepth", "dO")]
        ref, noise = R.bwd(*args, depth_count=L), R.bwd_noise(*args, depth_count=L)
        for name, g, r, n in zip(NAMES, grads, ref, noise):
            compare(name + ":" + kind, g, r, n)
    inp = synth.make_inputs(B, H, H, T, d, L, dtype="bf16", seed=761, device="cuda", with_dO=True)
    grads = run_bwd_gpu(inp, L, scale=1.0)
    args = [synth.to_f64(inp[k]) for k in ("Q", "Kseq", "Vseq", "Kdepth", "Vdepth", "dO")]
    ref, noise = R.bwd(*args, depth_count=L, scale=1.0), R.bwd_noise(*args, depth_count=L, scale=1.0)
    for name, g, r, n in zip(NAMES, grads, ref, noise):
        compare(name + ":scale1", g, r, n)


@pytest.mark.parametrize("d,Hq,Hk", [(128, 4, 4), (64, 16, 2)])
@pytest.mark.parametrize("kind,kw", KINDS)
def test_decode_structured(kind, kw, d, Hq, Hk):
    """Decoding step on structured caches: the slices of the sequence cache have very different
    maxima (rising), or the depth slots dominate / vanish in the merge."""
    from paper_2603_15619_amd import moda_attn_decode

    B, T, L = 2, 3000, 6
    inp = structured(kind, kw, B, Hq, Hk, T, d, L, seed=770 + d)
    Q = inp["Q"][:, :, -1].contiguous()
    Kd, Vd = inp["Kdepth"][:, :, -1].contiguous(), inp["Vdepth"][:, :, -1].contiguous()
    O, LSE = moda_attn_decode(Q, inp["Kseq"], inp["Vseq"], Kd, Vd)
    torch.cuda.synchronize()
    f = synth.to_f64
    rows = np.array([T - 1], dtype=np.int32)
    Oref, Lref = R.fwd_rows(f(Q)[:, :, None], f(inp["Kseq"]), f(inp["Vseq"]), f(Kd)[:, :, None], f(Vd)[:, :, None],
                            rows, depth_count=L)
    eo = np.abs(f(O) - Oref[:, :, 0]).max()
    el = np.abs(f(LSE) - Lref[:, :, 0]).max()
    print("decode structured", kind, kw, "d=%d  max|dO| = %.3e  max|dLSE| = %.3e" % (d, eo, el), flush=True)
    assert np.isfinite(f(O)).all() and eo <= 2e-2 and el <= 1e-3
