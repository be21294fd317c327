"""GPU parity: libmoda backward (through the C ABI) against the fp64 CPU oracle.

The backward consumes O and LSE of the library's own forward.  Inputs are bf16; gradients come
back in bf16 after fp32 accumulation.

Tolerance.  The paper gives no figure for the backward (it only times it, Table 2), so the bound
is derived from the arithmetic and follows the length of the sums.  A gradient element is a sum
over N (query, key) pairs of terms that each carry a weight p or a logit gradient e; the kernels
round p and e to bf16 before the matrix products, and delta = <dO, O> is formed from the forward's
bf16 output.  Each of those roundings is a relative error of at most U = 2^-8 (bf16 keeps 8
significant bits), uniformly distributed, i.e. of standard deviation at most U / sqrt(3), and
they are independent from pair
to pair, so the error of the sum has standard deviation (U / sqrt(3)) * noise, where
noise = sqrt(sum of the squared terms) (+ the delta contribution) is what the checker's
`bwd_noise` returns: it grows like sqrt(N) * |typical term|.  The result is then rounded to bf16
once (relative U).  Per element:

    |got - ref| <= KSIGMA * (U / sqrt(3)) * noise + 1.25 U |ref| + FLOOR

with KSIGMA = 6 (the largest of 1e8 Gaussian deviates is about 5.7 sigma), 1.25 U instead of U
for the output rounding so that the fp32 accumulation order and the exp2 approximation have
room, and FLOOR = 1e-6 for elements whose reference is zero.  (A CPU emulation of exactly these
roundings, on the first shape of test_bwd_shapes, gives errors of 1.0 standard deviations rms
and at most 0.5 of this bound.)
"""
import math

import numpy as np
import pytest
import torch

from oracle import moda_ref as R
from paper_2603_15619_amd import synth

pytestmark = pytest.mark.gpu

U = 2.0 ** -8
KSIGMA = 6.0
FLOOR = 1e-6
NAMES = ("dQ", "dKseq", "dVseq", "dKdepth", "dVdepth")


def tolerance(ref, noise):
    return KSIGMA * (U / math.sqrt(3.0)) * noise + 1.25 * U * np.abs(ref) + FLOOR


def run_gpu(inp, L, causal=True, scale=None):
    from paper_2603_15619_amd import moda_attn_bwd, moda_attn_fwd

    O, LSE = moda_attn_fwd(inp["Q"], inp["Kseq"], inp["Vseq"], inp["Kdepth"], inp["Vdepth"],
                           depth_count=L, causal=causal, scale=scale)
    grads = moda_attn_bwd(inp["Q"], inp["Kseq"], inp["Vseq"], inp["Kdepth"], inp["Vdepth"], O, LSE,
                          inp["dO"], depth_count=L, causal=causal, scale=scale)
    torch.cuda.synchronize()
    return grads


def compare(name, got, ref, noise):
    got = synth.to_f64(got)
    assert np.isfinite(got).all(), name
    err = np.abs(got - ref)
    tol = tolerance(ref, noise)
    ratio = float((err / tol).max()) if err.size else 0.0
    sig = float((err / np.maximum((U / math.sqrt(3.0)) * noise, 1e-30))[noise > 0].max()) if (noise > 0).any() else 0.0
    print("   %-8s max|err| = %.3e  max|ref| = %.3e  max noise = %.3e  worst err/tol = %.3f  (err in sigmas of "
          "the noise model, output rounding included: %.2f)" %
          (name, err.max() if err.size else 0.0, np.abs(ref).max() if ref.size else 0.0,
           noise.max() if noise.size else 0.0, ratio, sig), flush=True)
    assert ratio <= 1.0, name


def check_full(B, H, T, d, L, seed, causal=True, depth_alloc=None, scale=None, Hk=None, inp=None):
    Hk = H if Hk is None else Hk
    print("bwd case", dict(B=B, Hq=H, Hk=Hk, T=T, d=d, L=L, seed=seed, causal=causal, depth_alloc=depth_alloc),
          flush=True)
    if inp is None:
        inp = synth.make_inputs(B, H, Hk, T, d, L, dtype="bf16", seed=seed, device="cuda",
                                depth_alloc=depth_alloc, with_dO=True)
    grads = run_gpu(inp, L, causal, scale)
    args = [synth.to_f64(inp[k]) for k in ("Q", "Kseq", "Vseq", "Kdepth", "Vdepth", "dO")]
    ref = R.bwd(*args, depth_count=L, causal=causal, scale=scale)
    noise = R.bwd_noise(*args, depth_count=L, causal=causal, scale=scale)
    for name, g, r, n in zip(NAMES, grads, ref, noise):
        if r is None:
            assert g is None
            continue
        compare(name, g, r, n)


@pytest.mark.parametrize("T,d,L", [(300, 128, 5), (200, 64, 3), (130, 128, 0), (257, 128, 15),
                                   (64, 64, 9), (1, 128, 2), (500, 128, 17)])
def test_bwd_shapes(T, d, L):
    check_full(2, 2, T, d, L, 300 + T + L)


def test_bwd_non_causal_and_slot_stride():
    check_full(1, 2, 333, 128, 3, 21, causal=False)
    check_full(1, 2, 300, 128, 4, 22, depth_alloc=6)
    check_full(1, 3, 260, 64, 2, 23, scale=0.2)


def test_bwd_deterministic():
    inp = synth.make_inputs(1, 2, 2, 400, 128, 7, dtype="bf16", seed=24, device="cuda", with_dO=True)
    a = run_gpu(inp, 7)
    b = run_gpu(inp, 7)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_bwd_rejects_unsupported():
    from paper_2603_15619_amd import MODAError

    inp = synth.make_inputs(1, 128, 1, 64, 128, 2, dtype="bf16", seed=25, device="cuda", with_dO=True)
    with pytest.raises(MODAError):  # more than 64 query heads per key/value head
        run_gpu(inp, 2)


@pytest.mark.parametrize("Hq,Hk,T,d,L,La", [(4, 2, 300, 128, 5, None), (8, 1, 200, 64, 3, 4), (6, 2, 257, 128, 0, 2),
                                            (8, 2, 130, 64, 9, None), (2, 1, 64, 128, 0, 0), (16, 2, 500, 64, 17, None),
                                            (16, 1, 200, 128, 5, 7), (24, 1, 130, 64, 3, None), (12, 1, 257, 128, 4, None)])
def test_bwd_grouped_queries(Hq, Hk, T, d, L, La):
    """G = Hq / Hk query heads share a key/value head: the gradients of the shared sequence
    and depth keys / values sum over the group (G = 2, 3, 4, 8, 12, 16, 24; the paper's models
    use G = 2, its kernel benchmarks G = 8 and, in two rows, 16 and 32)."""
    check_full(2, Hq, T, d, L, 500 + T + L, depth_alloc=La, Hk=Hk)


def test_bwd_grouped_queries_non_causal_deterministic():
    check_full(1, 4, 333, 128, 3, 26, causal=False, Hk=2)
    inp = synth.make_inputs(1, 8, 2, 400, 64, 7, dtype="bf16", seed=27, device="cuda", with_dO=True)
    a = run_gpu(inp, 7)
    b = run_gpu(inp, 7)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_config5_t256_slice_full():
    """B=8, H=16, d=128, depth_count=15: the T=256 problem, all five gradients in full."""
    check_full(8, 16, 256, 128, 15, 4)


def test_config5_full_size_sampled():
    """B=8, H=16, d=128, T=4096, depth_count=15: row-local gradients on sampled rows of
    every (b, h), and dKseq / dVseq in full for two (b, h) against a full-T oracle."""
    B, H, T, d, L = 8, 16, 4096, 128, 15
    inp = synth.make_inputs(B, H, H, T, d, L, dtype="bf16", seed=4, device="cuda", with_dO=True)
    dQ, dK, dV, dKd, dVd = run_gpu(inp, L)
    rows = synth.sample_rows(T, n_random=16, edge=4, tile=512, seed=4)
    ridx = torch.from_numpy(rows.astype(np.int64)).cuda()
    pick = lambda t: synth.to_f64(t.index_select(2, ridx))
    rargs = (pick(inp["Q"]), synth.to_f64(inp["Kseq"]), synth.to_f64(inp["Vseq"]),
             pick(inp["Kdepth"]), pick(inp["Vdepth"]), pick(inp["dO"]), rows)
    rq, rkd, rvd = R.bwd_rows(*rargs, depth_count=L)
    nq, nkd, nvd = R.bwd_noise_rows(*rargs, depth_count=L)
    compare("dQ", dQ.index_select(2, ridx), rq, nq)
    compare("dKdepth", dKd.index_select(2, ridx), rkd, nkd)
    compare("dVdepth", dVd.index_select(2, ridx), rvd, nvd)
    # two (b, h) slabs in full: (0, 0) and (B-1, H-1)
    for (b, h) in [(0, 0), (B - 1, H - 1)]:
        sl = lambda t: synth.to_f64(t[b:b + 1, h:h + 1])
        sargs = (sl(inp["Q"]), sl(inp["Kseq"]), sl(inp["Vseq"]), sl(inp["Kdepth"]), sl(inp["Vdepth"]), sl(inp["dO"]))
        ref = R.bwd(*sargs, depth_count=L)
        noise = R.bwd_noise(*sargs, depth_count=L)
        compare("dKseq[%d,%d]" % (b, h), dK[b:b + 1, h:h + 1], ref[1], noise[1])
        compare("dVseq[%d,%d]" % (b, h), dV[b:b + 1, h:h + 1], ref[2], noise[2])
    for g in (dQ, dK, dV, dKd, dVd):
        assert torch.isfinite(g.float()).all()


@pytest.mark.parametrize("Hq,Hk,L", [(2, 2, 1), (2, 2, 5), (2, 2, 7), (4, 2, 3)])
def test_bwd_unattended_slots_may_hold_nan(Hq, Hk, L):
    """Slots >= depth_count of a cache that is still being filled hold NaN bit patterns: they
    take no part, and their gradients are written as zero."""
    inp = synth.make_inputs(1, Hq, Hk, 200, 128, L, dtype="bf16", seed=28, device="cuda", depth_alloc=8,
                            with_dO=True)
    inp["Kdepth"][:, :, :, L:] = float("nan")
    inp["Vdepth"][:, :, :, L:] = float("nan")
    grads = run_gpu(inp, L)
    clean = {k: (None if v is None else v.clone()) for k, v in inp.items()}
    clean["Kdepth"][:, :, :, L:] = 0
    clean["Vdepth"][:, :, :, L:] = 0
    cargs = [synth.to_f64(clean[k]) for k in ("Q", "Kseq", "Vseq", "Kdepth", "Vdepth", "dO")]
    ref = R.bwd(*cargs, depth_count=L)
    noise = R.bwd_noise(*cargs, depth_count=L)
    for name, g, r, n in zip(NAMES, grads, ref, noise):
        compare(name, g, r, n)
    assert torch.count_nonzero(grads[3][:, :, :, L:].float()) == 0
    assert torch.count_nonzero(grads[4][:, :, :, L:].float()) == 0


def test_bwd_paper_kernel_benchmark_heads_t256():
    """Head geometry of the paper's kernel benchmark (Hq=64, Hk=8, d=64, 64 slots) on a T=256 problem,
    all five gradients in full."""
    check_full(1, 64, 256, 64, 64, 29, Hk=8)


def test_bwd_many_heads_short_sequence():
    """A case that a randomised sweep once found above a flat 2e-2 bound: 16 query heads on one
    key/value head, T = 257, d = 128, 2 of 5 slots attended (|dK| up to 8: long sums of large
    terms)."""
    check_full(3, 16, 257, 128, 2, 1046, depth_alloc=5, Hk=1)


@pytest.mark.parametrize("Hq,Hk,T,d,L", [(32, 1, 200, 64, 5), (64, 2, 130, 64, 3), (64, 1, 100, 128, 4),
                                         (48, 1, 150, 128, 2), (20, 2, 130, 64, 7)])
def test_bwd_wide_groups(Hq, Hk, T, d, L):
    """Groups of more than 8 query heads (G = 10, 32, 48, 64): the depth-slot gradients sum over
    the whole group in fp32 and are rounded once."""
    check_full(1, Hq, T, d, L, 600 + Hq + T, Hk=Hk)


def test_bwd_paper_table2_groups_and_slot_counts():
    """Table 2's other axes on T = 256 problems, all five gradients in full: G = 32 (Hq = 256,
    Hk = 8, 64 slots) and 128 / 256 slots at G = 8 (d = 64)."""
    check_full(1, 256, 256, 64, 64, 30, Hk=8)
    check_full(1, 16, 256, 64, 128, 31, Hk=2)
    check_full(1, 8, 256, 64, 256, 32, Hk=1)


def test_bwd_paper_shape_full_length_sampled():
    """A Table 2 shape at full length (row 1: T = 4096, Hq = 64, Hk = 8, d = 64, 64 slots): the
    row-local gradients on sampled rows of every head."""
    B, Hq, Hk, T, d, L = 1, 64, 8, 4096, 64, 64
    inp = synth.make_inputs(B, Hq, Hk, T, d, L, dtype="bf16", seed=33, device="cuda", with_dO=True)
    dQ, dK, dV, dKd, dVd = run_gpu(inp, L)
    rows = synth.sample_rows(T, n_random=8, edge=2, tile=1024, seed=33)
    ridx = torch.from_numpy(rows.astype(np.int64)).cuda()
    pick = lambda t: synth.to_f64(t.index_select(2, ridx))
    rargs = (pick(inp["Q"]), synth.to_f64(inp["Kseq"]), synth.to_f64(inp["Vseq"]),
             pick(inp["Kdepth"]), pick(inp["Vdepth"]), pick(inp["dO"]), rows)
    rq, rkd, rvd = R.bwd_rows(*rargs, depth_count=L)
    nq, nkd, nvd = R.bwd_noise_rows(*rargs, depth_count=L)
    compare("dQ", dQ.index_select(2, ridx), rq, nq)
    compare("dKdepth", dKd.index_select(2, ridx), rkd, nkd)
    compare("dVdepth", dVd.index_select(2, ridx), rvd, nvd)
    for g in (dQ, dK, dV, dKd, dVd):
        assert torch.isfinite(g.float()).all()
