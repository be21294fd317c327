"""GPU parity: the decoding step (moda_attn_decode, through the C ABI) against the fp64 checker.

A decoding step is the operator at the last position of the attended prefix, so the checker's
row-sampled forward with rows = [T-1] is its definition; the depth cache of the step holds the
new token's slots only.  Tolerances: the forward's (2e-2 on O, 1e-3 on LSE, bf16 inputs)."""
import numpy as np
import pytest
import torch

from oracle import moda_ref as R
from paper_2603_15619_amd import synth

pytestmark = pytest.mark.gpu


def check(B, Hq, Hk, T, d, L, seed, kv_alloc=None, depth_alloc=None, scale=None):
    from paper_2603_15619_amd import moda_attn_decode

    kv_alloc = T if kv_alloc is None else kv_alloc
    La = L if depth_alloc is None else depth_alloc
    print("decode case", dict(B=B, Hq=Hq, Hk=Hk, T=T, d=d, L=L, kv_alloc=kv_alloc, depth_alloc=La, seed=seed), flush=True)
    # sequence cache of kv_alloc rows (the rows past T hold NaN: never attended);
    # one query row and one position's depth slots per sequence
    inp = synth.make_inputs(B, Hq, Hk, kv_alloc, d, 0, dtype="bf16", seed=seed, device="cuda")
    one = synth.make_inputs(B, Hq, Hk, 1, d, La, dtype="bf16", seed=seed + 1, device="cuda")
    Kc, Vc = inp["Kseq"], inp["Vseq"]
    Kc[:, :, T:] = float("nan")
    Vc[:, :, T:] = float("nan")
    Q = one["Q"][:, :, 0].contiguous()
    Kd = None if La == 0 else one["Kdepth"][:, :, 0].contiguous()
    Vd = None if La == 0 else one["Vdepth"][:, :, 0].contiguous()
    if La > L:
        Kd[:, :, L:] = float("nan")
        Vd[:, :, L:] = float("nan")
    O, LSE = moda_attn_decode(Q, Kc, Vc, Kd, Vd, T=T, depth_count=L, scale=scale)
    torch.cuda.synchronize()
    rows = np.array([T - 1], dtype=np.int32)
    f = synth.to_f64
    kd = None if La == 0 else np.nan_to_num(f(Kd))[:, :, None]
    vd = None if La == 0 else np.nan_to_num(f(Vd))[:, :, None]
    Oref, Lref = R.fwd_rows(f(Q)[:, :, None], f(Kc[:, :, :T]), f(Vc[:, :, :T]), kd, vd, rows, depth_count=L,
                            scale=scale)
    eo = np.abs(f(O) - Oref[:, :, 0]).max()
    el = np.abs(f(LSE) - Lref[:, :, 0]).max()
    print("   max|dO| = %.3e   max|dLSE| = %.3e" % (eo, el), flush=True)
    assert np.isfinite(f(O)).all() and eo <= 2e-2 and el <= 1e-3


@pytest.mark.parametrize("B,Hq,Hk,T,d,L", [(2, 4, 4, 1000, 128, 15), (1, 8, 1, 777, 64, 5), (3, 6, 2, 300, 128, 0),
                                           (1, 16, 16, 5000, 128, 31), (2, 32, 2, 257, 64, 70), (1, 2, 2, 1, 128, 3),
                                           (1, 2, 1, 17, 64, 0), (4, 16, 8, 4096, 128, 15),
                                           # more than 4 heads per group: the matrix-pipe kernel (5 heads; 40 heads =
                                           # two chunks; the paper's kernel geometry on a long ragged cache; no slots)
                                           (1, 10, 2, 333, 128, 7), (1, 40, 1, 1500, 64, 33),
                                           (1, 64, 8, 20011, 64, 64), (2, 16, 2, 2049, 128, 0)])
def test_decode_shapes(B, Hq, Hk, T, d, L):
    check(B, Hq, Hk, T, d, L, 900 + T + L)


@pytest.mark.parametrize("seed", range(12))
def test_decode_random_shapes(seed):
    """Seeded random shapes: group sizes on both sides of the switch between the two partial
    kernels, ragged cache lengths, cache and slot strides larger than what is attended."""
    rng = np.random.default_rng(4200 + seed)
    d = int(rng.choice([64, 128]))
    Hk = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 16, 33]))
    B = int(rng.integers(1, 4))
    T = int(rng.integers(1, 3000))
    L = int(rng.choice([0, 1, 5, 31, 32, 33, 100]))
    kv_alloc = T + int(rng.integers(0, 70))
    depth_alloc = L + int(rng.integers(0, 5))
    check(B, G * Hk, Hk, T, d, L, 4300 + seed, kv_alloc=kv_alloc, depth_alloc=depth_alloc)


def test_decode_cache_strides_and_scale():
    check(2, 4, 2, 500, 128, 3, 31, kv_alloc=1024, depth_alloc=8)
    check(1, 8, 8, 129, 64, 2, 32, kv_alloc=130, scale=0.3)
    check(1, 8, 1, 500, 64, 3, 36, kv_alloc=600, depth_alloc=8, scale=0.2)


def test_decode_long_cache():
    """B=2, H=16, T=65536: many slices per (batch, head)."""
    check(2, 16, 16, 65536, 128, 15, 33)


def test_decode_matches_last_row_of_prefill():
    """The step's output equals the last row of the full forward over the same prefix (within
    the forward's tolerance on both)."""
    from paper_2603_15619_amd import moda_attn_decode, moda_attn_fwd

    inp = synth.make_inputs(1, 4, 2, 700, 128, 6, dtype="bf16", seed=34, device="cuda")
    O, LSE = moda_attn_fwd(inp["Q"], inp["Kseq"], inp["Vseq"], inp["Kdepth"], inp["Vdepth"])
    Od, Ld = moda_attn_decode(inp["Q"][:, :, -1].contiguous(), inp["Kseq"], inp["Vseq"],
                              inp["Kdepth"][:, :, -1].contiguous(), inp["Vdepth"][:, :, -1].contiguous())
    torch.cuda.synchronize()
    assert (O[:, :, -1].float() - Od.float()).abs().max().item() <= 2e-2
    assert (LSE[:, :, -1] - Ld).abs().max().item() <= 1e-3


def test_decode_rejects_bad_arguments():
    from paper_2603_15619_amd import MODAError, moda_attn_decode

    inp = synth.make_inputs(1, 2, 2, 64, 128, 0, dtype="bf16", seed=35, device="cuda")
    q = inp["Q"][:, :, 0].contiguous()
    with pytest.raises(MODAError):
        moda_attn_decode(q, inp["Kseq"], inp["Vseq"], T=65)  # longer than the cache
    with pytest.raises(MODAError):
        moda_attn_decode(q, inp["Kseq"], inp["Vseq"], T=0)
    with pytest.raises(MODAError):
        moda_attn_decode(q.float(), inp["Kseq"].float(), inp["Vseq"].float())  # bf16 only
