"""Seeded synthetic inputs for MoDA attention.

Holds no attention arithmetic: it only draws iid N(0,1) tensors of the shapes the
operator takes (paper section 2.2; the paper's kernel benchmarks use random
tensors of stated shape) and converts tensors for the CPU checker.  Both the HIP
path and the tests' fp64 checker consume the SAME buffers produced here: a
tensor is drawn once, on the device it will be used on, and the checker gets an
exact upcast of a copy of it.

Layouts: Q, dO [B,Hq,T,d]; Kseq, Vseq [B,Hk,T,d]; Kdepth, Vdepth
[B,Hk,T,depth_alloc,d] (slots >= depth_count are filled too, so a kernel that
reads them by mistake is caught).
"""
import numpy as np
import torch

_DTYPES = {"bf16": torch.bfloat16, "f32": torch.float32}

# Tensor ids keep the streams of different tensors of one call apart.
_TENSOR_IDS = {"Q": 0, "Kseq": 1, "Vseq": 2, "Kdepth": 3, "Vdepth": 4, "dO": 5}


def _randn(shape, dtype, seed, tensor_id, device):
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed) * 16 + tensor_id)
    n = 1
    for s in shape:
        n *= int(s)
    if n == 0:
        return torch.empty(shape, dtype=dtype, device=device)
    # Draw in slabs along dim 0 so a multi-GB bf16 tensor never needs an fp32 twin.
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    step = 1 << 28
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        flat[lo:hi] = torch.randn(hi - lo, generator=gen, device=device, dtype=torch.float32).to(dtype)
    return out


def make_inputs(B, Hq, Hk, T, d, depth_count, dtype="bf16", seed=0, device="cpu",
                depth_alloc=None, with_dO=False):
    """Return a dict of torch tensors on `device` (Kdepth/Vdepth are None when
    depth_alloc == 0)."""
    tdt = _DTYPES[dtype]
    depth_alloc = depth_count if depth_alloc is None else depth_alloc
    assert depth_alloc >= depth_count >= 0
    out = {
        "Q": _randn((B, Hq, T, d), tdt, seed, _TENSOR_IDS["Q"], device),
        "Kseq": _randn((B, Hk, T, d), tdt, seed, _TENSOR_IDS["Kseq"], device),
        "Vseq": _randn((B, Hk, T, d), tdt, seed, _TENSOR_IDS["Vseq"], device),
        "Kdepth": None,
        "Vdepth": None,
    }
    if depth_alloc > 0:
        out["Kdepth"] = _randn((B, Hk, T, depth_alloc, d), tdt, seed, _TENSOR_IDS["Kdepth"], device)
        out["Vdepth"] = _randn((B, Hk, T, depth_alloc, d), tdt, seed, _TENSOR_IDS["Vdepth"], device)
    if with_dO:
        out["dO"] = _randn((B, Hq, T, d), tdt, seed, _TENSOR_IDS["dO"], device)
    return out


def to_f64(t):
    """Exact upcast of a torch tensor (any device, bf16/f32) to a float64 numpy array."""
    if t is None:
        return None
    return t.detach().to("cpu").to(torch.float64).numpy()


def sample_rows(T, n_random=64, edge=8, tile=256, seed=0):
    """Query positions for sampled checks of a long problem: the first and last
    `edge` rows, the rows either side of every `tile` boundary (capped), and
    `n_random` seeded random rows.  Sorted, unique."""
    rows = set(range(min(edge, T))) | set(range(max(0, T - edge), T))
    bounds = list(range(tile, T, tile))
    if len(bounds) > 32:
        idx = np.linspace(0, len(bounds) - 1, 32).astype(int)
        bounds = [bounds[i] for i in idx]
    for b in bounds:
        rows.update((b - 1, b))
    rng = np.random.default_rng(seed)
    if T > 0 and n_random > 0:
        rows.update(int(x) for x in rng.integers(0, T, size=n_random))
    return np.array(sorted(rows), dtype=np.int32)
