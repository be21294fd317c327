"""Seeded synthetic inputs for MoDA attention.

Holds no attention arithmetic: it only draws iid N(0,1) tensors of the shapes the
operator takes (paper section 2.2; the paper's kernel benchmarks use random
tensors of stated shape) and converts tensors for the CPU checker.  Device tensors
are filled by the build's own counter-based generator (synth_csrc/moda_synth.hip,
libmoda_synth.so: hash of (seed, tensor id, index) -> Box-Muller, on the device).  Both the HIP
path and the tests' fp64 checker consume the SAME buffers produced here: a
tensor is drawn once, on the device it will be used on, and the checker gets an
exact upcast of a copy of it.

Layouts: Q, dO [B,Hq,T,d]; Kseq, Vseq [B,Hk,T,d]; Kdepth, Vdepth
[B,Hk,T,depth_alloc,d] (slots >= depth_count are filled too, so a kernel that
reads them by mistake is caught).
"""
import ctypes
import os

import numpy as np
import torch

_SYNTH_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmoda_synth.so")
_synth_lib = None


def _device_generator():
    """libmoda_synth.so: the build's own counter-based N(0,1) generator, run on the device
    (torch only provides the memory).  Raises if it has not been built."""
    global _synth_lib
    if _synth_lib is None:
        if not os.path.exists(_SYNTH_LIB_PATH):
            raise FileNotFoundError("%s not found: build it with `python -m paper_2603_15619_amd.build`"
                                    % _SYNTH_LIB_PATH)
        L = ctypes.CDLL(_SYNTH_LIB_PATH)
        L.moda_synth_normal.argtypes = [ctypes.c_void_p, ctypes.c_ulonglong, ctypes.c_ulonglong, ctypes.c_uint,
                                        ctypes.c_int, ctypes.c_void_p]
        L.moda_synth_normal.restype = ctypes.c_int
        _synth_lib = L
    return _synth_lib


_DTYPES = {"bf16": torch.bfloat16, "f32": torch.float32}

# Tensor ids keep the streams of different tensors of one call apart.
_TENSOR_IDS = {"Q": 0, "Kseq": 1, "Vseq": 2, "Kdepth": 3, "Vdepth": 4, "dO": 5}


def _randn(shape, dtype, seed, tensor_id, device):
    n = 1
    for s in shape:
        n *= int(s)
    if n == 0:
        return torch.empty(shape, dtype=dtype, device=device)
    if torch.device(device).type == "cuda":
        # on the device: the build's own generator fills the tensor in place
        out = torch.empty(shape, dtype=dtype, device=device)
        with torch.cuda.device(out.device):
            rc = _device_generator().moda_synth_normal(
                ctypes.c_void_p(out.data_ptr()), n, int(seed), int(tensor_id), 1 if dtype == torch.bfloat16 else 0,
                ctypes.c_void_p(torch.cuda.current_stream(out.device).cuda_stream))
        if rc != 0:
            raise RuntimeError("moda_synth_normal rejected its arguments")
        return out
    # host tensors (CPU-only experiments): torch's generator
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed) * 16 + tensor_id)
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


def make_structured_inputs(kind, B, Hq, Hk, T, d, depth_count, seed=0, device="cpu", depth_alloc=None,
                           with_dO=False, scale=None, slope=0.15, excess_log2=6.5, tile=64):
    """bf16 inputs whose LOGITS have a chosen structure (the iid N(0,1) recipe of make_inputs
    never makes a later key tile dominate an earlier one, so an online softmax's rescaling step
    is hardly exercised).  `scale` is the softmax scale the call will use (default 1/sqrt(d)).
    Starting from make_inputs' tensors:
      "rising"         the sequence keys' logits rise by about `slope` (natural-log units) per
                       key position: every key tile's maximum exceeds the previous one's by
                       slope * tile, the running maximum is raised on every tile and earlier
                       contributions are scaled down by large factors;
      "plateau"        the logits of the keys from the second tile on sit about `excess_log2`
                       powers of two above those of the first tile (a maximum that was fixed on
                       the first tile stays below what follows, by a bounded amount);
      "depth_dominant" depth slot 0 of every position is a multiple of the query itself (of the
                       first query head of its group): its logit towers over all others;
      "seq_dominant"   every depth key is a negative multiple of the query: the depth slots'
                       weights vanish next to the sequence keys'.
    Only Q, Kseq and Kdepth are shaped; values stay N(0,1)."""
    import math

    inp = make_inputs(B, Hq, Hk, T, d, depth_count, dtype="bf16", seed=seed, device=device,
                      depth_alloc=depth_alloc, with_dO=with_dO)
    sc = float(scale) if scale else 1.0 / math.sqrt(d)
    qmag = 4.0
    pos = torch.arange(T, device=device, dtype=torch.float32).view(1, 1, T, 1)
    if kind in ("rising", "plateau"):
        # Q = qmag in every channel + noise; a key whose channels all hold c then has the logit
        # sc * qmag * d * c (+ noise terms): c is chosen per position
        if kind == "rising":
            c = slope * pos / (sc * qmag * d)
            knoise = 0.5
        else:
            c = (pos >= tile).float() * (excess_log2 * math.log(2.0)) / (sc * qmag * d)
            knoise = 0.02
        inp["Q"] = (qmag + 0.25 * inp["Q"].float()).to(torch.bfloat16)
        inp["Kseq"] = (c + knoise * inp["Kseq"].float()).to(torch.bfloat16)
        if inp["Kdepth"] is not None and kind == "plateau":
            inp["Kdepth"] = (knoise * inp["Kdepth"].float()).to(torch.bfloat16)
    elif kind in ("depth_dominant", "seq_dominant"):
        if inp["Kdepth"] is None:
            raise ValueError("%s needs depth slots" % kind)
        G = Hq // Hk
        q0 = inp["Q"][:, ::G].float()  # first query head of every group, [B,Hk,T,d]
        if kind == "depth_dominant":
            inp["Kdepth"][:, :, :, 0] = (2.0 * q0).to(torch.bfloat16)
        else:
            qall = inp["Q"].float().view(B, Hk, G, T, d).mean(dim=2)
            inp["Kdepth"] = (-2.0 * G * qall.unsqueeze(3) + 0.1 * inp["Kdepth"].float()).to(torch.bfloat16)
    else:
        raise ValueError("unknown kind %r" % kind)
    return inp


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
