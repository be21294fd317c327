"""ctypes front end of the fp64 CPU oracle (oracle/moda_ref.c).

Test infrastructure only.  Every function takes numpy arrays (any float dtype;
they are upcast exactly to float64, so bf16/fp32 input rounding is not part of
the error budget) and returns float64 numpy arrays.  All arithmetic happens in
the C file; this module only marshals arguments.

Operator definition: paper section 2.2 (Mixture-of-Depths Attention), Eq. 2,
Algorithm 1.  Layouts: Q [B,Hq,T,d]; Kseq/Vseq [B,Hk,T,d];
Kdepth/Vdepth [B,Hk,T,depth_alloc,d]; LSE [B,Hq,T].
"""
import ctypes
import math

import numpy as np

from .build import build_oracle

_lib = None
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int)


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build_oracle(force=False))
        for name in ("moda_ref_fwd_f64", "moda_ref_fwd_rows_f64", "moda_ref_weights_f64",
                     "moda_ref_bwd_f64", "moda_ref_bwd_rows_f64", "moda_ref_bwd_noise_f64",
                     "moda_ref_bwd_noise_rows_f64", "moda_ref_num_threads"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().moda_ref_num_threads())


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(_dp)


def _dims(Q, Kseq, Kdepth, depth_count):
    B, Hq, _, d = Q.shape
    _, Hk, T, _ = Kseq.shape
    if Kdepth is None:
        depth_alloc = 0
        if depth_count is None:
            depth_count = 0
    else:
        depth_alloc = Kdepth.shape[3]
        if depth_count is None:
            depth_count = depth_alloc
    return B, Hq, Hk, T, d, depth_alloc, depth_count


def _scale(scale, d):
    return float(scale) if scale is not None and scale > 0 else 1.0 / math.sqrt(d)


def fwd(Q, Kseq, Vseq, Kdepth=None, Vdepth=None, depth_count=None, causal=True, scale=None):
    """Full forward.  Returns (O [B,Hq,T,d], LSE [B,Hq,T]) in float64."""
    Q, Kseq, Vseq, Kdepth, Vdepth = map(_f64, (Q, Kseq, Vseq, Kdepth, Vdepth))
    B, Hq, Hk, T, d, da, dc = _dims(Q, Kseq, Kdepth, depth_count)
    assert Q.shape[2] == T
    O = np.empty((B, Hq, T, d), np.float64)
    LSE = np.empty((B, Hq, T), np.float64)
    rc = lib().moda_ref_fwd_f64(_p(Q), _p(Kseq), _p(Vseq), _p(Kdepth), _p(Vdepth), _p(O), _p(LSE),
                                B, Hq, Hk, T, d, da, dc, int(bool(causal)),
                                ctypes.c_double(_scale(scale, d)))
    if rc != 0:
        raise ValueError("moda_ref_fwd_f64 rejected its arguments")
    return O, LSE


def fwd_rows(Q_rows, Kseq, Vseq, Kdepth_rows, Vdepth_rows, rows, depth_count=None, causal=True,
             scale=None):
    """Forward for the listed positions only.  Q_rows [B,Hq,R,d], depth rows
    [B,Hk,R,depth_alloc,d], Kseq/Vseq full.  Returns (O_rows, LSE_rows)."""
    Q_rows, Kseq, Vseq, Kdepth_rows, Vdepth_rows = map(
        _f64, (Q_rows, Kseq, Vseq, Kdepth_rows, Vdepth_rows))
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    B, Hq, Hk, T, d, da, dc = _dims(Q_rows, Kseq, Kdepth_rows, depth_count)
    R = rows.shape[0]
    assert Q_rows.shape[2] == R
    O = np.empty((B, Hq, R, d), np.float64)
    LSE = np.empty((B, Hq, R), np.float64)
    rc = lib().moda_ref_fwd_rows_f64(_p(Q_rows), _p(Kseq), _p(Vseq), _p(Kdepth_rows),
                                     _p(Vdepth_rows), rows.ctypes.data_as(_ip), R, _p(O), _p(LSE),
                                     B, Hq, Hk, T, d, da, dc, int(bool(causal)),
                                     ctypes.c_double(_scale(scale, d)))
    if rc != 0:
        raise ValueError("moda_ref_fwd_rows_f64 rejected its arguments")
    return O, LSE


def weights(Q, Kseq, Vseq, Kdepth, Vdepth, b, h, t, depth_count=None, causal=True, scale=None):
    """Softmax weights of query (b,h,t) over [visible sequence keys..., depth slots...]."""
    Q, Kseq, Vseq, Kdepth, Vdepth = map(_f64, (Q, Kseq, Vseq, Kdepth, Vdepth))
    B, Hq, Hk, T, d, da, dc = _dims(Q, Kseq, Kdepth, depth_count)
    n = (t + 1 if causal else T) + dc
    w = np.empty(n, np.float64)
    rc = lib().moda_ref_weights_f64(_p(Q), _p(Kseq), _p(Vseq), _p(Kdepth), _p(Vdepth), b, h, t,
                                    _p(w), B, Hq, Hk, T, d, da, dc, int(bool(causal)),
                                    ctypes.c_double(_scale(scale, d)))
    if rc != 0:
        raise ValueError("moda_ref_weights_f64 rejected its arguments")
    return w


def bwd(Q, Kseq, Vseq, Kdepth, Vdepth, dO, depth_count=None, causal=True, scale=None):
    """Full backward.  Returns (dQ, dKseq, dVseq, dKdepth, dVdepth); the depth
    gradients are None when there is no depth tensor."""
    Q, Kseq, Vseq, Kdepth, Vdepth, dO = map(_f64, (Q, Kseq, Vseq, Kdepth, Vdepth, dO))
    B, Hq, Hk, T, d, da, dc = _dims(Q, Kseq, Kdepth, depth_count)
    dQ = np.empty_like(Q)
    dK = np.empty_like(Kseq)
    dV = np.empty_like(Vseq)
    dKd = None if Kdepth is None else np.empty_like(Kdepth)
    dVd = None if Vdepth is None else np.empty_like(Vdepth)
    rc = lib().moda_ref_bwd_f64(_p(Q), _p(Kseq), _p(Vseq), _p(Kdepth), _p(Vdepth), _p(dO), _p(dQ),
                                _p(dK), _p(dV), _p(dKd), _p(dVd), B, Hq, Hk, T, d, da, dc,
                                int(bool(causal)), ctypes.c_double(_scale(scale, d)))
    if rc != 0:
        raise ValueError("moda_ref_bwd_f64 rejected its arguments")
    return dQ, dK, dV, dKd, dVd


def bwd_rows(Q_rows, Kseq, Vseq, Kdepth_rows, Vdepth_rows, dO_rows, rows, depth_count=None,
             causal=True, scale=None):
    """Row-local gradients (dQ_rows, dKdepth_rows, dVdepth_rows) for the listed positions."""
    Q_rows, Kseq, Vseq, Kdepth_rows, Vdepth_rows, dO_rows = map(
        _f64, (Q_rows, Kseq, Vseq, Kdepth_rows, Vdepth_rows, dO_rows))
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    B, Hq, Hk, T, d, da, dc = _dims(Q_rows, Kseq, Kdepth_rows, depth_count)
    R = rows.shape[0]
    dQ = np.empty_like(Q_rows)
    dKd = None if Kdepth_rows is None else np.empty_like(Kdepth_rows)
    dVd = None if Vdepth_rows is None else np.empty_like(Vdepth_rows)
    rc = lib().moda_ref_bwd_rows_f64(_p(Q_rows), _p(Kseq), _p(Vseq), _p(Kdepth_rows),
                                     _p(Vdepth_rows), _p(dO_rows), rows.ctypes.data_as(_ip), R,
                                     _p(dQ), _p(dKd), _p(dVd), B, Hq, Hk, T, d, da, dc,
                                     int(bool(causal)), ctypes.c_double(_scale(scale, d)))
    if rc != 0:
        raise ValueError("moda_ref_bwd_rows_f64 rejected its arguments")
    return dQ, dKd, dVd


def bwd_noise(Q, Kseq, Vseq, Kdepth, Vdepth, dO, depth_count=None, causal=True, scale=None):
    """Rounding-noise scale of every gradient element (same shapes as bwd's results): the
    standard deviation, per unit relative rounding error, of the error of an implementation
    that rounds the softmax weights, the logit gradients and the forward's output before it
    sums (first-order model, see moda_ref_bwd_noise_f64 in the C file)."""
    Q, Kseq, Vseq, Kdepth, Vdepth, dO = map(_f64, (Q, Kseq, Vseq, Kdepth, Vdepth, dO))
    B, Hq, Hk, T, d, da, dc = _dims(Q, Kseq, Kdepth, depth_count)
    nQ = np.empty_like(Q)
    nK = np.empty_like(Kseq)
    nV = np.empty_like(Vseq)
    nKd = None if Kdepth is None else np.empty_like(Kdepth)
    nVd = None if Vdepth is None else np.empty_like(Vdepth)
    rc = lib().moda_ref_bwd_noise_f64(_p(Q), _p(Kseq), _p(Vseq), _p(Kdepth), _p(Vdepth), _p(dO), _p(nQ),
                                      _p(nK), _p(nV), _p(nKd), _p(nVd), B, Hq, Hk, T, d, da, dc,
                                      int(bool(causal)), ctypes.c_double(_scale(scale, d)))
    if rc != 0:
        raise ValueError("moda_ref_bwd_noise_f64 rejected its arguments")
    return nQ, nK, nV, nKd, nVd


def bwd_noise_rows(Q_rows, Kseq, Vseq, Kdepth_rows, Vdepth_rows, dO_rows, rows, depth_count=None,
                   causal=True, scale=None):
    """Rounding-noise scale of the row-local gradients (nQ_rows, nKdepth_rows, nVdepth_rows)."""
    Q_rows, Kseq, Vseq, Kdepth_rows, Vdepth_rows, dO_rows = map(
        _f64, (Q_rows, Kseq, Vseq, Kdepth_rows, Vdepth_rows, dO_rows))
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    B, Hq, Hk, T, d, da, dc = _dims(Q_rows, Kseq, Kdepth_rows, depth_count)
    R = rows.shape[0]
    nQ = np.empty_like(Q_rows)
    nKd = None if Kdepth_rows is None else np.empty_like(Kdepth_rows)
    nVd = None if Vdepth_rows is None else np.empty_like(Vdepth_rows)
    rc = lib().moda_ref_bwd_noise_rows_f64(_p(Q_rows), _p(Kseq), _p(Vseq), _p(Kdepth_rows),
                                           _p(Vdepth_rows), _p(dO_rows), rows.ctypes.data_as(_ip), R,
                                           _p(nQ), _p(nKd), _p(nVd), B, Hq, Hk, T, d, da, dc,
                                           int(bool(causal)), ctypes.c_double(_scale(scale, d)))
    if rc != 0:
        raise ValueError("moda_ref_bwd_noise_rows_f64 rejected its arguments")
    return nQ, nKd, nVd


def depth_append(Kdepth, Vdepth, K, V, slot):
    """The depth stream's write step (paper section 2.2: after the operator, the layer's
    key-value pair is appended to the depth stream): returns copies of Kdepth, Vdepth
    [B,Hk,T,depth_alloc,d] in which slot `slot` of every position holds K, V [B,Hk,T,d] and
    every other slot is unchanged.  Plain array indexing, any dtype, no arithmetic."""
    Kd, Vd = np.array(Kdepth, copy=True), np.array(Vdepth, copy=True)
    if not 0 <= slot < Kd.shape[3]:
        raise IndexError("slot out of range")
    Kd[:, :, :, slot, :] = K
    Vd[:, :, :, slot, :] = V
    return Kd, Vd
