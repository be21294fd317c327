"""ctypes binding of the libmoda C ABI (include/moda.h).

Argument marshalling only: torch tensors supply device memory and the stream;
every step of the attention runs in the HIP kernels of libmoda.so.  There is no
fallback: if the library is missing or a call is rejected, an exception is raised.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# MODA_LIB_PATH points at another build of the same library (e.g. an experiment)
LIB_PATH = os.environ.get("MODA_LIB_PATH") or os.path.join(HERE, "libmoda.so")

MODA_F32, MODA_BF16 = 0, 1
EXPORTS = ("moda_attn_fwd", "moda_attn_fwd_tuned", "moda_attn_bwd_workspace_bytes", "moda_attn_bwd", "moda_depth_append",
           "moda_attn_decode", "moda_attn_decode_workspace_bytes", "moda_attn_decode_noalloc",
           "moda_attn_decode_noalloc_max_bytes",
           "moda_calibrate_mfma", "moda_calibrate_mfma_operand_bytes", "moda_calibrate_mfma_sink_bytes",
           "moda_status_string", "moda_version", "moda_kernels_per_call")


class MODAShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hk", ctypes.c_int32),
                ("T", ctypes.c_int32), ("d", ctypes.c_int32), ("depth_alloc", ctypes.c_int32),
                ("depth_count", ctypes.c_int32), ("causal", ctypes.c_int32),
                ("scale", ctypes.c_float), ("dtype", ctypes.c_int32)]


class MODAFwdTuning(ctypes.Structure):
    _fields_ = [("waves", ctypes.c_int32), ("heads_per_tile", ctypes.c_int32), ("head_group", ctypes.c_int32),
                ("depth_path", ctypes.c_int32)]


class MODAError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libmoda: %s (status %d)" % (text, code))
        self.code = code


_lib = None


def lib():
    """Load libmoda.so (built by paper_2603_15619_amd.build).  Raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: build it with `python -m paper_2603_15619_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        sp = ctypes.POINTER(MODAShape)
        L.moda_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, sp, vp]
        L.moda_attn_fwd.restype = ctypes.c_int
        L.moda_attn_fwd_tuned.argtypes = [vp, vp, vp, vp, vp, vp, vp, sp, ctypes.POINTER(MODAFwdTuning), vp]
        L.moda_attn_fwd_tuned.restype = ctypes.c_int
        L.moda_attn_bwd_workspace_bytes.argtypes = [sp]
        L.moda_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.moda_attn_bwd.argtypes = [vp] * 14 + [ctypes.c_size_t, sp, vp]
        L.moda_attn_bwd.restype = ctypes.c_int
        L.moda_depth_append.argtypes = [vp, vp, vp, vp, ctypes.c_int32, sp, vp]
        L.moda_depth_append.restype = ctypes.c_int
        L.moda_attn_decode_workspace_bytes.argtypes = [sp]
        L.moda_attn_decode_workspace_bytes.restype = ctypes.c_size_t
        L.moda_attn_decode.argtypes = [vp] * 7 + [ctypes.c_int32, vp, ctypes.c_size_t, sp, vp]
        L.moda_attn_decode.restype = ctypes.c_int
        L.moda_attn_decode_noalloc.argtypes = [vp] * 7 + [ctypes.c_int32, sp, vp]
        L.moda_attn_decode_noalloc.restype = ctypes.c_int
        L.moda_attn_decode_noalloc_max_bytes.argtypes = []
        L.moda_attn_decode_noalloc_max_bytes.restype = ctypes.c_size_t
        L.moda_calibrate_mfma_operand_bytes.argtypes = []
        L.moda_calibrate_mfma_operand_bytes.restype = ctypes.c_size_t
        L.moda_calibrate_mfma_sink_bytes.argtypes = [ctypes.c_int32]
        L.moda_calibrate_mfma_sink_bytes.restype = ctypes.c_size_t
        L.moda_calibrate_mfma.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32, vp]
        L.moda_calibrate_mfma.restype = ctypes.c_double
        L.moda_status_string.argtypes = [ctypes.c_int]
        L.moda_status_string.restype = ctypes.c_char_p
        L.moda_version.restype = ctypes.c_int
        L.moda_kernels_per_call.argtypes = [sp, ctypes.c_int]
        L.moda_kernels_per_call.restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().moda_status_string(code).decode()


def _check(code):
    if code != 0:
        raise MODAError(code, status_string(code))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return MODA_BF16
    if t.dtype == torch.float32:
        return MODA_F32
    raise TypeError("libmoda supports bf16 and fp32 tensors, got %s" % t.dtype)


def make_shape(Q, Kseq, Kdepth, depth_count, causal, scale):
    B, Hq, T, d = Q.shape
    Hk = Kseq.shape[1]
    depth_alloc = 0 if Kdepth is None else Kdepth.shape[3]
    if depth_count is None:
        depth_count = depth_alloc
    return MODAShape(B, Hq, Hk, T, d, depth_alloc, depth_count, int(bool(causal)),
                     float(scale) if scale else 0.0, _dtype_code(Q))


def _require(t, name, shape, dtype, device):
    if t is None:
        return
    if not t.is_cuda:
        raise ValueError("%s must live in device memory" % name)
    if t.device != device or t.dtype != dtype:
        raise ValueError("%s: device/dtype differ from Q" % name)
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s: expected shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)


def _stream(device):
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def moda_attn_fwd(Q, Kseq, Vseq, Kdepth=None, Vdepth=None, depth_count=None, causal=True,
                  scale=None, out=None, lse=None, tuning=None):
    """O, LSE = MoDA attention forward on the current stream of Q's device.

    Q [B,Hq,T,d]; Kseq/Vseq [B,Hk,T,d]; Kdepth/Vdepth [B,Hk,T,depth_alloc,d] or
    None; slots [0, depth_count) of each position are attended (default: all).
    `tuning` = dict(waves=, heads_per_tile=, head_group=, depth_path=) calls moda_attn_fwd_tuned (the bf16
    kernel's launch geometry chosen by the caller; missing keys keep the library's choice).
    """
    s = make_shape(Q, Kseq, Kdepth, depth_count, causal, scale)
    dev, dt = Q.device, Q.dtype
    _require(Q, "Q", (s.B, s.Hq, s.T, s.d), dt, dev)
    _require(Kseq, "Kseq", (s.B, s.Hk, s.T, s.d), dt, dev)
    _require(Vseq, "Vseq", (s.B, s.Hk, s.T, s.d), dt, dev)
    _require(Kdepth, "Kdepth", (s.B, s.Hk, s.T, s.depth_alloc, s.d), dt, dev)
    _require(Vdepth, "Vdepth", (s.B, s.Hk, s.T, s.depth_alloc, s.d), dt, dev)
    if out is None:
        out = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty((s.B, s.Hq, s.T), dtype=torch.float32, device=dev)
    _require(out, "out", Q.shape, dt, dev)
    _require(lse, "lse", (s.B, s.Hq, s.T), torch.float32, dev)
    with torch.cuda.device(dev):
        if tuning is None:
            _check(lib().moda_attn_fwd(_ptr(Q), _ptr(Kseq), _ptr(Vseq), _ptr(Kdepth), _ptr(Vdepth),
                                       _ptr(out), _ptr(lse), ctypes.byref(s), _stream(dev)))
        else:
            tn = MODAFwdTuning(int(tuning.get("waves", 0)), int(tuning.get("heads_per_tile", 0)),
                               int(tuning.get("head_group", 0)), int(tuning.get("depth_path", 0)))
            _check(lib().moda_attn_fwd_tuned(_ptr(Q), _ptr(Kseq), _ptr(Vseq), _ptr(Kdepth), _ptr(Vdepth),
                                             _ptr(out), _ptr(lse), ctypes.byref(s), ctypes.byref(tn), _stream(dev)))
    return out, lse


def moda_attn_bwd_workspace_bytes(shape: MODAShape) -> int:
    return int(lib().moda_attn_bwd_workspace_bytes(ctypes.byref(shape)))


def moda_attn_bwd(Q, Kseq, Vseq, Kdepth, Vdepth, O, LSE, dO, depth_count=None, causal=True,
                  scale=None, workspace=None):
    """(dQ, dKseq, dVseq, dKdepth, dVdepth) on the current stream of Q's device."""
    s = make_shape(Q, Kseq, Kdepth, depth_count, causal, scale)
    dev, dt = Q.device, Q.dtype
    _require(Q, "Q", (s.B, s.Hq, s.T, s.d), dt, dev)
    _require(Kseq, "Kseq", (s.B, s.Hk, s.T, s.d), dt, dev)
    _require(Vseq, "Vseq", (s.B, s.Hk, s.T, s.d), dt, dev)
    _require(Kdepth, "Kdepth", (s.B, s.Hk, s.T, s.depth_alloc, s.d), dt, dev)
    _require(Vdepth, "Vdepth", (s.B, s.Hk, s.T, s.depth_alloc, s.d), dt, dev)
    _require(O, "O", Q.shape, dt, dev)
    _require(dO, "dO", Q.shape, dt, dev)
    _require(LSE, "LSE", (s.B, s.Hq, s.T), torch.float32, dev)
    dQ = torch.empty_like(Q)
    dK = torch.empty_like(Kseq)
    dV = torch.empty_like(Vseq)
    dKd = None if Kdepth is None else torch.empty_like(Kdepth)
    dVd = None if Vdepth is None else torch.empty_like(Vdepth)
    need = moda_attn_bwd_workspace_bytes(s)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        _check(lib().moda_attn_bwd(_ptr(Q), _ptr(Kseq), _ptr(Vseq), _ptr(Kdepth), _ptr(Vdepth),
                                   _ptr(O), _ptr(LSE), _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV),
                                   _ptr(dKd), _ptr(dVd), _ptr(workspace), ws_bytes,
                                   ctypes.byref(s), _stream(dev)))
    return dQ, dK, dV, dKd, dVd


def moda_depth_append(K, V, Kdepth, Vdepth, slot):
    """Depth-stream write step, in place on the current stream: K, V [B,Hk,T,d] become slot
    `slot` of Kdepth, Vdepth [B,Hk,T,depth_alloc,d]."""
    B, Hk, T, d = K.shape
    dev, dt = K.device, K.dtype
    _require(K, "K", (B, Hk, T, d), dt, dev)
    _require(V, "V", (B, Hk, T, d), dt, dev)
    if Kdepth is None or Vdepth is None or Kdepth.dim() != 5:
        raise ValueError("Kdepth / Vdepth: expected [B,Hk,T,depth_alloc,d] tensors")
    La = Kdepth.shape[3]
    _require(Kdepth, "Kdepth", (B, Hk, T, La, d), dt, dev)
    _require(Vdepth, "Vdepth", (B, Hk, T, La, d), dt, dev)
    s = MODAShape(B, Hk, Hk, T, d, La, 0, 1, 0.0, _dtype_code(K))
    with torch.cuda.device(dev):
        _check(lib().moda_depth_append(_ptr(K), _ptr(V), _ptr(Kdepth), _ptr(Vdepth), int(slot),
                                       ctypes.byref(s), _stream(dev)))
    return Kdepth, Vdepth


def moda_attn_decode(Q, Kseq, Vseq, Kdepth=None, Vdepth=None, T=None, depth_count=None, scale=None,
                     out=None, lse=None, workspace=None, noalloc=False):
    """O [B,Hq,d], LSE [B,Hq] for one new token per sequence: Q [B,Hq,d]; sequence cache
    Kseq/Vseq [B,Hk,kv_alloc,d] of which positions [0, T) are attended (default: all); the new
    token's depth slots Kdepth/Vdepth [B,Hk,depth_alloc,d] or None.  noalloc=True calls
    moda_attn_decode_noalloc (the library's own scratch array instead of a workspace; `out`
    and `lse` must then be given, so that this wrapper allocates nothing either)."""
    B, Hq, d = Q.shape
    Hk, kv_alloc = Kseq.shape[1], Kseq.shape[2]
    T = kv_alloc if T is None else int(T)
    La = 0 if Kdepth is None else Kdepth.shape[2]
    L = La if depth_count is None else int(depth_count)
    dev, dt = Q.device, Q.dtype
    _require(Q, "Q", (B, Hq, d), dt, dev)
    _require(Kseq, "Kseq", (B, Hk, kv_alloc, d), dt, dev)
    _require(Vseq, "Vseq", (B, Hk, kv_alloc, d), dt, dev)
    _require(Kdepth, "Kdepth", (B, Hk, La, d), dt, dev)
    _require(Vdepth, "Vdepth", (B, Hk, La, d), dt, dev)
    s = MODAShape(B, Hq, Hk, T, d, La, L, 1, float(scale) if scale else 0.0, _dtype_code(Q))
    if noalloc and (out is None or lse is None):
        raise ValueError("noalloc=True needs out= and lse=")
    if out is None:
        out = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty((B, Hq), dtype=torch.float32, device=dev)
    _require(out, "out", Q.shape, dt, dev)
    _require(lse, "lse", (B, Hq), torch.float32, dev)
    if noalloc:
        with torch.cuda.device(dev):
            _check(lib().moda_attn_decode_noalloc(_ptr(Q), _ptr(Kseq), _ptr(Vseq), _ptr(Kdepth), _ptr(Vdepth),
                                                  _ptr(out), _ptr(lse), int(kv_alloc), ctypes.byref(s), _stream(dev)))
        return out, lse
    need = int(lib().moda_attn_decode_workspace_bytes(ctypes.byref(s)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        _check(lib().moda_attn_decode(_ptr(Q), _ptr(Kseq), _ptr(Vseq), _ptr(Kdepth), _ptr(Vdepth), _ptr(out),
                                      _ptr(lse), int(kv_alloc), _ptr(workspace), ws_bytes, ctypes.byref(s),
                                      _stream(dev)))
    return out, lse


def moda_calibrate_mfma(operands, workgroups, iters, sink=None):
    """Enqueue the matrix-pipe calibration kernel on the current stream; returns the floating-point
    operations of the launch.  `operands`: bf16 tensor of moda_calibrate_mfma_operand_bytes() bytes."""
    dev = operands.device
    need = int(lib().moda_calibrate_mfma_operand_bytes())
    if operands.dtype != torch.bfloat16 or operands.numel() * 2 < need or not operands.is_contiguous():
        raise ValueError("operands: contiguous bf16 tensor of at least %d bytes" % need)
    sb = int(lib().moda_calibrate_mfma_sink_bytes(int(workgroups)))
    if sink is None:
        sink = torch.empty(sb // 4, dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        fl = float(lib().moda_calibrate_mfma(_ptr(operands), _ptr(sink), sink.numel() * 4, int(workgroups), int(iters),
                                             _stream(dev)))
    if fl <= 0:
        raise MODAError(5, "calibration launch rejected")
    return fl
