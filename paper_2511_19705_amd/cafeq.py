"""ctypes binding of libcafeq.so: argument marshalling only.

Every function takes torch CUDA tensors (used purely as device memory), builds the
C descriptors of include/cafeq.h and enqueues the call on torch's current stream.
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CAFEQ_LIBRARY", os.path.join(_HERE, "libcafeq.so"))

AXIS_COL, AXIS_ROW = 0, 1
Q_SYM, Q_MINMAX = 0, 1   # the symmetric absmax grid; the min/max grid of the paper's Eq. (1)
SIDE_T, SIDE_TINV = 0, 1
F32, BF16 = 0, 1
CALL_RTN, CALL_PROXY, CALL_DUAL, CALL_ADAPTIVE = 0, 1, 2, 3

EXPORTS = (
    "cafeq_strerror", "cafeq_version", "cafeq_workspace_bytes", "cafeq_block_inverse",
    "cafeq_rtn_quantize", "cafeq_apply_transform", "cafeq_proxy_loss_fwd_bwd",
    "cafeq_dual_proxy_loss_fwd_bwd", "cafeq_adaptive_round_step",
    "cafeq_orth_penalty", "cafeq_sgd_update", "cafeq_adam_update", "cafeq_optimize_single",
    "cafeq_optimize_pair", "cafeq_pqe", "cafeq_rtn_quantize_minmax", "cafeq_hadamard_rtn", "cafeq_hadamard_workspace_bytes",
    "cafeq_infer_single", "cafeq_infer_workspace_bytes", "cafeq_set_launch_timing", "cafeq_rtn_quantize_static", "cafeq_prepared_bytes", "cafeq_prepare_weights",
    "cafeq_stream_read_probe",
)


class CafeqError(RuntimeError):
    pass


class Mat(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64), ("dtype", ctypes.c_int32), ("prepared", ctypes.c_void_p)]


class Xform(ctypes.Structure):
    _fields_ = [("T", ctypes.c_void_p), ("Tinv", ctypes.c_void_p), ("k", ctypes.c_int32),
                ("nb", ctypes.c_int32), ("rep", ctypes.c_int32)]


class QuantCfg(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_int32), ("group", ctypes.c_int32), ("axis", ctypes.c_int32),
                ("mode", ctypes.c_int32)]


class LaunchTiming(ctypes.Structure):
    _fields_ = [("start", ctypes.POINTER(ctypes.c_void_p)), ("stop", ctypes.POINTER(ctypes.c_void_p)),
                ("capacity", ctypes.c_int32), ("count", ctypes.c_int32), ("every", ctypes.c_int32),
                ("seen", ctypes.c_int32), ("kind", ctypes.c_int32)]


class OptCfg(ctypes.Structure):
    _fields_ = [("steps", ctypes.c_int32), ("lr", ctypes.c_float), ("lambda_orth", ctypes.c_float),
                ("normalize", ctypes.c_int32), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise CafeqError("libcafeq.so has not been built (run `python __graft_entry__.py`): " + LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    missing = [n for n in EXPORTS if not hasattr(lib, n)]
    if missing:
        raise CafeqError("libcafeq.so lacks exports: %s" % missing)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.cafeq_strerror.restype = ctypes.c_char_p
    lib.cafeq_strerror.argtypes = [i32]
    lib.cafeq_version.restype = i32
    lib.cafeq_workspace_bytes.restype = ctypes.c_size_t
    lib.cafeq_workspace_bytes.argtypes = [i32, ctypes.POINTER(Mat), ctypes.POINTER(Mat),
                                          ctypes.POINTER(Xform), ctypes.POINTER(QuantCfg)]
    lib.cafeq_block_inverse.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.cafeq_rtn_quantize.argtypes = [ctypes.POINTER(Mat), ctypes.POINTER(QuantCfg), vp, vp, vp, vp, vp]
    lib.cafeq_prepared_bytes.restype = ctypes.c_size_t
    lib.cafeq_prepared_bytes.argtypes = [ctypes.POINTER(Mat), i32]
    lib.cafeq_prepare_weights.argtypes = [ctypes.POINTER(Mat), i32, vp, vp]
    lib.cafeq_rtn_quantize_static.argtypes = [ctypes.POINTER(Mat), ctypes.POINTER(QuantCfg), vp, vp, vp, vp]
    lib.cafeq_apply_transform.argtypes = [ctypes.POINTER(Mat), ctypes.POINTER(Xform), i32, i32, vp, vp, vp]
    lib.cafeq_proxy_loss_fwd_bwd.argtypes = [ctypes.POINTER(Mat), ctypes.POINTER(Xform),
                                             ctypes.POINTER(QuantCfg), vp, vp, vp, vp, vp, vp]
    lib.cafeq_dual_proxy_loss_fwd_bwd.argtypes = [ctypes.POINTER(Mat), ctypes.POINTER(Mat),
                                                  ctypes.POINTER(Xform), ctypes.POINTER(QuantCfg),
                                                  ctypes.c_float, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.cafeq_adaptive_round_step.argtypes = [vp, vp, i64, i64, i64, i64, ctypes.POINTER(QuantCfg),
                                              i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    f32 = ctypes.c_float
    lib.cafeq_orth_penalty.argtypes = [vp, i32, i32, f32, vp, vp, vp, vp]
    lib.cafeq_sgd_update.argtypes = [vp, vp, f32, vp, i64, vp]
    f64 = ctypes.c_double
    lib.cafeq_adam_update.argtypes = [vp, vp, vp, vp, i32, f64, f64, f64, f64, i64, vp]
    lib.cafeq_optimize_single.argtypes = [ctypes.POINTER(Mat), vp, vp, i32, i32, i32, ctypes.POINTER(QuantCfg),
                                          ctypes.POINTER(OptCfg), vp, vp, vp, vp]
    lib.cafeq_optimize_pair.argtypes = [ctypes.POINTER(Mat), ctypes.POINTER(Mat), vp, vp, i32, i32, i32,
                                        ctypes.POINTER(QuantCfg), f32, ctypes.POINTER(OptCfg), vp, vp, vp, vp, vp]
    lib.cafeq_rtn_quantize_minmax.argtypes = [ctypes.POINTER(Mat), ctypes.POINTER(QuantCfg), vp, vp, vp, vp, vp, vp]
    lib.cafeq_hadamard_workspace_bytes.restype = ctypes.c_size_t
    lib.cafeq_hadamard_workspace_bytes.argtypes = [i64, i64, i32]
    lib.cafeq_infer_workspace_bytes.restype = ctypes.c_size_t
    lib.cafeq_infer_workspace_bytes.argtypes = [i32, i64]
    lib.cafeq_infer_single.argtypes = [vp, i32, i64, ctypes.POINTER(Xform), vp, vp, i64, i64, i32, vp, i64, vp, vp]
    lib.cafeq_hadamard_rtn.argtypes = [ctypes.POINTER(Mat), vp, i32, ctypes.POINTER(QuantCfg), vp, vp, vp, vp, vp, vp]
    lib.cafeq_pqe.argtypes = [vp, vp, i64, i64, i64, i64, ctypes.POINTER(QuantCfg), i32, i32, i32, vp, vp, vp, vp,
                              vp, vp, vp]
    lib.cafeq_set_launch_timing.argtypes = [ctypes.POINTER(LaunchTiming)]
    lib.cafeq_stream_read_probe.argtypes = [vp, ctypes.c_size_t, vp, vp]
    for n in EXPORTS[3:]:
        getattr(lib, n).restype = i32
    return lib


lib = _load()


def _check(rc):
    if rc != 0:
        raise CafeqError("cafeq call failed: %s (%d)" % (lib.cafeq_strerror(rc).decode(), rc))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def mat(t, prepared=None):
    """Descriptor of a 2-D CUDA tensor (float32 or bfloat16, unit column stride); `prepared`: the buffer
    prepare_weights() returned for it, or None."""
    if t.dim() != 2 or t.stride(1) != 1 or not t.is_cuda:
        raise CafeqError("need a 2-D CUDA tensor with unit column stride")
    if t.dtype == torch.float32:
        dt = F32
    elif t.dtype == torch.bfloat16:
        dt = BF16
    else:
        raise CafeqError("dtype must be float32 or bfloat16")
    return Mat(t.data_ptr(), t.shape[0], t.shape[1], t.stride(0), dt, prepared.data_ptr() if prepared is not None else 0)


def xform(T, Tinv, rep=1):
    for x in (T, Tinv):
        if x is not None and (x.dtype != torch.float32 or not x.is_contiguous() or x.dim() != 3):
            raise CafeqError("transform blocks must be contiguous float32 [nb][k][k]")
    return Xform(_ptr(T), _ptr(Tinv), T.shape[1], T.shape[0], rep)


_ws_cache = {}


def workspace(nbytes, device):
    """A cached scratch buffer (device memory owned by the binding, grown on demand)."""
    key = (device.type, device.index)
    buf = _ws_cache.get(key)
    if buf is None or buf.numel() < nbytes:
        buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
        _ws_cache[key] = buf
    return buf


def workspace_bytes(call_id, a, b=None, x=None, cfg=None):
    return int(lib.cafeq_workspace_bytes(call_id, ctypes.byref(a), ctypes.byref(b) if b else None,
                                         ctypes.byref(x) if x else None,
                                         ctypes.byref(cfg) if cfg else None))


def _scale_shape(rows, cols, group, axis):
    if axis == AXIS_COL:
        return (rows, cols // (group or cols))
    return (rows // (group or rows), cols)


def _minmax_shape(shape, mode):
    """Scale buffer of the fused calls: on the min/max grid the group minima follow the scales."""
    return shape if mode == Q_SYM else (2,) + tuple(shape)


def rtn_quantize(W, bits, group, axis=AXIS_COL, want_err=False):
    m = mat(W)
    cfg = QuantCfg(bits, group, axis, 0)
    R, C = W.shape
    codes = torch.empty((R, C), dtype=torch.int8, device=W.device)
    scales = torch.empty(_scale_shape(R, C, group, axis), dtype=torch.float32, device=W.device)
    err = torch.empty(1, dtype=torch.float32, device=W.device) if want_err else None
    ws = workspace(workspace_bytes(CALL_RTN, m, cfg=cfg), W.device) if want_err else None
    _check(lib.cafeq_rtn_quantize(ctypes.byref(m), ctypes.byref(cfg), _ptr(codes), _ptr(scales),
                                  _ptr(err), _ptr(ws), _stream()))
    return codes, scales, err


def prepare_weights(W, axis=AXIS_COL):
    """The prepared copy of W for transforms along `axis` (a uint8 tensor; see cafeq_prepare_weights)."""
    m = mat(W)
    nbytes = int(lib.cafeq_prepared_bytes(ctypes.byref(m), axis))
    if nbytes == 0:
        raise CafeqError("weights cannot be prepared for this axis (its length must be a multiple of 128)")
    buf = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    _check(lib.cafeq_prepare_weights(ctypes.byref(m), axis, _ptr(buf), _stream()))
    return buf


def rtn_quantize_static(W, codes, scales, err, bits, group, axis=AXIS_COL):
    """The quantizer with built-in scratch: the caller passes every output buffer; nothing is allocated."""
    m = mat(W)
    cfg = QuantCfg(bits, group, axis, 0)
    _check(lib.cafeq_rtn_quantize_static(ctypes.byref(m), ctypes.byref(cfg), _ptr(codes), _ptr(scales),
                                         _ptr(err), _stream()))


def block_inverse(T, want_rho=False):
    """Tinv (and optionally rho_row, rho_col) plus per-block status."""
    nb, k, _ = T.shape
    dev = T.device
    Tinv = torch.empty_like(T)
    rr = torch.empty(nb * k, dtype=torch.float32, device=dev) if want_rho else None
    rc_ = torch.empty(nb * k, dtype=torch.float32, device=dev) if want_rho else None
    status = torch.empty(nb, dtype=torch.int32, device=dev)
    x = Xform(_ptr(T), 0, k, nb, 1)
    ws = workspace(int(lib.cafeq_workspace_bytes(4, None, None, ctypes.byref(x), None)), dev)
    _check(lib.cafeq_block_inverse(_ptr(T), k, nb, _ptr(Tinv), _ptr(rr), _ptr(rc_), _ptr(status),
                                   _ptr(ws), _stream()))
    return (Tinv, rr, rc_, status) if want_rho else (Tinv, status)


def apply_transform(W, T, Tinv=None, axis=AXIS_COL, side=SIDE_T, rep=1):
    m = mat(W)
    x = xform(T, Tinv, rep)
    Z = torch.empty(W.shape, dtype=torch.float32, device=W.device)
    ws = workspace(int(lib.cafeq_workspace_bytes(5, None, None, ctypes.byref(x), None)), W.device)
    _check(lib.cafeq_apply_transform(ctypes.byref(m), ctypes.byref(x), axis, side, _ptr(Z), _ptr(ws), _stream()))
    return Z


def proxy_loss_fwd_bwd(W, T, Tinv, bits, group, axis=AXIS_COL, rep=1, want_grad=True, want_codes=False,
                       prepared=None, mode=Q_SYM):
    """Returns (losses[4], gradT or None, codes or None, scales or None).  With mode=Q_MINMAX the codes are
    unsigned bytes and `scales` is [2][...]: the scales, then the group minima."""
    m = mat(W, prepared)
    x = xform(T, Tinv, rep)
    cfg = QuantCfg(bits, group, axis, mode)
    dev = W.device
    losses = torch.empty(4, dtype=torch.float32, device=dev)
    grad = torch.empty_like(T) if want_grad else None
    R, C = W.shape
    codes = torch.empty((R, C), dtype=torch.int8, device=dev) if want_codes else None
    scales = torch.empty(_minmax_shape(_scale_shape(R, C, group, axis), mode), dtype=torch.float32,
                         device=dev) if want_codes else None
    nbytes = workspace_bytes(CALL_PROXY, m, x=x, cfg=cfg)
    if nbytes == 0:
        raise CafeqError("unsupported proxy-loss configuration (workspace query returned 0)")
    ws = workspace(nbytes, dev)
    _check(lib.cafeq_proxy_loss_fwd_bwd(ctypes.byref(m), ctypes.byref(x), ctypes.byref(cfg), _ptr(losses),
                                        _ptr(grad), _ptr(codes), _ptr(scales), _ptr(ws), _stream()))
    if want_codes and mode == Q_MINMAX:
        codes = codes.view(torch.uint8)
    return losses, grad, codes, scales


def dual_proxy_loss_fwd_bwd(A, B, T, Tinv, bits, group, rep=1, lse_t=5.0, want_grad=True, want_codes=False,
                            prepared=(None, None), mode=Q_SYM):
    """Returns (losses[6], gradT or None, (codesU, scalesU, codesV, scalesV) or None); mode as in
    proxy_loss_fwd_bwd."""
    ma, mb = mat(A, prepared[0]), mat(B, prepared[1])
    x = xform(T, Tinv, rep)
    cfg = QuantCfg(bits, group, 0, mode)
    dev = A.device
    losses = torch.empty(6, dtype=torch.float32, device=dev)
    grad = torch.empty_like(T) if want_grad else None
    outs = None
    cu = su = cv = sv = None
    if want_codes:
        cu = torch.empty(A.shape, dtype=torch.int8, device=dev)
        su = torch.empty(_minmax_shape(_scale_shape(A.shape[0], A.shape[1], group, AXIS_COL), mode),
                         dtype=torch.float32, device=dev)
        cv = torch.empty(B.shape, dtype=torch.int8, device=dev)
        sv = torch.empty(_minmax_shape(_scale_shape(B.shape[0], B.shape[1], group, AXIS_ROW), mode),
                         dtype=torch.float32, device=dev)
        outs = (cu, su, cv, sv) if mode == Q_SYM else (cu.view(torch.uint8), su, cv.view(torch.uint8), sv)
    nbytes = workspace_bytes(CALL_DUAL, ma, mb, x, cfg)
    if nbytes == 0:
        raise CafeqError("unsupported dual configuration (workspace query returned 0)")
    ws = workspace(nbytes, dev)
    _check(lib.cafeq_dual_proxy_loss_fwd_bwd(ctypes.byref(ma), ctypes.byref(mb), ctypes.byref(x),
                                             ctypes.byref(cfg), ctypes.c_float(lse_t), _ptr(losses), _ptr(grad),
                                             _ptr(cu), _ptr(su), _ptr(cv), _ptr(sv), _ptr(ws), _stream()))
    return losses, grad, outs


def adaptive_round_step(U, V, codesU, scalesU, codesV, scalesV, bits, group, k, rep=1, half=0):
    """One iteration of Alg. 1; codes/scales are updated in place.  Returns status[2*nb]."""
    for t in (U, V):
        if t.dtype != torch.float32 or not t.is_contiguous():
            raise CafeqError("U and V must be contiguous float32")
    nb = U.shape[1] // k
    cfg = QuantCfg(bits, group, 0, 0)
    mu, mv = mat(U), mat(V)
    x = Xform(0, 0, k, nb, rep)
    status = torch.zeros(2 * nb, dtype=torch.int32, device=U.device)
    nbytes = workspace_bytes(CALL_ADAPTIVE, mu, mv, x, cfg)
    if nbytes == 0:
        raise CafeqError("unsupported adaptive-rounding configuration (workspace query returned 0)")
    ws = workspace(nbytes, U.device)
    _check(lib.cafeq_adaptive_round_step(_ptr(U), _ptr(V), U.shape[0], U.shape[1], V.shape[0], V.shape[1],
                                         ctypes.byref(cfg), k, nb, rep, half, _ptr(codesU), _ptr(scalesU),
                                         _ptr(codesV), _ptr(scalesV), _ptr(status), _ptr(ws), _stream()))
    return status


def stream_read_probe(buf, sink=None):
    """One launch of the library's plain streaming read over the tensor `buf` (cafeq_stream_read_probe)."""
    if sink is None:
        sink = torch.zeros(1, dtype=torch.int32, device=buf.device)
    _check(lib.cafeq_stream_read_probe(_ptr(buf), ctypes.c_size_t(buf.numel() * buf.element_size()), _ptr(sink),
                                       _stream()))
    return sink


class LaunchTimer:
    """Caller-owned events around the fused-kernel launches (cafeq_set_launch_timing): `capacity` pairs of
    torch events are created up front; the library only records them.  every > 1: only every `every`-th launch
    is timed (an event pair holds the stream up for several microseconds).  kind: 0 the loss pass (fused transform
    kernel), 1 the gradient pass over the weights."""

    def __init__(self, capacity, every=1, kind=0):
        self.ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(capacity)]
        for a, b in self.ev:          # torch creates the underlying event on first use
            a.record()
            b.record()
        torch.cuda.synchronize()
        self.start = (ctypes.c_void_p * capacity)(*[a.cuda_event for a, _ in self.ev])
        self.stop = (ctypes.c_void_p * capacity)(*[b.cuda_event for _, b in self.ev])
        self.table = LaunchTiming(self.start, self.stop, capacity, 0, every, 0, kind)

    def __enter__(self):
        self.table.count = 0
        self.table.seen = 0
        _check(lib.cafeq_set_launch_timing(ctypes.byref(self.table)))
        return self

    def __exit__(self, *exc):
        _check(lib.cafeq_set_launch_timing(None))

    def durations_ms(self):
        """Per-launch durations (the caller has synchronised the stream)."""
        return [self.ev[i][0].elapsed_time(self.ev[i][1]) for i in range(self.table.count)]


def orth_penalty(T, lam, grad=None):
    """(value[1], grad) with grad incremented in place when given."""
    nb, k, _ = T.shape
    x = Xform(_ptr(T), 0, k, nb, 1)
    ws = workspace(int(lib.cafeq_workspace_bytes(6, None, None, ctypes.byref(x), None)), T.device)
    value = torch.empty(1, dtype=torch.float32, device=T.device)
    _check(lib.cafeq_orth_penalty(_ptr(T), k, nb, lam, _ptr(value), _ptr(grad), _ptr(ws), _stream()))
    return value, grad


def sgd_update(T, grad, lr, denom=None):
    _check(lib.cafeq_sgd_update(_ptr(T), _ptr(grad), lr, _ptr(denom), T.numel(), _stream()))


def adam_update(T, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    _check(lib.cafeq_adam_update(_ptr(T), _ptr(grad), _ptr(m), _ptr(v), step, lr, beta1, beta2, eps, T.numel(),
                                 _stream()))


def optimize_single(W, T, bits, group, axis=AXIS_COL, rep=1, lr=1.0, steps=10, lambda_orth=0.0, normalize=True,
                    mode=Q_SYM):
    """Gradient descent on the surrogate, T updated in place.  Returns (Tinv, history[steps][8], status)."""
    m = mat(W)
    nb, k, _ = T.shape
    Tinv = torch.empty_like(T)
    x = Xform(_ptr(T), _ptr(Tinv), k, nb, rep)
    cfg = QuantCfg(bits, group, axis, mode)
    opt = OptCfg(steps, lr, lambda_orth, 1 if normalize else 0, 0.0, 0.0, 0.0)
    ws = workspace(int(lib.cafeq_workspace_bytes(7, ctypes.byref(m), None, ctypes.byref(x), ctypes.byref(cfg))), W.device)
    history = torch.empty((max(steps, 1), 8), dtype=torch.float32, device=W.device)
    status = torch.empty(nb, dtype=torch.int32, device=W.device)
    _check(lib.cafeq_optimize_single(ctypes.byref(m), _ptr(T), _ptr(Tinv), k, nb, rep, ctypes.byref(cfg),
                                     ctypes.byref(opt), _ptr(history), _ptr(status), _ptr(ws), _stream()))
    return Tinv, history[:steps], status


def optimize_pair(A, B, T, bits, group, rep=1, lse_t=5.0, lr=1e-2, steps=10, lambda_orth=0.0, beta1=0.1,
                  beta2=0.999, eps=1e-8, prepared=(None, None), mode=Q_SYM):
    """Adam on the LogSumExp surrogate, T updated in place.  Returns (Tinv, history[steps][8], status)."""
    ma, mb = mat(A, prepared[0]), mat(B, prepared[1])
    nb, k, _ = T.shape
    Tinv = torch.empty_like(T)
    x = Xform(_ptr(T), _ptr(Tinv), k, nb, rep)
    cfg = QuantCfg(bits, group, 0, mode)
    opt = OptCfg(steps, lr, lambda_orth, 0, beta1, beta2, eps)
    ws = workspace(int(lib.cafeq_workspace_bytes(8, ctypes.byref(ma), ctypes.byref(mb), ctypes.byref(x),
                                                 ctypes.byref(cfg))), A.device)
    moments = torch.empty(2 * T.numel(), dtype=torch.float32, device=A.device)
    history = torch.empty((max(steps, 1), 8), dtype=torch.float32, device=A.device)
    status = torch.empty(nb, dtype=torch.int32, device=A.device)
    _check(lib.cafeq_optimize_pair(ctypes.byref(ma), ctypes.byref(mb), _ptr(T), _ptr(Tinv), k, nb, rep,
                                   ctypes.byref(cfg), lse_t, ctypes.byref(opt), _ptr(moments), _ptr(history),
                                   _ptr(status), _ptr(ws), _stream()))
    return Tinv, history[:steps], status


def pqe(U, V, codesU, scalesU, codesV, scalesV, bits, group, k, rep=1):
    """out[2] (device): sum of squared paired quantization errors over heads, and of the squared products."""
    nb = U.shape[1] // k
    mu, mv = mat(U), mat(V)
    x = Xform(0, 0, k, nb, rep)
    cfg = QuantCfg(bits, group, 0, 0)
    ws = workspace(int(lib.cafeq_workspace_bytes(9, ctypes.byref(mu), ctypes.byref(mv), ctypes.byref(x),
                                                 ctypes.byref(cfg))), U.device)
    out = torch.empty(2, dtype=torch.float32, device=U.device)
    _check(lib.cafeq_pqe(_ptr(U), _ptr(V), U.shape[0], U.shape[1], V.shape[0], V.shape[1], ctypes.byref(cfg), k, nb,
                         rep, _ptr(codesU), _ptr(scalesU), _ptr(codesV), _ptr(scalesV), _ptr(out), _ptr(ws), _stream()))
    return out


def rtn_quantize_minmax(W, bits, group, axis=AXIS_COL, want_err=False):
    """Eq. (1) grid: (codes uint8, scales, mins, err or None)."""
    m = mat(W)
    cfg = QuantCfg(bits, group, axis, 1)
    R, C = W.shape
    codes = torch.empty((R, C), dtype=torch.uint8, device=W.device)
    shape = _scale_shape(R, C, group, axis)
    scales = torch.empty(shape, dtype=torch.float32, device=W.device)
    mins = torch.empty(shape, dtype=torch.float32, device=W.device)
    err = torch.empty(1, dtype=torch.float32, device=W.device) if want_err else None
    ws = workspace(workspace_bytes(CALL_RTN, m, cfg=cfg), W.device) if want_err else None
    _check(lib.cafeq_rtn_quantize_minmax(ctypes.byref(m), ctypes.byref(cfg), _ptr(codes), _ptr(scales), _ptr(mins),
                                         _ptr(err), _ptr(ws), _stream()))
    return codes, scales, mins, err


def hadamard_rtn(W, signs, block, bits, group, want_z=False, want_codes=False):
    """Randomized-Hadamard baseline: (losses[2] = (err_sq, w_sq), Z or None, codes or None, scales or None)."""
    m = mat(W)
    cfg = QuantCfg(bits, group, AXIS_COL, 0)
    R, C = W.shape
    dev = W.device
    Z = torch.empty((R, C), dtype=torch.float32, device=dev) if want_z else None
    codes = torch.empty((R, C), dtype=torch.int8, device=dev) if want_codes else None
    scales = torch.empty((R, C // group), dtype=torch.float32, device=dev) if want_codes else None
    losses = torch.empty(2, dtype=torch.float32, device=dev)
    ws = workspace(int(lib.cafeq_hadamard_workspace_bytes(R, C, block)), dev)
    _check(lib.cafeq_hadamard_rtn(ctypes.byref(m), _ptr(signs), block, ctypes.byref(cfg), _ptr(Z), _ptr(codes),
                                  _ptr(scales), _ptr(losses), _ptr(ws), _stream()))
    return losses, Z, codes, scales


def infer_single(X, Tinv, codes, scales, group, out=None):
    """Y[n][out] = (X . blockdiag(Tinv)^T) . dequant(codes, scales)^T; Tinv None = no transform."""
    n, d = X.shape
    O = codes.shape[0]
    Y = out if out is not None else torch.empty((n, O), dtype=torch.float32, device=X.device)
    if Tinv is not None:
        nb, k, _ = Tinv.shape
        xf = Xform(None, _ptr(Tinv), k, nb, 1)
        ws = workspace(int(lib.cafeq_infer_workspace_bytes(n, d)), X.device)
        xfp = ctypes.byref(xf)
    else:
        ws, xfp = None, None
    _check(lib.cafeq_infer_single(_ptr(X), n, X.stride(0), xfp, _ptr(codes), _ptr(scales), O, d, group, _ptr(Y),
                                  Y.stride(0), _ptr(ws), _stream()))
    return Y
