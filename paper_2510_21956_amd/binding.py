"""ctypes binding with the same names as the C ABI in include/la.h.

Argument marshalling only.  There is no CPU fallback: if libla.so has not been
built, loading fails with an error that says how to build it.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libla.so")
_lib = None

LA_F32 = 0
LA_BF16 = 1

LA_MAX_TRACE = 8

EXPORTS = ("la_version", "la_status_string", "la_workspace_bytes", "la_forward", "la_backward",
           "la_forward_traced", "la_backward_traced", "la_saved_state_bytes", "la_forward_save",
           "la_backward_saved", "la_debug_override", "la_forward_static", "la_decode_state_bytes",
           "la_decode_step", "la_decode_prefill", "la_backward_ab", "la_forward_qknorm",
           "la_backward_qknorm", "la_forward_qknorm_save", "la_backward_qknorm_saved")


class la_trace(ctypes.Structure):
    """struct la_trace of include/la.h."""
    _fields_ = [("events", ctypes.POINTER(ctypes.c_void_p)),
                ("capacity", ctypes.c_int),
                ("recorded", ctypes.c_int),
                ("names", ctypes.c_char_p * LA_MAX_TRACE)]


class LaError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        super().__init__("%s failed: %s" % (where, la_status_string(code)))


def library_path():
    return _LIB_PATH


def load_library():
    """Load libla.so (built by paper_2510_21956_amd/build.py).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "HIP library %s not found; build it with "
            "`python -c 'import __graft_entry__ as g; g.build()'` "
            "(or python paper_2510_21956_amd/build.py).  There is no CPU fallback." % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, i, f = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
    lib.la_version.restype = i
    lib.la_version.argtypes = []
    lib.la_status_string.restype = ctypes.c_char_p
    lib.la_status_string.argtypes = [i]
    lib.la_workspace_bytes.restype = sz
    lib.la_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    lib.la_forward.restype = i
    lib.la_forward.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, f, f, i, i, vp, sz, vp]
    lib.la_backward.restype = i
    lib.la_backward.argtypes = [vp] * 9 + [i, i, i, i, f, f, i, i, vp, sz, vp]
    tp = ctypes.POINTER(la_trace)
    lib.la_forward_traced.restype = i
    lib.la_forward_traced.argtypes = lib.la_forward.argtypes + [tp]
    lib.la_backward_traced.restype = i
    lib.la_backward_traced.argtypes = lib.la_backward.argtypes + [tp]
    lib.la_saved_state_bytes.restype = sz
    lib.la_saved_state_bytes.argtypes = [i, i, i, i, i, i]
    lib.la_forward_save.restype = i
    lib.la_forward_save.argtypes = lib.la_forward.argtypes[:-1] + [vp, sz, vp, tp]
    lib.la_backward_saved.restype = i
    lib.la_backward_saved.argtypes = lib.la_backward.argtypes[:-1] + [vp, sz, vp, tp]
    lib.la_forward_static.restype = i
    lib.la_forward_static.argtypes = lib.la_forward.argtypes[:-3] + [vp]
    lib.la_decode_state_bytes.restype = sz
    lib.la_decode_state_bytes.argtypes = [i, i, i]
    lib.la_decode_step.restype = i
    lib.la_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, sz, i, i, i, i, f, f, i, vp]
    lib.la_decode_prefill.restype = i
    lib.la_decode_prefill.argtypes = [vp, vp, vp, sz, i, i, i, i, i, i, vp, sz, vp]
    lib.la_forward_qknorm.restype = i
    lib.la_forward_qknorm.argtypes = lib.la_forward_traced.argtypes
    lib.la_backward_qknorm.restype = i
    lib.la_backward_qknorm.argtypes = lib.la_backward_traced.argtypes
    lib.la_forward_qknorm_save.restype = i
    lib.la_forward_qknorm_save.argtypes = lib.la_forward_save.argtypes
    lib.la_backward_qknorm_saved.restype = i
    lib.la_backward_qknorm_saved.argtypes = lib.la_backward_saved.argtypes
    lib.la_backward_ab.restype = i
    lib.la_backward_ab.argtypes = [vp] * 7 + [i, i, i, i, f, f, i, i, vp, sz, vp]
    lib.la_debug_override.restype = None
    lib.la_debug_override.argtypes = [i, i]
    _lib = lib
    return lib


def la_version():
    return int(load_library().la_version())


def la_status_string(code):
    return load_library().la_status_string(int(code)).decode()


def la_debug_override(seg_len=0, force_generic=0):
    """la_debug_override of include/la.h (test / profiling hook; 0, 0 = automatic)."""
    load_library().la_debug_override(int(seg_len), int(bool(force_generic)))


def _dtype_code(t):
    if t.dtype == torch.float32:
        return LA_F32
    if t.dtype == torch.bfloat16:
        return LA_BF16
    raise TypeError("Q/K/V must be float32 or bfloat16, got %s" % t.dtype)


def la_workspace_bytes(B, H, N, D, dt, causal, is_backward):
    """is_backward: 0 forward, 1 backward, 2 backward that recomputes O / G (given as None)."""
    return int(load_library().la_workspace_bytes(B, H, N, D, dt, int(bool(causal)),
                                                 int(is_backward)))


def la_saved_state_bytes(B, H, N, D, dt, causal):
    return int(load_library().la_saved_state_bytes(B, H, N, D, dt, int(bool(causal))))


def _check_tensors(ref, *ts):
    for t in ts:
        if t is None:
            continue
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous device tensors")
        if t.device != ref.device:
            raise ValueError("tensors must live on one device")


def _stream_ptr(stream, device):
    s = torch.cuda.current_stream(device) if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(None if t is None else t.data_ptr())


def la_forward(Q, K, V, O, G, a, b, causal, workspace, stream=None):
    """la_forward of include/la.h on torch device tensors.

    Q, K, V, O: [B, H, N, D] float32 or bfloat16; G: [B, H, N] float32;
    workspace: uint8 device tensor of at least la_workspace_bytes(..., 0) bytes."""
    la_forward_traced(Q, K, V, O, G, a, b, causal, workspace, stream, None)


LA_STATIC_SCRATCH_BYTES = 32 << 20


def la_forward_static(Q, K, V, O, G, a, b, causal, stream=None):
    """la_forward_static of include/la.h: la_forward with the library's own static scratch."""
    if Q.dim() != 4:
        raise ValueError("Q must be [B, H, N, D]")
    B, H, N, D = Q.shape
    _check_tensors(Q, K, V, O, G)
    if K.shape != Q.shape or V.shape != Q.shape or O.shape != Q.shape:
        raise ValueError("shape mismatch")
    if not (K.dtype == V.dtype == O.dtype == Q.dtype):
        raise TypeError("dtype mismatch")
    if G is not None and (G.shape != Q.shape[:3] or G.dtype != torch.float32):
        raise ValueError("G must be [B, H, N] float32 (or None)")
    rc = load_library().la_forward_static(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(G), B, H, N, D,
                                          float(a), float(b), int(bool(causal)), _dtype_code(Q),
                                          _stream_ptr(stream, Q.device))
    if rc != 0:
        raise LaError(rc, "la_forward_static")


def la_forward_traced(Q, K, V, O, G, a, b, causal, workspace, stream=None, trace=None):
    """la_forward_traced of include/la.h; ``trace`` is a la_trace structure or None."""
    _forward(Q, K, V, O, G, a, b, causal, workspace, None, stream, trace, False)


def la_forward_save(Q, K, V, O, G, a, b, causal, workspace, saved, stream=None, trace=None):
    """la_forward_save of include/la.h; ``saved`` is a uint8 device tensor of at least
    la_saved_state_bytes(...) bytes (None when that is 0)."""
    _forward(Q, K, V, O, G, a, b, causal, workspace, saved, stream, trace, True)


def _saved_args(saved, ref):
    if saved is None:
        return ctypes.c_void_p(None), 0
    _check_tensors(ref, saved)
    return _ptr(saved), saved.numel() * saved.element_size()


def _forward(Q, K, V, O, G, a, b, causal, workspace, saved, stream, trace, save):
    if Q.dim() != 4:
        raise ValueError("Q must be [B, H, N, D]")
    B, H, N, D = Q.shape
    _check_tensors(Q, K, V, O, G, workspace)
    if K.shape != Q.shape or V.shape != Q.shape or O.shape != Q.shape:
        raise ValueError("shape mismatch")
    if not (K.dtype == V.dtype == O.dtype == Q.dtype):
        raise TypeError("dtype mismatch")
    if G is not None and (G.shape != Q.shape[:3] or G.dtype != torch.float32):
        raise ValueError("G must be [B, H, N] float32 (or None)")
    lib = load_library()
    head = (_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(G), B, H, N, D, float(a), float(b),
            int(bool(causal)), _dtype_code(Q), _ptr(workspace),
            workspace.numel() * workspace.element_size())
    tr = ctypes.byref(trace) if trace is not None else None
    if save == "qknorm":
        rc = lib.la_forward_qknorm(*head, _stream_ptr(stream, Q.device), tr)
    elif save == "qknorm_save":
        sp, sb = _saved_args(saved, Q)
        rc = lib.la_forward_qknorm_save(*head, sp, sb, _stream_ptr(stream, Q.device), tr)
    elif save:
        sp, sb = _saved_args(saved, Q)
        rc = lib.la_forward_save(*head, sp, sb, _stream_ptr(stream, Q.device), tr)
    else:
        rc = lib.la_forward_traced(*head, _stream_ptr(stream, Q.device), tr)
    if rc != 0:
        raise LaError(rc, "la_forward_save" if save else "la_forward")


def la_backward(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, stream=None):
    """la_backward of include/la.h on torch device tensors (see la_forward)."""
    la_backward_traced(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, stream, None)


def la_backward_traced(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, stream=None,
                       trace=None):
    """la_backward_traced of include/la.h; ``trace`` is a la_trace structure or None."""
    _backward(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, None, stream, trace, False)


def la_backward_saved(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, saved, stream=None,
                      trace=None):
    """la_backward_saved of include/la.h; ``saved`` as filled by la_forward_save."""
    _backward(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, saved, stream, trace, True)


def _backward(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, saved, stream, trace,
              use_saved):
    if Q.dim() != 4:
        raise ValueError("Q must be [B, H, N, D]")
    B, H, N, D = Q.shape
    _check_tensors(Q, K, V, O, G, dO, dQ, dK, dV, workspace)
    for name, t in (("K", K), ("V", V), ("O", O), ("dO", dO), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        if t is None:
            if name == "O":
                continue  # recomputed inside the call
            raise ValueError("%s is required" % name)
        if t.shape != Q.shape:
            raise ValueError("shape mismatch")
        if t.dtype != Q.dtype:
            raise TypeError("dtype mismatch")
    if G is not None and (G.shape != Q.shape[:3] or G.dtype != torch.float32):
        raise ValueError("G must be [B, H, N] float32 (or None)")
    lib = load_library()
    head = (_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(G), _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV),
            B, H, N, D, float(a), float(b), int(bool(causal)), _dtype_code(Q), _ptr(workspace),
            workspace.numel() * workspace.element_size())
    tr = ctypes.byref(trace) if trace is not None else None
    if use_saved == "qknorm":
        rc = lib.la_backward_qknorm(*head, _stream_ptr(stream, Q.device), tr)
    elif use_saved == "qknorm_save":
        sp, sb = _saved_args(saved, Q)
        rc = lib.la_backward_qknorm_saved(*head, sp, sb, _stream_ptr(stream, Q.device), tr)
    elif use_saved:
        sp, sb = _saved_args(saved, Q)
        rc = lib.la_backward_saved(*head, sp, sb, _stream_ptr(stream, Q.device), tr)
    else:
        rc = lib.la_backward_traced(*head, _stream_ptr(stream, Q.device), tr)
    if rc != 0:
        raise LaError(rc, "la_backward_saved" if use_saved else "la_backward")


def la_decode_state_bytes(B, H, D):
    return int(load_library().la_decode_state_bytes(B, H, D))


def la_decode_step(q, k, v, o, g, state, a, b, stream=None):
    """la_decode_step of include/la.h: q, k, v, o [B, H, T, D]; g [B, H, T] float32 or None;
    state: float32 device tensor of la_decode_state_bytes(B, H, D) bytes, updated in place."""
    if q.dim() != 4:
        raise ValueError("q must be [B, H, T, D]")
    B, H, T, D = q.shape
    _check_tensors(q, k, v, o, g, state)
    if k.shape != q.shape or v.shape != q.shape or o.shape != q.shape:
        raise ValueError("shape mismatch")
    if not (k.dtype == v.dtype == o.dtype == q.dtype) or state.dtype != torch.float32:
        raise TypeError("dtype mismatch")
    if g is not None and (g.shape != q.shape[:3] or g.dtype != torch.float32):
        raise ValueError("g must be [B, H, T] float32 (or None)")
    rc = load_library().la_decode_step(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(g), _ptr(state),
                                       state.numel() * 4, B, H, T, D, float(a), float(b),
                                       _dtype_code(q), _stream_ptr(stream, q.device))
    if rc != 0:
        raise LaError(rc, "la_decode_step")


def la_decode_prefill(K, V, state, accumulate, workspace, stream=None):
    """la_decode_prefill of include/la.h: K, V [B, H, N, D]."""
    if K.dim() != 4:
        raise ValueError("K must be [B, H, N, D]")
    B, H, N, D = K.shape
    _check_tensors(K, V, state, workspace)
    if V.shape != K.shape or V.dtype != K.dtype or state.dtype != torch.float32:
        raise ValueError("shape or dtype mismatch")
    rc = load_library().la_decode_prefill(_ptr(K), _ptr(V), _ptr(state), state.numel() * 4, B, H,
                                          N, D, _dtype_code(K), int(bool(accumulate)),
                                          _ptr(workspace),
                                          workspace.numel() * workspace.element_size(),
                                          _stream_ptr(stream, K.device))
    if rc != 0:
        raise LaError(rc, "la_decode_prefill")


def la_backward_ab(Q, K, V, O, G, dO, dab, a, b, causal, workspace, stream=None):
    """la_backward_ab of include/la.h; ``dab``: float32 device tensor of two elements."""
    if Q.dim() != 4:
        raise ValueError("Q must be [B, H, N, D]")
    B, H, N, D = Q.shape
    _check_tensors(Q, K, V, O, G, dO, dab, workspace)
    for t in (K, V, O, dO):
        if t.shape != Q.shape or t.dtype != Q.dtype:
            raise ValueError("shape or dtype mismatch")
    if G.shape != Q.shape[:3] or G.dtype != torch.float32:
        raise ValueError("G must be [B, H, N] float32")
    if dab.dtype != torch.float32 or dab.numel() < 2:
        raise ValueError("dab must hold two float32")
    rc = load_library().la_backward_ab(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(G), _ptr(dO),
                                       _ptr(dab), B, H, N, D, float(a), float(b),
                                       int(bool(causal)), _dtype_code(Q), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(),
                                       _stream_ptr(stream, Q.device))
    if rc != 0:
        raise LaError(rc, "la_backward_ab")


def la_forward_qknorm(Q, K, V, O, G, a, b, causal, workspace, stream=None, trace=None):
    """la_forward_qknorm of include/la.h: la_forward on raw Q, K, normalised row by row inside."""
    _forward(Q, K, V, O, G, a, b, causal, workspace, None, stream, trace, "qknorm")


def la_backward_qknorm(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, stream=None,
                       trace=None):
    """la_backward_qknorm of include/la.h: gradients for the raw Q, K."""
    _backward(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, None, stream, trace,
              "qknorm")


def la_forward_qknorm_save(Q, K, V, O, G, a, b, causal, workspace, saved, stream=None, trace=None):
    """la_forward_qknorm_save of include/la.h (``saved`` as for la_forward_save)."""
    _forward(Q, K, V, O, G, a, b, causal, workspace, saved, stream, trace, "qknorm_save")


def la_backward_qknorm_saved(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, saved,
                             stream=None, trace=None):
    """la_backward_qknorm_saved of include/la.h; ``saved`` as filled by la_forward_qknorm_save."""
    _backward(Q, K, V, O, G, dO, dQ, dK, dV, a, b, causal, workspace, saved, stream, trace,
              "qknorm_save")
