"""fp64 CPU oracle for linear attention (kernel a + b*x) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It never imports the HIP binding and shares no code with it.

The arithmetic lives in ``la_oracle.c`` (plain C, double precision, OpenMP over
the batch*head index); this module compiles it with gcc and exposes numpy-facing
wrappers.  Tensors are ``[B, H, N, D]`` (or ``[BH, N, D]``) float64 arrays.

Functions (paper passages in the C file's comments):
  forward_def / forward_rec       -- O, G by the definition / by running sums
  backward_def / backward_rec     -- dQ, dK, dV by the definition / running sums
  forward_def_rows                -- definition at selected rows of one slice
  decode                          -- incremental form with a carried state (App. B.1)
  grad_ab_def                     -- dL/da, dL/db by the definition
  normalise_rows / normalise_rows_backward -- the row normalisation of Sec. 3.3
  forward_qknorm / backward_qknorm -- attention on row-normalised Q, K, gradients for the raw Q, K
"""
import ctypes
import hashlib
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "la_oracle.c")
_lib = None


def _cpu_tag():
    """The library is built with -march=native, so one build serves one kind of CPU only:
    the file name carries a digest of this host's instruction-set flags, and a host with
    other flags builds its own copy instead of loading code it may not be able to run."""
    flags = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("flags"):
                flags = line
                break
    except OSError:
        pass
    return hashlib.sha1(flags.encode()).hexdigest()[:10]


_LIB = os.path.join(_HERE, "libla_oracle_%s.so" % _cpu_tag())


def build(force=False):
    """Compile la_oracle.c into a shared library next to it (gcc -O3 -march=native, OpenMP;
    -std=c11 keeps floating-point contraction and reassociation off)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lp = ctypes.POINTER(ctypes.c_long)
        L, I, F = ctypes.c_long, ctypes.c_int, ctypes.c_double
        lib.la_oracle_forward_def.argtypes = [dp, dp, dp, dp, dp, L, L, I, F, F, I]
        lib.la_oracle_forward_rec.argtypes = [dp, dp, dp, dp, dp, L, L, I, F, F, I]
        lib.la_oracle_forward_def_rows.argtypes = [dp, dp, dp, lp, L, dp, dp, L, I, F, F, I]
        lib.la_oracle_backward_def.argtypes = [dp, dp, dp, dp, dp, dp, dp, L, L, I, F, F, I]
        lib.la_oracle_backward_rec.argtypes = [dp, dp, dp, dp, dp, dp, dp, dp, dp,
                                               L, L, I, F, F, I]
        for f in (lib.la_oracle_forward_def, lib.la_oracle_forward_rec,
                  lib.la_oracle_forward_def_rows, lib.la_oracle_backward_def,
                  lib.la_oracle_backward_rec):
            f.restype = None
        lib.la_oracle_decode.argtypes = [dp, dp, dp, dp, dp, dp, L, L, I, F, F]
        lib.la_oracle_decode.restype = None
        lib.la_oracle_grad_ab_def.argtypes = [dp, dp, dp, dp, dp, L, L, I, F, F, I]
        lib.la_oracle_grad_ab_def.restype = None
        lib.la_oracle_normalise_rows.argtypes = [dp, dp, L, I]
        lib.la_oracle_normalise_rows.restype = None
        lib.la_oracle_normalise_rows_backward.argtypes = [dp, dp, dp, L, I]
        lib.la_oracle_normalise_rows_backward.restype = None
        lib.la_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads():
    """Threads the OpenMP loops will use (at most one per batch*head slice)."""
    return int(_load().la_oracle_num_threads())


def _p(x):
    return x.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _prep(*xs):
    out = []
    shape = xs[0].shape
    for x in xs:
        if x.shape != shape:
            raise ValueError("shape mismatch: %r vs %r" % (x.shape, shape))
        out.append(np.ascontiguousarray(x, dtype=np.float64))
    if len(shape) < 2:
        raise ValueError("need [..., N, D]")
    N, D = shape[-2], shape[-1]
    BH = int(np.prod(shape[:-2], dtype=np.int64)) if len(shape) > 2 else 1
    return out, shape, BH, N, D


def _forward(fn, Q, K, V, a, b, causal):
    (Q, K, V), shape, BH, N, D = _prep(Q, K, V)
    O = np.empty(shape, dtype=np.float64)
    G = np.empty(shape[:-1], dtype=np.float64)
    if BH * N * D:
        fn(_p(Q), _p(K), _p(V), _p(O), _p(G), BH, N, D, float(a), float(b), int(bool(causal)))
    return O, G


def forward_def(Q, K, V, a, b, causal):
    """O(N^2 D) definition (Sec. 2.2).  Returns (O, G)."""
    return _forward(_load().la_oracle_forward_def, Q, K, V, a, b, causal)


def forward_rec(Q, K, V, a, b, causal):
    """O(N D^2) running sums (Eq. fglast / xy).  Returns (O, G)."""
    return _forward(_load().la_oracle_forward_rec, Q, K, V, a, b, causal)


def forward_def_rows(q, k, v, rows, a, b, causal):
    """Definition at the given rows of one [N, D] slice.  Returns (o_rows, g_rows)."""
    (q, k, v), shape, BH, N, D = _prep(q, k, v)
    if BH != 1:
        raise ValueError("forward_def_rows takes one [N, D] slice")
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    if rows.size and (rows.min() < 0 or rows.max() >= N):
        raise ValueError("row index out of range")
    o = np.empty((rows.size, D), dtype=np.float64)
    g = np.empty((rows.size,), dtype=np.float64)
    _load().la_oracle_forward_def_rows(
        _p(q), _p(k), _p(v), rows.ctypes.data_as(ctypes.POINTER(ctypes.c_long)),
        rows.size, _p(o), _p(g), N, D, float(a), float(b), int(bool(causal)))
    return o, g


def backward_def(Q, K, V, dO, a, b, causal):
    """Gradients by the pairwise definition (Eq. bound + chain rule).  (dQ, dK, dV)."""
    (Q, K, V, dO), shape, BH, N, D = _prep(Q, K, V, dO)
    dQ, dK, dV = (np.empty(shape, dtype=np.float64) for _ in range(3))
    if BH * N * D:
        _load().la_oracle_backward_def(_p(Q), _p(K), _p(V), _p(dO), _p(dQ), _p(dK), _p(dV),
                                       BH, N, D, float(a), float(b), int(bool(causal)))
    return dQ, dK, dV


def backward_rec(Q, K, V, O, G, dO, a, b, causal):
    """Gradients by the running sums of Eq. back1/back2/endd from the stored set
    {Q, K, V, O, g}.  Returns (dQ, dK, dV)."""
    (Q, K, V, O, dO), shape, BH, N, D = _prep(Q, K, V, O, dO)
    G = np.ascontiguousarray(G, dtype=np.float64)
    if G.shape != shape[:-1]:
        raise ValueError("G must be [..., N]")
    dQ, dK, dV = (np.empty(shape, dtype=np.float64) for _ in range(3))
    if BH * N * D:
        _load().la_oracle_backward_rec(_p(Q), _p(K), _p(V), _p(O), _p(G), _p(dO),
                                       _p(dQ), _p(dK), _p(dV),
                                       BH, N, D, float(a), float(b), int(bool(causal)))
    return dQ, dK, dV


def decode_state_floats(D):
    """Doubles per slice of the carried state: [S (D*D) | z (D) | p (D) | count (1)]."""
    return D * D + 2 * D + 1


def decode(Q, K, V, state, a, b):
    """Incremental form (App. B.1): T new rows per slice, [..., T, D], appended to the
    prefix summarised by ``state`` ([..., decode_state_floats(D)], updated in place; zeros
    for an empty prefix).  Returns (O, G) of the new rows."""
    (Q, K, V), shape, BH, T, D = _prep(Q, K, V)
    if state.dtype != np.float64 or not state.flags.c_contiguous:
        raise ValueError("state must be a C-contiguous float64 array")
    if state.size != BH * decode_state_floats(D):
        raise ValueError("state has the wrong size")
    O = np.empty(shape, dtype=np.float64)
    G = np.empty(shape[:-1], dtype=np.float64)
    if BH * T * D:
        _load().la_oracle_decode(_p(Q), _p(K), _p(V), _p(O), _p(G), _p(state), BH, T, D,
                                 float(a), float(b))
    return O, G


def grad_ab_def(Q, K, V, dO, a, b, causal):
    """(dL/da, dL/db) of L = sum(O * dO) by the pairwise definition, over all slices."""
    (Q, K, V, dO), shape, BH, N, D = _prep(Q, K, V, dO)
    out = np.zeros(2, dtype=np.float64)
    if BH * N * D:
        _load().la_oracle_grad_ab_def(_p(Q), _p(K), _p(V), _p(dO), _p(out), BH, N, D,
                                      float(a), float(b), int(bool(causal)))
    return float(out[0]), float(out[1])


def normalise_rows(X):
    """xhat = x / ||x|| for every row of X [..., D] (Sec. 3.3)."""
    X = np.ascontiguousarray(X, dtype=np.float64)
    out = np.empty_like(X)
    D = X.shape[-1]
    if X.size:
        _load().la_oracle_normalise_rows(_p(X), _p(out), X.size // D, D)
    return out


def normalise_rows_backward(X, dXhat):
    """Gradient with respect to X of a loss whose gradient with respect to xhat is dXhat."""
    X = np.ascontiguousarray(X, dtype=np.float64)
    dXhat = np.ascontiguousarray(dXhat, dtype=np.float64)
    if dXhat.shape != X.shape:
        raise ValueError("shape mismatch")
    out = np.empty_like(X)
    D = X.shape[-1]
    if X.size:
        _load().la_oracle_normalise_rows_backward(_p(X), _p(dXhat), _p(out), X.size // D, D)
    return out


def forward_qknorm(Q, K, V, a, b, causal):
    """Row-normalise Q and K (Sec. 3.3), then the running-sum forward pass.  Returns (O, G)."""
    return forward_rec(normalise_rows(Q), normalise_rows(K), V, a, b, causal)


def backward_qknorm(Q, K, V, O, G, dO, a, b, causal):
    """Gradients with respect to the raw Q, K (and V) of attention on row-normalised Q, K,
    from the stored set {Q, K, V, O, g}: the running-sum backward pass on the normalised
    rows, then the backward of the normalisation."""
    dQh, dKh, dV = backward_rec(normalise_rows(Q), normalise_rows(K), V, O, G, dO, a, b, causal)
    return normalise_rows_backward(Q, dQh), normalise_rows_backward(K, dKh), dV
