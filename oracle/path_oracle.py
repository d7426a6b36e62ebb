"""ctypes front end of the fp64 CPU oracle in ``path_oracle.c``.

TEST INFRASTRUCTURE.  Only the tests, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this module; the GPU library
and its Python binding never do.  Nothing here touches the HIP path.

The oracle evaluates PaTH attention straight from its definition (paper
Sec. 2.1/2.2): for each query walk leftwards over the keys, logit against
``k_j`` first, then ``u <- (I - beta_j w_j w_j^T) u``; softmax in fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "path_oracle.c")
_LIB = os.path.join(_HERE, "libpath_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, -O2, strict IEEE: no -ffast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.path_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().path_oracle_num_threads())


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def fwd(q, k, v, w, beta, scale, rows=None, logf=None):
    """o, lse for all rows (``rows=None``) or for the token indices ``rows``.

    q,k,v,w: [B,H,L,d]; beta: [B,H,L]; logf (PaTH-FoX, optional): [B,H,L], the log of the
    forget gates.  Returns o [B,H,R,d], lse [B,H,R].
    """
    lib = _load()
    q, k, v, w, beta = map(_f64, (q, k, v, w, beta))
    if logf is not None:
        logf = _f64(logf)
        assert logf.shape == beta.shape
    B, H, L, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape and w.shape == q.shape
    assert beta.shape == (B, H, L)
    if rows is None:
        rows = np.arange(L, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    assert rows.ndim == 1 and (rows >= 0).all() and (rows < L).all()
    R = rows.shape[0]
    o = np.empty((B, H, R, d), dtype=np.float64)
    lse = np.empty((B, H, R), dtype=np.float64)
    if R:
        lib.path_oracle_fwd_rows(_p(q), _p(k), _p(v), _p(w), _p(beta), _p(logf) if logf is not None else None, _p(rows),
                                 ctypes.c_int(R), _p(o), _p(lse),
                                 ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(L),
                                 ctypes.c_int(d), ctypes.c_double(scale))
    return o, lse


def logits(q, k, w, beta, scale):
    """Dense scaled logits [L,L] of ONE head (q,k,w: [L,d]; beta: [L])."""
    lib = _load()
    q, k, w, beta = map(_f64, (q, k, w, beta))
    L, d = q.shape
    S = np.zeros((L, L), dtype=np.float64)
    lib.path_oracle_logits(_p(q), _p(k), _p(w), _p(beta), _p(S),
                           ctypes.c_int(L), ctypes.c_int(d), ctypes.c_double(scale))
    return S


def walk_norms(q, k, w, beta, i):
    """Norm of the walk vector of query ``i`` of ONE head at positions 0..i."""
    lib = _load()
    q, k, w, beta = map(_f64, (q, k, w, beta))
    L, d = q.shape
    n = np.zeros(L, dtype=np.float64)
    lib.path_oracle_walk_norms(_p(q), _p(k), _p(w), _p(beta), ctypes.c_int(int(i)),
                               _p(n), ctypes.c_int(L), ctypes.c_int(d))
    return n[: i + 1]


def bwd(q, k, v, w, beta, dO, scale, logf=None):
    """Gradients of sum(dO * o) w.r.t. q, k, v, w, beta (same shapes) -- and, with gates
    (PaTH-FoX, ``logf`` [B,H,L]), w.r.t. logf as a sixth result."""
    lib = _load()
    q, k, v, w, beta, dO = map(_f64, (q, k, v, w, beta, dO))
    B, H, L, d = q.shape
    outs = [np.empty_like(q) for _ in range(4)] + [np.empty((B, H, L), dtype=np.float64)]
    dlogf = None
    if logf is not None:
        logf = _f64(logf)
        assert logf.shape == beta.shape
        dlogf = np.empty((B, H, L), dtype=np.float64)
    lib.path_oracle_bwd(_p(q), _p(k), _p(v), _p(w), _p(beta), _p(logf) if logf is not None else None, _p(dO),
                        *[_p(x) for x in outs], _p(dlogf) if dlogf is not None else None,
                        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(L),
                        ctypes.c_int(d), ctypes.c_double(scale))
    return tuple(outs) + ((dlogf,) if dlogf is not None else ())
