"""Thin ctypes binding over ``libpath_attn.so`` (the C ABI of include/path_attn.h).

Argument marshalling only: every step of the hot path runs inside the HIP
kernels of the library.  PyTorch is used for device memory and the current
stream.  If the library has not been built the functions raise -- there is no
CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

PATH_F32 = 0
PATH_BF16 = 1
PATH_LAYOUT_BHLD = 0      # q, k, v, w, o [B,H,L,d]; beta, lse [B,H,L]
PATH_LAYOUT_BLHD = 1      # ...           [B,L,H,d]; ...       [B,L,H]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpath_attn.so")
_lib = None


class PathAttnError(RuntimeError):
    def __init__(self, code: int, name: str):
        super().__init__(f"path_attn: {name} (status {code})")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it first (python -m paper_2505_16381_amd.build). "
            "There is no fallback path.")
    # The process must hold ONE HIP runtime, the one PyTorch ships, because the tensors whose pointers
    # are handed to the library are allocated through it.  Importing torch first makes the loader
    # resolve this library's runtime dependency to that already loaded copy.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.path_status_str.restype = ctypes.c_char_p
    lib.path_status_str.argtypes = [ci]
    lib.path_attn_last_error.restype = ctypes.c_char_p
    lib.path_attn_last_error.argtypes = []
    lib.path_attn_workspace_bytes.restype = sz
    lib.path_attn_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
    lib.path_attn_fwd_workspace_layout.restype = ci
    lib.path_attn_fwd_workspace_layout.argtypes = [ci, ci, ci, ci, ci, ctypes.POINTER(sz)]
    lib.path_attn_fwd.restype = ci
    lib.path_attn_fwd.argtypes = [vp] * 7 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_fwd_prep.restype = ci
    lib.path_attn_fwd_prep.argtypes = [vp] * 5 + [ci, ci, ci, ci, ci, vp, sz, vp]
    lib.path_attn_fwd_sweep.restype = ci
    lib.path_attn_fwd_sweep.argtypes = [vp, vp, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_bwd.restype = ci
    lib.path_attn_bwd.argtypes = [vp] * 13 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_fox_fwd.restype = ci
    lib.path_attn_fox_fwd.argtypes = [vp] * 8 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_fox_bwd.restype = ci
    lib.path_attn_fox_bwd.argtypes = [vp] * 15 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_train_fwd.restype = ci
    lib.path_attn_train_fwd.argtypes = [vp] * 8 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_train_fwd_prep.restype = ci
    lib.path_attn_train_fwd_prep.argtypes = [vp] * 6 + [ci, ci, ci, ci, ci, vp, sz, vp]
    lib.path_attn_train_fwd_sweep.restype = ci
    lib.path_attn_train_fwd_sweep.argtypes = [vp, vp, ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_train_bwd.restype = ci
    lib.path_attn_train_bwd.argtypes = [vp] * 15 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_fwd_layout.restype = ci
    lib.path_attn_fwd_layout.argtypes = [vp] * 8 + [ci, ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_bwd_layout.restype = ci
    lib.path_attn_bwd_layout.argtypes = [vp] * 15 + [ci, ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_varlen_workspace_bytes.restype = sz
    lib.path_attn_varlen_workspace_bytes.argtypes = [ctypes.POINTER(ci), ci, ci, ci, ci, ci]
    lib.path_attn_varlen_fwd.restype = ci
    lib.path_attn_varlen_fwd.argtypes = [vp] * 8 + [ctypes.POINTER(ci), ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_varlen_bwd.restype = ci
    lib.path_attn_varlen_bwd.argtypes = [vp] * 15 + [ctypes.POINTER(ci), ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_decode_workspace_bytes.restype = sz
    lib.path_decode_workspace_bytes.argtypes = [ci, ci, ci]
    lib.path_key_prefill.restype = ci
    lib.path_key_prefill.argtypes = [vp, ci, ci, ci, ci, ci, vp, sz, vp, vp, ci, vp]
    lib.path_decode_step.restype = ci
    lib.path_decode_step.argtypes = [vp] * 7 + [ci, ci, vp, vp, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_attn_bwd_workspace_bytes_for_heads.restype = sz
    lib.path_attn_bwd_workspace_bytes_for_heads.argtypes = [ci, ci, ci, ci, ci, ci]
    lib.path_attn_bwd_heads_per_pass.restype = ci
    lib.path_attn_bwd_heads_per_pass.argtypes = [ci, ci, ci, ci, ci, sz]
    lib.path_attn_train_bwd_stages.restype = ci
    lib.path_attn_train_bwd_stages.argtypes = [ci] + [vp] * 15 + [ci, ci, ci, ci, ci, cf, ci, vp, sz, vp]
    lib.path_probe_mfma_flops.restype = ctypes.c_double
    lib.path_probe_mfma_flops.argtypes = [ci, ci]
    lib.path_probe_mfma.restype = ci
    lib.path_probe_mfma.argtypes = [vp, ci, ci, vp]
    lib.path_gate_prefill.restype = ci
    lib.path_gate_prefill.argtypes = [vp, ci, ci, ci, ci, vp, ci, vp]
    lib.path_decode_step_fox.restype = ci
    lib.path_decode_step_fox.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, vp, vp, ci, ci, ci, ctypes.c_float, ci, vp, ctypes.c_size_t, vp]
    lib.path_attn_ring_state_bytes.restype = ctypes.c_size_t
    lib.path_attn_ring_state_bytes.argtypes = [ci, ci, ci, ci]
    lib.path_attn_ring_regions.restype = ci
    lib.path_attn_ring_regions.argtypes = [ci, ci, ci, ci, ci, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
    lib.path_attn_ring_local.restype = ci
    lib.path_attn_ring_local.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ctypes.c_float, ci, vp, ctypes.c_size_t, vp]
    lib.path_attn_ring_hop.restype = ci
    lib.path_attn_ring_hop.argtypes = [vp, ci, ci, ci, vp, ctypes.c_size_t, ci, ci, ci, ctypes.c_float, ci, vp]
    lib.path_attn_ring_finish.restype = ci
    lib.path_attn_ring_finish.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp, ctypes.c_size_t, vp]
    lib.path_probe_mfma_operands.restype = ci
    lib.path_probe_mfma_operands.argtypes = [vp, ci, ci, ci, vp]
    lib.path_decode_static_scratch_bytes.restype = sz
    lib.path_decode_static_scratch_bytes.argtypes = []
    lib.path_decode_step_static.restype = ci
    lib.path_decode_step_static.argtypes = [vp] * 7 + [ci, ci, vp, vp, ci, ci, ci, cf, ci, vp]
    _lib = lib
    return lib


def path_status_str(code: int) -> str:
    return load_library().path_status_str(int(code)).decode()


def path_attn_workspace_bytes(B, H, L, d, dt, for_backward=False) -> int:
    return int(load_library().path_attn_workspace_bytes(B, H, L, d, dt, int(bool(for_backward))))


def path_attn_bwd_workspace_bytes_for_heads(B, H, L, d, dt, heads) -> int:
    """Bytes that let the self-contained backward pass over ``heads`` heads at a time (1 = the minimum)."""
    return int(load_library().path_attn_bwd_workspace_bytes_for_heads(B, H, L, d, dt, int(heads)))


def path_attn_bwd_heads_per_pass(B, H, L, d, dt, workspace_bytes) -> int:
    return int(load_library().path_attn_bwd_heads_per_pass(B, H, L, d, dt, int(workspace_bytes)))


def path_attn_fwd_workspace_layout(B, H, L, d, dt):
    """Byte offsets (kt, vt, dp, xinit, sd, total) of the forward workspace."""
    arr = (ctypes.c_size_t * 6)()
    _check(load_library().path_attn_fwd_workspace_layout(B, H, L, d, dt, arr))
    return tuple(int(x) for x in arr)


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def path_attn_last_error() -> str:
    return load_library().path_attn_last_error().decode()


def _check(code):
    if code != 0:
        detail = path_attn_last_error() if code == 6 else ""
        raise PathAttnError(code, path_status_str(code) + (f" [{detail}]" if detail else ""))


def _dt_of(t):
    import torch
    if t.dtype == torch.float32:
        return PATH_F32
    if t.dtype == torch.bfloat16:
        return PATH_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _workspace(nbytes, like, workspace):
    import torch
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=like.device)
    return workspace


def path_attn_fwd(q, k, v, w, beta, scale=None, causal=True, o=None, lse=None,
                  workspace=None, stream=None):
    """o, lse = PaTH attention forward.  q,k,v,w: [B,H,L,d]; beta: [B,H,L] (CUDA tensors)."""
    import torch
    lib = load_library()
    B, H, L, d = q.shape
    dt = _dt_of(q)
    for t in (q, k, v, w, beta):
        assert t.is_cuda and t.is_contiguous() and t.dtype == q.dtype
    assert k.shape == q.shape and v.shape == q.shape and w.shape == q.shape
    assert tuple(beta.shape) == (B, H, L)
    if scale is None:
        scale = float(d) ** -0.5
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, L), dtype=torch.float32, device=q.device)
    nbytes = path_attn_workspace_bytes(B, H, L, d, dt, False)
    workspace = _workspace(nbytes, q, workspace)
    _check(lib.path_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _ptr(o), _ptr(lse),
                             B, H, L, d, int(bool(causal)), float(scale), dt,
                             _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return o, lse


def path_attn_fwd_prep(q, k, v, w, beta, workspace, stream=None):
    """Stage 1 of the forward (chunk transform) into ``workspace``."""
    B, H, L, d = q.shape
    _check(load_library().path_attn_fwd_prep(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), B, H, L, d,
                                             _dt_of(q), _ptr(workspace), workspace.numel(),
                                             _stream_handle(stream)))


def path_attn_fwd_sweep(o, lse, scale, workspace, stream=None):
    """Stage 2 of the forward (sweep over key chunks) from ``workspace`` into o, lse."""
    B, H, L, d = o.shape
    _check(load_library().path_attn_fwd_sweep(_ptr(o), _ptr(lse), B, H, L, d, float(scale), _dt_of(o),
                                              _ptr(workspace), workspace.numel(), _stream_handle(stream)))


def path_attn_bwd(q, k, v, w, beta, o, lse, d_o, scale=None, causal=True,
                  workspace=None, stream=None):
    """dq, dk, dv, dw, dbeta = gradients of sum(d_o * o)."""
    import torch
    lib = load_library()
    B, H, L, d = q.shape
    dt = _dt_of(q)
    for t in (q, k, v, w, beta, o, d_o):
        assert t.is_cuda and t.is_contiguous() and t.dtype == q.dtype
    assert lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32
    if scale is None:
        scale = float(d) ** -0.5
    dq, dk, dv, dw = (torch.empty_like(q) for _ in range(4))
    dbeta = torch.empty_like(beta)
    nbytes = path_attn_workspace_bytes(B, H, L, d, dt, True)
    workspace = _workspace(nbytes, q, workspace)
    _check(lib.path_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _ptr(o), _ptr(lse),
                             _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dw), _ptr(dbeta),
                             B, H, L, d, int(bool(causal)), float(scale), dt,
                             _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return dq, dk, dv, dw, dbeta


def path_decode_workspace_bytes(B, H, d) -> int:
    return int(load_library().path_decode_workspace_bytes(B, H, d))


def path_key_prefill(v, fwd_workspace, kcache, vcache, stream=None):
    """Fills positions [0, L) of the caches [B,H,Lmax,d] after a prompt; ``fwd_workspace`` is the
    workspace path_attn_fwd / path_attn_fwd_prep used on that prompt."""
    B, H, L, d = v.shape
    _check(load_library().path_key_prefill(_ptr(v), B, H, L, d, _dt_of(v), _ptr(fwd_workspace), fwd_workspace.numel(),
                                           _ptr(kcache), _ptr(vcache), kcache.shape[2], _stream_handle(stream)))


def path_decode_step(q, k, v, w, beta, kcache, vcache, n, scale, workspace=None, stream=None):
    """One arriving token per (batch, head): q,k,v,w [B,H,d], beta [B,H]; n tokens already cached.
    Returns (o [B,H,d], lse [B,H]); the caches are updated in place."""
    import torch
    B, H, d = q.shape
    if workspace is None:
        workspace = torch.empty(path_decode_workspace_bytes(B, H, d), dtype=torch.uint8, device=q.device)
    o = torch.empty_like(q)
    lse = torch.empty((B, H), dtype=torch.float32, device=q.device)
    _check(load_library().path_decode_step(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _ptr(kcache), _ptr(vcache),
                                           int(n), kcache.shape[2], _ptr(o), _ptr(lse), B, H, d, float(scale), _dt_of(q),
                                           _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return o, lse


def path_gate_prefill(log_f, ccache, stream=None):
    """Running sums of the prompt's log gates log_f [B,H,L] into ccache [B,H,Lmax] (fp32)."""
    B, H, L = log_f.shape
    _check(load_library().path_gate_prefill(_ptr(log_f), B, H, L, _dt_of(log_f), _ptr(ccache), ccache.shape[2], _stream_handle(stream)))


def path_decode_step_fox(q, k, v, w, beta, log_f, kcache, vcache, ccache, n, scale, workspace=None, stream=None):
    """path_decode_step with forget gates: log_f [B,H] is the arriving token's log gate, ccache [B,H,Lmax] (fp32)
    the running sums of the cached tokens (updated in place)."""
    import torch
    B, H, d = q.shape
    if workspace is None:
        workspace = torch.empty(path_decode_workspace_bytes(B, H, d), dtype=torch.uint8, device=q.device)
    o = torch.empty_like(q)
    lse = torch.empty((B, H), dtype=torch.float32, device=q.device)
    _check(load_library().path_decode_step_fox(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _ptr(log_f), _ptr(kcache), _ptr(vcache),
                                               _ptr(ccache), int(n), kcache.shape[2], _ptr(o), _ptr(lse), B, H, d, float(scale), _dt_of(q),
                                               _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return o, lse


def path_decode_static_scratch_bytes() -> int:
    return int(load_library().path_decode_static_scratch_bytes())


def path_decode_step_static(q, k, v, w, beta, kcache, vcache, n, scale, o, lse, stream=None):
    """path_decode_step without a workspace and without any allocation: the caller passes the outputs
    o [B,H,d] and lse [B,H] (fp32) too; the split partials go to the library's own device array."""
    B, H, d = q.shape
    _check(load_library().path_decode_step_static(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _ptr(kcache), _ptr(vcache),
                                                  int(n), kcache.shape[2], _ptr(o), _ptr(lse), B, H, d, float(scale), _dt_of(q),
                                                  _stream_handle(stream)))
    return o, lse


def path_attn_fox_fwd(q, k, v, w, beta, log_f, scale=None, workspace=None, stream=None):
    """PaTH-FoX forward: as path_attn_fwd with log_f [B,H,L], the log of the forget gates."""
    import torch
    B, H, L, d = q.shape
    scale = float(d ** -0.5 if scale is None else scale)
    dt = _dt_of(q)
    o = torch.empty_like(q)
    lse = torch.empty((B, H, L), dtype=torch.float32, device=q.device)
    workspace = _workspace(path_attn_workspace_bytes(B, H, L, d, dt, False), q, workspace)
    _check(load_library().path_attn_fox_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _ptr(log_f), _ptr(o), _ptr(lse),
                                            B, H, L, d, 1, scale, dt, _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return o, lse


def path_attn_fox_bwd(q, k, v, w, beta, log_f, o, lse, d_o, scale=None, workspace=None, stream=None):
    """PaTH-FoX backward: returns (dq, dk, dv, dw, dbeta, dlog_f)."""
    import torch
    B, H, L, d = q.shape
    scale = float(d ** -0.5 if scale is None else scale)
    dt = _dt_of(q)
    outs = [torch.empty_like(q) for _ in range(4)] + [torch.empty_like(beta), torch.empty_like(log_f)]
    workspace = _workspace(path_attn_workspace_bytes(B, H, L, d, dt, True), q, workspace)
    _check(load_library().path_attn_fox_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _ptr(log_f), _ptr(o), _ptr(lse), _ptr(d_o),
                                            *[_ptr(x) for x in outs], B, H, L, d, 1, scale, dt,
                                            _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return tuple(outs)


def path_attn_train_fwd(q, k, v, w, beta, workspace, log_f=None, scale=None, stream=None):
    """Forward of the training pair: o, lse as path_attn_fwd (or path_attn_fox_fwd with log_f); `workspace`
    (backward-sized, path_attn_workspace_bytes(..., True)) keeps what path_attn_train_bwd starts from."""
    import torch
    B, H, L, d = q.shape
    scale = float(d ** -0.5 if scale is None else scale)
    dt = _dt_of(q)
    o = torch.empty_like(q)
    lse = torch.empty((B, H, L), dtype=torch.float32, device=q.device)
    _check(load_library().path_attn_train_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _ptr(log_f) if log_f is not None else None,
                                              _ptr(o), _ptr(lse), B, H, L, d, 1, scale, dt,
                                              _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return o, lse


def path_attn_train_bwd(q, k, v, w, beta, o, lse, d_o, workspace, log_f=None, scale=None, stream=None):
    """Backward of the training pair on the workspace path_attn_train_fwd left: (dq, dk, dv, dw, dbeta[, dlog_f])."""
    import torch
    B, H, L, d = q.shape
    scale = float(d ** -0.5 if scale is None else scale)
    dt = _dt_of(q)
    outs = [torch.empty_like(q) for _ in range(4)] + [torch.empty_like(beta)]
    dlog_f = torch.empty_like(log_f) if log_f is not None else None
    _check(load_library().path_attn_train_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _ptr(log_f) if log_f is not None else None,
                                              _ptr(o), _ptr(lse), _ptr(d_o), *[_ptr(x) for x in outs],
                                              _ptr(dlog_f) if dlog_f is not None else None, B, H, L, d, 1, scale, dt,
                                              _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return tuple(outs) + ((dlog_f,) if dlog_f is not None else ())


PATH_BWD_STAGE_SCAN, PATH_BWD_STAGE_KEYS_NEAR, PATH_BWD_STAGE_KEYS_FAR, PATH_BWD_STAGE_DDP, PATH_BWD_STAGE_CHUNK = 1, 2, 4, 8, 16
PATH_BWD_STAGE_ALL = 31


def path_attn_train_bwd_stages(stages, q, k, v, w, beta, o, lse, d_o, outs, workspace, log_f=None, dlog_f=None, scale=None, stream=None):
    """The selected stages of path_attn_train_bwd (PATH_BWD_STAGE_* bits) into the caller's gradient tensors
    ``outs`` = (dq, dk, dv, dw, dbeta); the stages must be called in the order of their values."""
    B, H, L, d = q.shape
    scale = float(d ** -0.5 if scale is None else scale)
    _check(load_library().path_attn_train_bwd_stages(int(stages), _ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta),
                                                     _ptr(log_f) if log_f is not None else None, _ptr(o), _ptr(lse), _ptr(d_o),
                                                     *[_ptr(x) for x in outs], _ptr(dlog_f) if dlog_f is not None else None,
                                                     B, H, L, d, 1, scale, _dt_of(q), _ptr(workspace), workspace.numel(),
                                                     _stream_handle(stream)))
    return outs


def path_probe_mfma(sink, waves_per_simd, iters, stream=None, random_operands=False):
    """Enqueues the register-resident MFMA chain (a measurement aid); returns the number of flops it performs.
    random_operands: operands of random sign and significand (what the kernels multiply) instead of smooth ones."""
    lib = load_library()
    if random_operands:
        _check(lib.path_probe_mfma_operands(_ptr(sink), int(waves_per_simd), int(iters), 1, _stream_handle(stream)))
    else:
        _check(lib.path_probe_mfma(_ptr(sink), int(waves_per_simd), int(iters), _stream_handle(stream)))
    return float(lib.path_probe_mfma_flops(int(waves_per_simd), int(iters)))


def path_attn_ring_state_bytes(B, H, L, d) -> int:
    return int(load_library().path_attn_ring_state_bytes(B, H, L, d))


def path_attn_ring_regions(B, H, L, d, dt):
    """[(offset, bytes)] of the workspace regions a hop reads: second-level keys, values, super-block products, gate sums."""
    off = (ctypes.c_size_t * 4)()
    nb = (ctypes.c_size_t * 4)()
    _check(load_library().path_attn_ring_regions(B, H, L, d, dt, off, nb))
    return [(int(off[i]), int(nb[i])) for i in range(4)]


def path_attn_ring_local(q, k, v, w, beta, state, workspace, log_f=None, scale=None, stream=None):
    """A device's own segment of a sequence-parallel forward: fills ``state`` (the sweep's per-query registers) and
    ``workspace`` (the segment's tiles, which segments to the right attend).  log_f: the segment's gates (PaTH-FoX)."""
    B, H, L, d = q.shape
    if scale is None:
        scale = float(d) ** -0.5
    _check(load_library().path_attn_ring_local(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _opt(log_f), _ptr(state), B, H, L, d,
                                               float(scale), _dt_of(q), _ptr(workspace), workspace.numel(), _stream_handle(stream)))


def path_attn_ring_hop(state, B, H, Lq, remote_workspace, Lk, d, dt, with_gates=False, scale=None, stream=None):
    """One hop: the queries of ``state`` attend every key of an earlier segment of Lk tokens (its workspace)."""
    if scale is None:
        scale = float(d) ** -0.5
    _check(load_library().path_attn_ring_hop(_ptr(state), B, H, Lq, _ptr(remote_workspace), remote_workspace.numel(), Lk, d,
                                             int(bool(with_gates)), float(scale), dt, _stream_handle(stream)))


def path_attn_ring_finish(state, o, lse, gates_workspace=None, stream=None):
    """o, lse from the state after the last hop (PaTH-FoX: with the workspace of the device's own segment)."""
    B, H, L, d = o.shape
    _check(load_library().path_attn_ring_finish(_ptr(state), _ptr(o), _ptr(lse), B, H, L, d, _dt_of(o), _opt(gates_workspace),
                                                gates_workspace.numel() if gates_workspace is not None else 0, _stream_handle(stream)))


def path_attn_train_fwd_prep(q, k, v, w, beta, workspace, log_f=None, stream=None):
    """First stage of path_attn_train_fwd: the transforms, into the backward-sized workspace."""
    B, H, L, d = q.shape
    _check(load_library().path_attn_train_fwd_prep(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta),
                                                   _ptr(log_f) if log_f is not None else None, B, H, L, d, _dt_of(q),
                                                   _ptr(workspace), workspace.numel(), _stream_handle(stream)))


def path_attn_train_fwd_sweep(o, lse, scale, workspace, with_gates=False, stream=None):
    """Second stage of path_attn_train_fwd: the sweep, on the workspace the first stage filled."""
    B, H, L, d = o.shape
    _check(load_library().path_attn_train_fwd_sweep(_ptr(o), _ptr(lse), int(bool(with_gates)), B, H, L, d, float(scale), _dt_of(o),
                                                    _ptr(workspace), workspace.numel(), _stream_handle(stream)))


def _opt(x):
    return _ptr(x) if x is not None else None


def _dims(q, layout):
    if layout == PATH_LAYOUT_BLHD:
        B, L, H, d = q.shape
    else:
        B, H, L, d = q.shape
    return B, H, L, d


def path_attn_fwd_layout(q, k, v, w, beta, layout, log_f=None, scale=None, workspace=None, stream=None):
    """Forward on [B,H,L,d] (PATH_LAYOUT_BHLD) or [B,L,H,d] (PATH_LAYOUT_BLHD) tensors; with log_f: PaTH-FoX.
    Returns (o, lse) in the same layout."""
    import torch
    B, H, L, d = _dims(q, layout)
    scale = float(d ** -0.5 if scale is None else scale)
    dt = _dt_of(q)
    o = torch.empty_like(q)
    lse = torch.empty(beta.shape, dtype=torch.float32, device=q.device)
    workspace = _workspace(path_attn_workspace_bytes(B, H, L, d, dt, False), q, workspace)
    _check(load_library().path_attn_fwd_layout(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _opt(log_f), _ptr(o), _ptr(lse),
                                               B, H, L, d, int(layout), 1, scale, dt, _ptr(workspace), workspace.numel(),
                                               _stream_handle(stream)))
    return o, lse


def path_attn_bwd_layout(q, k, v, w, beta, o, lse, d_o, layout, log_f=None, scale=None, workspace=None, stream=None):
    """Backward on either layout: (dq, dk, dv, dw, dbeta[, dlog_f]) in the layout of the inputs."""
    import torch
    B, H, L, d = _dims(q, layout)
    scale = float(d ** -0.5 if scale is None else scale)
    dt = _dt_of(q)
    outs = [torch.empty_like(q) for _ in range(4)] + [torch.empty_like(beta)]
    dlog_f = torch.empty_like(log_f) if log_f is not None else None
    workspace = _workspace(path_attn_workspace_bytes(B, H, L, d, dt, True), q, workspace)
    _check(load_library().path_attn_bwd_layout(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _opt(log_f), _ptr(o), _ptr(lse), _ptr(d_o),
                                               *[_ptr(x) for x in outs], _opt(dlog_f), B, H, L, d, int(layout), 1, scale, dt,
                                               _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return tuple(outs) + ((dlog_f,) if dlog_f is not None else ())


def _cu(cu_seqlens):
    cu = [int(x) for x in cu_seqlens]
    return (ctypes.c_int * len(cu))(*cu), len(cu) - 1


def path_attn_varlen_workspace_bytes(cu_seqlens, H, d, dt, for_backward=False) -> int:
    arr, n = _cu(cu_seqlens)
    return int(load_library().path_attn_varlen_workspace_bytes(arr, n, H, d, dt, int(bool(for_backward))))


def path_attn_varlen_fwd(q, k, v, w, beta, cu_seqlens, log_f=None, scale=None, workspace=None, stream=None):
    """Forward on packed sequences: q, k, v, w [T,H,d], beta [T,H]; cu_seqlens = host list of nseq+1 offsets."""
    import torch
    T, H, d = q.shape
    scale = float(d ** -0.5 if scale is None else scale)
    dt = _dt_of(q)
    arr, n = _cu(cu_seqlens)
    o = torch.empty_like(q)
    lse = torch.empty((T, H), dtype=torch.float32, device=q.device)
    workspace = _workspace(path_attn_varlen_workspace_bytes(cu_seqlens, H, d, dt, False), q, workspace)
    _check(load_library().path_attn_varlen_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _opt(log_f), _ptr(o), _ptr(lse),
                                               arr, n, H, d, 1, scale, dt, _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return o, lse


def path_attn_varlen_bwd(q, k, v, w, beta, o, lse, d_o, cu_seqlens, log_f=None, scale=None, workspace=None, stream=None):
    """Backward on packed sequences: (dq, dk, dv, dw, dbeta[, dlog_f])."""
    import torch
    T, H, d = q.shape
    scale = float(d ** -0.5 if scale is None else scale)
    dt = _dt_of(q)
    arr, n = _cu(cu_seqlens)
    outs = [torch.empty_like(q) for _ in range(4)] + [torch.empty_like(beta)]
    dlog_f = torch.empty_like(log_f) if log_f is not None else None
    workspace = _workspace(path_attn_varlen_workspace_bytes(cu_seqlens, H, d, dt, True), q, workspace)
    _check(load_library().path_attn_varlen_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(w), _ptr(beta), _opt(log_f), _ptr(o), _ptr(lse), _ptr(d_o),
                                               *[_ptr(x) for x in outs], _opt(dlog_f), arr, n, H, d, 1, scale, dt,
                                               _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    return tuple(outs) + ((dlog_f,) if dlog_f is not None else ())
