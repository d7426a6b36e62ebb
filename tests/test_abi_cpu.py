"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments with the documented codes before
anything is launched (no GPU needed: validation precedes every HIP call)."""
import ctypes
import os
import re

import pytest

import paper_2505_16381_amd as pa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "path_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(path_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = pa.load_library()
    names = _declared_functions()
    assert {"path_attn_fwd", "path_attn_bwd", "path_attn_workspace_bytes", "path_status_str", "path_attn_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    assert pa.path_status_str(0) == "PATH_OK"
    assert pa.path_status_str(4) == "PATH_ERR_UNSUPPORTED"
    assert pa.path_status_str(99) == "PATH_ERR_UNKNOWN"


def test_workspace_bytes():
    assert pa.path_attn_workspace_bytes(1, 2, 256, 64, pa.PATH_F32) > 0
    assert pa.path_attn_workspace_bytes(1, 2, 256, 96, pa.PATH_F32) == 0      # d not in {64,128}
    assert pa.path_attn_workspace_bytes(0, 2, 256, 64, pa.PATH_F32) == 0
    assert pa.path_attn_workspace_bytes(1, 2, 256, 64, 7) == 0
    a = pa.path_attn_workspace_bytes(1, 1, 64, 64, pa.PATH_BF16)
    b = pa.path_attn_workspace_bytes(1, 1, 65, 64, pa.PATH_BF16)               # ragged tail = one more chunk
    assert a < b <= 2 * a                                                       # per-chunk regions double, per-super-block ones do not
    off = pa.path_attn_fwd_workspace_layout(4, 16, 8192, 128, pa.PATH_BF16)
    assert list(off) == sorted(off) and all(o % 256 == 0 for o in off)
    assert off[5] <= pa.path_attn_workspace_bytes(4, 16, 8192, 128, pa.PATH_BF16)


def _fwd(lib, ptrs, B=1, H=1, L=64, d=64, causal=1, dt=0, ws=0x1000, ws_bytes=1 << 30):
    q, k, v, w, beta, o, lse = ptrs
    return lib.path_attn_fwd(q, k, v, w, beta, o, lse, B, H, L, d, causal, 0.125, dt, ws, ws_bytes, None)


def test_forward_argument_validation_without_gpu():
    lib = pa.load_library()
    ok = [0x1000] * 7                      # never dereferenced: every case below fails validation first
    assert _fwd(lib, [None] + ok[1:]) == 1                       # PATH_ERR_NULL
    assert _fwd(lib, ok[:6] + [None]) == 1
    assert _fwd(lib, ok, ws=None) == 1
    assert _fwd(lib, ok, dt=5) == 3                              # PATH_ERR_DTYPE
    assert _fwd(lib, ok, d=96) == 2                              # PATH_ERR_SHAPE
    assert _fwd(lib, ok, L=0) == 2
    assert _fwd(lib, ok, B=70000) == 2
    assert _fwd(lib, ok, causal=0) == 4                          # PATH_ERR_UNSUPPORTED
    assert lib.path_attn_fwd(*ok, 1, 1, 64, 64, 1, 0.0, 0, 0x1000, 1 << 30, None) == 4   # scale must be > 0
    assert _fwd(lib, ok, ws_bytes=16) == 5                       # PATH_ERR_WORKSPACE
    assert _fwd(lib, ok, ws=0x1010) == 5                         # workspace not 256-aligned
    assert _fwd(lib, [0x1004] + ok[1:]) == 7                     # PATH_ERR_ALIGN
    assert _fwd(lib, ok[:5] + [0x1008] + ok[6:]) == 7


def test_backward_argument_validation_without_gpu():
    lib = pa.load_library()
    args = [0x1000] * 13
    call = lambda a, **kw: lib.path_attn_bwd(*a, kw.get("B", 1), 1, kw.get("L", 64), kw.get("d", 64),
                                             kw.get("causal", 1), 0.125, kw.get("dt", 1),
                                             kw.get("ws", 0x1000), kw.get("wsb", 1 << 40), None)
    assert call([None] + args[1:]) == 1
    assert call(args, d=32) == 2
    assert call(args, dt=9) == 3
    assert call(args, causal=0) == 4
    assert call(args, wsb=8) == 5


def test_static_decode_step_rejects_problems_beyond_its_array_without_a_gpu():
    """The allocation-free decode step checks its arguments, and the size of its built-in scratch array, before
    any HIP call: beyond B*H = 252 (d = 128) or 496 (d = 64) it returns PATH_ERR_WORKSPACE with the reason."""
    lib = pa.load_library()
    assert pa.path_decode_static_scratch_bytes() == 8 * 1024 * 1024
    z = ctypes.c_void_p(0x1000)
    call = lambda BH, d: lib.path_decode_step_static(z, z, z, z, z, z, z, 5, 16, z, z, 1, BH, d, ctypes.c_float(0.1), pa.PATH_BF16, None)
    assert call(253, 128) == 5 and "static scratch" in pa.path_attn_last_error()
    assert call(497, 64) == 5
    assert pa.path_decode_workspace_bytes(1, 252, 128) <= 8 * 1024 * 1024 < pa.path_decode_workspace_bytes(1, 253, 128)
    assert pa.path_decode_workspace_bytes(1, 496, 64) <= 8 * 1024 * 1024 < pa.path_decode_workspace_bytes(1, 497, 64)
    assert lib.path_decode_step_static(None, z, z, z, z, z, z, 5, 16, z, z, 1, 2, 64, ctypes.c_float(0.1), pa.PATH_BF16, None) == 1
    assert lib.path_decode_step_static(z, z, z, z, z, z, z, 16, 16, z, z, 1, 2, 64, ctypes.c_float(0.1), pa.PATH_BF16, None) == 2


def test_ring_argument_validation_without_gpu():
    """The sequence-parallel entry points reject bad arguments before any HIP call."""
    lib = pa.load_library()
    z = 0x1000
    f = ctypes.c_float(0.125)
    assert pa.path_attn_ring_state_bytes(2, 3, 130, 128) == 2 * 3 * 3 * 2 * (2 * 4 * 1024 + 192) * 4
    assert pa.path_attn_ring_state_bytes(1, 1, 64, 96) == 0
    local = lambda q=z, st=z, L=64, d=64, scale=f, dt=0, ws=z, wsb=1 << 40: lib.path_attn_ring_local(q, z, z, z, z, None, st, 1, 1, L, d, scale, dt, ws, wsb, None)
    assert local(q=None) == 1 and local(st=None) == 1 and local(ws=None) == 1
    assert local(L=0) == 2 and local(d=80) == 2
    assert local(dt=7) == 3
    assert local(scale=ctypes.c_float(0.0)) == 4
    assert local(wsb=64) == 5
    assert local(st=0x1004) == 7
    hop = lambda st=z, Lq=64, ws=z, wsb=1 << 40, Lk=64, d=64, dt=0: lib.path_attn_ring_hop(st, 1, 1, Lq, ws, wsb, Lk, d, 0, f, dt, None)
    assert hop(st=None) == 1 and hop(ws=None) == 1
    assert hop(Lk=100) == 2 and "multiple of 64" in pa.path_attn_last_error()
    assert hop(Lq=0) == 2
    assert hop(wsb=128) == 5
    assert hop(dt=9) == 3
    fin = lambda st=z, o=z, lse=z, L=64, d=64, dt=1, gw=None, gwb=0: lib.path_attn_ring_finish(st, o, lse, 1, 1, L, d, dt, gw, gwb, None)
    assert fin(o=None) == 1 and fin(lse=None) == 1 and fin(st=None) == 1
    assert fin(d=100) == 2 and fin(dt=4) == 3 and fin(o=0x1002) == 7
    assert fin(gw=z, gwb=64) == 5
