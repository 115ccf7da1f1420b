"""Thin ctypes binding over liblocmoe.so (the C ABI declared in include/locmoe.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch appears here for device memory and streams, nothing else.  There is no CPU
fallback: if the shared library is missing, ``lib()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "liblocmoe.so")

LOCMOE_OK = 0
LOCMOE_ERR_NULL, LOCMOE_ERR_SHAPE, LOCMOE_ERR_ARG, LOCMOE_ERR_WORKSPACE, LOCMOE_ERR_HIP = -1, -2, -3, -4, -5
LOCMOE_F32, LOCMOE_BF16 = 0, 1

EXPORTS = ("locmoe_status_string", "locmoe_capacity_min", "locmoe_p_delta", "locmoe_capacity",
           "locmoe_workspace_bytes", "locmoe_gate", "locmoe_gate_sq", "locmoe_angle_stats", "locmoe_route",
           "locmoe_dispatch", "locmoe_dispatch_static",
           "locmoe_expert_ffn", "locmoe_expert_ffn_in", "locmoe_expert_ffn_out", "locmoe_combine",
           "locmoe_packed_weights_bytes", "locmoe_pack_weights", "locmoe_combine_bwd", "locmoe_route_bwd",
           "locmoe_dispatch_bwd", "locmoe_expert_ffn_in_save", "locmoe_transpose_weights",
           "locmoe_expert_ffn_dgrad", "locmoe_expert_ffn_wgrad", "locmoe_pack_weights_t",
           "locmoe_expert_ffn_ws", "locmoe_expert_ffn_in_ws", "locmoe_expert_ffn_out_ws",
           "locmoe_expert_ffn_in_save_ws", "locmoe_expert_ffn_dgrad_ws", "locmoe_gate_dense", "locmoe_route_hash")
LOCMOE_FFN_WS_BYTES = 128
LOCMOE_DISPATCH_STATIC_MAX_COUNTS = 262144


class locmoe_desc(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("E", C.c_int32), ("N", C.c_int32), ("h", C.c_int32),
                ("C", C.c_int32), ("x_dtype", C.c_int32), ("relu", C.c_int32), ("w_packed", C.c_int32),
                ("alpha", C.c_float),
                ("mu", C.c_float)]


class LocMoEError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"liblocmoe: {status_string(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    """Loads the shared library once.  Fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2401_13920_amd.build` "
                           "(or __graft_entry__.build()). There is no fallback path.")
    # PyTorch ships its own HIP runtime; it has to be resident before this library is mapped, so that both
    # resolve to one runtime (device pointers and streams come from torch).  Loaded the other way round, the
    # library binds to the system runtime and every launch on a torch stream fails.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    P, I32, SZ, DBL = C.c_void_p, C.c_int32, C.c_size_t, C.c_double
    D = C.POINTER(locmoe_desc)
    L.locmoe_status_string.restype = C.c_char_p
    L.locmoe_status_string.argtypes = [C.c_int]
    L.locmoe_capacity_min.argtypes = [I32, I32, DBL, I32, C.POINTER(DBL)]
    L.locmoe_p_delta.argtypes = [I32, DBL, C.POINTER(DBL)]
    L.locmoe_capacity.argtypes = [I32, I32, I32, DBL, DBL, C.POINTER(I32)]
    L.locmoe_workspace_bytes.restype = SZ
    L.locmoe_workspace_bytes.argtypes = [D]
    L.locmoe_gate.argtypes = [D, P, P, P]
    L.locmoe_gate_sq.argtypes = [D, P, P, P, P]
    L.locmoe_angle_stats.argtypes = [D, P, P, P, I32, I32] + [P] * 7
    L.locmoe_route.argtypes = [D] + [P] * 10 + [SZ, P]
    L.locmoe_dispatch.argtypes = [D] + [P] * 12 + [SZ, P]
    L.locmoe_dispatch_static.argtypes = [D] + [P] * 12
    L.locmoe_expert_ffn.argtypes = [D] + [P] * 8
    L.locmoe_expert_ffn_in.argtypes = [D] + [P] * 6
    L.locmoe_expert_ffn_out.argtypes = [D] + [P] * 6
    L.locmoe_combine.argtypes = [D] + [P] * 5
    L.locmoe_combine_bwd.argtypes = [D] + [P] * 7
    L.locmoe_route_bwd.argtypes = [D] + [P] * 11
    L.locmoe_dispatch_bwd.argtypes = [D] + [P] * 5
    L.locmoe_expert_ffn_in_save.argtypes = [D] + [P] * 7
    L.locmoe_transpose_weights.argtypes = [D] + [P] * 5
    L.locmoe_pack_weights_t.argtypes = [D] + [P] * 5
    L.locmoe_expert_ffn_dgrad.argtypes = [D] + [P] * 9
    L.locmoe_expert_ffn_wgrad.argtypes = [D] + [P] * 9
    L.locmoe_expert_ffn_ws.argtypes = [D] + [P] * 8 + [SZ, P]
    L.locmoe_expert_ffn_in_ws.argtypes = [D] + [P] * 6 + [SZ, P]
    L.locmoe_expert_ffn_out_ws.argtypes = [D] + [P] * 6 + [SZ, P]
    L.locmoe_expert_ffn_in_save_ws.argtypes = [D] + [P] * 7 + [SZ, P]
    L.locmoe_expert_ffn_dgrad_ws.argtypes = [D] + [P] * 9 + [SZ, P]
    L.locmoe_gate_dense.argtypes = [D, P, P, P, P]
    L.locmoe_route_hash.argtypes = [D, P, C.c_uint32, P, P, P, P]
    L.locmoe_packed_weights_bytes.restype = SZ
    L.locmoe_packed_weights_bytes.argtypes = [D]
    L.locmoe_pack_weights.argtypes = [D] + [P] * 5
    for n in EXPORTS:
        if n not in ("locmoe_status_string", "locmoe_workspace_bytes", "locmoe_packed_weights_bytes"):
            getattr(L, n).restype = C.c_int
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().locmoe_status_string(int(status)).decode()


def _check(st: int) -> None:
    if st != LOCMOE_OK:
        raise LocMoEError(st)


def _ptr(t) -> int | None:
    """Device (or host) address of a torch tensor / numpy array, None stays NULL."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("liblocmoe needs contiguous buffers")
    return t.data_ptr()


def _stream(stream) -> int | None:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_desc(T, d, E, N, h, Cap, dtype="bf16", relu=True, alpha=0.01, mu=0.01, w_packed=False) -> locmoe_desc:
    return locmoe_desc(T, d, E, N, h, Cap, LOCMOE_BF16 if dtype == "bf16" else LOCMOE_F32, 1 if relu else 0,
                       1 if w_packed else 0, alpha, mu)


# ---- host scalars ------------------------------------------------------------------------
def locmoe_p_delta(d: int, delta: float) -> float:
    out = C.c_double()
    _check(lib().locmoe_p_delta(d, delta, C.byref(out)))
    return out.value


def locmoe_capacity_min(E: int, d: int, delta: float, form: int = 1) -> float:
    out = C.c_double()
    _check(lib().locmoe_capacity_min(E, d, delta, form, C.byref(out)))
    return out.value


def locmoe_capacity(T: int, E: int, d: int, cf: float, delta: float) -> int:
    out = C.c_int32()
    _check(lib().locmoe_capacity(T, E, d, cf, delta, C.byref(out)))
    return out.value


def locmoe_workspace_bytes(desc: locmoe_desc) -> int:
    return int(lib().locmoe_workspace_bytes(C.byref(desc)))


# ---- device steps: same names and argument order as the C ABI --------------------------------
def locmoe_gate(desc, x, g, stream=None):
    _check(lib().locmoe_gate(C.byref(desc), _ptr(x), _ptr(g), _stream(stream)))


def locmoe_gate_sq(desc, x, g, q, stream=None):
    _check(lib().locmoe_gate_sq(C.byref(desc), _ptr(x), _ptr(g), _ptr(q), _stream(stream)))


def locmoe_gate_dense(desc, x, Wg, g, stream=None):
    _check(lib().locmoe_gate_dense(C.byref(desc), _ptr(x), _ptr(Wg), _ptr(g), _stream(stream)))


def locmoe_route_hash(desc, key, seed, eid, w, cnt, stream=None):
    _check(lib().locmoe_route_hash(C.byref(desc), _ptr(key), int(seed) & 0xFFFFFFFF, _ptr(eid), _ptr(w), _ptr(cnt),
                                   _stream(stream)))


def locmoe_angle_stats(desc, g, q, eid, shift, nbins, c_self, c_other, hist_self, hist_other, cmin, stats,
                       stream=None):
    _check(lib().locmoe_angle_stats(C.byref(desc), _ptr(g), _ptr(q), _ptr(eid), int(shift), int(nbins), _ptr(c_self),
                                    _ptr(c_other), _ptr(hist_self), _ptr(hist_other), _ptr(cmin), _ptr(stats),
                                    _stream(stream)))


def locmoe_route(desc, g, eps, home, e2n, eid, w, cnt, Psum, stats, ws, ws_bytes, stream=None):
    _check(lib().locmoe_route(C.byref(desc), _ptr(g), _ptr(eps), _ptr(home), _ptr(e2n), _ptr(eid), _ptr(w),
                              _ptr(cnt), _ptr(Psum), _ptr(stats), _ptr(ws), ws_bytes, _stream(stream)))


def locmoe_dispatch(desc, x, eid, e2n, pos, slot, kept, seg_off, node_off, buf_expert, row_token, send, ws,
                    ws_bytes, stream=None):
    _check(lib().locmoe_dispatch(C.byref(desc), _ptr(x), _ptr(eid), _ptr(e2n), _ptr(pos), _ptr(slot), _ptr(kept),
                                 _ptr(seg_off), _ptr(node_off), _ptr(buf_expert), _ptr(row_token), _ptr(send),
                                 _ptr(ws), ws_bytes, _stream(stream)))


def locmoe_dispatch_static(desc, x, eid, e2n, pos, slot, kept, seg_off, node_off, buf_expert, row_token, send,
                           stream=None):
    _check(lib().locmoe_dispatch_static(C.byref(desc), _ptr(x), _ptr(eid), _ptr(e2n), _ptr(pos), _ptr(slot),
                                        _ptr(kept), _ptr(seg_off), _ptr(node_off), _ptr(buf_expert),
                                        _ptr(row_token), _ptr(send), _stream(stream)))


def locmoe_expert_ffn(desc, send, seg_off, buf_expert, W_in, W_out, H_ws, out, stream=None):
    _check(lib().locmoe_expert_ffn(C.byref(desc), _ptr(send), _ptr(seg_off), _ptr(buf_expert), _ptr(W_in),
                                   _ptr(W_out), _ptr(H_ws), _ptr(out), _stream(stream)))


def locmoe_expert_ffn_in(desc, send, seg_off, buf_expert, W_in, H_ws, stream=None):
    _check(lib().locmoe_expert_ffn_in(C.byref(desc), _ptr(send), _ptr(seg_off), _ptr(buf_expert), _ptr(W_in),
                                      _ptr(H_ws), _stream(stream)))


def locmoe_expert_ffn_out(desc, H_ws, seg_off, buf_expert, W_out, out, stream=None):
    _check(lib().locmoe_expert_ffn_out(C.byref(desc), _ptr(H_ws), _ptr(seg_off), _ptr(buf_expert), _ptr(W_out),
                                       _ptr(out), _stream(stream)))


def locmoe_expert_ffn_ws(desc, send, seg_off, buf_expert, W_in, W_out, H_ws, out, ws, ws_bytes, stream=None):
    _check(lib().locmoe_expert_ffn_ws(C.byref(desc), _ptr(send), _ptr(seg_off), _ptr(buf_expert), _ptr(W_in),
                                      _ptr(W_out), _ptr(H_ws), _ptr(out), _ptr(ws), ws_bytes, _stream(stream)))


def locmoe_expert_ffn_in_ws(desc, send, seg_off, buf_expert, W_in, H_ws, ws, ws_bytes, stream=None):
    _check(lib().locmoe_expert_ffn_in_ws(C.byref(desc), _ptr(send), _ptr(seg_off), _ptr(buf_expert), _ptr(W_in),
                                         _ptr(H_ws), _ptr(ws), ws_bytes, _stream(stream)))


def locmoe_expert_ffn_out_ws(desc, H_ws, seg_off, buf_expert, W_out, out, ws, ws_bytes, stream=None):
    _check(lib().locmoe_expert_ffn_out_ws(C.byref(desc), _ptr(H_ws), _ptr(seg_off), _ptr(buf_expert), _ptr(W_out),
                                          _ptr(out), _ptr(ws), ws_bytes, _stream(stream)))


def locmoe_expert_ffn_in_save_ws(desc, send, seg_off, buf_expert, W_in, H_ws, Z, ws, ws_bytes, stream=None):
    _check(lib().locmoe_expert_ffn_in_save_ws(C.byref(desc), _ptr(send), _ptr(seg_off), _ptr(buf_expert),
                                              _ptr(W_in), _ptr(H_ws), _ptr(Z), _ptr(ws), ws_bytes, _stream(stream)))


def locmoe_expert_ffn_dgrad_ws(desc, dout, Z, seg_off, buf_expert, W_out_t, W_in_t, dZ, dsend, ws, ws_bytes,
                               stream=None):
    _check(lib().locmoe_expert_ffn_dgrad_ws(C.byref(desc), _ptr(dout), _ptr(Z), _ptr(seg_off), _ptr(buf_expert),
                                            _ptr(W_out_t), _ptr(W_in_t), _ptr(dZ), _ptr(dsend), _ptr(ws), ws_bytes,
                                            _stream(stream)))


def locmoe_packed_weights_bytes(desc: locmoe_desc) -> int:
    return int(lib().locmoe_packed_weights_bytes(C.byref(desc)))


def locmoe_pack_weights(desc, W_in, W_out, W_in_packed, W_out_packed, stream=None):
    _check(lib().locmoe_pack_weights(C.byref(desc), _ptr(W_in), _ptr(W_out), _ptr(W_in_packed), _ptr(W_out_packed),
                                     _stream(stream)))


def locmoe_combine(desc, out, slot, w, y, stream=None):
    _check(lib().locmoe_combine(C.byref(desc), _ptr(out), _ptr(slot), _ptr(w), _ptr(y), _stream(stream)))


def locmoe_combine_bwd(desc, dy, out, slot, w, dout, dw, stream=None):
    _check(lib().locmoe_combine_bwd(C.byref(desc), _ptr(dy), _ptr(out), _ptr(slot), _ptr(w), _ptr(dout), _ptr(dw),
                                    _stream(stream)))


def locmoe_route_bwd(desc, g, eps, home, e2n, eid, cnt, Psum, dw, coef, dg, stream=None):
    _check(lib().locmoe_route_bwd(C.byref(desc), _ptr(g), _ptr(eps), _ptr(home), _ptr(e2n), _ptr(eid), _ptr(cnt),
                                  _ptr(Psum), _ptr(dw), _ptr(coef), _ptr(dg), _stream(stream)))


def locmoe_dispatch_bwd(desc, dsend, slot, dg, dx, stream=None):
    _check(lib().locmoe_dispatch_bwd(C.byref(desc), _ptr(dsend), _ptr(slot), _ptr(dg), _ptr(dx), _stream(stream)))


def locmoe_expert_ffn_in_save(desc, send, seg_off, buf_expert, W_in, H_ws, Z, stream=None):
    _check(lib().locmoe_expert_ffn_in_save(C.byref(desc), _ptr(send), _ptr(seg_off), _ptr(buf_expert), _ptr(W_in),
                                           _ptr(H_ws), _ptr(Z), _stream(stream)))


def locmoe_transpose_weights(desc, W_in, W_out, W_in_t, W_out_t, stream=None):
    _check(lib().locmoe_transpose_weights(C.byref(desc), _ptr(W_in), _ptr(W_out), _ptr(W_in_t), _ptr(W_out_t),
                                          _stream(stream)))


def locmoe_pack_weights_t(desc, W_in, W_out, W_in_t_packed, W_out_t_packed, stream=None):
    _check(lib().locmoe_pack_weights_t(C.byref(desc), _ptr(W_in), _ptr(W_out), _ptr(W_in_t_packed),
                                       _ptr(W_out_t_packed), _stream(stream)))


def locmoe_expert_ffn_dgrad(desc, dout, Z, seg_off, buf_expert, W_out_t, W_in_t, dZ, dsend, stream=None):
    _check(lib().locmoe_expert_ffn_dgrad(C.byref(desc), _ptr(dout), _ptr(Z), _ptr(seg_off), _ptr(buf_expert),
                                         _ptr(W_out_t), _ptr(W_in_t), _ptr(dZ), _ptr(dsend), _stream(stream)))


def locmoe_expert_ffn_wgrad(desc, send, H, dout, dZ, seg_off, buf_expert, dW_in, dW_out, stream=None):
    _check(lib().locmoe_expert_ffn_wgrad(C.byref(desc), _ptr(send), _ptr(H), _ptr(dout), _ptr(dZ), _ptr(seg_off),
                                         _ptr(buf_expert), _ptr(dW_in), _ptr(dW_out), _stream(stream)))


# ---- buffer bundle: device allocations for one layer call (plumbing only) ---------------------
@dataclass
class Buffers:
    g: object
    eid: object
    w: object
    cnt: object
    Psum: object
    stats: object
    pos: object
    slot: object
    kept: object
    seg_off: object
    node_off: object
    buf_expert: object
    row_token: object
    send: object
    H: object
    out: object
    y: object
    ws: object
    ws_bytes: int
    ffn_ws: object = None      # LOCMOE_FFN_WS_BYTES of zeros: the tile queues of the *_ws expert FFN entry points


def alloc_buffers(desc: locmoe_desc, device="cuda") -> Buffers:
    import torch
    T, d, E, N, h, Cap = desc.T, desc.d, desc.E, desc.N, desc.h, desc.C
    xd = torch.bfloat16 if desc.x_dtype == LOCMOE_BF16 else torch.float32
    rows = E * Cap
    i32 = dict(dtype=torch.int32, device=device)
    f32 = dict(dtype=torch.float32, device=device)
    wsb = locmoe_workspace_bytes(desc)
    return Buffers(
        g=torch.empty(T, E, **f32), eid=torch.empty(T, **i32), w=torch.empty(T, **f32),
        cnt=torch.empty(E, **i32), Psum=torch.empty(E, **f32), stats=torch.empty(8, **f32),
        pos=torch.empty(T, **i32), slot=torch.empty(T, **i32), kept=torch.empty(E, **i32),
        seg_off=torch.empty(E + 1, **i32), node_off=torch.empty(N + 1, **i32), buf_expert=torch.empty(E, **i32),
        row_token=torch.empty(rows, **i32), send=torch.empty(rows, d, dtype=xd, device=device),
        H=torch.empty(rows, h, dtype=torch.bfloat16, device=device), out=torch.empty(rows, d, dtype=xd, device=device),
        y=torch.empty(T, d, dtype=xd, device=device), ws=torch.empty(wsb, dtype=torch.uint8, device=device),
        ws_bytes=wsb, ffn_ws=torch.zeros(LOCMOE_FFN_WS_BYTES, dtype=torch.uint8, device=device))


def forward(desc, x, home, e2n, W_in, W_out, b: Buffers, eps=None, stream=None):
    """Enqueues the five steps of the hot path back to back on one stream."""
    locmoe_gate(desc, x, b.g, stream)
    locmoe_route(desc, b.g, eps, home, e2n, b.eid, b.w, b.cnt, b.Psum, b.stats, b.ws, b.ws_bytes, stream)
    locmoe_dispatch(desc, x, b.eid, e2n, b.pos, b.slot, b.kept, b.seg_off, b.node_off, b.buf_expert, b.row_token,
                    b.send, b.ws, b.ws_bytes, stream)
    locmoe_expert_ffn_ws(desc, b.send, b.seg_off, b.buf_expert, W_in, W_out, b.H, b.out, b.ffn_ws,
                         LOCMOE_FFN_WS_BYTES, stream)
    locmoe_combine(desc, b.out, b.slot, b.w, b.y, stream)
    return b.y


# ---- training: forward that keeps what the backward needs, and the backward chain ------------------
@dataclass
class GradBuffers:
    Z: object
    dout: object
    dw: object
    dZ: object
    dsend: object
    coef: object
    dg: object
    dx: object
    dW_in: object
    dW_out: object


def alloc_grad_buffers(desc: locmoe_desc, device="cuda") -> GradBuffers:
    import torch
    T, d, E, h, Cap = desc.T, desc.d, desc.E, desc.h, desc.C
    xd = torch.bfloat16 if desc.x_dtype == LOCMOE_BF16 else torch.float32
    rows = E * Cap
    bf = dict(dtype=torch.bfloat16, device=device)
    f32 = dict(dtype=torch.float32, device=device)
    return GradBuffers(
        Z=torch.empty(rows, h, **bf), dout=torch.empty(rows, d, dtype=xd, device=device), dw=torch.empty(T, **f32),
        dZ=torch.empty(rows, h, **bf), dsend=torch.empty(rows, d, dtype=xd, device=device),
        coef=torch.empty(E, **f32), dg=torch.empty(T, E, **f32), dx=torch.empty(T, d, dtype=xd, device=device),
        dW_in=torch.empty(E, h, d, **bf), dW_out=torch.empty(E, d, h, **bf))


def forward_train(desc, x, home, e2n, W_in, W_out, b: Buffers, gb: GradBuffers, eps=None, stream=None):
    """The forward path with the pre-activation Z kept for the backward."""
    locmoe_gate(desc, x, b.g, stream)
    locmoe_route(desc, b.g, eps, home, e2n, b.eid, b.w, b.cnt, b.Psum, b.stats, b.ws, b.ws_bytes, stream)
    locmoe_dispatch(desc, x, b.eid, e2n, b.pos, b.slot, b.kept, b.seg_off, b.node_off, b.buf_expert, b.row_token,
                    b.send, b.ws, b.ws_bytes, stream)
    locmoe_expert_ffn_in_save_ws(desc, b.send, b.seg_off, b.buf_expert, W_in, b.H, gb.Z, b.ffn_ws,
                                 LOCMOE_FFN_WS_BYTES, stream)
    locmoe_expert_ffn_out_ws(desc, b.H, b.seg_off, b.buf_expert, W_out, b.out, b.ffn_ws, LOCMOE_FFN_WS_BYTES, stream)
    locmoe_combine(desc, b.out, b.slot, b.w, b.y, stream)
    return b.y


def backward(desc, dy, home, e2n, W_in_t, W_out_t, b: Buffers, gb: GradBuffers, eps=None, stream=None):
    """Enqueues the backward steps on one stream, in reverse order of the forward; W_in_t / W_out_t are the
    transposed weights in the layout desc.w_packed names.  Leaves dx, dW_in, dW_out in gb."""
    locmoe_combine_bwd(desc, dy, b.out, b.slot, b.w, gb.dout, gb.dw, stream)
    locmoe_expert_ffn_dgrad_ws(desc, gb.dout, gb.Z, b.seg_off, b.buf_expert, W_out_t, W_in_t, gb.dZ, gb.dsend,
                               b.ffn_ws, LOCMOE_FFN_WS_BYTES, stream)
    locmoe_expert_ffn_wgrad(desc, b.send, b.H, gb.dout, gb.dZ, b.seg_off, b.buf_expert, gb.dW_in, gb.dW_out, stream)
    locmoe_route_bwd(desc, b.g, eps, home, e2n, b.eid, b.cnt, b.Psum, gb.dw, gb.coef, gb.dg, stream)
    locmoe_dispatch_bwd(desc, gb.dsend, b.slot, gb.dg, gb.dx, stream)
    return gb.dx
