"""Thin ctypes binding of liblsrm.so: argument marshalling only.

Same names as the C entry points (include/lsrm.h).  Tensors are torch CUDA tensors
used purely as device memory; every step of the path runs in the HIP library.  There
is no CPU fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblsrm.so")

LSRM_OK = 0
LSRM_ERR_INVALID_ARG = -1
LSRM_ERR_UNSUPPORTED = -2
LSRM_ERR_WORKSPACE = -3
LSRM_ERR_HIP = -4
LSRM_ERR_TOO_LARGE = -5
LSRM_STATIC_ROUTE_SCRATCH_BYTES = 1 << 20
LSRM_WS_ROUTE, LSRM_WS_FORWARD, LSRM_WS_BACKWARD, LSRM_WS_ROUTE_3D = 0, 1, 2, 3


class LsrmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


class lsrm_nsa_params(ctypes.Structure):
    _fields_ = [("n_obj", ctypes.c_int32), ("n_views", ctypes.c_int32), ("grid", ctypes.c_int32),
                ("block", ctypes.c_int32), ("h_q", ctypes.c_int32), ("h_kv", ctypes.c_int32),
                ("d", ctypes.c_int32), ("topk", ctypes.c_int32), ("window", ctypes.c_int32),
                ("n_seg", ctypes.c_int32), ("seg_offsets", ctypes.POINTER(ctypes.c_int32)),
                ("scale", ctypes.c_float), ("gate_channels", ctypes.c_int32), ("window_mode", ctypes.c_int32),
                ("d_block_count", ctypes.c_void_p), ("kv_packed", ctypes.c_int32),
                ("d_group_offsets", ctypes.c_void_p), ("n_groups", ctypes.c_int32)]


class lsrm_route3d_params(ctypes.Structure):
    _fields_ = [("prefilter", ctypes.c_int32), ("k_v2v", ctypes.c_int32), ("k_v2i", ctypes.c_int32),
                ("k_i2v", ctypes.c_int32), ("k_i2i", ctypes.c_int32), ("per_token", ctypes.c_int32)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_05182_amd.build` "
                      "(there is no CPU fallback)")
_lib = ctypes.CDLL(LIB_PATH)
_vp, _sz = ctypes.c_void_p, ctypes.c_size_t
_pp = ctypes.POINTER(lsrm_nsa_params)
_lib.lsrm_strerror.restype = ctypes.c_char_p
_lib.lsrm_strerror.argtypes = [ctypes.c_int32]
_lib.lsrm_workspace_bytes.restype = _sz
_lib.lsrm_workspace_bytes.argtypes = [_pp, ctypes.c_int]
_lib.lsrm_route_blocks.restype = ctypes.c_int32
_lib.lsrm_route_blocks.argtypes = [_pp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.lsrm_route_blocks_static.restype = ctypes.c_int32
_lib.lsrm_route_blocks_static.argtypes = [_pp, _vp, _vp, _vp, _vp, _vp]
_lib.lsrm_route_blocks_3d.restype = ctypes.c_int32
_lib.lsrm_route_blocks_3d.argtypes = [_pp, ctypes.POINTER(lsrm_route3d_params), _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.lsrm_nsa_compress.restype = ctypes.c_int32
_lib.lsrm_nsa_compress.argtypes = [_pp, _vp, _vp, _vp, _vp, _vp]
_lib.lsrm_nsa_compress_pack.restype = ctypes.c_int32
_lib.lsrm_nsa_compress_pack.argtypes = [_pp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.lsrm_nsa_forward.restype = ctypes.c_int32
_lib.lsrm_nsa_forward.argtypes = [_pp] + [_vp] * 11 + [_sz, _vp, _vp, _vp]
_lib.lsrm_nsa_backward.restype = ctypes.c_int32
_lib.lsrm_nsa_backward.argtypes = [_pp] + [_vp] * 14 + [_sz, _vp, _vp, _vp]


def strerror(status: int) -> str:
    return _lib.lsrm_strerror(status).decode()


def make_params(n_obj, n_views, grid, heads, d, topk, window, seg_offsets=None, scale=0.0, h_kv=None,
                block=64, gate_channels=False, window_mode=0, block_count=None, group_offsets=None) -> lsrm_nsa_params:
    """block_count: int32 device tensor [N/64] of active tokens per block, or None; group_offsets: int32 device tensor
    [n_groups + 1] (spatial blocks as runs of 64-slot blocks), or None (both kept alive by the struct)."""
    p = lsrm_nsa_params()
    if group_offsets is not None:
        assert group_offsets.is_cuda and group_offsets.dtype == torch.int32 and group_offsets.is_contiguous()
        p._group_keepalive = group_offsets
        p.d_group_offsets = group_offsets.data_ptr()
        p.n_groups = group_offsets.numel() - 1
    p.gate_channels = 1 if gate_channels else 0
    p.window_mode = window_mode
    if block_count is not None:
        assert block_count.is_cuda and block_count.dtype == torch.int32 and block_count.is_contiguous()
        p._count_keepalive = block_count
        p.d_block_count = block_count.data_ptr()
    p.n_obj, p.n_views, p.grid, p.block = n_obj, n_views, grid, block
    p.h_q, p.h_kv, p.d, p.topk, p.window = heads, heads if not h_kv else h_kv, d, topk, window
    p.scale = scale
    if seg_offsets is None:
        p.n_seg, p.seg_offsets = 0, None
    else:
        arr = (ctypes.c_int32 * len(seg_offsets))(*[int(x) for x in seg_offsets])
        p._keepalive = arr
        p.n_seg = len(seg_offsets) - 1
        p.seg_offsets = ctypes.cast(arr, ctypes.POINTER(ctypes.c_int32))
    return p


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def _check(rc, where):
    if rc != LSRM_OK:
        raise LsrmError(rc, where)


def lsrm_workspace_bytes(p: lsrm_nsa_params, which: int) -> int:
    return int(_lib.lsrm_workspace_bytes(ctypes.byref(p), which))


def lsrm_route_blocks(p, pos, cams, idx, dist2=None, ws=None, stream=None):
    """pos fp32 [n_obj,3], cams fp32 [M,16] -> idx int32 [NB,K] (and dist2 fp32 [NB,K])."""
    nbytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(_lib.lsrm_route_blocks(ctypes.byref(p), _ptr(pos), _ptr(cams), _ptr(idx), _ptr(dist2), _ptr(ws),
                                  nbytes, _stream(stream)), "lsrm_route_blocks")


def lsrm_route_blocks_static(p, pos, cams, idx, dist2=None, stream=None):
    """lsrm_route_blocks without a workspace: the library's fixed per-GPU scratch is used (no allocation)."""
    _check(_lib.lsrm_route_blocks_static(ctypes.byref(p), _ptr(pos), _ptr(cams), _ptr(idx), _ptr(dist2),
                                         _stream(stream)), "lsrm_route_blocks_static")


def lsrm_route_blocks_3d(p, r, pos, pos_img, cams, idx, dist2=None, ws=None, stream=None):
    """pos fp32 [n_obj,3], pos_img fp32 [n_img,3], cams fp32 [M,16] -> idx int32 [NB,topk] (and dist2)."""
    nbytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(_lib.lsrm_route_blocks_3d(ctypes.byref(p), ctypes.byref(r) if r is not None else None, _ptr(pos),
                                     _ptr(pos_img), _ptr(cams), _ptr(idx), _ptr(dist2), _ptr(ws), nbytes,
                                     _stream(stream)), "lsrm_route_blocks_3d")


def lsrm_nsa_compress(p, k, v, kc, vc, stream=None):
    """k, v bf16 [N,H,d] -> kc, vc bf16 [N/64,H,d]."""
    _check(_lib.lsrm_nsa_compress(ctypes.byref(p), _ptr(k), _ptr(v), _ptr(kc), _ptr(vc), _stream(stream)),
           "lsrm_nsa_compress")


def lsrm_nsa_compress_pack(p, k, v, kc, vc, ws, stream=None):
    """lsrm_nsa_compress that also leaves the repacked k, v in the forward workspace `ws`; the forward call that
    follows takes params with kv_packed = 1."""
    nbytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(_lib.lsrm_nsa_compress_pack(ctypes.byref(p), _ptr(k), _ptr(v), _ptr(kc), _ptr(vc), _ptr(ws), nbytes,
                                       _stream(stream)), "lsrm_nsa_compress_pack")


def _event(ev):
    """torch.cuda.Event -> raw hipEvent_t handle (the event must have been created)."""
    if ev is None:
        return None
    if not ev.cuda_event:
        ev.record()  # torch creates the underlying event lazily
    return ev.cuda_event


def lsrm_nsa_forward(p, q, k, v, kc, vc, idx, gates, out, lse=None, out_branch=None, ws=None, stream=None,
                     ev_attn_start=None, ev_attn_stop=None):
    nbytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(_lib.lsrm_nsa_forward(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(kc), _ptr(vc), _ptr(idx),
                                 _ptr(gates), _ptr(out), _ptr(lse), _ptr(out_branch), _ptr(ws), nbytes,
                                 _stream(stream), _event(ev_attn_start), _event(ev_attn_stop)), "lsrm_nsa_forward")


def lsrm_nsa_backward(p, q, k, v, kc, vc, idx, gates, lse, out_branch, dout, dq, dk, dv, ws=None, stream=None,
                      ev_start=None, ev_stop=None):
    nbytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(_lib.lsrm_nsa_backward(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(kc), _ptr(vc), _ptr(idx),
                                  _ptr(gates), _ptr(lse), _ptr(out_branch), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv),
                                  _ptr(ws), nbytes, _stream(stream), _event(ev_start), _event(ev_stop)),
           "lsrm_nsa_backward")


def alloc_workspace(p, which: int, device="cuda") -> torch.Tensor:
    n = lsrm_workspace_bytes(p, which)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)
