"""ctypes front end of the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu-baseline leg import this
package.  It knows nothing about the HIP library: arrays in, arrays out, all numpy.
See lsrm_oracle.c for what each function computes and which passage of the paper
it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lsrm_oracle.c")
# LSRM_ORACLE_SANITIZE=1 selects a build with AddressSanitizer and UndefinedBehaviorSanitizer (the process must
# have been started with the AddressSanitizer runtime preloaded: see tests/test_oracle_sanitizers.py)
_SANITIZE = os.environ.get("LSRM_ORACLE_SANITIZE", "0") == "1"
_LIB = os.path.join(_HERE, "liblsrm_oracle_asan.so" if _SANITIZE else "liblsrm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile lsrm_oracle.c with gcc (no fused multiply-add: routing is compared bit for bit)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        extra = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"] \
            if _SANITIZE else []
        cmd = ["gcc", "-O1" if _SANITIZE else "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", *extra, "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def centroids(pos: np.ndarray) -> np.ndarray:
    pos = _f32(pos)
    n_obj = pos.shape[0]
    out = np.empty((n_obj // 64, 3), dtype=np.float32)
    _load().oracle_centroids(ctypes.c_int(n_obj), _p(pos, ctypes.c_float), _p(out, ctypes.c_float))
    return out


def route(pos: np.ndarray, cams: np.ndarray, grid: int, topk: int):
    """-> (idx int32 [NB, K], dist2 float32 [NB, K])."""
    pos, cams = _f32(pos), _f32(cams)
    n_obj, m = pos.shape[0], cams.shape[0]
    nb = n_obj // 64 + m * (grid // 8) ** 2
    idx = np.empty((nb, topk), dtype=np.int32)
    d2 = np.empty((nb, topk), dtype=np.float32)
    _load().oracle_route(ctypes.c_int(n_obj), ctypes.c_int(m), ctypes.c_int(grid), ctypes.c_int(topk),
                         _p(pos, ctypes.c_float), _p(cams, ctypes.c_float), _p(idx, ctypes.c_int32),
                         _p(d2, ctypes.c_float))
    return idx, d2


def route_3d(pos, pos_img, cams, grid: int, width: int, prefilter: int, k_v2v: int, k_v2i: int, k_i2v: int,
             k_i2i: int, per_token: bool = False, queries=None):
    """The four selection rules -> (idx int32 [rows, width], dist2 float32 [rows, width]); a row holds the
    selected volume blocks, then the selected image blocks, then -1.  Queries are blocks (point = block
    centroid) or, with per_token, tokens (point = the token's own coordinate); `queries` lists the query
    ids to evaluate (default: all, in order)."""
    pos, pos_img, cams = _f32(pos), _f32(pos_img), _f32(cams)
    n_obj, m = pos.shape[0], cams.shape[0]
    assert pos_img.shape[0] == m * grid * grid
    n_all = n_obj + pos_img.shape[0] if per_token else n_obj // 64 + m * (grid // 8) ** 2
    qs = None if queries is None else _i32(np.asarray(queries))
    rows = n_all if qs is None else qs.shape[0]
    idx = np.empty((rows, width), dtype=np.int32)
    d2 = np.empty((rows, width), dtype=np.float32)
    _load().oracle_route_3d(ctypes.c_int(n_obj), ctypes.c_int(m), ctypes.c_int(grid), ctypes.c_int(width),
                            ctypes.c_int(prefilter), ctypes.c_int(k_v2v), ctypes.c_int(k_v2i), ctypes.c_int(k_i2v),
                            ctypes.c_int(k_i2i), ctypes.c_int(1 if per_token else 0), _p(qs, ctypes.c_int32),
                            ctypes.c_int(rows), _p(pos, ctypes.c_float), _p(pos_img, ctypes.c_float),
                            _p(cams, ctypes.c_float), _p(idx, ctypes.c_int32), _p(d2, ctypes.c_float))
    return idx, d2


def _counts(block_count, nb):
    if block_count is None:
        return None
    cnt = _i32(block_count)
    assert cnt.shape == (nb,) and cnt.min() >= 1 and cnt.max() <= 64, "active tokens per block: 1..64"
    return cnt


def _groups(group_offsets, nb):
    """Spatial blocks as runs of 64-slot blocks: ascending offsets [ng + 1], first 0, last nb; None = no groups."""
    if group_offsets is None:
        return 0, None
    off = _i32(group_offsets)
    assert off.ndim == 1 and off.shape[0] >= 2 and off[0] == 0 and off[-1] == nb and np.all(np.diff(off) >= 1)
    return off.shape[0] - 1, off


def pool(x: np.ndarray, block_count=None, group_offsets=None) -> np.ndarray:
    """x fp32 [N, H, d] -> block means fp32 [N/64, H, d] (over the first block_count[b] tokens of
    block b when block_count is given, 1..64 each); with group_offsets one mean per spatial block, [ng, H, d]."""
    x = _f32(x)
    n, h, d = x.shape
    ng, off = _groups(group_offsets, n // 64)
    out = np.empty((ng if ng else n // 64, h, d), dtype=np.float32)
    cnt = _counts(block_count, n // 64)
    _load().oracle_pool(ctypes.c_int64(n), ctypes.c_int(h), ctypes.c_int(d), _p(x, ctypes.c_float),
                        _p(cnt, ctypes.c_int32), ctypes.c_int(ng), _p(off, ctypes.c_int32), _p(out, ctypes.c_float))
    return out


def nsa_forward(q, k, v, kc, vc, idx, gates, seg_offsets, window, scale=0.0, qblocks=None,
                want_lse=False, want_branches=False, window_mode=0, block_count=None, group_offsets=None):
    """NSA forward for the query blocks in `qblocks` (all blocks if None).

    q [N, H, d]; k, v [N, h_kv, d] and kc, vc [NB, h_kv, d] with h_kv dividing H (grouped-query
    heads); gates [N, H, 3] (per head) or [N, 3, H, d] (per channel).
    window_mode 0: sliding window of `window` tokens inside the segment; 1: the query's own block.
    block_count [NB] (optional): active tokens per block (kc, vc pooled with the same counts).
    group_offsets [ng + 1] (optional): spatial blocks as runs of 64-slot blocks; kc, vc are then [ng, h_kv, d] (pooled
    with the same groups), the compressed branch sees one pair per group and the own-block window the whole group.
    Returns out fp32 [nq*64, H, d] (compact over the listed blocks) and, on request,
    lse fp32 [3, nq*64, H] and the three branch outputs fp32 [3, nq*64, H, d].
    """
    q, k, v, kc, vc, gates = map(_f32, (q, k, v, kc, vc, gates))
    idx, seg = _i32(idx), _i32(seg_offsets)
    n, h, d = q.shape
    h_kv = k.shape[1]
    assert h % h_kv == 0 and v.shape == k.shape and kc.shape[1] == h_kv and vc.shape == kc.shape
    assert gates.shape in ((n, h, 3), (n, 3, h, d))
    ng, goff = _groups(group_offsets, n // 64)
    assert kc.shape[0] == (ng if ng else n // 64)
    gate_channels = 1 if gates.ndim == 4 else 0
    topk = idx.shape[1] if idx.ndim == 2 else 0
    if qblocks is None:
        qblocks = np.arange(n // 64, dtype=np.int32)
    qblocks = _i32(qblocks)
    nq = qblocks.shape[0]
    out = np.empty((nq * 64, h, d), dtype=np.float32)
    lse = np.empty((3, nq * 64, h), dtype=np.float32) if want_lse else None
    ob = np.empty((3, nq * 64, h, d), dtype=np.float32) if want_branches else None
    _load().oracle_nsa_forward(
        ctypes.c_int64(n), ctypes.c_int(h), ctypes.c_int(h_kv), ctypes.c_int(d), ctypes.c_int(topk),
        ctypes.c_int(window), ctypes.c_int(window_mode), _p(_counts(block_count, n // 64), ctypes.c_int32),
        ctypes.c_float(scale), ctypes.c_int(seg.shape[0] - 1), _p(seg, ctypes.c_int32),
        _p(q, ctypes.c_float), _p(k, ctypes.c_float), _p(v, ctypes.c_float), _p(kc, ctypes.c_float),
        _p(vc, ctypes.c_float), _p(idx, ctypes.c_int32), _p(gates, ctypes.c_float), ctypes.c_int(gate_channels),
        _p(qblocks, ctypes.c_int32), ctypes.c_int(nq), ctypes.c_int(ng), _p(goff, ctypes.c_int32),
        _p(out, ctypes.c_float), _p(lse, ctypes.c_float), _p(ob, ctypes.c_float))
    res = [out]
    if want_lse:
        res.append(lse)
    if want_branches:
        res.append(ob)
    return res[0] if len(res) == 1 else tuple(res)


def nsa_backward(q, k, v, kc, vc, idx, gates, seg_offsets, window, dout, scale=0.0, window_mode=0, block_count=None,
                 group_offsets=None):
    """-> (dq fp32 [N, H, d], dk, dv fp32 [N, h_kv, d]); single-threaded definition, small inputs only.
    Shapes and gate layouts as in nsa_forward."""
    q, k, v, kc, vc, gates, dout = map(_f32, (q, k, v, kc, vc, gates, dout))
    idx, seg = _i32(idx), _i32(seg_offsets)
    n, h, d = q.shape
    h_kv = k.shape[1]
    assert h % h_kv == 0 and gates.shape in ((n, h, 3), (n, 3, h, d))
    ng, goff = _groups(group_offsets, n // 64)
    assert kc.shape[0] == (ng if ng else n // 64)
    topk = idx.shape[1] if idx.ndim == 2 else 0
    dq = np.empty_like(q)
    dk, dv = np.empty_like(k), np.empty_like(k)
    _load().oracle_nsa_backward(
        ctypes.c_int64(n), ctypes.c_int(h), ctypes.c_int(h_kv), ctypes.c_int(d), ctypes.c_int(topk),
        ctypes.c_int(window), ctypes.c_int(window_mode), _p(_counts(block_count, n // 64), ctypes.c_int32),
        ctypes.c_float(scale), ctypes.c_int(seg.shape[0] - 1),
        _p(seg, ctypes.c_int32), _p(q, ctypes.c_float), _p(k, ctypes.c_float), _p(v, ctypes.c_float),
        _p(kc, ctypes.c_float), _p(vc, ctypes.c_float), _p(idx, ctypes.c_int32), _p(gates, ctypes.c_float),
        ctypes.c_int(1 if gates.ndim == 4 else 0), _p(dout, ctypes.c_float), ctypes.c_int(ng), _p(goff, ctypes.c_int32),
        _p(dq, ctypes.c_float), _p(dk, ctypes.c_float), _p(dv, ctypes.c_float))
    return dq, dk, dv


def nsa_backward_sampled(q, k, v, kc, vc, idx, gates, seg_offsets, window, dout, qblocks, kblocks, heads,
                         kv_heads=None, scale=0.0, window_mode=0):
    """Gradients for a sample: dq [len(qblocks)*64, len(heads), d] of the listed query blocks and query
    heads, and dk, dv [len(kblocks)*64, len(kv_heads), d] of the listed key blocks and key/value heads (all
    queries contribute, through every query head of the key/value head's group).  kv_heads defaults to
    `heads` when every query head has its own key/value head.  Shapes and gate layouts as in nsa_forward."""
    q, k, v, kc, vc, gates, dout = map(_f32, (q, k, v, kc, vc, gates, dout))
    idx, seg = _i32(idx), _i32(seg_offsets)
    n, h, d = q.shape
    h_kv = k.shape[1]
    assert h % h_kv == 0 and gates.shape in ((n, h, 3), (n, 3, h, d))
    if kv_heads is None:
        assert h_kv == h, "grouped heads: say which key/value heads dk, dv are wanted for"
        kv_heads = heads
    qb, kb, hs, kvs = (_i32(np.asarray(a)) for a in (qblocks, kblocks, heads, kv_heads))
    assert hs.size == 0 or (hs.min() >= 0 and hs.max() < h)
    assert kvs.size == 0 or (kvs.min() >= 0 and kvs.max() < h_kv)
    topk = idx.shape[1] if idx.ndim == 2 else 0
    dq = np.empty((qb.shape[0] * 64, hs.shape[0], d), dtype=np.float32)
    dk = np.empty((kb.shape[0] * 64, kvs.shape[0], d), dtype=np.float32)
    dv = np.empty_like(dk)
    _load().oracle_nsa_backward_sampled(
        ctypes.c_int64(n), ctypes.c_int(h), ctypes.c_int(h_kv), ctypes.c_int(d), ctypes.c_int(topk),
        ctypes.c_int(window), ctypes.c_int(window_mode), ctypes.c_float(scale), ctypes.c_int(seg.shape[0] - 1),
        _p(seg, ctypes.c_int32), _p(q, ctypes.c_float), _p(k, ctypes.c_float), _p(v, ctypes.c_float),
        _p(kc, ctypes.c_float), _p(vc, ctypes.c_float), _p(idx, ctypes.c_int32), _p(gates, ctypes.c_float),
        ctypes.c_int(1 if gates.ndim == 4 else 0), _p(dout, ctypes.c_float),
        _p(qb, ctypes.c_int32), ctypes.c_int(qb.shape[0]), _p(kb, ctypes.c_int32), ctypes.c_int(kb.shape[0]),
        _p(hs, ctypes.c_int32), ctypes.c_int(hs.shape[0]), _p(kvs, ctypes.c_int32), ctypes.c_int(kvs.shape[0]),
        _p(dq, ctypes.c_float), _p(dk, ctypes.c_float), _p(dv, ctypes.c_float))
    return dq, dk, dv
