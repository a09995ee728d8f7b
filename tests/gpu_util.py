"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run the
HIP library through its binding, fetch results as numpy."""
import numpy as np
import torch

from paper_2604_05182_amd import inputs as I


def bf16_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bf16_host(t: torch.Tensor) -> np.ndarray:
    """bf16 device tensor -> float32 numpy."""
    return t.float().cpu().numpy()


def params_for(B, cfg, seg_offsets="default", scale=0.0, topk=None, window=None, window_mode=0, block_count=None,
               group_offsets=None):
    seg = None if isinstance(seg_offsets, str) else seg_offsets
    cnt = None if block_count is None else torch.from_numpy(np.ascontiguousarray(block_count, dtype=np.int32)).cuda()
    grp = None if group_offsets is None else torch.from_numpy(np.ascontiguousarray(group_offsets, dtype=np.int32)).cuda()
    return B.make_params(cfg.n_obj, cfg.n_views, cfg.grid, cfg.heads, cfg.d,
                         cfg.topk if topk is None else topk, cfg.window if window is None else window,
                         seg_offsets=seg, scale=scale, h_kv=cfg.kv_heads, gate_channels=cfg.gate_channels,
                         window_mode=window_mode, block_count=cnt, group_offsets=grp)


def run_route(B, cfg, pos, cams, want_dist=True):
    p = params_for(B, cfg)
    d_pos = torch.from_numpy(pos).cuda()
    d_cams = torch.from_numpy(cams).cuda()
    idx = torch.full((cfg.nb, cfg.topk), -7, dtype=torch.int32, device="cuda")
    d2 = torch.full((cfg.nb, cfg.topk), -1.0, dtype=torch.float32, device="cuda") if want_dist else None
    ws = B.alloc_workspace(p, B.LSRM_WS_ROUTE)
    B.lsrm_route_blocks(p, d_pos, d_cams, idx, d2, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), (d2.cpu().numpy() if want_dist else None)


def run_route_3d(B, cfg, pos, pos_img, cams, width, prefilter, k_v2v, k_v2i, k_i2v, k_i2i, want_dist=True,
                 per_token=False):
    p = params_for(B, cfg, topk=width)
    r = B.lsrm_route3d_params(prefilter, k_v2v, k_v2i, k_i2v, k_i2i, 1 if per_token else 0)
    d_pos, d_img, d_cams = (torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in (pos, pos_img, cams))
    rows = cfg.n if per_token else cfg.nb
    idx = torch.full((rows, width), -7, dtype=torch.int32, device="cuda")
    d2 = torch.full((rows, width), -1.0, dtype=torch.float32, device="cuda") if want_dist else None
    ws = B.alloc_workspace(p, B.LSRM_WS_ROUTE_3D)
    B.lsrm_route_blocks_3d(p, r, d_pos, d_img, d_cams, idx, d2, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), (d2.cpu().numpy() if want_dist else None)


def run_compress(B, cfg, k_bits, v_bits, block_count=None, group_offsets=None):
    p = params_for(B, cfg, block_count=block_count, group_offsets=group_offsets)
    dk, dv = bf16_dev(k_bits), bf16_dev(v_bits)
    n_pairs = cfg.nb if group_offsets is None else len(group_offsets) - 1
    kc = torch.empty((n_pairs, cfg.kv_heads, cfg.d), dtype=torch.bfloat16, device="cuda")
    vc = torch.empty_like(kc)
    B.lsrm_nsa_compress(p, dk, dv, kc, vc)
    torch.cuda.synchronize()
    return dk, dv, kc, vc


def run_forward(B, cfg, q_bits, k_bits, v_bits, idx, gates, seg_offsets="default", scale=0.0,
                want_aux=False, window=None, window_mode=0, block_count=None, fused_pack=False, group_offsets=None):
    """compress + forward on the device.  Returns dict of numpy results (+ device kc, vc).
    fused_pack: lsrm_nsa_compress_pack, then the forward with kv_packed = 1 (one pass over k and v for both)."""
    topk = idx.shape[1]
    p = params_for(B, cfg, seg_offsets=seg_offsets, scale=scale, topk=topk, window=window, window_mode=window_mode,
                   block_count=block_count, group_offsets=group_offsets)
    dq = bf16_dev(q_bits)
    if fused_pack:
        dk, dv = bf16_dev(k_bits), bf16_dev(v_bits)
        n_pairs = cfg.nb if group_offsets is None else len(group_offsets) - 1
        kc = torch.empty((n_pairs, cfg.kv_heads, cfg.d), dtype=torch.bfloat16, device="cuda")
        vc = torch.empty_like(kc)
        ws = B.alloc_workspace(p, B.LSRM_WS_FORWARD)
        ws.fill_(0xFF)   # NaN patterns: an image the fused pass fails to write shows
        B.lsrm_nsa_compress_pack(p, dk, dv, kc, vc, ws)
        p.kv_packed = 1
    else:
        dk, dv, kc, vc = run_compress(B, cfg, k_bits, v_bits, block_count, group_offsets)
    d_idx = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).cuda()
    d_g = torch.from_numpy(gates).cuda()
    out = torch.empty((cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((3, cfg.n, cfg.heads), dtype=torch.float32, device="cuda") if want_aux else None
    ob = torch.empty((3, cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device="cuda") if want_aux else None
    if not fused_pack:
        ws = B.alloc_workspace(p, B.LSRM_WS_FORWARD)
    B.lsrm_nsa_forward(p, dq, dk, dv, kc, vc, d_idx, d_g, out, lse, ob, ws)
    torch.cuda.synchronize()
    res = {"out": bf16_host(out), "kc": bf16_host(kc), "vc": bf16_host(vc)}
    if want_aux:
        res["lse"] = lse.cpu().numpy()
        res["ob"] = bf16_host(ob)
    return res


def run_backward(B, cfg, q_bits, k_bits, v_bits, idx, gates, dout_bits, seg_offsets="default", scale=0.0, window=None,
                 window_mode=0, block_count=None, group_offsets=None):
    """compress + forward (saving lse and branch outputs) + backward on the device -> dq, dk, dv as float32 numpy."""
    topk = idx.shape[1]
    p = params_for(B, cfg, seg_offsets=seg_offsets, scale=scale, topk=topk, window=window, window_mode=window_mode,
                   block_count=block_count, group_offsets=group_offsets)
    dq_in, ddo = bf16_dev(q_bits), bf16_dev(dout_bits)
    dk_in, dv_in, kc, vc = run_compress(B, cfg, k_bits, v_bits, block_count, group_offsets)
    d_idx = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).cuda()
    d_g = torch.from_numpy(gates).cuda()
    out = torch.empty((cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((3, cfg.n, cfg.heads), dtype=torch.float32, device="cuda")
    ob = torch.empty((3, cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device="cuda")
    ws = B.alloc_workspace(p, B.LSRM_WS_FORWARD)
    B.lsrm_nsa_forward(p, dq_in, dk_in, dv_in, kc, vc, d_idx, d_g, out, lse, ob, ws)
    gq = torch.full_like(out, float("nan"))
    gk, gv = torch.full_like(dk_in, float("nan")), torch.full_like(dk_in, float("nan"))
    wsb = B.alloc_workspace(p, B.LSRM_WS_BACKWARD)
    B.lsrm_nsa_backward(p, dq_in, dk_in, dv_in, kc, vc, d_idx, d_g, lse, ob, ddo, gq, gk, gv, wsb)
    torch.cuda.synchronize()
    return bf16_host(gq), bf16_host(gk), bf16_host(gv)


def attention_errors(got: np.ndarray, ref: np.ndarray):
    """(max-abs error, relative L2 error) in float64."""
    g, r = got.astype(np.float64), ref.astype(np.float64)
    diff = g - r
    return float(np.abs(diff).max()), float(np.sqrt((diff ** 2).sum() / max((r ** 2).sum(), 1e-300)))


MAX_ABS_TOL = 2e-2   # attention outputs, bf16 inputs
REL_L2_TOL = 5e-3
