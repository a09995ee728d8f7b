"""The allocation-free routing entry point (`lsrm_route_blocks_static`, for callers that cannot call
hipMalloc) against `lsrm_route_blocks`: same table and squared distances bit for bit, through the raw C
symbols, on two calls in a row that share the library's fixed scratch, the second on a smaller problem."""
import ctypes

import numpy as np
import pytest

from paper_2604_05182_amd import inputs as I

pytestmark = pytest.mark.gpu


def _route_both(B, torch, cfg):
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    p = B.make_params(cfg.n_obj, cfg.n_views, cfg.grid, cfg.heads, cfg.d, cfg.topk, cfg.window)
    d_pos, d_cams = torch.from_numpy(pos).cuda(), torch.from_numpy(cams).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for static in (False, True):
        idx = torch.full((cfg.nb, cfg.topk), -7, dtype=torch.int32, device="cuda")
        d2 = torch.full((cfg.nb, cfg.topk), -1.0, dtype=torch.float32, device="cuda")
        if static:
            rc = B._lib.lsrm_route_blocks_static(ctypes.byref(p), d_pos.data_ptr(), d_cams.data_ptr(), idx.data_ptr(),
                                                 d2.data_ptr(), stream)
        else:
            ws = B.alloc_workspace(p, B.LSRM_WS_ROUTE)
            rc = B._lib.lsrm_route_blocks(ctypes.byref(p), d_pos.data_ptr(), d_cams.data_ptr(), idx.data_ptr(),
                                          d2.data_ptr(), ws.data_ptr(), ws.numel(), stream)
        assert rc == B.LSRM_OK, B.strerror(rc)
        torch.cuda.synchronize()
        out.append((idx.cpu().numpy(), d2.cpu().numpy()))
    return out


def test_static_scratch_routing_matches_the_workspace_entry_point():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_05182_amd import binding as B
    big = I.CONFIGS[3]          # 2048 object blocks x 12 views of projections in the scratch
    small = I.small_config(name="na-small", n_obj=1088, n_views=3, grid=24, topk=7, seed=4, points="ellipsoids")
    for cfg in (big, small):    # the second call finds the first one's projections in the scratch
        print(f"[no-alloc] {cfg.name}: {cfg.nb_obj} object blocks x {cfg.n_views} views", flush=True)
        (idx_ws, d2_ws), (idx_st, d2_st) = _route_both(B, torch, cfg)
        assert (idx_ws != -7).all()
        assert np.array_equal(idx_st, idx_ws)
        assert np.array_equal(d2_st.view(np.uint32), d2_ws.view(np.uint32))
    # a problem whose projections exceed the fixed array is refused, and nothing is launched
    huge = B.make_params(64 * 131072, 2, 8, 1, 64, 4, 64)
    t = torch.zeros(16, device="cuda")
    rc = B._lib.lsrm_route_blocks_static(ctypes.byref(huge), t.data_ptr(), t.data_ptr(), t.data_ptr(), None, None)
    assert rc == B.LSRM_ERR_TOO_LARGE
    assert "fixed scratch" in B.strerror(rc)
