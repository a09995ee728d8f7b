"""The layer step recorded into a HIP graph and replayed.

The library launches kernels only (no allocation, no memset or copy nodes, no host synchronisation), so a
caller may capture routing (the allocation-free entry point), the pooling / packing pass, the forward and the
backward into a graph.  Every replay is compared bit for bit with the eager results, with eager work and
synchronisations between the replays.
"""
import numpy as np
import pytest

from paper_2604_05182_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,heads,h_kv,topk", [(128, 2, 2, 6), (64, 3, 3, 5), (32, 4, 2, 20)])
def test_step_replayed_from_a_graph_matches_eager(d, heads, h_kv, topk):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_05182_amd import binding as B
    import gpu_util as G
    cfg = I.small_config(name=f"graph-d{d}", n_obj=1088, n_views=3, grid=24, heads=heads, d=d, topk=topk, window=192,
                         seed=33, h_kv=h_kv, points="ellipsoids")
    print(f"[graph] {cfg.name}: {cfg.n} tokens, {heads} heads on {h_kv}, top-k {topk}", flush=True)
    dev = torch.device("cuda:0")
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    d_pos = torch.from_numpy(I.make_points(cfg)).to(dev)
    d_cams = torch.from_numpy(I.make_cameras(cfg)).to(dev)
    d_q, d_k, d_v = (G.bf16_dev(b) for b in (q_bits, k_bits, v_bits))
    d_gates = torch.from_numpy(I.make_gates(cfg)).to(dev)
    d_dout = G.bf16_dev(I.make_dout(cfg))
    p = B.make_params(cfg.n_obj, cfg.n_views, cfg.grid, cfg.heads, cfg.d, cfg.topk, cfg.window, h_kv=cfg.kv_heads)
    p.kv_packed = 1
    ws_fwd = B.alloc_workspace(p, B.LSRM_WS_FORWARD)
    ws_bwd = B.alloc_workspace(p, B.LSRM_WS_BACKWARD)

    def buffers():
        return dict(idx=torch.full((cfg.nb, cfg.topk), -7, dtype=torch.int32, device=dev),
                    kc=torch.zeros((cfg.nb, cfg.kv_heads, cfg.d), dtype=torch.bfloat16, device=dev),
                    vc=torch.zeros((cfg.nb, cfg.kv_heads, cfg.d), dtype=torch.bfloat16, device=dev),
                    out=torch.zeros((cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device=dev),
                    lse=torch.zeros((3, cfg.n, cfg.heads), dtype=torch.float32, device=dev),
                    ob=torch.zeros((3, cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device=dev),
                    dq=torch.zeros_like(d_q), dk=torch.zeros_like(d_k), dv=torch.zeros_like(d_v))

    def step(b):
        B.lsrm_route_blocks_static(p, d_pos, d_cams, b["idx"], None)
        B.lsrm_nsa_compress_pack(p, d_k, d_v, b["kc"], b["vc"], ws_fwd)
        B.lsrm_nsa_forward(p, d_q, d_k, d_v, b["kc"], b["vc"], b["idx"], d_gates, b["out"], b["lse"], b["ob"], ws_fwd)
        B.lsrm_nsa_backward(p, d_q, d_k, d_v, b["kc"], b["vc"], b["idx"], d_gates, b["lse"], b["ob"], d_dout, b["dq"],
                            b["dk"], b["dv"], ws_bwd)

    eager = buffers()
    step(eager)  # (also the first call of the static entry point on this device: its address lookup is not captured)
    torch.cuda.synchronize()
    want = {k: v.cpu().numpy().view(np.uint8).copy() if v.dtype != torch.bfloat16 else G.bf16_host(v).copy()
            for k, v in eager.items()}
    assert (eager["idx"].cpu().numpy() != -7).all()

    held = buffers()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(held)
    for replay in range(3):
        # eager work of the program's own between the replays: clear the outputs, run an eager step elsewhere
        for t in held.values():
            t.fill_(1)
        scratch = buffers()
        step(scratch)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in held.items():
            got = v.cpu().numpy().view(np.uint8) if v.dtype != torch.bfloat16 else G.bf16_host(v)
            assert np.array_equal(got, want[k]), f"replay {replay}: {k} differs from the eager result"
        print(f"[graph] {cfg.name}: replay {replay} identical to eager", flush=True)
