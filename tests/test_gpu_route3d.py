"""GPU parity of the four-rule routing (lsrm_route_blocks_3d) against the CPU oracle: indices
and squared distances bit for bit, on generated scenes, hand-built cases and the full-size
configuration."""
import numpy as np
import pytest

from paper_2604_05182_amd import inputs as I
import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_05182_amd import binding
    return binding


def _log(msg):
    print(msg, flush=True)


def _same(got, ref):
    idx, d2 = got
    ref_idx, ref_d2 = ref
    assert np.array_equal(idx, ref_idx)
    assert np.array_equal(d2.view(np.uint32), ref_d2.view(np.uint32))


# (config, width, prefilter, k_v2v, k_v2i, k_i2v, k_i2i)
CASES = [
    (I.small_config(name="r3-small", n_obj=512, n_views=2, grid=16, seed=3), 8, 2, 3, 4, 2, 3),
    # odd sizes: 17 object blocks, 3 views of 3x3 tiles, a prefilter above 64 is clipped to 9
    (I.small_config(name="r3-ragged", n_obj=1088, n_views=3, grid=24, seed=4, points="ellipsoids", near_views=1),
     40, 100, 9, 27, 17, 20),
    # budgets larger than the candidate lists: padding inside the row
    (I.small_config(name="r3-pad", n_obj=128, n_views=1, grid=16, seed=5), 12, 3, 5, 7, 5, 7),
    # one-sided budgets
    (I.small_config(name="r3-vol-only", n_obj=2048, n_views=2, grid=16, seed=6), 6, 2, 6, 0, 5, 0),
    (I.small_config(name="r3-img-only", n_obj=2048, n_views=5, grid=32, seed=7), 10, 4, 0, 10, 0, 9),
    # more object blocks than fit in LDS beside the candidates: keys are recomputed
    (I.small_config(name="r3-nocache", n_obj=7744 * 64, n_views=2, grid=8, seed=8), 6, 1, 4, 2, 3, 2),
    # the full-size scene with the paper's stage-2 budgets (volume 8, image 2M)
    (I.CONFIGS[3], 32, 4, 8, 24, 8, 24),
    (I.CONFIGS[4], 44, 4, 8, 36, 8, 36),
    # the paper's stage-3 budgets at 16 views: 16 volume + 64 image blocks, rows of 80
    (I.CONFIGS[6], 80, 4, 16, 64, 16, 64),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0].name)
def test_route_3d_bit_exact(B, oracle_lib, case):
    cfg, width, pre, kvv, kvi, kiv, kii = case
    _log(f"[route3d] {cfg.name} n_obj={cfg.n_obj} views={cfg.n_views} grid={cfg.grid} width={width} "
         f"B^i={pre} budgets={kvv},{kvi},{kiv},{kii}")
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    pimg = I.make_points_img(cfg, cams)
    ref = oracle_lib.route_3d(pos, pimg, cams, cfg.grid, width, pre, kvv, kvi, kiv, kii)
    _same(G.run_route_3d(B, cfg, pos, pimg, cams, width, pre, kvv, kvi, kiv, kii), ref)


def test_route_3d_hand_case_and_hidden_view(B, oracle_lib):
    # the fixture scene of the CPU pins (ties, minimum over the point set, prefilter cut) ...
    pos = np.zeros((128, 3), dtype=np.float32)
    pos[64:] = (1, 0, 0)
    pimg = np.zeros((256, 3), dtype=np.float32)
    pimg[:64] = (2, 0, 0)
    pimg[17] = (0, 0, 0.5)
    pimg[64:128] = (0.5, 0.5, 0)
    pimg[192:] = (1, 0, 1)
    cam = np.zeros((1, 16), dtype=np.float32)
    cam[0, :9] = np.eye(3).reshape(-1)
    cam[0, 9:12] = (0, 0, 4)
    cam[0, 12:] = (16, 16, 8, 8)
    cfg = I.small_config(name="r3-hand", n_obj=128, n_views=1, grid=16)
    _log("[route3d] hand case")
    got = G.run_route_3d(B, cfg, pos, pimg, cam, 4, 2, 2, 2, 1, 1)
    assert got[0][0].tolist() == [0, 1, 2, 3] and got[1][0].tolist() == [0.0, 1.0, 0.25, 0.5]
    assert got[0][2].tolist() == [1, 5, -1, -1]
    _same(got, oracle_lib.route_3d(pos, pimg, cam, 16, 4, 2, 2, 2, 1, 1))
    # ... and a second view that has every query point behind its image plane
    cams = np.concatenate([cam, cam])
    cams[1, 11] = -4
    cfg2 = I.small_config(name="r3-hidden", n_obj=128, n_views=2, grid=16)
    pimg2 = np.concatenate([pimg, np.zeros((256, 3), dtype=np.float32)])
    _log("[route3d] hidden view")
    got = G.run_route_3d(B, cfg2, pos, pimg2, cams, 6, 4, 2, 4, 2, 4)
    assert (got[0][:, 2:] < 2 + 4).all()          # no tile of the second view is ever selected
    _same(got, oracle_lib.route_3d(pos, pimg2, cams, 16, 6, 4, 2, 4, 2, 4))


def test_route_3d_without_distances_and_as_forward_table(B, oracle_lib):
    cfg = I.small_config(name="r3-fwd", n_obj=512, n_views=2, grid=16, heads=2, d=64, topk=6, window=128, seed=12)
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    pimg = I.make_points_img(cfg, cams)
    _log("[route3d] table feeds the forward")
    idx, none = G.run_route_3d(B, cfg, pos, pimg, cams, 6, 3, 2, 3, 2, 4, want_dist=False)
    assert none is None
    ref_idx, _ = oracle_lib.route_3d(pos, pimg, cams, cfg.grid, 6, 3, 2, 3, 2, 4)
    assert np.array_equal(idx, ref_idx)
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates = I.make_gates(cfg)
    res = G.run_forward(B, cfg, q_bits, k_bits, v_bits, idx, gates)
    q, k, v = (I.bf16_bits_to_f32(a) for a in (q_bits, k_bits, v_bits))
    ref_out = oracle_lib.nsa_forward(q, k, v, oracle_lib.pool(k), oracle_lib.pool(v), ref_idx, gates,
                                     cfg.seg_offsets(), cfg.window)
    ref_out = ref_out[0] if isinstance(ref_out, tuple) else ref_out
    max_abs, rel = G.attention_errors(res["out"], ref_out)
    assert max_abs <= G.MAX_ABS_TOL and rel <= G.REL_L2_TOL


def test_route_3d_error_codes(B):
    import torch
    cfg = I.small_config(n_obj=128, n_views=1, grid=16)
    p = G.params_for(B, cfg, topk=4)
    t = torch.zeros(4096, dtype=torch.float32, device="cuda")
    i = torch.zeros(4096, dtype=torch.int32, device="cuda")
    with pytest.raises(B.LsrmError) as e:        # budgets exceed the row width
        B.lsrm_route_blocks_3d(p, B.lsrm_route3d_params(2, 3, 2, 1, 1), t, t, t, i, None, t)
    assert e.value.status == B.LSRM_ERR_INVALID_ARG
    with pytest.raises(B.LsrmError) as e:        # no workspace
        B.lsrm_route_blocks_3d(p, B.lsrm_route3d_params(2, 2, 2, 1, 1), t, t, t, i, None, None)
    assert e.value.status == B.LSRM_ERR_WORKSPACE


@pytest.mark.parametrize("cfg,budgets", [
    (I.small_config(name="r3-tok-small", n_obj=512, n_views=2, grid=16, seed=3), (8, 2, 3, 4, 2, 3)),
    (I.small_config(name="r3-tok-mid", n_obj=8192, n_views=4, grid=32, seed=9, points="ellipsoids", near_views=1),
     (24, 4, 8, 16, 8, 16)),
], ids=lambda c: c.name if hasattr(c, "name") else "")
def test_route_3d_per_token_bit_exact(B, oracle_lib, cfg, budgets):
    """One query per token (its own coordinate as the query point), every row against the oracle."""
    width, pre, kvv, kvi, kiv, kii = budgets
    _log(f"[route3d] per token {cfg.name} n={cfg.n}")
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    pimg = I.make_points_img(cfg, cams)
    ref = oracle_lib.route_3d(pos, pimg, cams, cfg.grid, width, pre, kvv, kvi, kiv, kii, per_token=True)
    got = G.run_route_3d(B, cfg, pos, pimg, cams, width, pre, kvv, kvi, kiv, kii, per_token=True)
    assert got[0].shape == (cfg.n, width)
    _same(got, ref)


def test_route_3d_per_token_full_size_sampled(B, oracle_lib):
    """Config 4 at full size (428032 query tokens); the oracle evaluates a sample of them."""
    cfg = I.CONFIGS[4]
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    pimg = I.make_points_img(cfg, cams)
    rng = np.random.default_rng(17)
    pick = np.unique(np.concatenate([[0, cfg.n_obj - 1, cfg.n_obj, cfg.n - 1], rng.integers(0, cfg.n, size=1500)]))
    _log(f"[route3d] per token config 4, oracle on {len(pick)} of {cfg.n} tokens")
    ref = oracle_lib.route_3d(pos, pimg, cams, cfg.grid, 44, 4, 8, 36, 8, 36, per_token=True, queries=pick)
    idx, d2 = G.run_route_3d(B, cfg, pos, pimg, cams, 44, 4, 8, 36, 8, 36, per_token=True)
    _same((idx[pick], d2[pick]), ref)
