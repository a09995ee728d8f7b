"""Pins for the routing oracle (Sec. 3.3, block-level reading): hand-built cases whose
answers follow from geometry, invariants of an exact top-k, and an independent float64
recomputation through a 3x4 projection matrix."""
import numpy as np
import pytest

from paper_2604_05182_amd import inputs as I

pytestmark = pytest.mark.filterwarnings("ignore")


def _cam(R, t, fx, fy, cx, cy):
    c = np.zeros(16, dtype=np.float32)
    c[:9] = np.asarray(R, dtype=np.float32).reshape(-1)
    c[9:12] = t
    c[12:] = (fx, fy, cx, cy)
    return c


def _golden(name):
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    rows = [l.split("#")[0].split() for l in open(path) if l.split("#")[0].strip()]
    return rows


def test_centroid_exact_dyadic(oracle_lib):
    # positions that are multiples of 1/8: fp32 sums are exact, so the mean is exact
    rng = np.random.default_rng(0)
    pos = (rng.integers(-8, 9, size=(128, 3)) / 8.0).astype(np.float32)
    c = oracle_lib.centroids(pos)
    ref = pos.astype(np.float64).reshape(2, 64, 3).mean(1)
    assert np.array_equal(c.astype(np.float64), ref)


def test_centroid_close_to_float64_mean(oracle_lib):
    cfg = I.small_config(n_obj=1024)
    pos = I.make_points(cfg)
    c = oracle_lib.centroids(pos)
    ref = pos.astype(np.float64).reshape(-1, 64, 3).mean(1)
    assert np.abs(c - ref).max() < 1e-6


def test_on_axis_point_ties_resolve_to_lowest_ids(oracle_lib):
    # identity rotation, camera 3 units behind the origin on -z: the origin projects to
    # (cx, cy) = (8, 8), equidistant (d2 = 32) from the four tile centres of a 16x16 grid.
    pos = np.zeros((64, 3), dtype=np.float32)
    cams = _cam(np.eye(3), (0, 0, 3), 10.0, 10.0, 8.0, 8.0)[None]
    idx, d2 = oracle_lib.route(pos, cams, grid=16, topk=4)
    assert idx[0].tolist() == [1, 2, 3, 4]            # nb_obj = 1, tiles are global ids 1..4
    assert d2[0].tolist() == [32.0, 32.0, 32.0, 32.0]
    # image rows: the only object block, then -1 padding
    assert idx[1:, 0].tolist() == [0, 0, 0, 0]
    assert (idx[1:, 1:] == -1).all() and np.isinf(d2[1:, 1:]).all()


def test_hand_case_from_fixture(oracle_lib):
    # tests/golden/routing_hand_case.txt: values worked out by hand from the pinhole model
    rows = _golden("routing_hand_case.txt")
    expect_idx = [int(x) for x in rows[0]]
    expect_d2 = [float(x) for x in rows[1]]
    pos = np.tile(np.array([[1.0, 1.0, 0.0]], dtype=np.float32), (64, 1))
    cams = _cam(np.eye(3), (0, 0, 2), 8.0, 8.0, 8.0, 8.0)[None]
    idx, d2 = oracle_lib.route(pos, cams, grid=16, topk=4)
    assert idx[0].tolist() == expect_idx
    assert d2[0].tolist() == expect_d2


def test_behind_camera_is_infinitely_far(oracle_lib):
    pos = np.zeros((128, 3), dtype=np.float32)
    pos[64:] = (0, 0, -5.0)          # second block is behind the camera (z = -2)
    cams = _cam(np.eye(3), (0, 0, 3), 10.0, 10.0, 8.0, 8.0)[None]
    idx, d2 = oracle_lib.route(pos, cams, grid=16, topk=2)
    assert np.isinf(d2[1]).all() and idx[1].tolist() == [2, 3]   # ranked by id alone
    # every tile prefers block 0; block 1 comes second at +inf
    assert (idx[2:, 0] == 0).all() and (idx[2:, 1] == 1).all() and np.isinf(d2[2:, 1]).all()


@pytest.mark.parametrize("points", ["uniform", "ellipsoids"])
def test_invariants_and_float64_recomputation(oracle_lib, points):
    cfg = I.small_config(n_obj=2048, n_views=3, grid=32, topk=5, points=points, seed=11)
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    idx, d2 = oracle_lib.route(pos, cams, cfg.grid, cfg.topk)
    nbo, nt = cfg.nb_obj, cfg.n_tiles
    assert idx.shape == (cfg.nb, cfg.topk)
    assert (np.diff(d2, axis=1) >= 0).all()
    assert ((idx[:nbo] >= nbo) & (idx[:nbo] < cfg.nb)).all()
    assert ((idx[nbo:] >= 0) & (idx[nbo:] < nbo)).all()
    for row in idx:
        assert len(set(row.tolist())) == cfg.topk
    # independent float64 formulation: homogeneous 3x4 matrices, argsort
    cent = pos.astype(np.float64).reshape(nbo, 64, 3).mean(1)
    hom = np.concatenate([cent, np.ones((nbo, 1))], axis=1)
    tg = cfg.grid // 8
    centres = np.array([[8 * tj + 4, 8 * ti + 4] for ti in range(tg) for tj in range(tg)], dtype=np.float64)
    D = np.empty((nbo, nt))
    for m in range(cfg.n_views):
        c = cams[m].astype(np.float64)
        Kmat = np.array([[c[12], 0, c[14]], [0, c[13], c[15]], [0, 0, 1]])
        P = Kmat @ np.concatenate([c[:9].reshape(3, 3), c[9:12, None]], axis=1)
        uvw = hom @ P.T
        uv = uvw[:, :2] / uvw[:, 2:3]
        D[:, m * tg * tg:(m + 1) * tg * tg] = ((uv[:, None, :] - centres[None]) ** 2).sum(-1)
    mism = 0
    for b in range(nbo):
        ref = np.argsort(D[b], kind="stable")[:cfg.topk] + nbo
        if not np.array_equal(ref, idx[b]):
            # only allowed when fp32 rounding reorders a near-tie
            srt = np.sort(D[b])
            assert np.min(np.diff(srt[:cfg.topk + 1])) < 1e-3 * max(1.0, srt[cfg.topk]), b
            mism += 1
        assert np.allclose(d2[b], np.sort(D[b])[:cfg.topk], rtol=1e-4, atol=1e-4)
    for t in range(nt):
        ref = np.argsort(D[:, t], kind="stable")[:cfg.topk]
        if not np.array_equal(ref, idx[nbo + t]):
            srt = np.sort(D[:, t])
            assert np.min(np.diff(srt[:cfg.topk + 1])) < 1e-3 * max(1.0, srt[cfg.topk]), t
            mism += 1
        assert np.allclose(d2[nbo + t], np.sort(D[:, t])[:cfg.topk], rtol=1e-4, atol=1e-4)
    assert mism <= 2


def test_full_k_is_a_permutation_and_transpose_consistent(oracle_lib):
    cfg = I.small_config(n_obj=512, n_views=2, grid=16, seed=3)   # 8 object blocks, 8 tiles
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    idx, d2 = oracle_lib.route(pos, cams, cfg.grid, 8)
    nbo = cfg.nb_obj
    for b in range(nbo):
        assert sorted(idx[b].tolist()) == list(range(nbo, nbo + 8))
    for t in range(8):
        assert sorted(idx[nbo + t].tolist()) == list(range(nbo))
    # the same distance is seen from both sides of the pair (object block b, tile t)
    for b in range(nbo):
        for k in range(8):
            t = idx[b, k] - nbo
            kk = idx[nbo + t].tolist().index(b)
            assert d2[b, k] == d2[nbo + t, kk]


def test_k_larger_than_candidates_pads(oracle_lib):
    cfg = I.small_config(n_obj=128, n_views=1, grid=8, seed=5)    # 2 object blocks, 1 tile
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    idx, d2 = oracle_lib.route(pos, cams, cfg.grid, 3)
    assert idx[0].tolist() == [2, -1, -1] and idx[1].tolist() == [2, -1, -1]
    assert sorted(idx[2, :2].tolist()) == [0, 1] and idx[2, 2] == -1
