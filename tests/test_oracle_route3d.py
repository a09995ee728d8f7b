"""Pins for the oracle of the four geometric selection rules (Sec. 3.3, block level): a
hand-worked fixture, closed forms on lattices, special cases that reduce to a plain argsort,
and a float64 brute force through homogeneous projection matrices on generated scenes."""
import os

import numpy as np
import pytest

from paper_2604_05182_amd import inputs as I


def _cam(R, t, fx, fy, cx, cy):
    c = np.zeros(16, dtype=np.float32)
    c[:9] = np.asarray(R, dtype=np.float32).reshape(-1)
    c[9:12] = t
    c[12:] = (fx, fy, cx, cy)
    return c


def _hand_scene():
    pos = np.zeros((128, 3), dtype=np.float32)
    pos[64:] = (1, 0, 0)
    pimg = np.zeros((256, 3), dtype=np.float32)
    pimg[:64] = (2, 0, 0)
    pimg[17] = (0, 0, 0.5)
    pimg[64:128] = (0.5, 0.5, 0)
    pimg[128:192] = (0, 0, 0)
    pimg[192:] = (1, 0, 1)
    cams = _cam(np.eye(3), (0, 0, 4), 16.0, 16.0, 8.0, 8.0)[None]
    return pos, pimg, cams


def test_hand_case_from_fixture(oracle_lib):
    path = os.path.join(os.path.dirname(__file__), "golden", "route3d_hand_case.txt")
    rows = [l.split("#")[0].strip() for l in open(path) if l.split("#")[0].strip()]
    exp_idx = np.array([[int(x) for x in r.split("|")[0].split()] for r in rows], dtype=np.int32)
    exp_d2 = np.array([[float(x) for x in r.split("|")[1].split()] for r in rows], dtype=np.float32)
    pos, pimg, cams = _hand_scene()
    idx, d2 = oracle_lib.route_3d(pos, pimg, cams, grid=16, width=4, prefilter=2, k_v2v=2, k_v2i=2, k_i2v=1,
                                  k_i2i=1)
    assert np.array_equal(idx, exp_idx)
    assert np.array_equal(d2, exp_d2)


def test_prefilter_wide_enough_reaches_the_nearest_set(oracle_lib):
    # same scene, prefilter = all four tiles: block 0 now finds tile 2 (distance 0) first
    pos, pimg, cams = _hand_scene()
    idx, d2 = oracle_lib.route_3d(pos, pimg, cams, grid=16, width=4, prefilter=4, k_v2v=1, k_v2i=3, k_i2v=0,
                                  k_i2i=4)
    assert idx[0].tolist() == [0, 4, 2, 3] and d2[0].tolist() == [0.0, 0.0, 0.25, 0.5]
    # image rows hold image blocks only (i2v budget 0); tile 2 sits on p of block 0
    assert idx[4].tolist() == [4, 2, 3, 5] and d2[4].tolist() == [0.0, 0.25, 0.5, 2.0]


def test_volume_rule_on_a_lattice(oracle_lib):
    # block j = 64 copies of (j, 0, 0): the k nearest centres of block i are ranked by (|i-j|, j)
    nbo, k = 16, 5
    pos = np.repeat(np.stack([np.arange(nbo), np.zeros(nbo), np.zeros(nbo)], 1), 64, axis=0).astype(np.float32)
    cams = _cam(np.eye(3), (0, 0, 50), 1.0, 1.0, 4.0, 4.0)[None]
    pimg = np.tile(np.array([[3.5, 0.0, 0.0]], dtype=np.float32), (64, 1))       # one tile, grid 8
    idx, d2 = oracle_lib.route_3d(pos, pimg, cams, grid=8, width=k, prefilter=1, k_v2v=k, k_v2i=0, k_i2v=2,
                                  k_i2i=0)
    for i in range(nbo):
        order = sorted(range(nbo), key=lambda j: (abs(i - j), j))[:k]
        assert idx[i].tolist() == order
        assert d2[i].tolist() == [float((i - j) ** 2) for j in order]
    # the tile's representative (3.5, 0, 0) lies midway between blocks 3 and 4: tie -> lower id
    assert idx[nbo].tolist() == [3, 4, -1, -1, -1] and d2[nbo, :2].tolist() == [0.25, 0.25]


def test_view_behind_the_query_contributes_nothing(oracle_lib):
    # view 0 looks along +z from z = -4 (p in front), view 1 has p behind its image plane
    pos = np.zeros((64, 3), dtype=np.float32)
    cams = np.stack([_cam(np.eye(3), (0, 0, 4), 8.0, 8.0, 4.0, 4.0), _cam(np.eye(3), (0, 0, -4), 8.0, 8.0, 4.0, 4.0)])
    pimg = np.zeros((128, 3), dtype=np.float32)
    pimg[:64] = (0, 0, 3)      # tile of view 0: 3-D distance 9
    pimg[64:] = (0, 0, 0)      # tile of view 1: distance 0, but not visible from p
    idx, d2 = oracle_lib.route_3d(pos, pimg, cams, grid=8, width=3, prefilter=1, k_v2v=1, k_v2i=2, k_i2v=1, k_i2i=2)
    assert idx[0].tolist() == [0, 1, -1] and d2[0].tolist() == [0.0, 9.0, np.inf]
    # the tile of view 1 (its points project fine into view 0, and into view 1 not at all)
    assert idx[2].tolist() == [0, 1, -1] and d2[2].tolist() == [0.0, 9.0, np.inf]
    # the tile of view 0, p = (0,0,3): z = 7 in view 0, z = -1 in view 1
    assert idx[1].tolist() == [0, 1, -1] and d2[1].tolist() == [9.0, 0.0, np.inf]


def _brute_force(pos, pimg, cams, grid, prefilter, k_vol, k_img):
    """float64, homogeneous 3x4 matrices; returns per query block the ranked volume list and the
    ranked image list with distances (full candidate lists, not truncated)."""
    nbo = pos.shape[0] // 64
    tg = grid // 8
    tpv = tg * tg
    m_views = cams.shape[0]
    pts = np.concatenate([pos, pimg]).astype(np.float64).reshape(-1, 64, 3)
    rep = pts.mean(1)
    centres = np.array([[8 * tj + 4, 8 * ti + 4] for ti in range(tg) for tj in range(tg)], dtype=np.float64)
    mats = []
    for m in range(m_views):
        c = cams[m].astype(np.float64)
        kmat = np.array([[c[12], 0, c[14]], [0, c[13], c[15]], [0, 0, 1]])
        mats.append(kmat @ np.concatenate([c[:9].reshape(3, 3), c[9:12, None]], axis=1))
    out = []
    for b in range(rep.shape[0]):
        p = rep[b]
        dv = ((rep[:nbo] - p) ** 2).sum(1)
        cand = []
        for m in range(m_views):
            uvw = mats[m] @ np.append(p, 1.0)
            if uvw[2] <= 1e-6:
                continue
            uv = uvw[:2] / uvw[2]
            d2d = ((centres - uv) ** 2).sum(1)
            near = np.argsort(d2d, kind="stable")[:prefilter]
            gap = np.sort(d2d)[prefilter] - np.sort(d2d)[prefilter - 1] if prefilter < tpv else np.inf
            for t in near:
                tile = m * tpv + int(t)
                dmin = ((pts[nbo + tile] - p) ** 2).sum(1).min()
                cand.append((dmin, nbo + tile, gap))
        out.append((dv, cand))
    return out


@pytest.mark.parametrize("points,seed", [("uniform", 21), ("ellipsoids", 22)])
def test_float64_brute_force_on_generated_scenes(oracle_lib, points, seed):
    cfg = I.small_config(n_obj=1024, n_views=3, grid=32, points=points, seed=seed, near_views=1)
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    pimg = I.make_points_img(cfg, cams)
    pre, kv2v, kv2i, ki2v, ki2i = 4, 3, 5, 2, 6
    width = 8
    idx, d2 = oracle_lib.route_3d(pos, pimg, cams, cfg.grid, width, pre, kv2v, kv2i, ki2v, ki2i)
    nbo = cfg.nb_obj
    ref = _brute_force(pos, pimg, cams, cfg.grid, pre, None, None)
    loose = 0
    for b in range(cfg.nb):
        kv, ki = (kv2v, kv2i) if b < nbo else (ki2v, ki2i)
        dv, cand = ref[b]
        row, drow = idx[b], d2[b]
        # layout: kv volume ids, ki image ids, padding
        assert ((row[:kv] >= 0) & (row[:kv] < nbo)).all()
        assert ((row[kv:kv + ki] >= nbo) & (row[kv:kv + ki] < cfg.nb)).all()
        assert (row[kv + ki:] == -1).all() and np.isinf(drow[kv + ki:]).all()
        assert (np.diff(drow[:kv]) >= 0).all() and (np.diff(drow[kv:kv + ki]) >= 0).all()
        assert len(set(row[:kv + ki].tolist())) == kv + ki
        # volume part against float64
        order = np.argsort(dv, kind="stable")
        assert np.allclose(drow[:kv], dv[order[:kv]], rtol=1e-5, atol=1e-6)
        if not np.array_equal(order[:kv], row[:kv]):
            srt = dv[order]
            assert np.min(np.diff(srt[:kv + 1])) < 1e-5
            loose += 1
        # image part against float64 (candidates whose prefilter cut is a near tie may differ)
        assert len(cand) >= ki
        cand.sort(key=lambda c: (c[0], c[1]))
        want = [c[1] for c in cand[:ki]]
        if want != row[kv:kv + ki].tolist():
            tight = min(c[2] for c in cand) < 1e-3 or np.min(np.diff([c[0] for c in cand[:ki + 1]])) < 1e-5
            assert tight, b
            loose += 1
        else:
            assert np.allclose(drow[kv:kv + ki], [c[0] for c in cand[:ki]], rtol=1e-5, atol=1e-6)
    assert loose <= 3


def test_point_sets_of_one_point_reduce_to_argsort(oracle_lib):
    # every tile's 64 points coincide and the prefilter admits every tile of a view: the image
    # rule is then a plain nearest-neighbour search over one point per tile
    cfg = I.small_config(n_obj=256, n_views=2, grid=16, seed=5)
    rng = np.random.default_rng(9)
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    one = rng.uniform(-0.7, 0.7, size=(cfg.n_tiles, 3)).astype(np.float32)
    pimg = np.repeat(one, 64, axis=0)
    idx, d2 = oracle_lib.route_3d(pos, pimg, cams, cfg.grid, 8, cfg.tiles_per_view, 0, 8, 0, 8)
    rep = np.concatenate([pos.reshape(-1, 64, 3).astype(np.float64).mean(1), one.astype(np.float64)])
    for b in range(cfg.nb):
        dist = ((one.astype(np.float64) - rep[b]) ** 2).sum(1)
        assert idx[b].tolist() == (np.argsort(dist, kind="stable") + cfg.nb_obj).tolist()
        assert np.allclose(d2[b], np.sort(dist), rtol=1e-5, atol=1e-6)


def test_budgets_larger_than_the_candidate_lists_pad(oracle_lib):
    cfg = I.small_config(n_obj=128, n_views=1, grid=16, seed=6)
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    pimg = I.make_points_img(cfg, cams)
    idx, d2 = oracle_lib.route_3d(pos, pimg, cams, cfg.grid, 12, 3, 5, 7, 5, 7)
    for b in range(cfg.nb):
        assert sorted(idx[b, :2].tolist()) == [0, 1]                 # only two volume blocks exist
        assert ((idx[b, 2:5] >= 2) & (idx[b, 2:5] < 6)).all()        # three candidates survive the prefilter
        assert (idx[b, 5:] == -1).all() and np.isinf(d2[b, 5:]).all()


def test_per_token_queries(oracle_lib):
    """The rules as the paper words them, one query per token (Sec. 3.3): the query point is the
    token's own coordinate.  Pins: tokens of a block whose points coincide route like the block;
    a subset of queries equals the rows of the full table; and the hand scene's odd point."""
    pos, pimg, cams = _hand_scene()
    args = dict(grid=16, width=4, prefilter=2, k_v2v=2, k_v2i=2, k_i2v=1, k_i2i=1)
    blk_idx, blk_d2 = oracle_lib.route_3d(pos, pimg, cams, **args)
    tok_idx, tok_d2 = oracle_lib.route_3d(pos, pimg, cams, per_token=True, **args)
    assert tok_idx.shape == (128 + 256, 4)
    # blocks of coincident points (object blocks 0, 1; tiles 1, 2, 3): every token routes like its block
    for b in (0, 1, 3, 4, 5):
        assert (tok_idx[64 * b:64 * b + 64] == blk_idx[b]).all() and (tok_d2[64 * b:64 * b + 64] == blk_d2[b]).all()
    # tile 0: 63 tokens at (2,0,0), token 17 at (0,0,0.5)
    #   p = (2,0,0): nearest centre b1 (1); projects to (16, 8): t1, t3 at 32 -> t1: 2.25+0.25 = 2.5, t3: 1+1 = 2 -> t3
    #   p = (0,0,0.5): b0 0.25 < b1 1.25; projects to (8,8): tie -> t0, t1; t0 contains the token itself: 0
    assert tok_idx[128].tolist() == [1, 5, -1, -1] and tok_d2[128].tolist()[:2] == [1.0, 2.0]
    assert tok_idx[128 + 17].tolist() == [0, 2, -1, -1] and tok_d2[128 + 17].tolist()[:2] == [0.25, 0.0]
    pick = np.array([300, 0, 145, 64], dtype=np.int32)
    sub_idx, sub_d2 = oracle_lib.route_3d(pos, pimg, cams, per_token=True, queries=pick, **args)
    assert np.array_equal(sub_idx, tok_idx[pick]) and np.array_equal(sub_d2, tok_d2[pick])


def test_per_token_float64_brute_force(oracle_lib):
    cfg = I.small_config(n_obj=512, n_views=2, grid=16, points="ellipsoids", seed=31)
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    pimg = I.make_points_img(cfg, cams)
    idx, d2 = oracle_lib.route_3d(pos, pimg, cams, cfg.grid, 6, 2, 2, 4, 2, 4, per_token=True)
    pts = np.concatenate([pos, pimg]).astype(np.float64)
    cent = pts.reshape(-1, 64, 3).mean(1)
    nbo = cfg.nb_obj
    tg = cfg.grid // 8
    centres = np.array([[8 * tj + 4, 8 * ti + 4] for ti in range(tg) for tj in range(tg)], dtype=np.float64)
    loose = exact = 0
    for i in range(0, cfg.n, 7):
        p = pts[i]
        dv = ((cent[:nbo] - p) ** 2).sum(1)
        order = np.argsort(dv, kind="stable")[:2]
        assert np.array_equal(order, idx[i, :2]) or np.min(np.diff(np.sort(dv)[:3])) < 1e-5
        cand, gaps = [], []
        for m in range(cfg.n_views):
            c = cams[m].astype(np.float64)
            x = c[:9].reshape(3, 3) @ p + c[9:12]
            if x[2] <= 1e-6:
                continue
            uv = np.array([c[12] * x[0] / x[2] + c[14], c[13] * x[1] / x[2] + c[15]])
            d2d = ((centres - uv) ** 2).sum(1)
            near = np.argsort(d2d, kind="stable")[:2]
            srt = np.sort(d2d)
            gaps.append(srt[2] - srt[1])     # how clear the prefilter's cut is in this view
            for t in near:
                tile = m * tg * tg + int(t)
                rows = slice(cfg.n_obj + 64 * tile, cfg.n_obj + 64 * tile + 64)
                cand.append((((pts[rows] - p) ** 2).sum(1).min(), nbo + tile))
        cand.sort()
        if [c[1] for c in cand[:4]] != idx[i, 2:6].tolist():
            # only where fp32 rounding decides: a patch centre reprojects onto an axis of symmetry of
            # the 2 x 2 tile grid, or two candidates are equally far
            assert min(gaps) < 1e-3 or np.min(np.diff([c[0] for c in cand[:5]])) < 1e-5, i
            loose += 1
        else:
            assert np.allclose(d2[i, 2:6], [c[0] for c in cand[:4]], rtol=1e-5, atol=1e-6)
            exact += 1
    assert exact >= 60
