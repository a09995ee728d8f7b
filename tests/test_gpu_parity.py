"""GPU parity: the HIP library (through its C boundary) against the CPU oracle, element
by element, on the same seeded inputs.

Bars: routed indices and squared distances bit-exact; pooled keys/values within one
bf16 rounding of the fp32 mean; attention outputs within max-abs 2e-2 and relative L2
5e-3 of the oracle (bf16 inputs, fp32 oracle arithmetic in double accumulators).
"""
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


# ----------------------------------------------------------------------------- routing
ROUTE_CASES = [
    I.small_config(name="r-small", n_obj=512, n_views=2, grid=16, topk=3, seed=3),
    I.small_config(name="r-ragged", n_obj=1088, n_views=3, grid=24, topk=7, seed=4, points="ellipsoids"),
    I.small_config(name="r-fullk", n_obj=512, n_views=2, grid=16, topk=8, seed=5),
    I.small_config(name="r-pad", n_obj=128, n_views=1, grid=8, topk=3, seed=5),
    # more object blocks than the routing kernel keeps in LDS: exercises its recompute path
    I.small_config(name="r-nocache", n_obj=7744 * 64, n_views=2, grid=8, topk=6, seed=6),
    I.CONFIGS[1], I.CONFIGS[2], I.CONFIGS[3], I.CONFIGS[4],
]


@pytest.mark.parametrize("cfg", ROUTE_CASES, ids=lambda c: c.name)
def test_route_bit_exact(B, oracle_lib, cfg):
    _log(f"[route] {cfg.name} n_obj={cfg.n_obj} views={cfg.n_views} grid={cfg.grid} K={cfg.topk}")
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    ref_idx, ref_d2 = oracle_lib.route(pos, cams, cfg.grid, cfg.topk)
    idx, d2 = G.run_route(B, cfg, pos, cams)
    assert np.array_equal(idx, ref_idx)
    assert np.array_equal(d2.view(np.uint32), ref_d2.view(np.uint32))


def test_route_ties_and_behind_camera(B, oracle_lib):
    cfg = I.small_config(name="r-hand", n_obj=128, n_views=1, grid=16, topk=4)
    pos = np.zeros((128, 3), dtype=np.float32)
    pos[64:] = (0, 0, -5.0)
    cams = np.zeros((1, 16), dtype=np.float32)
    cams[0, :9] = np.eye(3).reshape(-1)
    cams[0, 9:12] = (0, 0, 3)
    cams[0, 12:] = (10, 10, 8, 8)
    ref_idx, ref_d2 = oracle_lib.route(pos, cams, 16, 4)
    idx, d2 = G.run_route(B, cfg, pos, cams)
    assert idx[0].tolist() == [2, 3, 4, 5] and d2[0].tolist() == [32.0] * 4
    assert np.array_equal(idx, ref_idx) and np.array_equal(d2.view(np.uint32), ref_d2.view(np.uint32))


def test_route_without_distances(B, oracle_lib):
    cfg = ROUTE_CASES[0]
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    idx, _ = G.run_route(B, cfg, pos, cams, want_dist=False)
    assert np.array_equal(idx, oracle_lib.route(pos, cams, cfg.grid, cfg.topk)[0])


# ----------------------------------------------------------------------------- pooling
@pytest.mark.parametrize("cfg", [I.small_config(name="p-small", heads=2, d=64),
                                 I.small_config(name="p-d128", heads=3, d=128, n_obj=448, grid=24),
                                 I.CONFIGS[1]], ids=lambda c: c.name)
def test_compress(B, oracle_lib, cfg):
    _log(f"[compress] {cfg.name}")
    _, k_bits, v_bits = I.make_qkv(cfg)
    _, _, kc, vc = G.run_compress(B, cfg, k_bits, v_bits)
    for got, bits in ((kc, k_bits), (vc, v_bits)):
        ref = oracle_lib.pool(I.bf16_bits_to_f32(bits))
        got = G.bf16_host(got)
        # one rounding to bf16 (relative 2^-9) plus fp32 summation noise
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-6)


# ----------------------------------------------------------------------------- forward
def _forward_case(B, oracle_lib, cfg, idx=None, seg="default", scale=0.0, qblocks=None, window=None, window_mode=0,
                  block_count=None):
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates = I.make_gates(cfg)
    if idx is None:
        idx, _ = oracle_lib.route(I.make_points(cfg), I.make_cameras(cfg), cfg.grid, cfg.topk)
    seg_arr = cfg.seg_offsets() if isinstance(seg, str) else np.asarray(seg, dtype=np.int32)
    window = cfg.window if window is None else window
    if block_count is not None:
        # whatever sits in the inactive slots of K and V must never be looked at: make it NaN
        inactive = (np.arange(cfg.n) % 64) >= np.repeat(np.asarray(block_count), 64)
        k_bits, v_bits = k_bits.copy(), v_bits.copy()
        k_bits[inactive] = 0x7FC0
        v_bits[inactive] = 0x7FC0
    res = G.run_forward(B, cfg, q_bits, k_bits, v_bits, idx, gates, seg_offsets=seg, scale=scale,
                        want_aux=True, window=window, window_mode=window_mode, block_count=block_count)
    q, k, v = (I.bf16_bits_to_f32(a) for a in (q_bits, k_bits, v_bits))
    kc, vc = oracle_lib.pool(k, block_count), oracle_lib.pool(v, block_count)
    ref_out, ref_lse, ref_ob = oracle_lib.nsa_forward(q, k, v, kc, vc, idx, gates, seg_arr, window, scale=scale,
                                                      qblocks=qblocks, want_lse=True, want_branches=True,
                                                      window_mode=window_mode, block_count=block_count)
    if qblocks is not None:
        rows = (np.asarray(qblocks)[:, None] * 64 + np.arange(64)[None]).reshape(-1)
        res = {"out": res["out"][rows], "lse": res["lse"][:, rows], "ob": res["ob"][:, rows]}
    if block_count is not None:
        # rows of inactive slots are unspecified: compare the active ones
        blocks = np.arange(cfg.nb) if qblocks is None else np.asarray(qblocks)
        act = (np.arange(64)[None, :] < np.asarray(block_count)[blocks][:, None]).reshape(-1)
        res = {"out": res["out"][act], "lse": res["lse"][:, act], "ob": res["ob"][:, act]}
        ref_out, ref_lse, ref_ob = ref_out[act], ref_lse[:, act], ref_ob[:, act]
    return res, ref_out, ref_lse, ref_ob


def _assert_forward(res, ref_out, ref_lse, ref_ob, tag):
    ma, rl = G.attention_errors(res["out"], ref_out)
    _log(f"[forward] {tag}: out max-abs {ma:.3e} rel-L2 {rl:.3e}")
    assert ma <= G.MAX_ABS_TOL and rl <= G.REL_L2_TOL
    for b, name in enumerate(("cmp", "sel", "win")):
        ma, rl = G.attention_errors(res["ob"][b], ref_ob[b])
        _log(f"           branch {name}: max-abs {ma:.3e} rel-L2 {rl:.3e}")
        assert ma <= G.MAX_ABS_TOL and rl <= G.REL_L2_TOL
    fin = np.isfinite(ref_lse)
    assert np.array_equal(np.isfinite(res["lse"]), fin)
    assert np.array_equal(np.isneginf(res["lse"]), np.isneginf(ref_lse))
    assert np.abs(res["lse"][fin] - ref_lse[fin]).max() <= 2e-2


@pytest.mark.parametrize("d", [32, 64, 128])
def test_forward_small(B, oracle_lib, d):
    cfg = I.small_config(name=f"f-small-d{d}", n_obj=512, n_views=2, grid=16, heads=2, d=d, topk=3, window=128)
    _log(f"[forward] {cfg.name}")
    _assert_forward(*_forward_case(B, oracle_lib, cfg), cfg.name)


@pytest.mark.parametrize("d", [32, 64, 128])
def test_forward_ragged_and_holes(B, oracle_lib, d):
    """NB not a multiple of 4 or 32, odd head count, -1 holes, an empty routed row, a window
    that is not a multiple of the block, explicit scale."""
    cfg = I.small_config(name=f"f-ragged-d{d}", n_obj=1088, n_views=3, grid=24, heads=3, d=d, topk=5,
                         window=200, seed=21)
    _log(f"[forward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(5)
    idx = np.stack([rng.choice(cfg.nb, size=cfg.topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[rng.random(idx.shape) < 0.2] = -1
    idx[2] = -1
    _assert_forward(*_forward_case(B, oracle_lib, cfg, idx=idx, scale=0.2), cfg.name)


@pytest.mark.parametrize("d,heads,h_kv,gate_channels", [(64, 8, 2, False), (64, 3, 1, True), (128, 4, 2, True),
                                                        (128, 2, 2, True), (32, 4, 4, False),
                                                        # the paper's heads: 32 query heads of 32 channels on 2
                                                        (32, 32, 2, True)])
def test_forward_grouped_heads_and_channel_gates(B, oracle_lib, d, heads, h_kv, gate_channels):
    """Query heads sharing key/value heads (App. A) and one gate per output channel."""
    cfg = I.small_config(name=f"gqa-d{d}-h{heads}-kv{h_kv}-ch{int(gate_channels)}", n_obj=640, n_views=2, grid=16,
                         heads=heads, d=d, topk=3, window=160, seed=31, h_kv=h_kv, gate_channels=gate_channels)
    _log(f"[forward] {cfg.name}")
    res, ref_out, ref_lse, ref_ob = _forward_case(B, oracle_lib, cfg)
    _assert_forward(res, ref_out, ref_lse, ref_ob, cfg.name)


def _block_counts(cfg, seed):
    rng = np.random.default_rng(seed)
    cnt = rng.integers(1, 65, size=cfg.nb).astype(np.int32)
    cnt[:6] = (64, 1, 33, 32, 31, 64)
    return cnt


@pytest.mark.parametrize("d,window_mode,with_counts", [(64, 1, False), (128, 1, False), (64, 0, True), (128, 0, True),
                                                       (64, 1, True), (128, 1, True), (32, 1, True)])
def test_forward_own_block_window_and_active_counts(B, oracle_lib, d, window_mode, with_counts):
    """Window branch over the query's own block (App. A) and blocks with fewer than 64 active
    tokens (Sec. 3.2), alone and together; ragged block count, holes in the routing table."""
    cfg = I.small_config(name=f"f-own{window_mode}-cnt{int(with_counts)}-d{d}", n_obj=1088, n_views=3, grid=24, heads=3,
                         d=d, topk=5, window=200, seed=41)
    _log(f"[forward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(6)
    idx = np.stack([rng.choice(cfg.nb, size=cfg.topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[rng.random(idx.shape) < 0.2] = -1
    idx[:, 0] = np.minimum(np.arange(cfg.nb), 5)      # the special counts (1, 31, 32, 33) are routed to
    cnt = _block_counts(cfg, 7) if with_counts else None
    res, ref_out, ref_lse, ref_ob = _forward_case(B, oracle_lib, cfg, idx=idx, window_mode=window_mode, block_count=cnt)
    _assert_forward(res, ref_out, ref_lse, ref_ob, cfg.name)


def test_compress_with_active_counts(B, oracle_lib):
    cfg = I.small_config(name="p-counts", n_obj=1088, n_views=3, grid=24, heads=3, d=64, seed=42)
    cnt = _block_counts(cfg, 8)
    _, k_bits, v_bits = I.make_qkv(cfg)
    # poison the inactive slots: they must not reach the averages
    act = (np.arange(cfg.n) % 64) < np.repeat(cnt, 64)
    k_bits = k_bits.copy()
    k_bits[~act] = 0x7FC0          # bf16 NaN
    _, _, kc, vc = G.run_compress(B, cfg, k_bits, v_bits, cnt)
    for got, bits in ((kc, k_bits), (vc, v_bits)):
        ref = oracle_lib.pool(I.bf16_bits_to_f32(bits), cnt)
        got = G.bf16_host(got)
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-6)


@pytest.mark.parametrize("d,heads,h_kv,with_counts", [(64, 2, 2, False), (128, 3, 3, False), (32, 8, 2, False),
                                                      (128, 2, 2, True), (64, 4, 1, True)])
def test_compress_pack_then_forward(B, oracle_lib, d, heads, h_kv, with_counts):
    """lsrm_nsa_compress_pack (pooling and repacking in one pass over k and v) followed by the forward with
    kv_packed = 1: the pooled pairs against the oracle's means, the attention outputs against the oracle, and
    bit for bit against the two-pass route when both are given the same pooled pairs."""
    cfg = I.small_config(name=f"f-fused-d{d}-h{heads}-kv{h_kv}-cnt{int(with_counts)}", n_obj=1088, n_views=3, grid=24,
                         heads=heads, d=d, topk=5, window=200, seed=43, h_kv=h_kv)
    _log(f"[compress_pack + forward] {cfg.name} nb={cfg.nb}")
    cnt = _block_counts(cfg, 9) if with_counts else None
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates = I.make_gates(cfg)
    idx, _ = oracle_lib.route(I.make_points(cfg), I.make_cameras(cfg), cfg.grid, cfg.topk)
    if cnt is not None:
        inactive = (np.arange(cfg.n) % 64) >= np.repeat(cnt, 64)
        k_bits, v_bits = k_bits.copy(), v_bits.copy()
        k_bits[inactive] = 0x7FC0
        v_bits[inactive] = 0x7FC0
    res = G.run_forward(B, cfg, q_bits, k_bits, v_bits, idx, gates, want_aux=True, block_count=cnt, fused_pack=True)
    q, k, v = (I.bf16_bits_to_f32(a) for a in (q_bits, k_bits, v_bits))
    kc, vc = oracle_lib.pool(k, cnt), oracle_lib.pool(v, cnt)
    for got, ref in ((res["kc"], kc), (res["vc"], vc)):
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-6)
    ref_out, ref_lse, ref_ob = oracle_lib.nsa_forward(q, k, v, kc, vc, idx, gates, cfg.seg_offsets(), cfg.window,
                                                      want_lse=True, want_branches=True, block_count=cnt)
    sel = slice(None) if cnt is None else (np.arange(cfg.n) % 64) < np.repeat(cnt, 64)
    got = {"out": res["out"][sel], "lse": res["lse"][:, sel], "ob": res["ob"][:, sel]}
    _assert_forward(got, ref_out[sel], ref_lse[:, sel], ref_ob[:, sel], cfg.name)
    # the images of the fused pass are those of the forward's own packing: same pooled pairs in, same bits out
    import torch
    p = G.params_for(B, cfg, block_count=cnt)
    dq, dk, dv = (G.bf16_dev(a) for a in (q_bits, k_bits, v_bits))
    kc_d, vc_d = (torch.from_numpy(I.f32_to_bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
                  for a in (res["kc"], res["vc"]))
    out2 = torch.empty((cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device="cuda")
    B.lsrm_nsa_forward(p, dq, dk, dv, kc_d, vc_d, torch.from_numpy(idx).cuda(), torch.from_numpy(gates).cuda(), out2,
                       None, None, B.alloc_workspace(p, B.LSRM_WS_FORWARD))
    torch.cuda.synchronize()
    assert np.array_equal(G.bf16_host(out2)[sel], res["out"][sel])


def test_forward_dense_equivalence(B, oracle_lib):
    """Single segment, window covering the sequence, every block routed: the selected and
    window branches both equal plain full attention (compared with the oracle's)."""
    cfg = I.small_config(name="f-dense", n_obj=512, n_views=0, grid=0, heads=2, d=64, topk=8, window=1024)
    idx = np.tile(np.arange(8, dtype=np.int32), (8, 1))
    res, ref_out, ref_lse, ref_ob = _forward_case(B, oracle_lib, cfg, idx=idx, seg=[0, 512])
    _assert_forward(res, ref_out, ref_lse, ref_ob, cfg.name)
    ma, _ = G.attention_errors(res["ob"][1], res["ob"][2])
    assert ma <= 2e-2


def test_forward_zero_window_and_topk_one(B, oracle_lib):
    cfg = I.small_config(name="f-w0", n_obj=256, n_views=1, grid=16, heads=1, d=64, topk=1, window=0)
    _assert_forward(*_forward_case(B, oracle_lib, cfg), cfg.name)


@pytest.mark.parametrize("d", [32, 64, 128])
def test_forward_large_scale_moves_the_running_max(B, oracle_lib, d):
    """Scores many units apart (score standard deviation about 5 nats): the running maximum is raised
    several times per row, including while probabilities of the previous tile are still waiting to be
    accumulated.  (Not larger: with a near one-hot softmax the outputs are single V rows of magnitude 4,
    whose bf16 rounding alone reaches the absolute tolerance.)"""
    cfg = I.small_config(name=f"f-bigscale-d{d}", n_obj=2048, n_views=2, grid=16, heads=2, d=d, topk=6, window=384,
                         seed=33)
    _log(f"[forward] {cfg.name}")
    _assert_forward(*_forward_case(B, oracle_lib, cfg, scale={32: 0.85, 64: 0.6, 128: 0.45}[d]), cfg.name)


def test_forward_config1_full(B, oracle_lib):
    cfg = I.CONFIGS[1]
    _log(f"[forward] config 1 full ({cfg.n} tokens)")
    _assert_forward(*_forward_case(B, oracle_lib, cfg), "config1")


@pytest.mark.parametrize("cid,n_random", [(2, 24), (3, 12)])
def test_forward_full_size_sampled(B, oracle_lib, cid, n_random):
    """Full-size launch, oracle on a sample of query blocks: first and last block of every segment plus
    random ones, all heads.  (Configs 4 and 6 have their own, larger samples in test_gpu_full_size.py.)"""
    cfg = I.CONFIGS[cid]
    qblocks = I.sample_query_blocks(cfg, n_random)
    _log(f"[forward] config {cid} full-size launch, oracle on {len(qblocks)} query blocks")
    idx = None
    if cid in I.ROUTE3D:   # routed by the four geometric rules (table from the oracle; the GPU routing has its own tests)
        cams = I.make_cameras(cfg)
        idx, _ = oracle_lib.route_3d(I.make_points(cfg), I.make_points_img(cfg, cams), cams, cfg.grid, cfg.topk,
                                     **I.ROUTE3D[cid])
    _assert_forward(*_forward_case(B, oracle_lib, cfg, idx=idx, qblocks=qblocks), f"config{cid}-sampled")


def test_forward_is_deterministic(B, oracle_lib):
    cfg = I.small_config(name="f-det", n_obj=512, n_views=2, grid=16, heads=2, d=64, topk=3, window=128)
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates = I.make_gates(cfg)
    idx, _ = oracle_lib.route(I.make_points(cfg), I.make_cameras(cfg), cfg.grid, cfg.topk)
    a = G.run_forward(B, cfg, q_bits, k_bits, v_bits, idx, gates)["out"]
    b = G.run_forward(B, cfg, q_bits, k_bits, v_bits, idx, gates)["out"]
    assert np.array_equal(a, b)


@pytest.mark.parametrize("d,topk,with_counts", [(64, 64, False), (128, 64, False), (32, 128, False), (64, 128, False),
                                                 (128, 128, False), (128, 80, False), (32, 80, True), (128, 100, True)])
def test_forward_wide_routing_rows(B, oracle_lib, d, topk, with_counts):
    """Routing rows of 64 entries (every lane of the list holder is used) and of 65..128 (two registers: the
    paper's stage-3 budget is 16 volume + 4 blocks per view, 80 at 16 views), some rows full, some with holes
    on either side of entry 64, neighbouring rows overlapping as routed rows do."""
    cfg = I.small_config(name=f"f-topk{topk}-d{d}-cnt{int(with_counts)}", n_obj=8192, n_views=2, grid=16, heads=1, d=d,
                         topk=topk, window=64, seed=61)
    _log(f"[forward] {cfg.name}")
    rng = np.random.default_rng(12)
    idx = np.stack([(rng.choice(cfg.nb - 8, size=topk, replace=False) + (r // 4) % 8) for r in range(cfg.nb)]).astype(np.int32)
    idx[0::4] = idx[1::4]                               # pairs of identical rows inside a workgroup's group
    idx[1::3][rng.random(idx[1::3].shape) < 0.3] = -1
    idx[5, :70] = -1                                     # a row whose valid entries all sit past entry 64
    cnt = _block_counts(cfg, 10) if with_counts else None
    _assert_forward(*_forward_case(B, oracle_lib, cfg, idx=idx, block_count=cnt), cfg.name)


@pytest.mark.parametrize("d,topk", [(64, 6), (128, 9), (32, 5)])
def test_forward_rows_that_share_and_repeat_blocks(B, oracle_lib, d, topk):
    """Routing rows built to stress the step schedule of the selected branch: the four rows of a workgroup
    identical, overlapping in part (pairs, triples), disjoint, a block listed twice or three times in a row
    (it is attended that many times) while its neighbours list it once, holes in the middle of rows, rows of
    different lengths, an empty row."""
    cfg = I.small_config(name=f"f-share-d{d}", n_obj=1088, n_views=3, grid=24, heads=2, d=d, topk=topk, window=64,
                         seed=81)
    _log(f"[forward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(17)
    idx = np.full((cfg.nb, topk), -1, dtype=np.int32)
    for g in range(0, cfg.nb, 4):
        rows = range(g, min(g + 4, cfg.nb))
        kind = (g // 4) % 6
        common = rng.choice(cfg.nb, size=topk, replace=False)
        for r in rows:
            if kind == 0:      # identical rows (in a different order each)
                idx[r] = rng.permutation(common)
            elif kind == 1:    # half shared, half private
                own = rng.choice(cfg.nb, size=topk, replace=False)
                idx[r] = np.where(np.arange(topk) % 2 == 0, common, own)
            elif kind == 2:    # disjoint random rows
                idx[r] = rng.choice(cfg.nb, size=topk, replace=False)
            elif kind == 3:    # repeats: the first block twice or three times in odd rows, once in even rows
                idx[r] = common
                if r % 2:
                    idx[r, 1] = common[0]
                    if topk > 4:
                        idx[r, 4] = common[0]
            elif kind == 4:    # holes in the middle, rows of different lengths
                idx[r] = rng.permutation(common)
                idx[r, rng.random(topk) < 0.25 * (1 + r % 4)] = -1
            else:              # pairs share: rows 0, 1 one list, rows 2, 3 another, one row empty
                idx[r] = common if (r - g) < 2 else rng.choice(cfg.nb, size=topk, replace=False)
                if r - g == 3:
                    idx[r] = -1
    _assert_forward(*_forward_case(B, oracle_lib, cfg, idx=idx), cfg.name)


@pytest.mark.parametrize("n_obj,n_views", [(0, 3), (640, 0)])
def test_one_modality_only(B, oracle_lib, n_obj, n_views):
    """Sequences without object tokens, or without views: routing finds no candidates of the other
    modality (rows of -1), the selected branch is empty everywhere, the other two carry the layer."""
    cfg = I.small_config(name=f"f-obj{n_obj}-views{n_views}", n_obj=n_obj, n_views=n_views, grid=16, heads=2, d=64,
                         topk=3, window=96, seed=62)
    _log(f"[route+forward] {cfg.name}")
    pos = I.make_points(cfg) if n_obj else np.zeros((0, 3), dtype=np.float32)
    cams = I.make_cameras(cfg) if n_views else np.zeros((0, 16), dtype=np.float32)
    ref_idx, _ = oracle_lib.route(pos, cams, cfg.grid, cfg.topk)
    assert (ref_idx == -1).all()
    import torch
    p = G.params_for(B, cfg)
    d_idx = torch.full((cfg.nb, cfg.topk), -7, dtype=torch.int32, device="cuda")
    ws = B.alloc_workspace(p, B.LSRM_WS_ROUTE)
    dummy = torch.zeros(64, dtype=torch.float32, device="cuda")
    B.lsrm_route_blocks(p, torch.from_numpy(pos).cuda() if n_obj else dummy,
                        torch.from_numpy(cams).cuda() if n_views else dummy, d_idx, None, ws)
    torch.cuda.synchronize()
    assert np.array_equal(d_idx.cpu().numpy(), ref_idx)
    res, ref_out, ref_lse, ref_ob = _forward_case(B, oracle_lib, cfg, idx=ref_idx)
    _assert_forward(res, ref_out, ref_lse, ref_ob, cfg.name)
    assert np.all(res["ob"][1] == 0) and np.all(np.isneginf(res["lse"][1]))


def test_empty_problem_is_a_no_op(B):
    import torch
    p = B.make_params(0, 0, 16, 2, 64, 3, 128)
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(64, dtype=torch.float32, device="cuda")
    i = torch.zeros(64, dtype=torch.int32, device="cuda")
    B.lsrm_route_blocks(p, f, f, i, None, f)
    B.lsrm_nsa_compress(p, t, t, t, t)
    B.lsrm_nsa_forward(p, t, t, t, t, t, i, f, t, None, None, f)
    torch.cuda.synchronize()


# ----------------------------------------------------------------------------- error paths
def test_error_codes(B):
    import torch
    cfg = I.small_config()
    p = G.params_for(B, cfg)
    bad = B.make_params(cfg.n_obj, cfg.n_views, cfg.grid, cfg.heads, 96, cfg.topk, cfg.window)
    t = torch.empty(16, device="cuda")
    with pytest.raises(B.LsrmError) as e:
        B.lsrm_nsa_compress(bad, t, t, t, t)
    assert e.value.status == B.LSRM_ERR_UNSUPPORTED
    with pytest.raises(B.LsrmError) as e:
        B.lsrm_route_blocks(p, t, t, t, None, None)
    assert e.value.status == B.LSRM_ERR_WORKSPACE
    odd = B.make_params(cfg.n_obj + 1, cfg.n_views, cfg.grid, cfg.heads, cfg.d, cfg.topk, cfg.window)
    with pytest.raises(B.LsrmError) as e:
        B.lsrm_nsa_compress(odd, t, t, t, t)
    assert e.value.status == B.LSRM_ERR_INVALID_ARG
    assert B.lsrm_workspace_bytes(bad, B.LSRM_WS_FORWARD) == 0
