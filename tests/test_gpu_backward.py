"""GPU parity of lsrm_nsa_backward against the CPU oracle's analytic gradients, element by
element on small cases and on a sample of blocks and heads at the full size of config 5.
Tolerance as for the forward: max-abs <= 2e-2 and relative L2 <= 5e-3 per gradient tensor."""
import sys

import numpy as np
import pytest

from paper_2604_05182_amd import inputs as I

import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2604_05182_amd import binding
    return binding


def _log(msg):
    print(msg, file=sys.stderr, flush=True)


def _case(B, oracle_lib, cfg, idx=None, seg="default", scale=0.0, window=None, window_mode=0):
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates, dout_bits = I.make_gates(cfg), I.make_dout(cfg)
    if idx is None:
        idx, _ = oracle_lib.route(I.make_points(cfg), I.make_cameras(cfg), cfg.grid, cfg.topk)
    seg_arr = cfg.seg_offsets() if isinstance(seg, str) else np.asarray(seg, dtype=np.int32)
    window = cfg.window if window is None else window
    got = G.run_backward(B, cfg, q_bits, k_bits, v_bits, idx, gates, dout_bits, seg_offsets=seg, scale=scale,
                         window=window, window_mode=window_mode)
    q, k, v, dout = (I.bf16_bits_to_f32(a) for a in (q_bits, k_bits, v_bits, dout_bits))
    kc, vc = oracle_lib.pool(k), oracle_lib.pool(v)
    return got, (q, k, v, kc, vc, idx, gates, seg_arr, window, dout)


def _assert_grads(got, ref, tag):
    for name, g, r in zip(("dq", "dk", "dv"), got, ref):
        assert np.isfinite(g).all(), f"{tag} {name}: non-finite values"
        ma, rl = G.attention_errors(g, r)
        _log(f"[backward] {tag} {name}: max-abs {ma:.3e} rel-L2 {rl:.3e}  (|ref| max {np.abs(r).max():.3e})")
        assert ma <= G.MAX_ABS_TOL and rl <= G.REL_L2_TOL, (tag, name, ma, rl)


def test_backward_grouped_heads_large_gradients_elementwise(B, oracle_lib):
    """Sixteen query heads per key/value head with single-token blocks and dout as generated (not divided by the
    group size): dk and dv reach magnitudes where their bf16 storage alone exceeds the absolute bar, so they are
    checked element by element against a bar that grows with the row: 2e-2 for rows of order one plus 2^-7 of the
    largest reference value of the element's (token, head) row -- every channel of a row sums the same contributions
    with the same probabilities, so a channel's error follows the row's magnitude, not its own value (a bf16 result
    is within 2^-9 of its value; the operands' own bf16 roundings and the order of the fp32 sums take the rest) --
    and by relative L2 as everywhere."""
    cfg = I.small_config(name="b-group16-unscaled", n_obj=576, n_views=2, grid=16, heads=32, d=32, topk=4, window=160,
                         seed=71, h_kv=2, gate_channels=False)
    _log(f"[backward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(13)
    cnt = rng.integers(1, 65, size=cfg.nb).astype(np.int32)
    cnt[:6] = (64, 1, 33, 32, 31, 64)
    idx = np.stack([rng.choice(cfg.nb, size=cfg.topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[:, 0] = np.minimum(np.arange(cfg.nb), 5)
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates, dout_bits = I.make_gates(cfg), I.make_dout(cfg)
    q, k, v, dout = (I.bf16_bits_to_f32(a) for a in (q_bits, k_bits, v_bits, dout_bits))
    got = G.run_backward(B, cfg, q_bits, k_bits, v_bits, idx, gates, dout_bits, window_mode=1, block_count=cnt)
    kc, vc = oracle_lib.pool(k, cnt), oracle_lib.pool(v, cnt)
    ref = oracle_lib.nsa_backward(q, k, v, kc, vc, idx, gates, cfg.seg_offsets(), cfg.window, dout, window_mode=1,
                                  block_count=cnt)
    active = (np.arange(cfg.n) % 64) < np.repeat(cnt, 64)
    for name, g, r in zip(("dq", "dk", "dv"), got, ref):
        g, r = g[active], r[active]
        assert np.isfinite(g).all(), name
        excess = np.abs(g - r) - (G.MAX_ABS_TOL + np.abs(r).max(axis=-1, keepdims=True) * 2.0 ** -7)
        _, rl = G.attention_errors(g, r)
        _log(f"[backward] {cfg.name} {name}: |ref| max {np.abs(r).max():.3e}, worst excess over the bar "
             f"{excess.max():.3e}, rel-L2 {rl:.3e}")
        assert excess.max() <= 0.0 and rl <= G.REL_L2_TOL, (name, float(excess.max()), rl)


def test_backward_small(B, oracle_lib):
    cfg = I.small_config(name="b-small", n_obj=512, n_views=2, grid=16, heads=2, d=64, topk=3, window=128)
    _log(f"[backward] {cfg.name}")
    got, args = _case(B, oracle_lib, cfg)
    _assert_grads(got, oracle_lib.nsa_backward(*args), cfg.name)


def test_backward_ragged_and_holes(B, oracle_lib):
    """NB not a multiple of 32, odd head count, -1 holes, an empty routed row, key blocks nobody routes
    to, a window that is not a multiple of the block, explicit scale."""
    cfg = I.small_config(name="b-ragged", n_obj=1088, n_views=3, grid=24, heads=3, d=64, topk=5, window=200, seed=21)
    _log(f"[backward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(5)
    idx = np.stack([rng.choice(cfg.nb // 2, size=cfg.topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[rng.random(idx.shape) < 0.2] = -1
    idx[2] = -1
    got, args = _case(B, oracle_lib, cfg, idx=idx, scale=0.2)
    _assert_grads(got, oracle_lib.nsa_backward(*args, scale=0.2), cfg.name)


@pytest.mark.parametrize("d", [64, 128, 32])
def test_backward_repeated_and_popular_blocks(B, oracle_lib, d):
    """Rows that list a block twice (it is attended twice) and one block that every row lists (a reverse list
    longer than one 64-entry chunk, and by far the longest walk), with per-channel gates on grouped heads
    (the gradient rows change between branches even where a branch is empty)."""
    cfg = I.small_config(name=f"b-repeat-d{d}", n_obj=4096, n_views=2, grid=16, heads=4, d=d, topk=4, window=128,
                         seed=27, h_kv=2, gate_channels=True)
    _log(f"[backward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(11)
    idx = np.stack([rng.choice(cfg.nb, size=cfg.topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[:, 0] = 5                      # a popular block: nb entries in its reverse list
    idx[3::7, 2] = idx[3::7, 1]        # repeats inside a row
    idx[4::9, 3] = 5                   # the popular block twice in a row
    idx[6] = -1
    got, args = _case(B, oracle_lib, cfg, idx=idx)
    _assert_grads(got, oracle_lib.nsa_backward(*args), cfg.name)
    # no routed blocks and no window at all: only the compressed branch is left
    cfg0 = I.small_config(name="b-cmp-only", n_obj=512, n_views=2, grid=16, heads=4, d=64, topk=2, window=0, seed=28,
                          h_kv=2, gate_channels=True)
    idx0 = np.full((cfg0.nb, cfg0.topk), -1, dtype=np.int32)
    got, args = _case(B, oracle_lib, cfg0, idx=idx0)
    _assert_grads(got, oracle_lib.nsa_backward(*args), cfg0.name)


@pytest.mark.parametrize("d,topk", [(64, 128), (128, 80), (32, 100)])
def test_backward_wide_routing_rows(B, oracle_lib, d, topk):
    """Routing rows of 65..128 entries (the paper's stage-3 budgets at 16 views need 80), with holes on either
    side of entry 64 and a row whose valid entries all sit past it."""
    cfg = I.small_config(name=f"b-topk{topk}-d{d}", n_obj=8192, n_views=2, grid=16, heads=2, d=d, topk=topk, window=64,
                         seed=63)
    _log(f"[backward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(14)
    idx = np.stack([rng.choice(cfg.nb, size=topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[1::3][rng.random(idx[1::3].shape) < 0.3] = -1
    idx[5, :70] = -1
    got, args = _case(B, oracle_lib, cfg, idx=idx)
    # every block and head through the sampled function (the same arithmetic, spread over the host's threads)
    every = np.arange(cfg.nb, dtype=np.int32)
    _assert_grads(got, oracle_lib.nsa_backward_sampled(*args, every, every, list(range(cfg.heads))), cfg.name)


def test_backward_own_block_window(B, oracle_lib):
    """The window branch over the query's own block (App. A) instead of the sliding window."""
    cfg = I.small_config(name="b-ownblock", n_obj=1088, n_views=3, grid=24, heads=3, d=64, topk=5, window=200, seed=23)
    _log(f"[backward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(9)
    idx = np.stack([rng.choice(cfg.nb, size=cfg.topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[rng.random(idx.shape) < 0.2] = -1
    got, args = _case(B, oracle_lib, cfg, idx=idx, window_mode=1)
    _assert_grads(got, oracle_lib.nsa_backward(*args, window_mode=1), cfg.name)


@pytest.mark.parametrize("d,heads,h_kv,gate_channels", [(64, 6, 2, False), (64, 2, 2, True), (64, 4, 1, True),
                                                        (32, 2, 2, False), (128, 2, 2, False), (128, 4, 2, True),
                                                        # the paper's heads in small: 16 query heads per key/value head
                                                        (32, 32, 2, True),
                                                        # 9 query heads per key/value head: head ranges of 2, 2, 2, 2, 1
                                                        (32, 18, 2, False)])
def test_backward_head_shapes_and_gates(B, oracle_lib, d, heads, h_kv, gate_channels):
    """Head dimensions 32 / 64 / 128, query heads sharing key/value heads (a key/value head collects the
    gradients of its whole group), one gate per output channel; ragged block count, holes in the table."""
    cfg = I.small_config(name=f"b-d{d}-h{heads}-kv{h_kv}-ch{int(gate_channels)}", n_obj=576, n_views=2, grid=16,
                         heads=heads, d=d, topk=4, window=160, seed=51, h_kv=h_kv, gate_channels=gate_channels)
    _log(f"[backward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(11)
    idx = np.stack([rng.choice(cfg.nb, size=cfg.topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[rng.random(idx.shape) < 0.2] = -1
    got, args = _case(B, oracle_lib, cfg, idx=idx)
    assert got[1].shape == (cfg.n, h_kv, d)
    _assert_grads(got, oracle_lib.nsa_backward(*args), cfg.name)


@pytest.mark.parametrize("d,window_mode,heads,h_kv,gate_channels",
                         [(64, 0, 3, 3, False), (64, 1, 3, 3, False), (128, 1, 3, 3, False), (32, 0, 3, 3, False),
                          # grouped heads: the pass that adds the head ranges finishes the rows
                          (64, 0, 4, 2, False), (32, 1, 16, 2, False),
                          # per-channel gates: the gate * dout rows of padding slots (NaN dout) must never be read
                          (64, 0, 3, 3, True), (128, 1, 2, 2, True), (32, 0, 4, 2, True)])
def test_backward_with_active_counts(B, oracle_lib, d, window_mode, heads, h_kv, gate_channels):
    """Blocks with fewer than 64 active tokens: padding slots are neither queries nor keys (whatever sits in
    their rows of k, v and dout -- NaN here -- is never looked at) and get zero gradients."""
    cfg = I.small_config(name=f"b-counts-d{d}-w{window_mode}-h{heads}-kv{h_kv}-ch{int(gate_channels)}", n_obj=576,
                         n_views=2, grid=16, heads=heads, d=d, topk=4, window=160, seed=71, h_kv=h_kv,
                         gate_channels=gate_channels)
    _log(f"[backward] {cfg.name} nb={cfg.nb}")
    rng = np.random.default_rng(13)
    cnt = rng.integers(1, 65, size=cfg.nb).astype(np.int32)
    cnt[:6] = (64, 1, 33, 32, 31, 64)
    idx = np.stack([rng.choice(cfg.nb, size=cfg.topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[rng.random(idx.shape) < 0.2] = -1
    idx[:, 0] = np.minimum(np.arange(cfg.nb), 5)
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates, dout_bits = I.make_gates(cfg), I.make_dout(cfg)
    if heads != h_kv:
        # a key/value head sums the gradients of its group: dout / group (a power of two, exact in bf16) keeps
        # dk, dv at the magnitude the absolute tolerance was set for
        dout_bits = I.f32_to_bf16_bits(I.bf16_bits_to_f32(dout_bits) * np.float32(h_kv / heads))
    q, k, v, dout = (I.bf16_bits_to_f32(a) for a in (q_bits, k_bits, v_bits, dout_bits))
    inactive = (np.arange(cfg.n) % 64) >= np.repeat(cnt, 64)
    k_bits, v_bits, dout_bits = k_bits.copy(), v_bits.copy(), dout_bits.copy()
    for bits in (k_bits, v_bits, dout_bits):
        bits[inactive] = 0x7FC0
    got = G.run_backward(B, cfg, q_bits, k_bits, v_bits, idx, gates, dout_bits, window_mode=window_mode, block_count=cnt)
    kc, vc = oracle_lib.pool(k, cnt), oracle_lib.pool(v, cnt)
    ref = oracle_lib.nsa_backward(q, k, v, kc, vc, idx, gates, cfg.seg_offsets(), cfg.window, dout,
                                  window_mode=window_mode, block_count=cnt)
    _assert_grads(got, ref, cfg.name)
    for g in got:
        assert np.all(g[inactive] == 0)


def test_backward_zero_window_and_topk_one(B, oracle_lib):
    cfg = I.small_config(name="b-w0", n_obj=256, n_views=1, grid=16, heads=1, d=64, topk=1, window=0)
    got, args = _case(B, oracle_lib, cfg)
    _assert_grads(got, oracle_lib.nsa_backward(*args), cfg.name)


def test_backward_single_segment_wide_window(B, oracle_lib):
    """One segment, window wider than the sequence, every block routed by every block."""
    cfg = I.small_config(name="b-dense", n_obj=512, n_views=0, grid=0, heads=2, d=64, topk=8, window=1024)
    idx = np.tile(np.arange(8, dtype=np.int32), (8, 1))
    got, args = _case(B, oracle_lib, cfg, idx=idx, seg=[0, 512])
    _assert_grads(got, oracle_lib.nsa_backward(*args), cfg.name)


def test_backward_config5_full_size_sampled(B, oracle_lib):
    """Full-size launch of config 5; the oracle evaluates dq on sampled query blocks and dk, dv on
    sampled key blocks (contributions of every query of the sequence), three heads."""
    cfg = I.CONFIGS[5]
    qblocks = I.sample_query_blocks(cfg, 3)
    kblocks = I.sample_query_blocks(cfg, 2, seed=5)[::2]
    heads = [0, 7, cfg.heads - 1]
    _log(f"[backward] config 5 full-size launch; oracle on {len(qblocks)} query blocks, {len(kblocks)} key blocks, "
         f"heads {heads}")
    got, args = _case(B, oracle_lib, cfg)
    (q, k, v, kc, vc, idx, gates, seg_arr, window, dout) = args
    ref = oracle_lib.nsa_backward_sampled(q, k, v, kc, vc, idx, gates, seg_arr, window, dout, qblocks, kblocks, heads)
    rows_q = (np.asarray(qblocks)[:, None] * 64 + np.arange(64)[None]).reshape(-1)
    rows_k = (np.asarray(kblocks)[:, None] * 64 + np.arange(64)[None]).reshape(-1)
    sub = (got[0][rows_q][:, heads], got[1][rows_k][:, heads], got[2][rows_k][:, heads])
    _assert_grads(sub, ref, "config5-sampled")
    assert all(np.isfinite(g).all() for g in got)


def test_backward_wide_heads_many_tiles_sampled(B, oracle_lib):
    """Head dimension 128 (the shape of config 4's heads) on a sequence long enough for thousands of workgroups,
    several window tiles per key block and reverse lists of uneven length: sampled like the test above, plus
    two runs compared bit for bit."""
    cfg = I.small_config(name="b-d128-mid", n_obj=32768, n_views=4, grid=64, heads=2, d=128, topk=16, window=512,
                         seed=61)
    qblocks = I.sample_query_blocks(cfg, 3)
    kblocks = I.sample_query_blocks(cfg, 2, seed=5)[::2]
    heads = [0, 1]
    _log(f"[backward] {cfg.name}: N {cfg.n}; oracle on {len(qblocks)} query blocks, {len(kblocks)} key blocks")
    got, args = _case(B, oracle_lib, cfg)
    (q, k, v, kc, vc, idx, gates, seg_arr, window, dout) = args
    ref = oracle_lib.nsa_backward_sampled(q, k, v, kc, vc, idx, gates, seg_arr, window, dout, qblocks, kblocks, heads)
    rows_q = (np.asarray(qblocks)[:, None] * 64 + np.arange(64)[None]).reshape(-1)
    rows_k = (np.asarray(kblocks)[:, None] * 64 + np.arange(64)[None]).reshape(-1)
    sub = (got[0][rows_q][:, heads], got[1][rows_k][:, heads], got[2][rows_k][:, heads])
    _assert_grads(sub, ref, cfg.name)
    assert all(np.isfinite(g).all() for g in got)
    again, _ = _case(B, oracle_lib, cfg)
    for x, y in zip(got, again):
        assert np.array_equal(x, y)


def test_backward_is_deterministic(B, oracle_lib):
    cfg = I.small_config(name="b-det", n_obj=1024, n_views=2, grid=16, heads=2, d=64, topk=4, window=256)
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates, dout_bits = I.make_gates(cfg), I.make_dout(cfg)
    idx, _ = oracle_lib.route(I.make_points(cfg), I.make_cameras(cfg), cfg.grid, cfg.topk)
    a = G.run_backward(B, cfg, q_bits, k_bits, v_bits, idx, gates, dout_bits)
    b = G.run_backward(B, cfg, q_bits, k_bits, v_bits, idx, gates, dout_bits)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_backward_full_size_is_deterministic(B, oracle_lib):
    """Config 5 at full size, three calls in a row (workspaces reused with whatever the call before left
    in them, the chip fully loaded): a tile read before its copy has landed shows up as a difference."""
    cfg = I.CONFIGS[5]
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates, dout_bits = I.make_gates(cfg), I.make_dout(cfg)
    idx, _ = oracle_lib.route(I.make_points(cfg), I.make_cameras(cfg), cfg.grid, cfg.topk)
    _log("[backward] config 5, three runs")
    runs = [G.run_backward(B, cfg, q_bits, k_bits, v_bits, idx, gates, dout_bits) for _ in range(3)]
    for other in runs[1:]:
        for x, y in zip(runs[0], other):
            assert np.array_equal(x, y)
