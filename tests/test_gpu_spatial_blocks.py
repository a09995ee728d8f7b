"""GPU parity with spatial blocks larger than 64 tokens (Sec. 3.2: 8 x 8 x 8 volume blocks hold up to 512 active
tokens), given as groups of consecutive 64-slot blocks: one compressed pair per spatial block, the own-block window
over the whole spatial block, gradients handed back to all its active tokens.  Compress, forward and backward
against the oracle, element by element."""
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


def _groups(nb, rng, max_blocks=8):
    """Random spatial blocks of 1..max_blocks 64-slot blocks covering nb blocks; a few sizes forced in."""
    sizes = [1, max_blocks, 2, 3]
    while sum(sizes) < nb:
        sizes.append(int(rng.integers(1, max_blocks + 1)))
    over = sum(sizes) - nb
    while over > 0:                      # trim from the end
        take = min(over, sizes[-1] - 1) if sizes[-1] > 1 else 1
        if sizes[-1] - take <= 0:
            sizes.pop()
        else:
            sizes[-1] -= take
        over = sum(sizes) - nb
    assert sum(sizes) == nb and min(sizes) >= 1
    return np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)


def _case(cfg, seed, with_counts, topk, min_count=1):
    rng = np.random.default_rng(seed)
    goff = _groups(cfg.nb, rng)
    idx = np.stack([rng.choice(cfg.nb, size=topk, replace=False) for _ in range(cfg.nb)]).astype(np.int32)
    idx[rng.random(idx.shape) < 0.15] = -1
    cnt = None
    if with_counts:
        # a spatial block fills its 64-slot blocks in order: only its last block is partly filled; two blocks in the
        # middle of groups are made partial as well (the kernels mask per 64-slot block)
        cnt = np.full(cfg.nb, 64, dtype=np.int32)
        cnt[goff[1:] - 1] = rng.integers(min_count, 65, size=len(goff) - 1)
        cnt[goff[1] + 2] = 31
        cnt[goff[2]] = max(5, min_count)
    return goff, idx, cnt


def _poison(cfg, cnt, *bits):
    if cnt is None:
        return bits
    inactive = (np.arange(cfg.n) % 64) >= np.repeat(cnt, 64)
    out = []
    for b in bits:
        b = b.copy()
        b[inactive] = 0x7FC0
        out.append(b)
    return out


@pytest.mark.parametrize("d,heads,h_kv,window_mode,with_counts", [(64, 2, 2, 1, False), (128, 2, 2, 1, True),
                                                                  (64, 4, 2, 0, True), (32, 4, 1, 1, True),
                                                                  (128, 3, 3, 0, False)])
def test_forward_with_spatial_blocks(B, oracle_lib, d, heads, h_kv, window_mode, with_counts):
    cfg = I.small_config(name=f"g-fwd-d{d}-w{window_mode}-cnt{int(with_counts)}", n_obj=2368, n_views=2, grid=24,
                         heads=heads, d=d, topk=6, window=160, seed=91, h_kv=h_kv)
    goff, idx, cnt = _case(cfg, 3, with_counts, cfg.topk)
    _log(f"[spatial blocks] {cfg.name}: {cfg.nb} blocks of 64 slots in {len(goff) - 1} spatial blocks of "
         f"{np.diff(goff).min()}..{np.diff(goff).max()}")
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates = I.make_gates(cfg)
    k_bits, v_bits = _poison(cfg, cnt, k_bits, v_bits)
    for fused in (False, True):
        res = G.run_forward(B, cfg, q_bits, k_bits, v_bits, idx, gates, want_aux=True, window_mode=window_mode,
                            block_count=cnt, group_offsets=goff, fused_pack=fused)
        q, k, v = (I.bf16_bits_to_f32(a) for a in (q_bits, k_bits, v_bits))
        kc, vc = oracle_lib.pool(k, cnt, goff), oracle_lib.pool(v, cnt, goff)
        assert res["kc"].shape == kc.shape == (len(goff) - 1, h_kv, d)
        for got, ref in ((res["kc"], kc), (res["vc"], vc)):
            assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-6)
        ref_out, ref_lse, ref_ob = oracle_lib.nsa_forward(q, k, v, kc, vc, idx, gates, cfg.seg_offsets(), cfg.window,
                                                          want_lse=True, want_branches=True, window_mode=window_mode,
                                                          block_count=cnt, group_offsets=goff)
        act = np.ones(cfg.n, dtype=bool) if cnt is None else (np.arange(cfg.n) % 64) < np.repeat(cnt, 64)
        for name, got, ref in (("out", res["out"], ref_out), ("cmp", res["ob"][0], ref_ob[0]),
                               ("sel", res["ob"][1], ref_ob[1]), ("win", res["ob"][2], ref_ob[2])):
            ma, rl = G.attention_errors(got[act], ref[act])
            _log(f"    fused={fused} {name}: max-abs {ma:.3e} rel-L2 {rl:.3e}")
            assert ma <= G.MAX_ABS_TOL and rl <= G.REL_L2_TOL
        fin = np.isfinite(ref_lse[:, act])
        assert np.array_equal(np.isfinite(res["lse"][:, act]), fin)
        assert np.abs(res["lse"][:, act][fin] - ref_lse[:, act][fin]).max() <= 2e-2


@pytest.mark.parametrize("d,heads,h_kv,window_mode,with_counts", [(64, 2, 2, 1, False), (128, 2, 2, 1, True),
                                                                  (64, 4, 2, 0, True), (32, 4, 1, 1, True)])
def test_backward_with_spatial_blocks(B, oracle_lib, d, heads, h_kv, window_mode, with_counts):
    cfg = I.small_config(name=f"g-bwd-d{d}-w{window_mode}-cnt{int(with_counts)}", n_obj=1088, n_views=2, grid=16,
                         heads=heads, d=d, topk=4, window=160, seed=93, h_kv=h_kv)
    # (spatial blocks hold at least 8 active tokens here: a pooled pair hands the gradient it collects from every
    # query of the sequence to its tokens, divided by their number -- with a single token nothing averages the bf16
    # noise of those 1600 contributions down, and it reaches 0.03-0.05 on that one row)
    goff, idx, cnt = _case(cfg, 5, with_counts, cfg.topk, min_count=8)
    _log(f"[spatial blocks] {cfg.name}: {cfg.nb} blocks in {len(goff) - 1} spatial blocks")
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates, dout_bits = I.make_gates(cfg), I.make_dout(cfg)
    if heads != h_kv:   # keep the summed gradients of a key/value head at the magnitude the absolute bar was set for
        dout_bits = I.f32_to_bf16_bits(I.bf16_bits_to_f32(dout_bits) * np.float32(h_kv / heads))
    q, k, v, dout = (I.bf16_bits_to_f32(a) for a in (q_bits, k_bits, v_bits, dout_bits))
    k_bits, v_bits, dout_bits = _poison(cfg, cnt, k_bits, v_bits, dout_bits)
    got = G.run_backward(B, cfg, q_bits, k_bits, v_bits, idx, gates, dout_bits, window_mode=window_mode,
                         block_count=cnt, group_offsets=goff)
    kc, vc = oracle_lib.pool(k, cnt, goff), oracle_lib.pool(v, cnt, goff)
    ref = oracle_lib.nsa_backward(q, k, v, kc, vc, idx, gates, cfg.seg_offsets(), cfg.window, dout,
                                  window_mode=window_mode, block_count=cnt, group_offsets=goff)
    for name, g, r in zip(("dq", "dk", "dv"), got, ref):
        assert np.isfinite(g).all(), name
        ma, rl = G.attention_errors(g, r)
        _log(f"    {name}: max-abs {ma:.3e} rel-L2 {rl:.3e} (|ref| max {np.abs(r).max():.3e})")
        assert ma <= G.MAX_ABS_TOL and rl <= G.REL_L2_TOL, (name, ma, rl)
    if cnt is not None:
        inactive = (np.arange(cfg.n) % 64) >= np.repeat(cnt, 64)
        for g in got:
            assert np.all(g[inactive] == 0)


def test_group_arguments_are_checked(B):
    import torch
    off = torch.tensor([0, 2, 8], dtype=torch.int32, device="cuda")
    ok = B.make_params(512, 0, 16, 2, 64, 3, 128, group_offsets=off)
    assert B.lsrm_workspace_bytes(ok, B.LSRM_WS_FORWARD) > 0 and B.lsrm_workspace_bytes(ok, B.LSRM_WS_BACKWARD) > 0
    bad = B.make_params(512, 0, 16, 2, 64, 3, 128, group_offsets=off)
    bad.n_groups = 9          # more spatial blocks than 64-slot blocks
    assert B.lsrm_workspace_bytes(bad, B.LSRM_WS_FORWARD) == 0
    none = B.make_params(512, 0, 16, 2, 64, 3, 128)
    none.n_groups = 2         # a count without offsets
    assert B.lsrm_workspace_bytes(none, B.LSRM_WS_FORWARD) == 0
