"""GPU parity and run-to-run determinism at the full size of the configurations whose timings are quoted
(config 4: the benchmark's; config 6: the paper's head shape; config 3 shapes for the backward), in the launch
configuration the benchmark times.  The oracle cannot finish these sizes, so it evaluates samples:

forward   first and last block of every segment, 8 random query blocks for every combination of (position of
          the block inside its workgroup's group of 4, which of the 8 contiguous ranges of groups -- one per
          XCD -- the group falls in), and the blocks on either side of every range boundary: about 300 query
          blocks at config 4, all heads, every output element of those blocks;
backward  dq on sampled query blocks, dk and dv on sampled key blocks (a popular one, i.e. one with the
          longest reverse routing list, among them) to which every query of the sequence contributes.

Inputs and device results of a configuration are made once per module and shared by its tests.
Bars as everywhere: max-abs <= 2e-2 and relative L2 <= 5e-3, lse within 2e-2, determinism bit for bit.
"""
import sys

import numpy as np
import pytest

from paper_2604_05182_amd import inputs as I
import gpu_util as G

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

N_CHUNKS = 4


def _log(msg):
    print(msg, file=sys.stderr, flush=True)


class _Case:
    """Seeded inputs of one configuration on the host and the device, the forward run twice into the same buffers."""

    def __init__(self, B, oracle_lib, cid):
        import torch
        self.cid, self.cfg = cid, I.CONFIGS[cid]
        cfg = self.cfg
        _log(f"[full-size] config {cid}: generating inputs ({cfg.n} tokens, {cfg.heads} heads on {cfg.kv_heads}, d {cfg.d})")
        self.q_bits, self.k_bits, self.v_bits = I.make_qkv(cfg)
        self.gates, self.dout_bits = I.make_gates(cfg), I.make_dout(cfg)
        cams = I.make_cameras(cfg)
        if cid in I.ROUTE3D:
            self.idx, _ = oracle_lib.route_3d(I.make_points(cfg), I.make_points_img(cfg, cams), cams, cfg.grid, cfg.topk,
                                              **I.ROUTE3D[cid])
        else:
            self.idx, _ = oracle_lib.route(I.make_points(cfg), cams, cfg.grid, cfg.topk)
        self.seg = cfg.seg_offsets()
        self.p = G.params_for(B, cfg)
        self.dq, self.dk, self.dv = (G.bf16_dev(a) for a in (self.q_bits, self.k_bits, self.v_bits))
        self.kc = torch.empty((cfg.nb, cfg.kv_heads, cfg.d), dtype=torch.bfloat16, device="cuda")
        self.vc = torch.empty_like(self.kc)
        B.lsrm_nsa_compress(self.p, self.dk, self.dv, self.kc, self.vc)
        self.d_idx = torch.from_numpy(self.idx).cuda()
        self.d_g = torch.from_numpy(self.gates).cuda()
        self.out = torch.empty((cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device="cuda")
        self.lse = torch.empty((3, cfg.n, cfg.heads), dtype=torch.float32, device="cuda")
        self.ob = torch.empty((3, cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device="cuda")
        self.ws = B.alloc_workspace(self.p, B.LSRM_WS_FORWARD)
        _log(f"[full-size] config {cid}: forward, first launch")
        self._forward(B)
        torch.cuda.synchronize()
        first = (self.out.clone(), self.lse.clone(), self.ob.clone())
        # second launch into the same outputs and the same workspace, which now holds the first launch's tile
        # images and gated sums; the outputs are poisoned in between so that a row left unwritten shows
        self.out.fill_(float("nan"))
        self.lse.fill_(float("nan"))
        self.ob.fill_(float("nan"))
        _log(f"[full-size] config {cid}: forward, second launch")
        self._forward(B)
        torch.cuda.synchronize()
        # bit patterns, so that NaN == NaN and -0 != +0
        self.identical = [bool(torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a.view(torch.int32),
                                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b.view(torch.int32)))
                          for a, b in zip(first, (self.out, self.lse, self.ob))]
        del first
        self._f32 = None

    def _forward(self, B):
        B.lsrm_nsa_forward(self.p, self.dq, self.dk, self.dv, self.kc, self.vc, self.d_idx, self.d_g, self.out,
                           self.lse, self.ob, self.ws)

    def host_f32(self, oracle_lib):
        """q, k, v, pooled k, v as fp32 (made on first use: several GB at config 4)."""
        if self._f32 is None:
            q, k, v = (I.bf16_bits_to_f32(a) for a in (self.q_bits, self.k_bits, self.v_bits))
            self._f32 = (q, k, v, oracle_lib.pool(k), oracle_lib.pool(v))
        return self._f32


_cases = {}


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_05182_amd import binding
    yield binding
    _cases.clear()


def _case(B, oracle_lib, cid):
    # one configuration at a time stays resident (config 4 holds about 25 GB of device memory)
    if cid not in _cases:
        _cases.clear()
        import torch
        torch.cuda.empty_cache()
        _cases[cid] = _Case(B, oracle_lib, cid)
    return _cases[cid]


def _deterministic(B, oracle_lib, cid):
    """Two launches at full size, the chip fully loaded and the workspaces reused: out, lse and the branch
    outputs must agree bit for bit (a tile read before its copy has landed, or a missed wait between an MFMA
    and its reader, shows up here and not at small sizes)."""
    c = _case(B, oracle_lib, cid)
    assert c.identical == [True, True, True], f"out / lse / out_branch identical: {c.identical}"


def _forward_chunk(B, oracle_lib, cid, chunk):
    import torch
    c = _case(B, oracle_lib, cid)
    cfg = c.cfg
    sample = I.sample_query_blocks_stratified(cfg, 8 if cid == 4 else 2)
    qblocks = sample[chunk::N_CHUNKS]
    _log(f"[full-size] config {cid} forward: oracle on {len(qblocks)} of {len(sample)} sampled query blocks "
         f"(chunk {chunk} of {N_CHUNKS}), all {cfg.heads} heads")
    q, k, v, kc, vc = c.host_f32(oracle_lib)
    ref_out, ref_lse, ref_ob = oracle_lib.nsa_forward(q, k, v, kc, vc, c.idx, c.gates, c.seg, cfg.window,
                                                      qblocks=qblocks, want_lse=True, want_branches=True)
    rows = torch.from_numpy((qblocks.astype(np.int64)[:, None] * 64 + np.arange(64)[None]).reshape(-1)).cuda()
    got_out = G.bf16_host(c.out[rows])
    got_lse = c.lse[:, rows].cpu().numpy()
    got_ob = G.bf16_host(c.ob[:, rows])
    tag = f"config{cid}-chunk{chunk}"
    ma, rl = G.attention_errors(got_out, ref_out)
    _log(f"[full-size] {tag}: out max-abs {ma:.3e} rel-L2 {rl:.3e}")
    assert ma <= G.MAX_ABS_TOL and rl <= G.REL_L2_TOL
    for b, name in enumerate(("cmp", "sel", "win")):
        ma, rl = G.attention_errors(got_ob[b], ref_ob[b])
        _log(f"              branch {name}: max-abs {ma:.3e} rel-L2 {rl:.3e}")
        assert ma <= G.MAX_ABS_TOL and rl <= G.REL_L2_TOL
    assert np.isfinite(got_lse).all() and np.isfinite(ref_lse).all()
    assert np.abs(got_lse - ref_lse).max() <= 2e-2


def _popular_and_plain_key_blocks(cfg, idx):
    """Key blocks for the dk/dv sample: the block most query blocks route to, the last one nobody or hardly
    anybody routes to, an object block and an image block in the middle, the first and the last block."""
    hits = np.bincount(idx[idx >= 0].reshape(-1), minlength=cfg.nb)
    picks = [int(np.argmax(hits)), int(cfg.nb - 1 - np.argmin(hits[::-1])), cfg.nb_obj // 2,
             cfg.nb_obj + cfg.n_tiles // 2, 0, cfg.nb - 1]
    return np.array(sorted(set(picks)), dtype=np.int32), hits


def _backward_sampled(B, oracle_lib, cid):
    """lsrm_nsa_backward at the full size of the shapes whose backward timings are quoted, consuming the lse
    and branch outputs of the full-size forward of the same case."""
    import torch
    c = _case(B, oracle_lib, cid)
    cfg = c.cfg
    ddo = G.bf16_dev(c.dout_bits)
    gq = torch.full_like(c.out, float("nan"))
    gk, gv = torch.full_like(c.dk, float("nan")), torch.full_like(c.dk, float("nan"))
    wsb = B.alloc_workspace(c.p, B.LSRM_WS_BACKWARD)
    _log(f"[full-size] config {cid} shapes: backward launch")
    B.lsrm_nsa_backward(c.p, c.dq, c.dk, c.dv, c.kc, c.vc, c.d_idx, c.d_g, c.lse, c.ob, ddo, gq, gk, gv, wsb)
    torch.cuda.synchronize()
    del wsb
    for name, t in (("dq", gq), ("dk", gk), ("dv", gv)):
        assert bool(torch.isfinite(t.float()).all()), f"{name}: non-finite values"
    qblocks = I.sample_query_blocks(cfg, 3)
    kblocks, hits = _popular_and_plain_key_blocks(cfg, c.idx)
    group = cfg.heads // cfg.kv_heads
    if group == 1:
        heads = [5] if cid == 4 else [0, 7, cfg.heads - 1]     # one head at config 4: every query's softmax over
        kv_heads = heads                                        # 6688 pooled keys costs the oracle a minute per head
    else:
        kv_heads = [1]
        heads = [0, group - 1, group, cfg.heads - 1]            # dq: both groups; dk, dv: all 16 heads of group 1
    _log(f"[full-size] config {cid} shapes backward: oracle on {len(qblocks)} query blocks (heads {heads}), key blocks "
         f"{kblocks.tolist()} (routed to by {hits[kblocks].tolist()} query blocks; key/value heads {kv_heads})")
    q, k, v, kc, vc = c.host_f32(oracle_lib)
    dout = I.bf16_bits_to_f32(c.dout_bits)
    ref = oracle_lib.nsa_backward_sampled(q, k, v, kc, vc, c.idx, c.gates, c.seg, cfg.window, dout, qblocks, kblocks,
                                          heads, kv_heads=kv_heads)
    rows_q = torch.from_numpy((qblocks.astype(np.int64)[:, None] * 64 + np.arange(64)[None]).reshape(-1)).cuda()
    rows_k = torch.from_numpy((kblocks.astype(np.int64)[:, None] * 64 + np.arange(64)[None]).reshape(-1)).cuda()
    got = (G.bf16_host(gq[rows_q][:, heads]), G.bf16_host(gk[rows_k][:, kv_heads]), G.bf16_host(gv[rows_k][:, kv_heads]))
    for name, g, r in zip(("dq", "dk", "dv"), got, ref):
        ma, rl = G.attention_errors(g, r)
        _log(f"[full-size] config {cid} shapes backward {name}: max-abs {ma:.3e} rel-L2 {rl:.3e} (|ref| max "
             f"{np.abs(r).max():.3e})")
        assert ma <= G.MAX_ABS_TOL and rl <= G.REL_L2_TOL, (name, ma, rl)


# Tests of one configuration are kept together: its inputs and device buffers are made once.
def test_config4_forward_is_deterministic(B, oracle_lib):
    _deterministic(B, oracle_lib, 4)


@pytest.mark.parametrize("chunk", range(N_CHUNKS))
def test_config4_forward_stratified_sample(B, oracle_lib, chunk):
    _forward_chunk(B, oracle_lib, 4, chunk)


def test_config4_shapes_backward_sampled(B, oracle_lib):
    _backward_sampled(B, oracle_lib, 4)


def test_config6_forward_is_deterministic(B, oracle_lib):
    _deterministic(B, oracle_lib, 6)


@pytest.mark.parametrize("chunk", range(N_CHUNKS))
def test_config6_forward_stratified_sample(B, oracle_lib, chunk):
    _forward_chunk(B, oracle_lib, 6, chunk)


def test_config6_shapes_backward_sampled(B, oracle_lib):
    _backward_sampled(B, oracle_lib, 6)


def test_config3_shapes_backward_sampled(B, oracle_lib):
    _backward_sampled(B, oracle_lib, 3)
