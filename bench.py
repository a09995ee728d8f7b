#!/usr/bin/env python3
"""Benchmark of the NSA layer hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: lsrm_route_blocks ->
lsrm_nsa_compress_pack (block averages and the forward's repacking of k, v in one pass) ->
lsrm_nsa_forward, inputs already resident in HBM (--two-pass: lsrm_nsa_compress and a forward that
repacks k, v itself).  The metric is
effective attention TFLOP/s (4 d h x attended (query, key) pairs; masked or padded work
does not count) and ms per layer.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..6] [--no-cpu-baseline]

--config 5 times the backward instead (config 2 shapes): a step is one lsrm_nsa_backward call on
resident inputs and saved forward results; effective FLOPs = 2.5 x the forward's (5 contractions).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16

# HBM bytes per launch of the attention kernel (fetched + written), from rocprofv3 FETCH_SIZE / WRITE_SIZE
# runs of this script scaled by the same counters of a plain 1 GiB copy; the readings and the commands are
# in profiles/nsa_forward_kernel_config4_hbm_traffic.txt.  Only the workloads that were profiled appear.
MEASURED_HBM_BYTES = {4: 56.5e9 + 3.5e9}


def cpu_baseline(cfg, arrays, idx, target_seconds=20.0):
    """Times the CPU oracle (as it stands) on a bounded sample of query blocks."""
    import oracle
    from paper_2604_05182_amd import inputs as I
    q, k, v = (I.bf16_bits_to_f32(a) for a in arrays["qkv_bits"])
    t0 = time.perf_counter()
    kc, vc = oracle.pool(k), oracle.pool(v)
    t_pool = time.perf_counter() - t0
    seg = cfg.seg_offsets()
    threads = oracle.num_threads()
    # calibrate on a few blocks, then size the sample for about target_seconds
    probe = I.sample_query_blocks(cfg, 0)[:max(2, threads // 4)]
    t0 = time.perf_counter()
    oracle.nsa_forward(q, k, v, kc, vc, idx, arrays["gates"], seg, cfg.window, qblocks=probe)
    per_block = (time.perf_counter() - t0) / len(probe)
    n_blocks = int(min(cfg.nb, max(threads, target_seconds / max(per_block, 1e-6))))
    blocks = I.sample_query_blocks(cfg, n_blocks, seed=1)[:n_blocks] if n_blocks < cfg.nb else np.arange(cfg.nb, dtype=np.int32)
    t0 = time.perf_counter()
    oracle.nsa_forward(q, k, v, kc, vc, idx, arrays["gates"], seg, cfg.window, qblocks=blocks)
    dt = time.perf_counter() - t0
    flops_per_block = cfg.forward_flops(int((idx >= 0).sum())) / cfg.nb
    return {
        "value": round(flops_per_block * len(blocks) / dt / 1e12, 6),
        "unit": "TFLOP/s",
        "cores": threads,
        "kind": "oracle",
        "sample": f"forward oracle on {len(blocks)} of {cfg.nb} query blocks (all heads), {dt:.1f} s; "
                  f"pooling of all K,V {t_pool:.1f} s not included; extrapolated ms/layer "
                  f"{dt / len(blocks) * cfg.nb * 1e3:.0f}",
    }


def cpu_baseline_backward(cfg, arrays, idx, dout_bits, target_seconds=20.0):
    """Times the CPU oracle's sampled gradient function on a bounded sample (query blocks only: dq)."""
    import oracle
    from paper_2604_05182_amd import inputs as I
    q, k, v = (I.bf16_bits_to_f32(a) for a in arrays["qkv_bits"])
    dout = I.bf16_bits_to_f32(dout_bits)
    kc, vc = oracle.pool(k), oracle.pool(v)
    seg = cfg.seg_offsets()
    threads = oracle.num_threads()
    heads = list(range(cfg.heads))
    none = np.zeros((0,), dtype=np.int32)
    probe = I.sample_query_blocks(cfg, 0)[:2]
    t0 = time.perf_counter()
    oracle.nsa_backward_sampled(q, k, v, kc, vc, idx, arrays["gates"], seg, cfg.window, dout, probe, none, heads)
    per_block = (time.perf_counter() - t0) / len(probe)
    n_blocks = int(min(cfg.nb, max(threads, target_seconds / max(per_block, 1e-6))))
    blocks = I.sample_query_blocks(cfg, n_blocks, seed=1)[:n_blocks]
    t0 = time.perf_counter()
    oracle.nsa_backward_sampled(q, k, v, kc, vc, idx, arrays["gates"], seg, cfg.window, dout, blocks, none, heads)
    dt = time.perf_counter() - t0
    flops_per_block = 2.5 * cfg.forward_flops(int((idx >= 0).sum())) / cfg.nb
    return {
        "value": round(flops_per_block * len(blocks) / dt / 1e12, 6),
        "unit": "TFLOP/s",
        "cores": threads,
        "kind": "oracle",
        "sample": f"gradient oracle (one pass computing dq; dk and dv accumulate in the same pass) on the rows of "
                  f"{len(blocks)} of {cfg.nb} query blocks, all heads, {dt:.1f} s; extrapolated ms/layer "
                  f"{dt / len(blocks) * cfg.nb * 1e3:.0f}",
    }


def run_backward_bench(args, cfg, B, I, p, dev, tensors, workspaces, host, route):
    import torch
    d_q, d_k, d_v, d_kc, d_vc, d_idx, d_gates, d_out, d_pos, d_cams = tensors
    ws_route, ws_fwd = workspaces
    q_bits, k_bits, v_bits, gates = host
    dout_bits = I.make_dout(cfg)
    d_dout = torch.from_numpy(dout_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    d_lse = torch.empty((3, cfg.n, cfg.heads), dtype=torch.float32, device=dev)
    d_ob = torch.empty((3, cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device=dev)
    d_dq, d_dk, d_dv = torch.empty_like(d_q), torch.empty_like(d_k), torch.empty_like(d_k)
    ws_bwd = B.alloc_workspace(p, B.LSRM_WS_BACKWARD)
    # forward results the backward consumes (not timed)
    route()
    B.lsrm_nsa_compress(p, d_k, d_v, d_kc, d_vc)
    B.lsrm_nsa_forward(p, d_q, d_k, d_v, d_kc, d_vc, d_idx, d_gates, d_out, d_lse, d_ob, ws_fwd)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    for row in ev:
        for e in row:
            e.record()

    def step(i=None):
        e = ev[i] if i is not None else [None, None]
        B.lsrm_nsa_backward(p, d_q, d_k, d_v, d_kc, d_vc, d_idx, d_gates, d_lse, d_ob, d_dout, d_dq, d_dk, d_dv, ws_bwd,
                            ev_start=e[0], ev_stop=e[1])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    ms_call = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    idx = d_idx.cpu().numpy()
    flops = 2.5 * cfg.forward_flops(int((idx >= 0).sum()))
    value = flops / (ms_step * 1e-3) / 1e12
    call_tflops = flops / (ms_call * 1e-3) / 1e12
    result = {
        "metric": "NSA layer backward effective TFLOP/s (lsrm_nsa_backward), 1 MI355X",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": f"config {args.config} ({cfg.name}): {cfg.n_obj} object + {cfg.n_views}x{cfg.grid}x{cfg.grid} "
                        f"image tokens = {cfg.n}, {cfg.heads} heads"
                        + (f" on {cfg.kv_heads} key/value heads" if cfg.kv_heads != cfg.heads else "")
                        + f", d {cfg.d}, block 64, top-k {cfg.topk}, window {cfg.window}"
                        + (", per-channel gates" if cfg.gate_channels else "") + "; gradients of q, k, v",
            "effective_flops": flops,
            "pct_of_bf16_mfma_peak": round(100.0 * value / BF16_MFMA_PEAK_TFLOPS, 2),
        },
        "breakdown_ms": {"backward_call": round(ms_call, 4)},
        "roofline": {
            "kernel": "all kernels of lsrm_nsa_backward (HIP events around the call's launches; per-kernel split in "
                      "profiles/)",
            "bound": "mfma", "achieved": round(call_tflops, 3), "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(call_tflops / BF16_MFMA_PEAK_TFLOPS, 4), "traffic": None,
        },
    }
    if not args.no_cpu_baseline and cfg.kv_heads == cfg.heads and not cfg.gate_channels:
        result["cpu_baseline"] = cpu_baseline_backward(cfg, {"qkv_bits": (q_bits, k_bits, v_bits), "gates": gates}, idx,
                                                       dout_bits)
    print(json.dumps(result), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4,
                    help="workload id 1..4 forward (default 4: the largest single-GPU config), 5 backward, "
                         "6 forward with the paper's head shape (32 x 32 on 2 key/value heads, channel gates, "
                         "four-rule routing)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--backward", action="store_true",
                    help="time lsrm_nsa_backward on the chosen config's shapes instead of the forward step (config 5 "
                         "always does)")
    ap.add_argument("--topk", type=int, default=None, help="override the config's routed top-k (experiments)")
    ap.add_argument("--window", type=int, default=None, help="override the config's window (experiments)")
    ap.add_argument("--routing", choices=("projected", "four-rule"), default="projected",
                    help="routing table: the configs' projected-centroid rule (default) or the four geometric "
                         "selection rules (lsrm_route_blocks_3d: B^i = 4, a quarter of top-k volume blocks, the "
                         "rest image blocks)")
    ap.add_argument("--serial", action="store_true",
                    help="routing, pooling/packing and forward on one stream (default: routing on a second stream "
                         "beside the pooling/packing pass)")
    ap.add_argument("--two-pass", action="store_true",
                    help="lsrm_nsa_compress, then a forward that repacks k and v itself, instead of the default "
                         "lsrm_nsa_compress_pack + forward with kv_packed (one pass over k and v for both)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-size kernel to scale rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings against)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2604_05182_amd import inputs as I
    from paper_2604_05182_amd import binding as B  # raises if the HIP library is not built

    cfg = I.CONFIGS[args.config]
    if args.topk is not None or args.window is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, topk=cfg.topk if args.topk is None else args.topk,
                                  window=cfg.window if args.window is None else args.window,
                                  name=cfg.name + "-override")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    # ---- seeded synthetic inputs, moved to HBM before anything is timed
    pos, cams = I.make_points(cfg), I.make_cameras(cfg)
    q_bits, k_bits, v_bits = I.make_qkv(cfg)
    gates = I.make_gates(cfg)

    def bf16_dev(bits):
        return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)

    d_pos, d_cams = torch.from_numpy(pos).to(dev), torch.from_numpy(cams).to(dev)
    d_q, d_k, d_v = bf16_dev(q_bits), bf16_dev(k_bits), bf16_dev(v_bits)
    d_gates = torch.from_numpy(gates).to(dev)
    p = B.make_params(cfg.n_obj, cfg.n_views, cfg.grid, cfg.heads, cfg.d, cfg.topk, cfg.window, h_kv=cfg.kv_heads,
                      gate_channels=cfg.gate_channels)
    d_idx = torch.empty((cfg.nb, cfg.topk), dtype=torch.int32, device=dev)
    d_kc = torch.empty((cfg.nb, cfg.kv_heads, cfg.d), dtype=torch.bfloat16, device=dev)
    d_vc = torch.empty_like(d_kc)
    d_out = torch.empty((cfg.n, cfg.heads, cfg.d), dtype=torch.bfloat16, device=dev)
    ws_route = B.alloc_workspace(p, B.LSRM_WS_ROUTE)
    ws_fwd = B.alloc_workspace(p, B.LSRM_WS_FORWARD)
    if not (args.two_pass or args.config == 5 or args.backward):
        p.kv_packed = 1
    four_rule = args.routing == "four-rule" or args.config in I.ROUTE3D
    if four_rule:
        k_vol = I.ROUTE3D[args.config]["k_v2v"] if args.config in I.ROUTE3D else cfg.topk // 4
        r3d = B.lsrm_route3d_params(4, k_vol, cfg.topk - k_vol, k_vol, cfg.topk - k_vol)
        d_pos_img = torch.from_numpy(I.make_points_img(cfg, cams)).to(dev)
        ws_route = B.alloc_workspace(p, B.LSRM_WS_ROUTE_3D)

    def route(stream=None):
        if four_rule:
            B.lsrm_route_blocks_3d(p, r3d, d_pos, d_pos_img, d_cams, d_idx, None, ws_route, stream=stream)
        else:
            B.lsrm_route_blocks(p, d_pos, d_cams, d_idx, None, ws_route, stream=stream)

    if args.config == 5 or args.backward:
        run_backward_bench(args, cfg, B, I, p, dev, (d_q, d_k, d_v, d_kc, d_vc, d_idx, d_gates, d_out, d_pos, d_cams),
                           (ws_route, ws_fwd), (q_bits, k_bits, v_bits, gates), route)
        return

    n_ev = args.steps
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(n_ev)]
    warm_ev = [torch.cuda.Event(enable_timing=True) for _ in range(8)]
    for row in ev + [warm_ev]:
        for e in row:
            e.record()  # creates the underlying hipEvent handles
    # Routing (positions and cameras -> table) and pooling/packing (K, V -> pooled pairs and tile images) do not depend
    # on each other: the step runs routing on a second stream (default priority) beside the pooling/packing pass, and
    # the forward waits for both.  --serial puts the three calls on one stream.
    main_stream = torch.cuda.current_stream()
    side_stream = main_stream if args.serial else torch.cuda.Stream()

    def step(i=None):
        e = ev[i] if i is not None else warm_ev
        e[0].record(main_stream)
        if not args.serial:
            side_stream.wait_event(e[0])  # the previous step's forward has read the routing table
        e[6].record(side_stream)
        route(stream=side_stream)
        e[1].record(side_stream)
        if args.two_pass:
            B.lsrm_nsa_compress(p, d_k, d_v, d_kc, d_vc)
        else:
            B.lsrm_nsa_compress_pack(p, d_k, d_v, d_kc, d_vc, ws_fwd)
        e[2].record(main_stream)
        if not args.serial:
            main_stream.wait_event(e[1])
        e[7].record(main_stream)
        B.lsrm_nsa_forward(p, d_q, d_k, d_v, d_kc, d_vc, d_idx, d_gates, d_out, None, None, ws_fwd,
                           ev_attn_start=e[3], ev_attn_stop=e[4])
        e[5].record(main_stream)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall * 1e3 / args.steps
    ms_route = float(np.mean([e[6].elapsed_time(e[1]) for e in ev]))
    ms_compress = float(np.mean([(e[0] if not args.serial else e[1]).elapsed_time(e[2]) for e in ev]))
    ms_fwd_call = float(np.mean([e[7].elapsed_time(e[5]) for e in ev]))
    ms_attn = float(np.mean([e[3].elapsed_time(e[4]) for e in ev]))

    idx = d_idx.cpu().numpy()
    n_valid = int((idx >= 0).sum())
    flops = cfg.forward_flops(n_valid)
    value = flops / (ms_step * 1e-3) / 1e12
    attn_tflops = flops / (ms_attn * 1e-3) / 1e12

    result = {
        "metric": "NSA layer effective TFLOP/s (route + compress + fused forward), 1 MI355X",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"config {args.config} ({cfg.name}): {cfg.n_obj} object + {cfg.n_views}x{cfg.grid}x{cfg.grid} image "
                        f"tokens = {cfg.n}, {cfg.heads} heads"
                        + (f" on {cfg.kv_heads} key/value heads" if cfg.kv_heads != cfg.heads else "")
                        + f", d {cfg.d}, block 64, top-k {cfg.topk}, window {cfg.window}"
                        + (", per-channel gates" if cfg.gate_channels else "")
                        + (f", four-rule routing (B^i 4, {k_vol} volume + {cfg.topk - k_vol} image blocks)"
                           if four_rule else ""),
            "effective_flops": flops,
            "pct_of_bf16_mfma_peak": round(100.0 * value / BF16_MFMA_PEAK_TFLOPS, 2),
            "streams": "one" if args.serial else "routing on a second stream beside the pooling/packing pass",
        },
        "breakdown_ms": {"route": round(ms_route, 4), "compress": round(ms_compress, 4),
                         "forward_call": round(ms_fwd_call, 4), "attention_kernel": round(ms_attn, 4)},
        "roofline": {
            "kernel": "nsa_forward_kernel",
            "bound": "mfma",
            "achieved": round(attn_tflops, 3),
            "peak": BF16_MFMA_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(attn_tflops / BF16_MFMA_PEAK_TFLOPS, 4),
            "traffic": (MEASURED_HBM_BYTES.get(args.config)
                        if args.topk is None and args.window is None and not four_rule else None),
            "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated)",
        },
    }
    # the whole lsrm_nsa_forward call (step schedule, packing of the pooled pairs, attention kernel; with --two-pass also
    # the packing of k and v) against the same peak
    call_tflops = flops / (ms_fwd_call * 1e-3) / 1e12
    result["roofline_call"] = {"call": "lsrm_nsa_forward", "bound": "mfma", "achieved": round(call_tflops, 3),
                               "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                               "frac": round(call_tflops / BF16_MFMA_PEAK_TFLOPS, 4)}
    if cfg.d <= 64:
        # At d <= 64 the softmax arithmetic, not the matrix pipe, bounds the kernel: a 32 x 32 score tile costs 8 MFMAs
        # at d = 64 (4 at d = 32) but always 1024 exponentials.  Per score element and head the kernel issues one
        # fused scale-and-subtract, one exponential (a quarter-rate instruction: 4 issue slots), one add into the row
        # sum and half a packed bf16 conversion -- 6.5 slots; 8 are charged, the rest being the share of the
        # per-tile work (operand address updates, overflow test of the optimistic running maximum, masks at the
        # edges).  Peak issue rate: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz.  At d = 64 the matrix-pipe time at the
        # bf16 peak is half of the vector-pipe time at this peak, at d = 32 a quarter.
        p_all = cfg.forward_pairs(n_valid)
        slots = 8.0 * cfg.heads * (p_all["cmp"] + p_all["sel"] + p_all["win"])
        peak = 256 * 4 * 16 * 2.4e9 / 1e12
        ach = slots / (ms_attn * 1e-3) / 1e12
        result["roofline"] = {"kernel": "nsa_forward_kernel", "bound": "alu", "achieved": round(ach, 3),
                              "peak": round(peak, 2), "unit": "T fp32 lane-op slots/s", "frac": round(ach / peak, 4),
                              "traffic": None,
                              "mfma_tflops": round(attn_tflops, 3),
                              "mfma_frac": round(attn_tflops / BF16_MFMA_PEAK_TFLOPS, 4)}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, {"qkv_bits": (q_bits, k_bits, v_bits), "gates": gates}, idx)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
