"""Seeded synthetic workloads for the NSA layer (inputs only, no method arithmetic).

Everything here produces *inputs*: object points, their Morton order, pinhole
cameras, bf16 Q/K/V, gates.  Routing, pooling and attention live elsewhere (the
HIP library on one side, the CPU oracle on the other); both sides consume the
arrays made here, so neither needs the other.

Sequence layout (object tokens first, then the views):
  token index  [0, n_obj)                      object tokens in Morton order
  then per view m = 0..M-1, S*S patch tokens, tile-major: the (S/8)x(S/8) tile
  grid is walked row-major, and the 8x8 patches of a tile are row-major inside it.
Hence every block is 64 consecutive tokens and block id = token index // 64.

bf16 tensors are carried as numpy uint16 bit patterns.
"""
from __future__ import annotations

import math
import os
from dataclasses import dataclass, field

import numpy as np

BLOCK = 64


@dataclass(frozen=True)
class NSAConfig:
    name: str
    n_obj: int
    n_views: int
    grid: int          # S: patches per image side
    heads: int
    d: int
    topk: int
    window: int
    points: str        # "uniform" | "ellipsoids"
    near_views: int = 0  # views placed at half distance
    seed: int = 0
    h_kv: int = 0        # key/value heads (0 = same as `heads`); query head i reads head i // (heads / h_kv)
    gate_channels: bool = False  # gates per output channel [N, 3, H, d] instead of per head [N, H, 3]

    @property
    def kv_heads(self) -> int:
        return self.h_kv if self.h_kv > 0 else self.heads

    @property
    def n_img(self) -> int:
        return self.n_views * self.grid * self.grid

    @property
    def n(self) -> int:
        return self.n_obj + self.n_img

    @property
    def nb_obj(self) -> int:
        return self.n_obj // BLOCK

    @property
    def tiles_per_view(self) -> int:
        return (self.grid // 8) ** 2

    @property
    def n_tiles(self) -> int:
        return self.n_views * self.tiles_per_view

    @property
    def nb(self) -> int:
        return self.nb_obj + self.n_tiles

    def seg_offsets(self) -> np.ndarray:
        s2 = self.grid * self.grid
        return np.array([0, self.n_obj] + [self.n_obj + (m + 1) * s2 for m in range(self.n_views)],
                        dtype=np.int32)

    def window_pairs(self) -> int:
        """Exact number of (query, key) pairs of the window branch, with segment clipping."""
        total = 0
        offs = self.seg_offsets()
        half = self.window // 2
        for a, b in zip(offs[:-1], offs[1:]):
            length = int(b - a)
            i = np.arange(length, dtype=np.int64)
            lo = np.maximum(0, i - half)
            hi = np.minimum(length, i + half)
            total += int((hi - lo).sum())
        return total

    def forward_pairs(self, n_valid_idx: int | None = None) -> dict:
        if n_valid_idx is None:
            n_valid_idx = self.nb * self.topk
        return {"cmp": self.n * self.nb, "sel": BLOCK * BLOCK * n_valid_idx, "win": self.window_pairs()}

    def forward_flops(self, n_valid_idx: int | None = None) -> float:
        p = self.forward_pairs(n_valid_idx)
        return 4.0 * self.d * self.heads * (p["cmp"] + p["sel"] + p["win"])


CONFIGS = {
    1: NSAConfig("tiny", 4096, 2, 32, 4, 64, 4, 256, "uniform", seed=1001),
    2: NSAConfig("mid", 32768, 6, 64, 16, 64, 16, 512, "uniform", seed=1002),
    3: NSAConfig("large", 131072, 12, 64, 16, 64, 16, 512, "ellipsoids", seed=1003),
    4: NSAConfig("extreme", 262144, 18, 96, 16, 128, 32, 1024, "ellipsoids", near_views=2, seed=1004),
    5: NSAConfig("mid-backward", 32768, 6, 64, 16, 64, 16, 512, "uniform", seed=1002),
    # The paper's attention heads (App. A: 32 query heads of 32 channels on 2 key/value heads, one gate
    # per output channel) with its stage-3 routing budgets (hyper-parameter table of the appendix: 16 volume
    # + 4 M image blocks, M = 16 views of 512 / 8 = 64 patches a side); routed with the four geometric rules.
    6: NSAConfig("paper-heads", 131072, 16, 64, 32, 32, 80, 512, "ellipsoids", seed=1006, h_kv=2, gate_channels=True),
}
ROUTE3D = {6: dict(prefilter=4, k_v2v=16, k_v2i=64, k_i2v=16, k_i2i=64)}  # four-rule budgets of such configs


def small_config(name="unit", n_obj=512, n_views=2, grid=16, heads=2, d=64, topk=3, window=128,
                 points="uniform", seed=7, near_views=0, h_kv=0, gate_channels=False) -> NSAConfig:
    """A config small enough for pure-Python / dense-matrix checks."""
    return NSAConfig(name, n_obj, n_views, grid, heads, d, topk, window, points, near_views, seed, h_kv,
                     gate_channels)


# ----------------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    if b.size < (1 << 22):
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
    out = np.empty(b.shape, dtype=np.float32)
    src, dst = b.reshape(-1), out.reshape(-1).view(np.uint32)
    step = 1 << 22

    def work(i):
        np.left_shift(src[i:i + step], np.uint32(16), out=dst[i:i + step], dtype=np.uint32, casting="unsafe")

    _parallel_for(range(0, src.size, step), work)
    return out


def _n_workers() -> int:
    try:
        return max(1, min(16, len(os.sched_getaffinity(0))))
    except AttributeError:
        return max(1, min(16, os.cpu_count() or 1))


def _parallel_for(items, fn):
    """Runs fn over items on a few threads (numpy releases the GIL in its inner loops)."""
    from concurrent.futures import ThreadPoolExecutor
    items = list(items)
    if len(items) <= 1:
        for it in items:
            fn(it)
        return
    with ThreadPoolExecutor(max_workers=_n_workers()) as pool:
        list(pool.map(fn, items))


# ----------------------------------------------------------------------------- geometry
def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def _random_rotation(rng: np.random.Generator) -> np.ndarray:
    a = rng.standard_normal((3, 3))
    q, r = np.linalg.qr(a)
    q = q * np.sign(np.diag(r))
    if np.linalg.det(q) < 0:
        q[:, 0] = -q[:, 0]
    return q


def _ellipsoid_union_points(n: int, rng: np.random.Generator) -> np.ndarray:
    n_e = int(rng.integers(3, 9))
    centres = rng.uniform(-0.4, 0.4, size=(n_e, 3))
    axes = rng.uniform(0.15, 0.5, size=(n_e, 3))
    rots = np.stack([_random_rotation(rng) for _ in range(n_e)])
    # Knud Thomsen's approximate ellipsoid area, used only as a sampling weight
    p = 1.6075
    a, b, c = axes[:, 0], axes[:, 1], axes[:, 2]
    area = 4 * np.pi * (((a * b) ** p + (a * c) ** p + (b * c) ** p) / 3.0) ** (1.0 / p)
    prob = area / area.sum()
    out = np.empty((0, 3))
    while out.shape[0] < n:
        m = int((n - out.shape[0]) * 1.5) + 1024
        which = rng.choice(n_e, size=m, p=prob)
        g = rng.standard_normal((m, 3))
        g /= np.linalg.norm(g, axis=1, keepdims=True)
        local = g * axes[which]
        world = np.einsum("nij,nj->ni", rots[which], local) + centres[which]
        keep = np.ones(m, dtype=bool)
        for e in range(n_e):
            rel = np.einsum("ji,nj->ni", rots[e], world - centres[e]) / axes[e]
            inside = (rel * rel).sum(1) < 1.0 - 1e-9
            keep &= ~(inside & (which != e))
        out = np.concatenate([out, world[keep]], axis=0)
    out = out[:n]
    r = np.linalg.norm(out, axis=1).max()
    if r > 0.98:
        out = out * (0.98 / r)
    return out


def morton_order(pos: np.ndarray) -> np.ndarray:
    """Stable argsort by 30-bit Morton code (10 bits per axis over [-1, 1])."""
    q = np.clip(np.floor((pos.astype(np.float64) + 1.0) * 512.0), 0, 1023).astype(np.uint64)

    def spread(v):
        v = v & np.uint64(0x3FF)
        v = (v | (v << np.uint64(16))) & np.uint64(0x030000FF)
        v = (v | (v << np.uint64(8))) & np.uint64(0x0300F00F)
        v = (v | (v << np.uint64(4))) & np.uint64(0x030C30C3)
        v = (v | (v << np.uint64(2))) & np.uint64(0x09249249)
        return v

    code = spread(q[:, 0]) | (spread(q[:, 1]) << np.uint64(1)) | (spread(q[:, 2]) << np.uint64(2))
    return np.argsort(code, kind="stable")


def make_points(cfg: NSAConfig) -> np.ndarray:
    """Object-token positions, float32 [n_obj, 3], already in Morton (sequence) order."""
    rng = _rng(cfg.seed, 1)
    if cfg.points == "uniform":
        pts = rng.uniform(-1.0, 1.0, size=(cfg.n_obj, 3))
    elif cfg.points == "ellipsoids":
        pts = _ellipsoid_union_points(cfg.n_obj, rng)
    else:
        raise ValueError(cfg.points)
    pts = pts.astype(np.float32)
    return np.ascontiguousarray(pts[morton_order(pts)])


CAM_FLOATS = 16  # R[9] row-major world->camera, t[3], fx, fy, cx, cy


def make_cameras(cfg: NSAConfig, radius: float = 2.5, fov_deg: float = 40.0) -> np.ndarray:
    """Pinhole cameras looking at the origin, float32 [M, 16]; intrinsics in patch units.

    x_cam = R @ p + t, (u, v) = (fx * x/z + cx, fy * y/z + cy); the centre of patch
    (row r, column c) is at (u, v) = (c + 0.5, r + 0.5).
    """
    rng = _rng(cfg.seed, 2)
    cams = np.zeros((cfg.n_views, CAM_FLOATS), dtype=np.float64)
    up = np.array([0.0, 0.0, 1.0])
    f = (cfg.grid / 2.0) / math.tan(math.radians(fov_deg / 2.0))
    for m in range(cfg.n_views):
        while True:
            c = rng.standard_normal(3)
            c /= np.linalg.norm(c)
            if abs(c @ up) <= 0.99:
                break
        rad = radius * (0.5 if m < cfg.near_views else 1.0)
        centre = c * rad
        fwd = -c
        right = np.cross(fwd, up)
        right /= np.linalg.norm(right)
        down = np.cross(fwd, right)
        rot = np.stack([right, down, fwd])
        t = -rot @ centre
        cams[m, :9] = rot.reshape(-1)
        cams[m, 9:12] = t
        cams[m, 12:16] = (f, f, cfg.grid / 2.0, cfg.grid / 2.0)
    return cams.astype(np.float32)


def image_token_patch(cfg: NSAConfig):
    """(view, row, col) int arrays [n_img] of every image token, in sequence (tile-major) order."""
    s, tg = cfg.grid, cfg.grid // 8
    i = np.arange(cfg.n_img, dtype=np.int64)
    view, r = i // (s * s), i % (s * s)
    tile, inner = r // BLOCK, r % BLOCK
    row = (tile // tg) * 8 + inner // 8
    col = (tile % tg) * 8 + inner % 8
    return view, row, col


def make_points_img(cfg: NSAConfig, cams: np.ndarray) -> np.ndarray:
    """A 3-D point for every image token, float32 [n_img, 3] in sequence order: where the ray
    through the patch centre first meets a rough sphere around the origin (radius drawn per
    token from U(0.6, 0.8)); a ray that misses takes its point nearest to the origin.  Stands
    in for the rendered surface point of a patch (synthetic: no renderer, no trained volume)."""
    rng = _rng(cfg.seed, 3)
    view, row, col = image_token_patch(cfg)
    c = cams.astype(np.float64)
    rot = c[:, :9].reshape(-1, 3, 3)
    centre = -np.einsum("mji,mj->mi", rot, c[:, 9:12])             # -R^T t
    fx, fy, cx, cy = (c[view, 12 + j] for j in range(4))
    d_cam = np.stack([(col + 0.5 - cx) / fx, (row + 0.5 - cy) / fy, np.ones(cfg.n_img)], axis=1)
    d = np.einsum("nji,nj->ni", rot[view], d_cam)                   # R^T d_cam
    d /= np.linalg.norm(d, axis=1, keepdims=True)
    o = centre[view]
    radius = rng.uniform(0.6, 0.8, size=cfg.n_img)
    b = (o * d).sum(1)
    disc = b * b - ((o * o).sum(1) - radius * radius)
    s_hit = -b - np.sqrt(np.maximum(disc, 0.0))
    s_par = np.where(disc >= 0.0, s_hit, -b)
    return np.ascontiguousarray((o + s_par[:, None] * d).astype(np.float32))


# ----------------------------------------------------------------------------- tensors
def _normal_bf16(shape, seed: int, stream: int, chunk_rows: int = 1 << 12) -> np.ndarray:
    """N(0,1) rounded to bf16.  Chunk c of 4096 rows draws from its own counter-based Philox
    stream keyed by (seed, stream, c), so the result does not depend on the thread count."""
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(shape[0], -1)

    def work(c):
        r0 = c * chunk_rows
        r1 = min(shape[0], r0 + chunk_rows)
        rng = np.random.Generator(np.random.Philox(key=[seed, (stream << 32) + c]))
        x = rng.standard_normal((r1 - r0, flat.shape[1]), dtype=np.float32)
        flat[r0:r1] = f32_to_bf16_bits(x)

    _parallel_for(range((shape[0] + chunk_rows - 1) // chunk_rows), work)
    return out


def make_qkv(cfg: NSAConfig):
    """(q, k, v) bf16 bit patterns, uint16: q [N, H, d], k and v [N, h_kv, d]; values ~ N(0, 1)
    rounded to bf16."""
    return tuple(_normal_bf16((cfg.n, cfg.heads if i == 0 else cfg.kv_heads, cfg.d), cfg.seed, 10 + i)
                 for i in range(3))


def make_gates(cfg: NSAConfig) -> np.ndarray:
    """Gate weights sigmoid(N(0,1)), float32, branch order (cmp, sel, win): [N, H, 3], or
    [N, 3, H, d] when the config asks for one gate per output channel."""
    rng = _rng(cfg.seed, 20)
    shape = (cfg.n, 3, cfg.heads, cfg.d) if cfg.gate_channels else (cfg.n, cfg.heads, 3)
    g = rng.standard_normal(shape, dtype=np.float32)
    return (1.0 / (1.0 + np.exp(-g.astype(np.float64)))).astype(np.float32)


def make_dout(cfg: NSAConfig) -> np.ndarray:
    return _normal_bf16((cfg.n, cfg.heads, cfg.d), cfg.seed, 30)


def sample_query_blocks(cfg: NSAConfig, n_random: int, seed: int = 0) -> np.ndarray:
    """First and last block of every segment plus n_random others (sorted, unique)."""
    offs = cfg.seg_offsets() // BLOCK
    edge = set()
    for a, b in zip(offs[:-1], offs[1:]):
        edge.add(int(a))
        edge.add(int(b) - 1)
    rng = _rng(cfg.seed + 77 + seed, 40)
    extra = rng.choice(cfg.nb, size=min(n_random, cfg.nb), replace=False)
    return np.array(sorted(edge | set(int(e) for e in extra)), dtype=np.int32)


def sample_query_blocks_stratified(cfg: NSAConfig, per_stratum: int, slots: int = 4, ranges: int = 8,
                                   seed: int = 0) -> np.ndarray:
    """First and last block of every segment, `per_stratum` random blocks for every combination of
    (block id mod `slots`, which of `ranges` equal contiguous ranges of block groups the block falls in), and
    the blocks on either side of every range boundary (sorted, unique).  A group is `slots` consecutive
    blocks; the ranges are ceil(groups / ranges) groups long."""
    groups = (cfg.nb + slots - 1) // slots
    per_range = (groups + ranges - 1) // ranges
    blocks = np.arange(cfg.nb)
    slot, rng_id = blocks % slots, (blocks // slots) // per_range
    picked = set(int(b) for b in sample_query_blocks(cfg, 0))
    rng = _rng(cfg.seed + 91 + seed, 41)
    for s in range(slots):
        for r in range(ranges):
            pool = blocks[(slot == s) & (rng_id == r)]
            if pool.size:
                picked.update(int(b) for b in rng.choice(pool, size=min(per_stratum, pool.size), replace=False))
    for r in range(1, ranges):
        edge = r * per_range * slots
        picked.update(b for b in (edge - 1, edge) if 0 <= b < cfg.nb)
    return np.array(sorted(picked), dtype=np.int32)
