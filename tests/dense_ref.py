"""Dense-mask formulation of the NSA layer in float64 numpy / torch.

An independent second formulation used to pin the CPU oracle: instead of gathering
key lists per query, every branch is an ordinary masked softmax attention over a
full score matrix (App. A, Eq. nsa_1: three separate softmaxes, gated sum).  Only
usable for small N.
"""
import numpy as np


def group_ids(n, group_offsets):
    """Spatial block (group) of every token; group_offsets [ng + 1] in 64-slot blocks, None: one group per block."""
    if group_offsets is None:
        return np.arange(n) // 64
    off = np.asarray(group_offsets)
    return np.repeat(np.repeat(np.arange(len(off) - 1), np.diff(off)), 64)


def pooled(x, block_count=None, group_offsets=None):
    """Mean over the active tokens of every spatial block: a membership matrix times x, over its row sums."""
    n, h, d = x.shape
    active = np.ones(n, dtype=bool) if block_count is None else (np.arange(n) % 64) < np.repeat(np.asarray(block_count), 64)
    gid = group_ids(n, group_offsets)
    member = ((gid[None, :] == np.arange(gid.max() + 1)[:, None]) & active[None, :]).astype(x.dtype)   # [groups, n]
    return np.einsum("gn,nhc->ghc", member, x) / member.sum(axis=1)[:, None, None]


def masks(n, idx, seg_offsets, window, window_mode=0, block_count=None, group_offsets=None):
    """Boolean [n, n] masks of the selected and window branches.  window_mode 1: the window is the
    query's own block (its whole spatial block with group_offsets).  block_count: slots at or beyond a
    block's count are nobody's key."""
    nb = n // 64
    sel = np.zeros((n, n), dtype=bool)
    for qb in range(nb):
        for kb in idx[qb]:
            if kb >= 0:
                sel[qb * 64:(qb + 1) * 64, kb * 64:(kb + 1) * 64] = True
    seg_id = np.full(n, -1)
    for s, (a, b) in enumerate(zip(seg_offsets[:-1], seg_offsets[1:])):
        seg_id[a:b] = s
    i = np.arange(n)[:, None]
    j = np.arange(n)[None, :]
    win = (seg_id[:, None] == seg_id[None, :]) & (seg_id[:, None] >= 0) & (j - i >= -(window // 2)) & (j - i < window // 2)
    if window_mode == 1:
        gid = group_ids(n, group_offsets)
        win = gid[:, None] == gid[None, :]
    if block_count is not None:
        active = (np.arange(n) % 64) < np.repeat(np.asarray(block_count), 64)
        sel = sel & active[None, :]
        win = win & active[None, :]
    return sel, win


def masked_attention(q, k, v, mask, scale):
    """q [n,d], k,v [m,d], mask [n,m] -> (o [n,d], lse [n], p [n,m])."""
    s = (q @ k.T) * scale
    s = np.where(mask, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        p = np.where(l > 0, e / l, 0.0)
        lse = np.where(l[:, 0] > 0, m[:, 0] + np.log(l[:, 0]), -np.inf)
    return p @ v, lse, p


def dense_nsa(q, k, v, idx, gates, seg_offsets, window, scale=None, window_mode=0, block_count=None,
              group_offsets=None):
    """All float64.  Returns out [N,H,d], branches [3,N,H,d], lse [3,N,H].
    Grouped-query heads (k, v with fewer heads than q) are expanded to one key/value head per
    query head first; gates are [N,H,3] or, per channel, [N,3,H,d]."""
    q, k, v, gates = (np.asarray(a, dtype=np.float64) for a in (q, k, v, gates))
    n, h, d = q.shape
    if k.shape[1] != h:
        k, v = (np.repeat(a, h // a.shape[1], axis=1) for a in (k, v))
    scale = 1.0 / np.sqrt(d) if not scale else scale
    kc, vc = pooled(k, block_count, group_offsets), pooled(v, block_count, group_offsets)
    sel, win = masks(n, idx, seg_offsets, window, window_mode, block_count, group_offsets)
    allc = np.ones((n, kc.shape[0]), dtype=bool)
    ob = np.zeros((3, n, h, d))
    lse = np.zeros((3, n, h))
    for hh in range(h):
        ob[0, :, hh], lse[0, :, hh], _ = masked_attention(q[:, hh], kc[:, hh], vc[:, hh], allc, scale)
        ob[1, :, hh], lse[1, :, hh], _ = masked_attention(q[:, hh], k[:, hh], v[:, hh], sel, scale)
        ob[2, :, hh], lse[2, :, hh], _ = masked_attention(q[:, hh], k[:, hh], v[:, hh], win, scale)
    if gates.ndim == 4:
        out = np.einsum("nbhc,bnhc->nhc", gates, ob)
    else:
        out = sum(gates[:, :, b, None] * ob[b] for b in range(3))
    return out, ob, lse


def dense_nsa_torch_grads(q, k, v, idx, gates, seg_offsets, window, dout, scale=None, window_mode=0, block_count=None,
                          group_offsets=None):
    """Library autograd (float64) through the dense-mask formulation -> dq, dk, dv."""
    import torch
    tq, tk0, tv0 = (torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True) for a in (q, k, v))
    g = torch.tensor(np.asarray(gates, dtype=np.float64))
    n, h, d = tq.shape
    # grouped-query heads: every query head gets a view of its key/value head (autograd sums the group)
    tk, tv = (t.repeat_interleave(h // t.shape[1], dim=1) for t in (tk0, tv0))
    if g.ndim == 4:   # per-channel gates [N, 3, H, d] -> [N, H, 3, d]
        g = g.permute(0, 2, 1, 3)
    else:
        g = g[..., None]
    scale = 1.0 / np.sqrt(d) if not scale else scale
    sel, win = masks(n, idx, seg_offsets, window, window_mode, block_count, group_offsets)
    sel, win = torch.tensor(sel), torch.tensor(win)
    if group_offsets is not None:
        act_tok = np.ones(n, dtype=bool) if block_count is None else (np.arange(n) % 64) < np.repeat(np.asarray(block_count), 64)
        gid = group_ids(n, group_offsets)
        member = torch.tensor(((gid[None, :] == np.arange(gid.max() + 1)[:, None]) & act_tok[None, :]).astype(np.float64))
        kc = torch.einsum("gn,nhc->ghc", member, tk) / member.sum(1)[:, None, None]
        vc = torch.einsum("gn,nhc->ghc", member, tv) / member.sum(1)[:, None, None]
        active_q = torch.tensor(act_tok.astype(np.float64))
    elif block_count is None:
        kc = tk.reshape(n // 64, 64, h, d).mean(1)
        vc = tv.reshape(n // 64, 64, h, d).mean(1)
        active_q = torch.ones(n, dtype=torch.float64)
    else:
        cnt = torch.tensor(np.asarray(block_count), dtype=torch.float64)
        act = (torch.arange(64)[None, :] < cnt[:, None]).to(torch.float64)          # [NB, 64]
        kc = (tk.reshape(n // 64, 64, h, d) * act[:, :, None, None]).sum(1) / cnt[:, None, None]
        vc = (tv.reshape(n // 64, 64, h, d) * act[:, :, None, None]).sum(1) / cnt[:, None, None]
        active_q = act.reshape(-1)     # padding slots are not queries: their outputs carry no loss

    def att(qh, kh, vh, mask):
        s = (qh @ kh.T) * scale
        if mask is not None:
            s = s.masked_fill(~mask, float("-inf"))
            empty = ~mask.any(dim=1, keepdim=True)
            s = torch.where(empty, torch.zeros_like(s), s)
            p = torch.softmax(s, dim=1)
            p = torch.where(empty, torch.zeros_like(p), p)
        else:
            p = torch.softmax(s, dim=1)
        return p @ vh

    out = torch.zeros_like(tq)
    outs = []
    for hh in range(h):
        o = (g[:, hh, 0] * att(tq[:, hh], kc[:, hh], vc[:, hh], None)
             + g[:, hh, 1] * att(tq[:, hh], tk[:, hh], tv[:, hh], sel)
             + g[:, hh, 2] * att(tq[:, hh], tk[:, hh], tv[:, hh], win))
        outs.append(o)
    out = torch.stack(outs, dim=1)
    (out * torch.tensor(np.asarray(dout, dtype=np.float64)) * active_q[:, None, None]).sum().backward()
    return tq.grad.numpy(), tk0.grad.numpy(), tv0.grad.numpy()
