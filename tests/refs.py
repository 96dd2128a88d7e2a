"""Independent numpy statements of window attention, used only to pin the oracle.

Nothing here is shared with ``oracle/`` or with the HIP library.  Two routes:

* ``global_attention``: attention over ALL tokens of an image at once with an
  additive [HW, HW] matrix that encodes "same shifted window", the wrap mask and
  the relative bias.  It never forms a window tensor.
* ``dense_window_msa``: the textbook shifted-window attention done with array
  copies (roll, reshape into windows, einsum, explicit mask tensor, reverse).
"""
import numpy as np


def _softmax(s, axis=-1):
    s = s - s.max(axis=axis, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=axis, keepdims=True)


def global_additive_matrix(H, W, M, s, table_h):
    """[HW, HW] additive term for one head; table_h is the head's column [(2M-1)^2].

    Tokens are taken at their positions (pi, pj) in x.  A token's coordinate in
    the rolled frame is (pi - s) mod H; a token was wrapped along an axis iff
    its original coordinate is < s.  Two tokens interact iff they fall in the
    same window of the rolled frame; inside a window, pairs with different wrap
    flags get -100, all other pairs get the bias of their coordinate offset.
    """
    pi, pj = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    pi, pj = pi.reshape(-1), pj.reshape(-1)
    fi, fj = (pi - s) % H, (pj - s) % W
    win = (fi // M) * (W // M) + (fj // M)
    wrap = 2 * (pi < s).astype(int) + (pj < s).astype(int)
    r, c = fi % M, fj % M
    same_win = win[:, None] == win[None, :]
    same_wrap = wrap[:, None] == wrap[None, :]
    dr = r[:, None] - r[None, :] + (M - 1)
    dc = c[:, None] - c[None, :] + (M - 1)
    idx = np.clip(dr, 0, 2 * M - 2) * (2 * M - 1) + np.clip(dc, 0, 2 * M - 2)
    add = np.where(same_win, table_h[idx], -np.inf)
    add = np.where(same_win & ~same_wrap, -100.0, add)
    return add


def global_attention(feat, w_qkv, b_qkv, table, nheads, M, s, dqk=0):
    """Multi-head attention core without output projection, via global attention.

    feat [B,H,W,Cc]; w_qkv [2Q+Cc,Cc]; b_qkv [2Q+Cc], Q = nheads*dqk channels of q and of k
    (dqk = 0: Q = Cc); table [(2M-1)^2, nheads].
    Returns [B,H,W,Cc] at the tokens' own positions.
    """
    B, H, W, Cc = feat.shape
    d = Cc // nheads
    e = dqk or d
    Q = nheads * e
    t = feat.reshape(B, H * W, Cc).astype(np.float64)
    qkv = t @ w_qkv.T.astype(np.float64) + b_qkv
    q, k, v = qkv[..., :Q], qkv[..., Q:2 * Q], qkv[..., 2 * Q:]
    out = np.empty_like(t)
    for h in range(nheads):
        sl, sle = slice(h * d, (h + 1) * d), slice(h * e, (h + 1) * e)
        add = global_additive_matrix(H, W, M, s, table[:, h].astype(np.float64))
        sc = np.einsum("bnd,bmd->bnm", q[..., sle], k[..., sle]) / np.sqrt(e) + add[None]
        out[..., sl] = _softmax(sc) @ v[..., sl]
    return out.reshape(B, H, W, Cc)


def grouped_by_composition(x, p, heads, groups, M, s, cascade=True, core=global_attention, dqk=0):
    """GSWA as a chain of plain multi-head cores on channel slices + one dense projection."""
    B, H, W, C = x.shape
    Cg, hg = C // groups, heads // groups
    outs = []
    prev = None
    for g in range(groups):
        f = x[..., g * Cg:(g + 1) * Cg].astype(np.float64)
        if g > 0 and cascade:
            f = f + prev
        prev = core(f, p["w_qkv"][g], p["b_qkv"][g], p["table"][:, g * hg:(g + 1) * hg], hg, M, s,
                    **({"dqk": dqk} if dqk else {}))
        outs.append(prev)
    a = np.concatenate(outs, axis=-1)
    return a @ p["w_proj"].T.astype(np.float64) + p["b_proj"], a


def dense_window_msa(feat, w_qkv, b_qkv, table, nheads, M, s, dqk=0):
    """Textbook (shifted-)window multi-head attention core with array copies; no projection.
    dqk: channels per head of q and k when they differ from those of v."""
    B, H, W, Cc = feat.shape
    d, N = Cc // nheads, M * M
    e = dqk or d
    f = np.roll(feat.astype(np.float64), shift=(-s, -s), axis=(1, 2)) if s else feat.astype(np.float64)

    def to_windows(a):
        ch = a.shape[-1]
        return a.reshape(B, H // M, M, W // M, M, ch).transpose(0, 1, 3, 2, 4, 5).reshape(-1, N, ch)

    win = to_windows(f)                                            # [nW*B, N, Cc]
    proj = win @ w_qkv.T + b_qkv
    qk = proj[..., :2 * nheads * e].reshape(-1, N, 2, nheads, e).transpose(2, 0, 3, 1, 4)
    q, k = qk[0], qk[1]                                            # [nWB, h, N, e]
    v = proj[..., 2 * nheads * e:].reshape(-1, N, nheads, d).transpose(0, 2, 1, 3)
    att = np.einsum("whnd,whmd->whnm", q, k) * e ** -0.5

    # relative position index table
    coords = np.stack(np.meshgrid(np.arange(M), np.arange(M), indexing="ij")).reshape(2, -1)
    rel = coords[:, :, None] - coords[:, None, :] + (M - 1)        # [2, N, N]
    rel_index = rel[0] * (2 * M - 1) + rel[1]
    att = att + table[rel_index].transpose(2, 0, 1)[None]          # [1, h, N, N]

    if s:
        label = np.zeros((1, H, W, 1))
        cuts = (slice(0, -M), slice(-M, -s), slice(-s, None))
        cnt = 0
        for hs in cuts:
            for ws in cuts:
                label[:, hs, ws, :] = cnt
                cnt += 1
        lw = label.reshape(1, H // M, M, W // M, M, 1).transpose(0, 1, 3, 2, 4, 5).reshape(-1, N)
        mask = np.where(lw[:, :, None] != lw[:, None, :], -100.0, 0.0)   # [nW, N, N]
        nW = mask.shape[0]
        att = att.reshape(B, nW, nheads, N, N) + mask[None, :, None]
        att = att.reshape(-1, nheads, N, N)
    o = (_softmax(att) @ v).transpose(0, 2, 1, 3).reshape(-1, N, Cc)
    o = o.reshape(B, H // M, W // M, M, M, Cc).transpose(0, 1, 3, 2, 4, 5).reshape(B, H, W, Cc)
    return np.roll(o, shift=(s, s), axis=(1, 2)) if s else o


def as_f64(p):
    return {k: np.asarray(v, dtype=np.float64) for k, v in p.items()}
