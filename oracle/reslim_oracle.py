"""CPU oracle for the Reslim ViT forward under TILES (ORBIT-2, Sec. 4.1 and 4.2).

TEST INFRASTRUCTURE ONLY.  Plain numpy in float64, written step by step from the
paper's description; slow on purpose, no blocking or fusion.  It shares no code
with the HIP library and is imported only by tests, the smoke check and the
benchmark's CPU-baseline leg.  Library primitives used as steps: `@` (matmul),
`np.exp`, `scipy.special.erf`.

Where the paper is silent the reading taken is stated beside the function.  Parts whose *choice of operation* the paper
does not fix (the residual path's upsampler and kernel, the decoder reduced to a
linear projection) are "parity unpinned" against the paper; they are pinned only
against textbook definitions (bilinear interpolation, zero-padded correlation).

Two forms of the whole forward are given:
  * `reslim_forward`         embeds once, gathers tokens tile-major, runs every
                             tile, keeps interiors (the batched form);
  * `reslim_forward_literal` Sec. 4.2 taken literally: cut the input field into
                             haloed tiles, run the *untiled* model on each cut,
                             drop the halo of each output, stitch.
Their agreement to rounding is one of the oracle's pins.
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# ============================================================================
# Sec. 4.2  TILES: partition, halo, crop + stitch indices  (integers only)
# ============================================================================
def tiles_partition(Hp: int, Wp: int, Ty: int, Tx: int, halo: int):
    """Tile table for a patch grid of Hp x Wp cut into Ty x Tx tiles (Sec. 4.2).

    Readings: the cut is balanced (tile row i covers patch rows
    [floor(i*Hp/Ty), floor((i+1)*Hp/Ty))), the halo is `halo` patches wide and is
    clipped at the domain edge, tokens inside a tile are ordered row-major over
    the haloed box, tiles are ordered row-major over the tile grid.

    Returns (tiles, gather_idx, interior_src, n_h):
      tiles[t]        dict with interior box y0,y1,x0,x1, haloed box Y0,Y1,X0,X1
                      (patch units, half-open), tok_off, n_tok
      gather_idx[k]   global patch id (y*Wp + x) of tile-major token k
      interior_src[g] tile-major token index holding global patch g inside the one
                      tile whose interior (not halo) contains it
    """
    if min(Hp, Wp, Ty, Tx) < 1 or halo < 0 or Ty > Hp or Tx > Wp:
        raise ValueError("invalid tiling")
    tiles: List[dict] = []
    gather: List[int] = []
    interior_src = [-1] * (Hp * Wp)
    off = 0
    for i in range(Ty):
        y0, y1 = (i * Hp) // Ty, ((i + 1) * Hp) // Ty
        for j in range(Tx):
            x0, x1 = (j * Wp) // Tx, ((j + 1) * Wp) // Tx
            Y0, Y1 = max(0, y0 - halo), min(Hp, y1 + halo)
            X0, X1 = max(0, x0 - halo), min(Wp, x1 + halo)
            n_tok = (Y1 - Y0) * (X1 - X0)
            tiles.append(dict(y0=y0, y1=y1, x0=x0, x1=x1, Y0=Y0, Y1=Y1, X0=X0, X1=X1,
                              tok_off=off, n_tok=n_tok))
            for y in range(Y0, Y1):
                for x in range(X0, X1):
                    k = off + (y - Y0) * (X1 - X0) + (x - X0)
                    gather.append(y * Wp + x)
                    if y0 <= y < y1 and x0 <= x < x1:
                        interior_src[y * Wp + x] = k
            off += n_tok
    return (tiles, np.asarray(gather, dtype=np.int32),
            np.asarray(interior_src, dtype=np.int32), off)


def attention_pair_count(tiles: Sequence[dict]) -> int:
    """Number of (query, key) pairs tile-local attention evaluates: sum of n_t^2.
    Sec. 4.2 states the cost as O(N^2 / T), linear in N for a fixed tile size."""
    return sum(t["n_tok"] ** 2 for t in tiles)


# ============================================================================
# Textbook pieces of a transformer block (Sec. 3: "self-attention and
# feedforward sub-layers"); reading: pre-LN ViT block, biases, erf-GELU.
# ============================================================================
def linear(x, w, b=None):
    """y = x W^T + b with W stored [out, in]."""
    y = np.asarray(x, F64) @ np.asarray(w, F64).T
    return y if b is None else y + np.asarray(b, F64)


def layer_norm(x, gamma, beta, eps: float = 1e-5):
    """Per-row normalisation over the last axis, biased variance, then affine."""
    x = np.asarray(x, F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, F64) + np.asarray(beta, F64)


def gelu(x):
    """Exact GELU: x * Phi(x), Phi the standard normal CDF."""
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def softmax(s, axis: int = -1):
    s = np.asarray(s, F64)
    e = np.exp(s - s.max(axis=axis, keepdims=True))
    return e / e.sum(axis=axis, keepdims=True)


def self_attention(q, k, v, heads: int):
    """Multi-head softmax(Q K^T / sqrt(dh)) V over ONE token set.
    q, k, v: [n, D]; head g owns columns [g*dh, (g+1)*dh)."""
    q, k, v = (np.asarray(a, F64) for a in (q, k, v))
    n, D = q.shape
    dh = D // heads
    out = np.empty((n, D), F64)
    for g in range(heads):
        c = slice(g * dh, (g + 1) * dh)
        p = softmax(q[:, c] @ k[:, c].T / math.sqrt(dh), axis=-1)
        out[:, c] = p @ v[:, c]
    return out


def tiles_attention(qkv, tiles: Sequence[dict], heads: int):
    """Sec. 4.2: self-attention restricted to each tile.  Halo tokens are ordinary
    members of their tile (queries and keys).
    qkv: [B, n_h, 3*D] with columns ordered (q | k | v), each split into heads.
    Returns [B, n_h, D]."""
    qkv = np.asarray(qkv, F64)
    B, n_h, D3 = qkv.shape
    D = D3 // 3
    out = np.empty((B, n_h, D), F64)
    for b in range(B):
        for t in tiles:
            r = slice(t["tok_off"], t["tok_off"] + t["n_tok"])
            blk = qkv[b, r]
            out[b, r] = self_attention(blk[:, :D], blk[:, D:2 * D], blk[:, 2 * D:], heads)
    return out


def tiles_attention_lse(qkv, tiles: Sequence[dict], heads: int):
    """Natural log of the softmax denominator of every query and head,
    log sum_j exp(q_i . k_j / sqrt(dh)) over the keys of query i's tile: [B, heads, n_h]."""
    qkv = np.asarray(qkv, F64)
    B, n_h, D3 = qkv.shape
    D = D3 // 3
    dh = D // heads
    out = np.empty((B, heads, n_h), F64)
    for b in range(B):
        for t in tiles:
            r = slice(t["tok_off"], t["tok_off"] + t["n_tok"])
            for g in range(heads):
                s = qkv[b, r, g * dh:(g + 1) * dh] @ qkv[b, r, D + g * dh:D + (g + 1) * dh].T / math.sqrt(dh)
                m = s.max(axis=-1)
                out[b, g, r] = m + np.log(np.exp(s - m[:, None]).sum(axis=-1))
    return out


def self_attention_bwd(q, k, v, d_out, heads: int):
    """Gradient of self_attention (one token set) with respect to q, k, v for an
    upstream gradient d_out of its output -- the chain rule written out (training of
    the model of Sec. 4.1 needs it; the paper gives no formula of its own):
        P = softmax(S), S = Q K^T / sqrt(dh), O = P V
        dV = P^T dO,   dP = dO V^T,   dS_ij = P_ij (dP_ij - sum_l P_il dP_il),
        dQ = dS K / sqrt(dh),   dK = dS^T Q / sqrt(dh).
    Returns (dq, dk, dv), each [n, D]."""
    q, k, v, d_out = (np.asarray(a, F64) for a in (q, k, v, d_out))
    n, D = q.shape
    dh = D // heads
    dq, dk, dv = np.empty((n, D), F64), np.empty((n, D), F64), np.empty((n, D), F64)
    sc = 1.0 / math.sqrt(dh)
    for g in range(heads):
        c = slice(g * dh, (g + 1) * dh)
        p = softmax(q[:, c] @ k[:, c].T * sc, axis=-1)
        dv[:, c] = p.T @ d_out[:, c]
        dp = d_out[:, c] @ v[:, c].T
        ds = p * (dp - (p * dp).sum(axis=-1, keepdims=True))
        dq[:, c] = ds @ k[:, c] * sc
        dk[:, c] = ds.T @ q[:, c] * sc
    return dq, dk, dv


def tiles_attention_bwd(qkv, d_out, tiles: Sequence[dict], heads: int):
    """Gradient of tiles_attention: tiles do not interact (Sec. 4.2), so it is the
    per-tile gradient.  qkv: [B, n_h, 3*D]; d_out: [B, n_h, D]; returns d_qkv
    [B, n_h, 3*D] with the same (q | k | v) column order."""
    qkv = np.asarray(qkv, F64)
    d_out = np.asarray(d_out, F64)
    B, n_h, D3 = qkv.shape
    D = D3 // 3
    d_qkv = np.empty((B, n_h, D3), F64)
    for b in range(B):
        for t in tiles:
            r = slice(t["tok_off"], t["tok_off"] + t["n_tok"])
            blk = qkv[b, r]
            dq, dk, dv = self_attention_bwd(blk[:, :D], blk[:, D:2 * D], blk[:, 2 * D:], d_out[b, r], heads)
            d_qkv[b, r, :D], d_qkv[b, r, D:2 * D], d_qkv[b, r, 2 * D:] = dq, dk, dv
    return d_qkv


def block_tokens(X, w: Dict[str, np.ndarray], layer: int, heads: int):
    """One pre-LN transformer block on ONE token set X[n, D]."""
    X = np.asarray(X, F64)
    D = X.shape[1]
    a = layer_norm(X, w["ln1_g"][layer], w["ln1_b"][layer])
    qkv = linear(a, w["w_qkv"][layer], w["b_qkv"][layer])
    o = self_attention(qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:], heads)
    X = X + linear(o, w["w_proj"][layer], w["b_proj"][layer])
    u = gelu(linear(layer_norm(X, w["ln2_g"][layer], w["ln2_b"][layer]),
                    w["w_fc1"][layer], w["b_fc1"][layer]))
    return X + linear(u, w["w_fc2"][layer], w["b_fc2"][layer])


# ---- gradients of the block's pieces (the paper trains the model, Sec. 5, and prints no
# formulas: each function is the chain rule through the forward function of the same name)
def linear_bwd(x, w, dy):
    """y = x W^T + b  =>  dx = dy W,  dW = dy^T x,  db = column sums of dy."""
    x, w, dy = (np.asarray(a, F64) for a in (x, w, dy))
    return dy @ w, dy.T @ x, dy.sum(axis=0)


def layer_norm_bwd(x, gamma, dy, eps: float = 1e-5):
    """Gradient of layer_norm.  With xh = (x - mu) / sigma, g = gamma * dy and means over the row:
    dx = (g - mean(g) - xh * mean(g * xh)) / sigma;  dgamma = sum_rows dy * xh;  dbeta = sum_rows dy."""
    x, gamma, dy = (np.asarray(a, F64) for a in (x, gamma, dy))
    mu = x.mean(axis=-1, keepdims=True)
    sig = np.sqrt(((x - mu) ** 2).mean(axis=-1, keepdims=True) + eps)
    xh = (x - mu) / sig
    g = dy * gamma
    dx = (g - g.mean(axis=-1, keepdims=True) - xh * (g * xh).mean(axis=-1, keepdims=True)) / sig
    return dx, (dy * xh).reshape(-1, x.shape[-1]).sum(axis=0), dy.reshape(-1, x.shape[-1]).sum(axis=0)


def gelu_grad(x):
    """d/dx [x Phi(x)] = Phi(x) + x phi(x), phi the standard normal density."""
    x = np.asarray(x, F64)
    return 0.5 * (1.0 + _erf(x / math.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


BLOCK_PARAMS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj", "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def block_tokens_bwd(X, w: Dict[str, np.ndarray], layer: int, heads: int, d_out):
    """Gradient of block_tokens (ONE token set) for an upstream gradient d_out of its output:
    returns (dX, {parameter name: gradient}) with the parameter names of BLOCK_PARAMS.
    The forward is replayed to get the intermediates, then walked backwards."""
    X, d_out = np.asarray(X, F64), np.asarray(d_out, F64)
    D = X.shape[1]
    a1 = layer_norm(X, w["ln1_g"][layer], w["ln1_b"][layer])
    qkv = linear(a1, w["w_qkv"][layer], w["b_qkv"][layer])
    o = self_attention(qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:], heads)
    x_mid = X + linear(o, w["w_proj"][layer], w["b_proj"][layer])
    a2 = layer_norm(x_mid, w["ln2_g"][layer], w["ln2_b"][layer])
    h = linear(a2, w["w_fc1"][layer], w["b_fc1"][layer])
    u = gelu(h)
    g = {}
    # x_out = x_mid + fc2(u)
    d_u, g["w_fc2"], g["b_fc2"] = linear_bwd(u, w["w_fc2"][layer], d_out)
    d_h = d_u * gelu_grad(h)
    d_a2, g["w_fc1"], g["b_fc1"] = linear_bwd(a2, w["w_fc1"][layer], d_h)
    d_ln, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(x_mid, w["ln2_g"][layer], d_a2)
    d_mid = d_out + d_ln
    # x_mid = X + proj(attention(qkv(ln1(X))))
    d_o, g["w_proj"], g["b_proj"] = linear_bwd(o, w["w_proj"][layer], d_mid)
    d_qkv = np.concatenate(self_attention_bwd(qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:], d_o, heads), axis=1)
    d_a1, g["w_qkv"], g["b_qkv"] = linear_bwd(a1, w["w_qkv"][layer], d_qkv)
    d_ln, g["ln1_g"], g["ln1_b"] = layer_norm_bwd(X, w["ln1_g"][layer], d_a1)
    return d_mid + d_ln, g


def reslim_block_bwd(X, tiles: Sequence[dict], w, layer: int, heads: int, d_out):
    """Gradient of reslim_block on the tile-major stream X[B, n_h, D]: every tile is its own
    token set (Sec. 4.2), the parameters are shared, so their gradients add over tiles and samples."""
    X, d_out = np.asarray(X, F64), np.asarray(d_out, F64)
    dX = np.empty_like(X)
    grads = None
    for b in range(X.shape[0]):
        for t in tiles:
            r = slice(t["tok_off"], t["tok_off"] + t["n_tok"])
            dX[b, r], g = block_tokens_bwd(X[b, r], w, layer, heads, d_out[b, r])
            grads = g if grads is None else {k: grads[k] + g[k] for k in g}
    return dX, grads


# ---- dynamic gradient scaling (Sec. 4.4 "Mixed Precision": gradients are taken of a loss multiplied
# by a scale S so that small ones survive bfloat16, divided by S again at the parameter update, and S
# adapts: the paper names PyTorch's scheme, whose documented rule is restated here)
def grads_unscale(grads: Dict[str, np.ndarray], scale: float):
    """Every gradient divided by the scale, and whether any of them holds a non-finite value."""
    out = {k: np.asarray(g, F64) / scale for k, g in grads.items()}
    return out, any(not np.isfinite(g).all() for g in out.values())


def grad_scale_update(scale: float, tracker: int, found_inf: bool, growth: float = 2.0, backoff: float = 0.5,
                      interval: int = 2000):
    """One step of the scale's schedule: a step with a non-finite gradient multiplies the scale by
    `backoff` and restarts the count; `interval` clean steps in a row multiply it by `growth`.
    Returns (scale, tracker)."""
    if found_inf:
        return scale * backoff, 0
    tracker += 1
    if tracker == interval:
        return scale * growth, 0
    return scale, tracker


def reslim_block(X, tiles: Sequence[dict], w, layer: int, heads: int):
    """One block applied to the tile-major stream X[B, n_h, D]: every tile is its
    own token set (Sec. 4.2)."""
    X = np.asarray(X, F64)
    out = np.empty_like(X)
    for b in range(X.shape[0]):
        for t in tiles:
            r = slice(t["tok_off"], t["tok_off"] + t["n_tok"])
            out[b, r] = block_tokens(X[b, r], w, layer, heads)
    return out


# ============================================================================
# Sec. 4.1  main path front end: per-variable tokenisation, cross-attention
# aggregation over variables, resolution embedding
# ============================================================================
def patch_embed(x, w, patch: int):
    """Tokenise every variable separately: e[b, n, v, :] = W_pe[v] vec(patch) +
    b_pe[v] + var_emb[v], vec row-major over the p x p pixels, n = py*Wp + px."""
    x = np.asarray(x, F64)
    B, V, H, W = x.shape
    p = patch
    Hp, Wp = H // p, W // p
    pix = x.reshape(B, V, Hp, p, Wp, p).transpose(0, 2, 4, 1, 3, 5).reshape(B, Hp * Wp, V, p * p)
    e = np.empty((B, Hp * Wp, V, w["w_pe"].shape[1]), F64)
    for v in range(V):
        e[:, :, v, :] = linear(pix[:, :, v, :], w["w_pe"][v], w["b_pe"][v]) + np.asarray(w["var_emb"][v], F64)
    return e


def variable_aggregation(e, w, heads: int):
    """Collapse the variable axis with cross-attention (Sec. 4.1): one learned
    query attends over the V embeddings of a patch, multi-head, then an output
    projection.  e: [..., V, D] -> [..., D]."""
    e = np.asarray(e, F64)
    D = e.shape[-1]
    dh = D // heads
    q = linear(np.asarray(w["agg_q0"], F64), w["agg_wq"], w["agg_bq"])      # [D]
    k = linear(e, w["agg_wk"], w["agg_bk"])                                 # [..., V, D]
    u = linear(e, w["agg_wv"], w["agg_bv"])
    o = np.empty(e.shape[:-2] + (D,), F64)
    for g in range(heads):
        c = slice(g * dh, (g + 1) * dh)
        a = softmax((k[..., c] * q[c]).sum(-1) / math.sqrt(dh), axis=-1)    # [..., V]
        o[..., c] = (a[..., None] * u[..., c]).sum(-2)
    return linear(o, w["agg_wo"], w["agg_bo"])


def embed_tokens(x, w, patch: int, heads: int, res_idx: int, pos_rows=None, chunk: int = 4096):
    """z[b, n, :] for every patch n of the field x[B, V, H, W]: tokenise, aggregate
    variables, add the positional row and the resolution-embedding row.
    `pos_rows[n]` names the row of `pos_emb` patch n uses (global position);
    default: n itself.  Adaptive compression is the identity (Sec. 4.1 allows it)."""
    x = np.asarray(x, F64)
    B, V, H, W = x.shape
    Hp, Wp = H // patch, W // patch
    N = Hp * Wp
    pos_rows = np.arange(N) if pos_rows is None else np.asarray(pos_rows)
    D = w["agg_wo"].shape[0]
    z = np.empty((B, N, D), F64)
    for b in range(B):
        # chunk over patch rows only to bound memory; no arithmetic depends on it
        rows_per = max(1, chunk // Wp)
        for r0 in range(0, Hp, rows_per):
            r1 = min(Hp, r0 + rows_per)
            e = patch_embed(x[b:b + 1, :, r0 * patch:r1 * patch, :], w, patch)[0]
            z[b, r0 * Wp:r1 * Wp] = variable_aggregation(e, w, heads)
    z += np.asarray(w["pos_emb"], F64)[pos_rows][None]
    z += np.asarray(w["res_emb"], F64)[res_idx]
    return z


# ============================================================================
# Sec. 4.1  decoder (linear projection + un-patchify) and residual path
# ============================================================================
def head_project(Xn, w):
    """Per-token linear projection to C * (p*s)^2 fine pixels."""
    return linear(Xn, w["w_head"], w["b_head"])


def unpatchify(P, Hp: int, Wp: int, C: int, ps: int):
    """P[B, Hp*Wp, C*ps*ps] (c slowest, then row, then column inside the patch)
    -> y[B, C, Hp*ps, Wp*ps]."""
    B = P.shape[0]
    return (np.asarray(P).reshape(B, Hp, Wp, C, ps, ps)
            .transpose(0, 3, 1, 4, 2, 5).reshape(B, C, Hp * ps, Wp * ps))


def bilinear_upsample(u, s: int):
    """u[..., h, w] -> [..., h*s, w*s]; output pixel centre d maps to source
    coordinate (d + 0.5)/s - 0.5, neighbours clamped to the array edge."""
    u = np.asarray(u, F64)
    h, wd = u.shape[-2:]

    def taps(n):
        src = (np.arange(n * s, dtype=F64) + 0.5) / s - 0.5
        i0 = np.floor(src).astype(np.int64)
        f = src - i0
        return np.clip(i0, 0, n - 1), np.clip(i0 + 1, 0, n - 1), f

    y0, y1, fy = taps(h)
    x0, x1, fx = taps(wd)
    rows = u[..., y0, :] * (1.0 - fy)[:, None] + u[..., y1, :] * fy[:, None]
    return rows[..., :, x0] * (1.0 - fx) + rows[..., :, x1] * fx


def conv3x3_same(u, wgt, bias):
    """Cross-correlation out[o, y, x] = b[o] + sum_{c,dy,dx} w[o,c,dy,dx] *
    u[c, y+dy-1, x+dx-1], zero outside the array.  u: [Cin, h, w]."""
    u = np.asarray(u, F64)
    wgt = np.asarray(wgt, F64)
    Cin, h, wd = u.shape
    pad = np.zeros((Cin, h + 2, wd + 2), F64)
    pad[:, 1:-1, 1:-1] = u
    out = np.zeros((wgt.shape[0], h, wd), F64) + np.asarray(bias, F64)[:, None, None]
    for dy in range(3):
        for dx in range(3):
            out += np.einsum("oc,chw->ohw", wgt[:, :, dy, dx], pad[:, dy:dy + h, dx:dx + wd])
    return out


def residual_path(x_box, w, s: int):
    """Residual path of Sec. 4.1 on one field cut x_box[V, h, w]: pick the output
    variables, upsample by s (bilinear), one 3x3 convolution with bias.
    Reading (paper names only "upsampling" and "lightweight convolutional layers")."""
    sel = np.asarray(x_box, F64)[np.asarray(w["out_var_idx"])]
    return conv3x3_same(bilinear_upsample(sel, s), w["w_res"], w["b_res"])


# ============================================================================
# Whole forward
# ============================================================================
def reslim_forward(x, w, cfg, return_intermediates: bool = False):
    """Batched form.  cfg needs: patch, scale, heads, depth, tiles_y, tiles_x,
    halo, res_idx, out_vars.  x: [B, V, H, W] -> y: [B, C, s*H, s*W]."""
    x = np.asarray(x, F64)
    B, V, H, W = x.shape
    p, s, C = cfg.patch, cfg.scale, cfg.out_vars
    Hp, Wp = H // p, W // p
    ps = p * s
    tiles, gather_idx, interior_src, n_h = tiles_partition(Hp, Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)

    z = embed_tokens(x, w, p, cfg.heads, cfg.res_idx)                 # [B, N, D]
    X = z[:, gather_idx, :]                                            # [B, n_h, D]
    inter = {"tokens": X.copy()} if return_intermediates else None
    for layer in range(cfg.depth):
        X = reslim_block(X, tiles, w, layer, cfg.heads)
        if inter is not None:
            inter[f"block{layer}"] = X.copy()
    Xn = layer_norm(X, w["lnf_g"], w["lnf_b"])
    P = head_project(Xn[:, interior_src, :], w)                        # halo dropped
    y_main = unpatchify(P, Hp, Wp, C, ps)

    R = np.empty_like(y_main)
    for t in tiles:
        box = x[:, :, t["Y0"] * p:t["Y1"] * p, t["X0"] * p:t["X1"] * p]
        iy0, ix0 = (t["y0"] - t["Y0"]) * ps, (t["x0"] - t["X0"]) * ps
        hy, hx = (t["y1"] - t["y0"]) * ps, (t["x1"] - t["x0"]) * ps
        for b in range(B):
            r = residual_path(box[b], w, s)
            R[b, :, t["y0"] * ps:t["y1"] * ps, t["x0"] * ps:t["x1"] * ps] = \
                r[:, iy0:iy0 + hy, ix0:ix0 + hx]
    y = y_main + R
    if inter is not None:
        inter["y_main"] = y_main
        inter["residual"] = R
        return y, inter
    return y


def untiled_forward(x_box, w, cfg, pos_rows):
    """The model with no tiling on one field cut x_box[V, h, w] (one sample):
    all tokens of the cut attend to each other.  Returns [C, s*h, s*w]."""
    p, s, C = cfg.patch, cfg.scale, cfg.out_vars
    V, h, wd = x_box.shape
    hp, wp = h // p, wd // p
    X = embed_tokens(np.asarray(x_box, F64)[None], w, p, cfg.heads, cfg.res_idx, pos_rows=pos_rows)[0]
    for layer in range(cfg.depth):
        X = block_tokens(X, w, layer, cfg.heads)
    P = head_project(layer_norm(X, w["lnf_g"], w["lnf_b"]), w)
    y = unpatchify(P[None], hp, wp, C, p * s)[0]
    return y + residual_path(x_box, w, s)


def forward_tile(x_b, w, cfg, tile: dict, Wp: int):
    """Sec. 4.2 for one tile of one sample x_b[V, H, W]: cut the haloed box out of
    the field, downscale it on its own, discard the halo.  Returns the fine
    interior [C, (y1-y0)*p*s, (x1-x0)*p*s]."""
    p, s = cfg.patch, cfg.scale
    ps = p * s
    t = tile
    box = np.asarray(x_b, F64)[:, t["Y0"] * p:t["Y1"] * p, t["X0"] * p:t["X1"] * p]
    pos_rows = np.array([y * Wp + x for y in range(t["Y0"], t["Y1"]) for x in range(t["X0"], t["X1"])])
    y = untiled_forward(box, w, cfg, pos_rows)
    iy0, ix0 = (t["y0"] - t["Y0"]) * ps, (t["x0"] - t["X0"]) * ps
    return y[:, iy0:iy0 + (t["y1"] - t["y0"]) * ps, ix0:ix0 + (t["x1"] - t["x0"]) * ps]


def reslim_forward_literal(x, w, cfg):
    """Literal form of Sec. 4.2: tile, downscale each tile separately, stitch."""
    x = np.asarray(x, F64)
    B, V, H, W = x.shape
    p, s = cfg.patch, cfg.scale
    ps = p * s
    Hp, Wp = H // p, W // p
    tiles, _, _, _ = tiles_partition(Hp, Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    y = np.empty((B, cfg.out_vars, H * s, W * s), F64)
    for b in range(B):
        for t in tiles:
            y[b, :, t["y0"] * ps:t["y1"] * ps, t["x0"] * ps:t["x1"] * ps] = forward_tile(x[b], w, cfg, t, Wp)
    return y


def rel_l2(a, ref) -> float:
    """max over leading planes of ||a - ref||_2 / ||ref||_2 (planes = all axes but
    the last two for >=3-D arrays, the whole array otherwise)."""
    a = np.asarray(a, F64)
    ref = np.asarray(ref, F64)
    if ref.ndim >= 3:
        a2 = a.reshape(-1, ref.shape[-2] * ref.shape[-1])
        r2 = ref.reshape(a2.shape)
        num = np.sqrt(((a2 - r2) ** 2).sum(-1))
        den = np.sqrt((r2 ** 2).sum(-1))
        return float((num / np.maximum(den, 1e-300)).max())
    return float(np.sqrt(((a - ref) ** 2).sum()) / max(np.sqrt((ref ** 2).sum()), 1e-300))


# --------------------------------------------------------------------------- Bayesian training loss
# Sec. 4.1, "Bayesian Training Loss" (the paper's one equation): a latitude-weighted
# squared error plus a total-variation prior over each pixel's spatial neighbours,
#     || y - x ||_D^2  +  sum_k sum_i sum_{j in C(i)} b_ij | x_ki - x_kj | .
# Readings where the text is silent:
#  * D = diag of cos(latitude of the pixel row), divided by its mean over the rows;
#    rows are the centres of an equiangular grid between lat_min and lat_max;
#  * C(i) = the 8 nearest pixels, clipped at the domain edge (no wrap-around);
#  * b_ij = (1 / distance) / (4 + 4 / sqrt(2)): inversely proportional to the Euclidean
#    pixel distance, normalised so a full neighbourhood sums to 1 (edge pixels are not
#    renormalised);
#  * both terms are averaged over the K N pixel values (the first term is called a
#    mean squared error), the prior carries an explicit weight (1 in the equation);
#  * x in the prior is the prediction; every ordered pair (i, j) counts, as the
#    double sum is written.
def lat_weights(Hf: int, lat_min: float = -90.0, lat_max: float = 90.0):
    """cos(latitude) at the Hf row centres, normalised to mean 1."""
    step = (lat_max - lat_min) / Hf
    lat = lat_min + (np.arange(Hf, dtype=F64) + 0.5) * step
    w = np.cos(np.deg2rad(lat))
    return w / w.mean()


def bayes_loss(pred, target, lat_w, tv_weight: float = 1.0):
    """Returns (total, data term, prior term) for pred, target [B, K, Hf, Wf]."""
    x = np.asarray(pred, F64)
    y = np.asarray(target, F64)
    lw = np.asarray(lat_w, F64)
    B, K, Hf, Wf = x.shape
    count = float(B * K * Hf * Wf)
    data = float((lw[None, None, :, None] * (y - x) ** 2).sum() / count)
    norm = 4.0 + 4.0 / np.sqrt(2.0)
    prior = 0.0
    for dy in (-1, 0, 1):
        for dx in (-1, 0, 1):
            if dy == 0 and dx == 0:
                continue
            b = (1.0 / np.sqrt(float(dy * dy + dx * dx))) / norm
            # pixels i = (r, c) whose neighbour j = (r + dy, c + dx) lies inside the grid
            r0, r1 = max(0, -dy), Hf - max(0, dy)
            c0, c1 = max(0, -dx), Wf - max(0, dx)
            if r1 <= r0 or c1 <= c0:
                continue
            prior += b * float(np.abs(x[:, :, r0:r1, c0:c1] - x[:, :, r0 + dy:r1 + dy, c0 + dx:c1 + dx]).sum())
    prior = tv_weight * prior / count
    return data + prior, data, prior
