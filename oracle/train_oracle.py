"""CPU oracle for one training step's gradients of the Reslim model under TILES (ORBIT-2
Sec. 4.1 architecture and Bayesian training loss, Sec. 4.2 tiling, Sec. 5: the model is trained).

TEST INFRASTRUCTURE ONLY: plain numpy in float64, slow, imported by tests only; shares no code
with the library.  The paper prints the loss (its one equation) and no gradient formula: every
function here is the chain rule through the forward function of the same name in
reslim_oracle.py, walked backwards step by step.  Pinned (tests/test_oracle_train_pins.py) to
PyTorch CPU autograd through a forward rebuilt from PyTorch's own operators, and to finite
differences.

Readings where the paper is silent:
  * |.| in the prior has no derivative at 0: the subgradient 0 is taken (sign(0) = 0), the choice
    PyTorch's autograd makes as well;
  * every parameter of reslim_oracle's forward gets a gradient, the input field and the target
    get none; `out_var_idx` (a selection) is not a parameter;
  * rows of the position and resolution tables that the forward does not read get zero.
"""
from __future__ import annotations

import math
from typing import Dict

import numpy as np

from . import reslim_oracle as ro

F64 = np.float64


# ---------------------------------------------------------------- loss
def bayes_loss_bwd(pred, target, lat_w, tv_weight: float = 1.0):
    """Gradient of reslim_oracle.bayes_loss (its total) with respect to the prediction.
    Data term: (2 / count) D_r (x - y).  Prior: every ordered pair (i, j) appears in the double
    sum, and the neighbourhood and the weights are symmetric, so pixel m collects
    2 b_mj sign(x_m - x_j) from each neighbour j; sign(0) = 0."""
    x = np.asarray(pred, F64)
    y = np.asarray(target, F64)
    lw = np.asarray(lat_w, F64)
    B, K, Hf, Wf = x.shape
    count = float(B * K * Hf * Wf)
    g = 2.0 * lw[None, None, :, None] * (x - y) / count
    norm = 4.0 + 4.0 / np.sqrt(2.0)
    for dy in (-1, 0, 1):
        for dx in (-1, 0, 1):
            if dy == 0 and dx == 0:
                continue
            b = (1.0 / np.sqrt(float(dy * dy + dx * dx))) / norm
            r0, r1 = max(0, -dy), Hf - max(0, dy)
            c0, c1 = max(0, -dx), Wf - max(0, dx)
            if r1 <= r0 or c1 <= c0:
                continue
            diff = x[:, :, r0:r1, c0:c1] - x[:, :, r0 + dy:r1 + dy, c0 + dx:c1 + dx]
            g[:, :, r0:r1, c0:c1] += (2.0 * tv_weight * b / count) * np.sign(diff)
    return g


# ---------------------------------------------------------------- back end
def unpatchify_bwd(dy, Hp: int, Wp: int, C: int, ps: int):
    """Transpose of reslim_oracle.unpatchify (a permutation): dy[B, C, Hp*ps, Wp*ps] -> [B, Hp*Wp, C*ps*ps]."""
    dy = np.asarray(dy, F64)
    B = dy.shape[0]
    return dy.reshape(B, C, Hp, ps, Wp, ps).transpose(0, 2, 4, 1, 3, 5).reshape(B, Hp * Wp, C * ps * ps)


def residual_path_bwd(x_box, w, s: int, d_r):
    """Gradient of reslim_oracle.residual_path on one field cut with respect to the convolution's
    weights and bias (the input field gets none): d_r[C, h*s, w*s] is the upstream gradient on
    the cut's fine grid (zero where the cut's output is discarded).
    d_w[o, c, dy, dx] = sum_{y, x} d_r[o, y, x] U_pad[c, y + dy, x + dx];  d_b[o] = sum d_r[o]."""
    sel = np.asarray(x_box, F64)[np.asarray(w["out_var_idx"])]
    U = ro.bilinear_upsample(sel, s)
    Cin, h, wd = U.shape
    pad = np.zeros((Cin, h + 2, wd + 2), F64)
    pad[:, 1:-1, 1:-1] = U
    d_r = np.asarray(d_r, F64)
    d_w = np.empty((d_r.shape[0], Cin, 3, 3), F64)
    for dy in range(3):
        for dx in range(3):
            d_w[:, :, dy, dx] = np.einsum("ohw,chw->oc", d_r, pad[:, dy:dy + h, dx:dx + wd])
    return d_w, d_r.sum(axis=(1, 2))


# ---------------------------------------------------------------- front end
def variable_aggregation_bwd(e, w, heads: int, d_z):
    """Gradient of reslim_oracle.variable_aggregation: e[T, V, D] (T tokens), d_z[T, D] ->
    (d_e[T, V, D], gradients of agg_q0, agg_wq, agg_bq, agg_wk, agg_bk, agg_wv, agg_bv, agg_wo, agg_bo).
    With s_gv = q_g . k_vg / sqrt(dh), a = softmax_v(s), o_g = sum_v a_gv u_vg, z = W_o o + b_o:
    d_o = d_z W_o;  d_a_gv = d_o_g . u_vg;  d_u_vg = a_gv d_o_g;  d_s = a (d_a - sum_v a d_a);
    d_q_g = sum d_s_gv k_vg / sqrt(dh) over tokens and v;  d_k_vg = d_s_gv q_g / sqrt(dh)."""
    e = np.asarray(e, F64)
    d_z = np.asarray(d_z, F64)
    T, V, D = e.shape
    dh = D // heads
    sc = 1.0 / math.sqrt(dh)
    q0 = np.asarray(w["agg_q0"], F64)
    q = ro.linear(q0, w["agg_wq"], w["agg_bq"])
    k = ro.linear(e, w["agg_wk"], w["agg_bk"])
    u = ro.linear(e, w["agg_wv"], w["agg_bv"])
    o = np.empty((T, D), F64)
    a_all = np.empty((T, heads, V), F64)
    for g in range(heads):
        c = slice(g * dh, (g + 1) * dh)
        a_all[:, g] = ro.softmax((k[..., c] * q[c]).sum(-1) * sc, axis=-1)
        o[:, c] = (a_all[:, g][..., None] * u[..., c]).sum(-2)
    grads = {}
    d_o, grads["agg_wo"], grads["agg_bo"] = ro.linear_bwd(o, w["agg_wo"], d_z)
    d_k = np.empty_like(k)
    d_u = np.empty_like(u)
    d_q = np.zeros(D, F64)
    for g in range(heads):
        c = slice(g * dh, (g + 1) * dh)
        a = a_all[:, g]                                             # [T, V]
        d_a = (u[..., c] * d_o[:, None, c]).sum(-1)                 # [T, V]
        d_u[..., c] = a[..., None] * d_o[:, None, c]
        d_s = a * (d_a - (a * d_a).sum(-1, keepdims=True))
        d_q[c] = (d_s[..., None] * k[..., c]).sum(axis=(0, 1)) * sc
        d_k[..., c] = d_s[..., None] * q[c] * sc
    d_e1, grads["agg_wk"], grads["agg_bk"] = ro.linear_bwd(e.reshape(T * V, D), w["agg_wk"], d_k.reshape(T * V, D))
    d_e2, grads["agg_wv"], grads["agg_bv"] = ro.linear_bwd(e.reshape(T * V, D), w["agg_wv"], d_u.reshape(T * V, D))
    grads["agg_wq"] = np.outer(d_q, q0)
    grads["agg_bq"] = d_q
    grads["agg_q0"] = np.asarray(w["agg_wq"], F64).T @ d_q
    return (d_e1 + d_e2).reshape(T, V, D), grads


def patch_embed_bwd(x, patch: int, d_e):
    """Gradient of reslim_oracle.patch_embed with respect to its parameters: x[B, V, H, W],
    d_e[B, N, V, D] -> d_w_pe[V, D, p*p], d_b_pe[V, D], d_var_emb[V, D] (the last two are equal:
    both are added to every token of the variable)."""
    x = np.asarray(x, F64)
    d_e = np.asarray(d_e, F64)
    B, V, H, W = x.shape
    p = patch
    Hp, Wp = H // p, W // p
    pix = x.reshape(B, V, Hp, p, Wp, p).transpose(0, 2, 4, 1, 3, 5).reshape(B * Hp * Wp, V, p * p)
    de = d_e.reshape(B * Hp * Wp, V, -1)
    d_w = np.einsum("tvd,tvk->vdk", de, pix)
    d_b = de.sum(axis=0)
    return d_w, d_b, d_b.copy()


def embed_tokens_bwd(x, w, patch: int, heads: int, res_idx: int, d_z):
    """Gradient of reslim_oracle.embed_tokens (untiled call, pos_rows = identity) with respect to
    every front-end parameter.  d_z[B, N, D]."""
    x = np.asarray(x, F64)
    d_z = np.asarray(d_z, F64)
    B, V, H, W = x.shape
    N, D = d_z.shape[1], d_z.shape[2]
    e = ro.patch_embed(x, w, patch)                                 # [B, N, V, D]
    d_e, grads = variable_aggregation_bwd(e.reshape(B * N, V, D), w, heads, d_z.reshape(B * N, D))
    grads["w_pe"], grads["b_pe"], grads["var_emb"] = patch_embed_bwd(x, patch, d_e.reshape(B, N, V, D))
    grads["pos_emb"] = d_z.sum(axis=0)                              # the table is shared by the samples
    grads["res_emb"] = np.zeros_like(np.asarray(w["res_emb"], F64))
    grads["res_emb"][res_idx] = d_z.sum(axis=(0, 1))
    return grads


# ---------------------------------------------------------------- whole step
def reslim_loss_and_grads(x, target, w, cfg, lat_w, tv_weight: float = 1.0):
    """One training step's forward and backward: returns ((total, data, prior), gradients of every
    parameter tensor by name, intermediates) for the batch x[B, V, H, W] with targets
    target[B, C, s*H, s*W].  Intermediates: "y", "d_y", "d_P" (head projection), "tokens_out" and
    "d_tokens_out" (tile-major stream after the last block and its gradient), "d_tokens_in" (gradient
    of the stream before the first block), "d_z" (patch order)."""
    x = np.asarray(x, F64)
    B, V, H, W = x.shape
    p, s, C = cfg.patch, cfg.scale, cfg.out_vars
    Hp, Wp = H // p, W // p
    ps = p * s
    tiles, gather_idx, interior_src, n_h = ro.tiles_partition(Hp, Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    # ---- forward, keeping what the backward needs
    z = ro.embed_tokens(x, w, p, cfg.heads, cfg.res_idx)
    X = z[:, gather_idx, :]
    stream = [X]
    for layer in range(cfg.depth):
        X = ro.reslim_block(X, tiles, w, layer, cfg.heads)
        stream.append(X)
    Xn = ro.layer_norm(X, w["lnf_g"], w["lnf_b"])
    Xn_int = Xn[:, interior_src, :]
    y = ro.unpatchify(ro.head_project(Xn_int, w), Hp, Wp, C, ps)
    for t in tiles:
        box = x[:, :, t["Y0"] * p:t["Y1"] * p, t["X0"] * p:t["X1"] * p]
        iy0, ix0 = (t["y0"] - t["Y0"]) * ps, (t["x0"] - t["X0"]) * ps
        hy, hx = (t["y1"] - t["y0"]) * ps, (t["x1"] - t["x0"]) * ps
        for b in range(B):
            y[b, :, t["y0"] * ps:t["y1"] * ps, t["x0"] * ps:t["x1"] * ps] += \
                ro.residual_path(box[b], w, s)[:, iy0:iy0 + hy, ix0:ix0 + hx]
    loss = ro.bayes_loss(y, target, lat_w, tv_weight)
    # ---- backward
    g: Dict[str, np.ndarray] = {}
    d_y = bayes_loss_bwd(y, target, lat_w, tv_weight)
    g["w_res"] = np.zeros_like(np.asarray(w["w_res"], F64))
    g["b_res"] = np.zeros_like(np.asarray(w["b_res"], F64))
    for t in tiles:
        box = x[:, :, t["Y0"] * p:t["Y1"] * p, t["X0"] * p:t["X1"] * p]
        iy0, ix0 = (t["y0"] - t["Y0"]) * ps, (t["x0"] - t["X0"]) * ps
        hy, hx = (t["y1"] - t["y0"]) * ps, (t["x1"] - t["x0"]) * ps
        for b in range(B):
            d_r = np.zeros((C, (t["Y1"] - t["Y0"]) * ps, (t["X1"] - t["X0"]) * ps), F64)
            d_r[:, iy0:iy0 + hy, ix0:ix0 + hx] = d_y[b, :, t["y0"] * ps:t["y1"] * ps, t["x0"] * ps:t["x1"] * ps]
            dw, db = residual_path_bwd(box[b], w, s, d_r)
            g["w_res"] += dw
            g["b_res"] += db
    d_P = unpatchify_bwd(d_y, Hp, Wp, C, ps)
    N = Hp * Wp
    d_int, g["w_head"], g["b_head"] = ro.linear_bwd(Xn_int.reshape(B * N, -1), w["w_head"], d_P.reshape(B * N, -1))
    d_Xn = np.zeros_like(Xn)
    d_Xn[:, interior_src, :] = d_int.reshape(B, N, -1)               # the halo's outputs are discarded: zero gradient
    d_X, g["lnf_g"], g["lnf_b"] = ro.layer_norm_bwd(stream[-1], w["lnf_g"], d_Xn)
    inter = {"y": y, "d_y": d_y, "d_P": d_P, "tokens_out": stream[-1], "d_tokens_out": d_X.copy()}
    for name in ro.BLOCK_PARAMS:
        g[name] = np.zeros_like(np.asarray(w[name], F64))
    for layer in reversed(range(cfg.depth)):
        d_X, gl = ro.reslim_block_bwd(stream[layer], tiles, w, layer, cfg.heads, d_X)
        for name in ro.BLOCK_PARAMS:
            g[name][layer] = gl[name]
    inter["d_tokens_in"] = d_X
    d_z = np.zeros_like(z)
    np.add.at(d_z, (slice(None), np.asarray(gather_idx)), d_X)        # every halo copy of a patch hands its gradient back
    inter["d_z"] = d_z
    g.update(embed_tokens_bwd(x, w, p, cfg.heads, cfg.res_idx, d_z))
    return loss, g, inter
