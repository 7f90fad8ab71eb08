"""Pins for the training-step oracle (oracle/train_oracle.py): every gradient against PyTorch CPU
autograd through a forward REBUILT from PyTorch's own operators (conv2d patch embedding,
multi_head_attention_forward aggregation, layer_norm, scaled_dot_product_attention per tile,
interpolate + conv2d residual path, pixel-shuffle-like un-patchify, the loss written with tensor
shifts) -- nothing of the oracle's code is on that side -- and against central finite differences
of the oracle's own loss.  CPU only."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import reslim_oracle as O
from oracle import train_oracle as TO
from paper_2505_04802_amd import workloads as WL

torch.set_default_dtype(torch.float64)


def small_cfg(**kw):
    base = WL.ReslimConfig("tr", batch=2, in_vars=3, out_vars=2, H=12, W=16, scale=2, patch=2,
                           embed_dim=16, heads=2, mlp_ratio=2, depth=2, tiles_y=2, tiles_x=2,
                           halo=1, dtype=0, seed=5, res_idx=1)
    return base.with_(**kw)


def inputs(cfg, std=0.25):
    w = {k: np.asarray(v, np.float64) if k != "out_var_idx" else v for k, v in WL.make_weights(cfg, std=std).items()}
    w["out_var_idx"] = np.array([2, 0][:cfg.out_vars], np.int32) if cfg.in_vars >= 3 else w["out_var_idx"]
    x = WL.make_fields(cfg).astype(np.float64)
    r = np.random.default_rng(cfg.seed + 100)
    target = r.standard_normal((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale))
    lat_w = O.lat_weights(cfg.H * cfg.scale, -60.0, 75.0)
    return w, x, target, lat_w


def torch_loss(P, x, target, lat_w, cfg, tv_weight):
    """The model of Sec. 4.1 under TILES (Sec. 4.2) and the Bayesian loss, from PyTorch operators."""
    p, s, C, D, heads = cfg.patch, cfg.scale, cfg.out_vars, cfg.embed_dim, cfg.heads
    B, V, H, W = x.shape
    Hp, Wp = H // p, W // p
    N, ps = Hp * Wp, p * s
    tiles, gather_idx, interior_src, n_h = O.tiles_partition(Hp, Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    xt = torch.from_numpy(x)
    # tokenise each variable with a strided convolution
    e = []
    for v in range(V):
        c = F.conv2d(xt[:, v:v + 1], P["w_pe"][v].reshape(D, 1, p, p), P["b_pe"][v], stride=p)      # [B, D, Hp, Wp]
        e.append(c.flatten(2).transpose(1, 2) + P["var_emb"][v])                                     # [B, N, D]
    e = torch.stack(e, dim=0).reshape(V, B * N, D)                                                   # keys: [V, tokens, D]
    q0 = P["agg_q0"].reshape(1, 1, D).expand(1, B * N, D)
    z, _ = F.multi_head_attention_forward(
        q0, e, e, D, heads, torch.cat([P["agg_wq"], P["agg_wk"], P["agg_wv"]]),
        torch.cat([P["agg_bq"], P["agg_bk"], P["agg_bv"]]), None, None, False, 0.0, P["agg_wo"], P["agg_bo"],
        training=False, need_weights=False)
    z = z.reshape(B, N, D) + P["pos_emb"][None] + P["res_emb"][cfg.res_idx]
    X = z[:, torch.as_tensor(gather_idx)]
    for l in range(cfg.depth):
        outs = []
        for t in tiles:
            Xt = X[:, t["tok_off"]:t["tok_off"] + t["n_tok"]]
            a = F.layer_norm(Xt, (D,), P["ln1_g"][l], P["ln1_b"][l], 1e-5)
            qkv = F.linear(a, P["w_qkv"][l], P["b_qkv"][l])
            sp = lambda m: m.reshape(B, -1, heads, D // heads).transpose(1, 2)
            o = F.scaled_dot_product_attention(sp(qkv[..., :D]), sp(qkv[..., D:2 * D]), sp(qkv[..., 2 * D:]))
            Xt = Xt + F.linear(o.transpose(1, 2).reshape(B, -1, D), P["w_proj"][l], P["b_proj"][l])
            h = F.gelu(F.linear(F.layer_norm(Xt, (D,), P["ln2_g"][l], P["ln2_b"][l], 1e-5), P["w_fc1"][l], P["b_fc1"][l]))
            outs.append(Xt + F.linear(h, P["w_fc2"][l], P["b_fc2"][l]))
        X = torch.cat(outs, dim=1)
    Xn = F.layer_norm(X, (D,), P["lnf_g"], P["lnf_b"], 1e-5)[:, torch.as_tensor(interior_src)]
    Pm = F.linear(Xn, P["w_head"], P["b_head"])                                                      # [B, N, C*ps*ps]
    y = Pm.reshape(B, Hp, Wp, C, ps, ps).permute(0, 3, 1, 4, 2, 5).reshape(B, C, Hp * ps, Wp * ps)
    sel = torch.as_tensor(np.asarray(P["out_var_idx"]), dtype=torch.long)
    pieces = torch.zeros_like(y)
    for t in tiles:
        box = xt[:, sel][:, :, t["Y0"] * p:t["Y1"] * p, t["X0"] * p:t["X1"] * p]
        r = F.conv2d(F.interpolate(box, scale_factor=s, mode="bilinear", align_corners=False), P["w_res"], P["b_res"], padding=1)
        iy0, ix0 = (t["y0"] - t["Y0"]) * ps, (t["x0"] - t["X0"]) * ps
        hy, hx = (t["y1"] - t["y0"]) * ps, (t["x1"] - t["x0"]) * ps
        pad = (t["x0"] * ps, (Wp - t["x1"]) * ps, t["y0"] * ps, (Hp - t["y1"]) * ps)
        pieces = pieces + F.pad(r[:, :, iy0:iy0 + hy, ix0:ix0 + hx], pad)
    y = y + pieces
    tt, lw = torch.from_numpy(target), torch.from_numpy(lat_w)
    data = (lw[None, None, :, None] * (tt - y) ** 2).mean()
    norm = 4.0 + 4.0 / math.sqrt(2.0)
    prior = 0.0
    Hf, Wf = y.shape[2:]
    for dy in (-1, 0, 1):
        for dx in (-1, 0, 1):
            if dy == 0 and dx == 0:
                continue
            a = y[:, :, max(0, -dy):Hf - max(0, dy), max(0, -dx):Wf - max(0, dx)]
            b = y[:, :, max(0, dy):Hf - max(0, -dy), max(0, dx):Wf - max(0, -dx)]
            prior = prior + (a - b).abs().sum() / math.sqrt(dy * dy + dx * dx) / norm
    prior = tv_weight * prior / y.numel()
    return data + prior, y


@pytest.mark.parametrize("kw", [dict(), dict(tiles_y=1, tiles_x=1, halo=0, depth=1), dict(halo=0, tiles_y=3, tiles_x=2, in_vars=2, out_vars=2)],
                         ids=["tiled_halo", "one_tile", "no_halo"])
def test_every_gradient_against_torch_autograd(kw):
    cfg = small_cfg(**kw)
    w, x, target, lat_w = inputs(cfg)
    tv = 0.7
    loss, g, inter = TO.reslim_loss_and_grads(x, target, w, cfg, lat_w, tv)
    P = {k: (torch.from_numpy(np.array(v, np.float64)).requires_grad_(True) if k != "out_var_idx" else v) for k, v in w.items()}
    tl, ty = torch_loss(P, x, target, lat_w, cfg, tv)
    assert abs(float(tl.detach()) - loss[0]) <= 1e-12 * max(1.0, abs(loss[0]))
    np.testing.assert_allclose(inter["y"], ty.detach().numpy(), atol=1e-11)
    tl.backward()
    names = [k for k in w if k != "out_var_idx"]
    assert sorted(names) == sorted(g)                      # a gradient for every parameter tensor, none missing
    for k in names:
        ref = P[k].grad.numpy()
        assert ref.shape == g[k].shape, k
        if k == "agg_bk":
            # a key bias moves all V scores of a head by the same amount and the softmax over the
            # variables does not see it: the gradient is exactly zero (both sides leave rounding noise)
            assert np.abs(ref).max() <= 1e-14 and np.abs(g[k]).max() <= 1e-14
            continue
        scale = np.abs(ref).max()
        assert scale > 0, k                                  # nothing else is trivially zero
        assert np.abs(g[k] - ref).max() <= 1e-9 * scale, (k, np.abs(g[k] - ref).max(), scale)
    # rows of the resolution table the forward does not read get zero; the row it reads does not
    assert not g["res_emb"][1 - cfg.res_idx].any() and g["res_emb"][cfg.res_idx].any()


def test_gradients_by_finite_differences_of_the_oracle_loss():
    """Central differences of the oracle's own loss value, one entry of every kind of tensor
    (smooth part only: the step stays far from the kinks of |.| for these seeds)."""
    cfg = small_cfg(depth=1)
    w, x, target, lat_w = inputs(cfg)
    loss, g, _ = TO.reslim_loss_and_grads(x, target, w, cfg, lat_w, 0.3)
    f = lambda ww: O.bayes_loss(O.reslim_forward(x, ww, cfg), target, lat_w, 0.3)[0]
    eps = 1e-6
    for name, idx in (("w_pe", (1, 3, 2)), ("b_pe", (0, 5)), ("var_emb", (2, 1)), ("agg_q0", (4,)), ("agg_wq", (3, 7)),
                      ("agg_wk", (2, 9)), ("agg_bv", (6,)), ("agg_wo", (1, 1)), ("pos_emb", (17, 3)), ("res_emb", (1, 2)),
                      ("w_qkv", (0, 20, 5)), ("ln2_g", (0, 4)), ("lnf_b", (3,)), ("w_head", (9, 2)), ("b_head", (30,)),
                      ("w_res", (1, 0, 2, 1)), ("b_res", (0,))):
        wp, wm = dict(w), dict(w)
        wp[name] = w[name].copy(); wm[name] = w[name].copy()
        wp[name][idx] += eps; wm[name][idx] -= eps
        fd = (f(wp) - f(wm)) / (2 * eps)
        assert abs(fd - g[name][idx]) <= 2e-6 * max(abs(fd), 1e-3), (name, fd, g[name][idx])


def test_loss_gradient_closed_forms():
    lw = O.lat_weights(6, -30.0, 30.0)
    x = np.zeros((1, 1, 6, 5))
    y = np.ones_like(x)
    # constant prediction: the prior's subgradient is 0 everywhere (sign(0) = 0), the data term is 2 D (x - y) / count
    g = TO.bayes_loss_bwd(x, y, lw, 5.0)
    np.testing.assert_allclose(g, -2.0 * lw[None, None, :, None] * np.ones_like(x) / x.size, atol=1e-15)
    # a single raised pixel in the interior: it gets +2 b for each of its 8 neighbours (sum of b = 1),
    # each neighbour gets -2 b_ij; target = prediction switches the data term off
    x[0, 0, 3, 2] = 1.0
    g = TO.bayes_loss_bwd(x, x, lw, 1.0)
    norm = 4.0 + 4.0 / math.sqrt(2.0)
    assert g[0, 0, 3, 2] == pytest.approx(2.0 / x.size)
    assert g[0, 0, 3, 1] == pytest.approx(-2.0 / norm / x.size) and g[0, 0, 2, 1] == pytest.approx(-2.0 / math.sqrt(2.0) / norm / x.size)
    assert g[0, 0, 0, 0] == 0.0
    assert abs(g.sum()) < 1e-15                                       # the prior only sees differences
    # finite differences on a random field (no two neighbours equal)
    r = np.random.default_rng(3)
    x, y = r.standard_normal((2, 2, 5, 7)), r.standard_normal((2, 2, 5, 7))
    lw = O.lat_weights(5)
    g = TO.bayes_loss_bwd(x, y, lw, 0.4)
    for idx in ((0, 0, 0, 0), (1, 1, 4, 6), (0, 1, 2, 3)):
        xp, xm = x.copy(), x.copy()
        xp[idx] += 1e-6; xm[idx] -= 1e-6
        fd = (O.bayes_loss(xp, y, lw, 0.4)[0] - O.bayes_loss(xm, y, lw, 0.4)[0]) / 2e-6
        assert abs(fd - g[idx]) < 1e-8


def test_transposes_and_halo_bookkeeping():
    r = np.random.default_rng(4)
    # un-patchify is a permutation: its gradient is the inverse permutation
    P = r.standard_normal((2, 3 * 4, 2 * 4 * 4))
    y = O.unpatchify(P, 3, 4, 2, 4)
    assert np.array_equal(TO.unpatchify_bwd(y, 3, 4, 2, 4), P)
    # the gradient of the gather adds up the halo copies: <gather(z), g> = <z, gather^T(g)>
    cfg = small_cfg()
    tiles, gather_idx, interior_src, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    z, gX = r.standard_normal((cfg.Hp * cfg.Wp, 3)), r.standard_normal((n_h, 3))
    gz = np.zeros_like(z)
    np.add.at(gz, np.asarray(gather_idx), gX)
    assert abs((z[gather_idx] * gX).sum() - (z * gz).sum()) < 1e-12
    # the residual path's weight gradient by the definition of the cross-correlation, in loops
    w, x, _, _ = inputs(cfg)
    box = x[0, :, :4, :6]
    d_r = r.standard_normal((cfg.out_vars, 8, 12))
    dw, db = TO.residual_path_bwd(box, w, 2, d_r)
    U = O.bilinear_upsample(box[np.asarray(w["out_var_idx"])], 2)
    o, c, dy, dx = 1, 0, 2, 0
    ref = sum(d_r[o, yy, xx] * U[c, yy + dy - 1, xx + dx - 1] for yy in range(8) for xx in range(12)
              if 0 <= yy + dy - 1 < 8 and 0 <= xx + dx - 1 < 12)
    assert dw[o, c, dy, dx] == pytest.approx(ref) and db[o] == pytest.approx(d_r[o].sum())
