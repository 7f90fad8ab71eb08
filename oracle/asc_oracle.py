"""CPU oracle for adaptive spatial compression (ORBIT-2, Sec. 4.1, paragraph
"Adaptive Spatial Compression", and the compression rows of Table 2(b)).

TEST INFRASTRUCTURE ONLY: plain numpy, slow, imported by tests, the smoke check
and the benchmark's CPU leg; shares no code with the library.

What the paper fixes: after the variable aggregation the embedding is mapped to
image space; a quad-tree splits every quadrant whose edge density (Canny edge
detection) exceeds a threshold until a minimum patch size is reached; the ViT
blocks run on one token per quad-tree leaf; a decompression step brings the
tokens back to the uniform patch grid before the decoder.  With compression
switched off the module is the identity.

What it leaves open, and the reading taken here (parity unpinned against the
paper for each of them, pinned against the definitions they reduce to):
  * image-space map: one linear map D -> p*p per token (weights given by the
    caller), un-patchified to the coarse grid;
  * the detector runs on an 8-bit image: per sample v -> floor((v - min) *
    (255 / (max - min)) + 0.5) in float32 (a constant field gives all zeros);
  * Canny's steps in integers: the 5x5 binomial-like smoothing mask with sum 159
    that textbooks give for sigma ~ 1.4 (rounded division), 3x3 Sobel
    derivatives, |gx| + |gy| as magnitude, the gradient direction quantised to
    four sectors at 22.5 / 67.5 degrees (fixed point, 15 fraction bits),
    non-maximum suppression along it (strictly greater than the neighbour on the
    up/left side, not smaller than the other), two thresholds with hysteresis
    over the 8-neighbourhood; image borders by replication for the two filters,
    pixels outside count as magnitude 0 in the suppression;
  * quad-tree: roots are max_leaf x max_leaf blocks of patches in row-major
    order, the grid padded (conceptually, with nothing in the padding) to a
    multiple of max_leaf; a node wholly outside the grid is dropped, a node that
    sticks out of it always splits, a node inside it of side s patches splits iff
    s > min_leaf and float32(count) > float32(tau) * float32(area in pixels);
    children in the order NW, NE, SW, SE, leaves listed depth-first;
  * a leaf's token is the arithmetic mean of the aggregated embeddings (position
    and resolution terms included) of its patches; decompression gives every
    patch its leaf's token.
"""
from __future__ import annotations

import numpy as np

from . import reslim_oracle as ro

F64 = np.float64

SMOOTH_MASK = np.array([[2, 4, 5, 4, 2],
                        [4, 9, 12, 9, 4],
                        [5, 12, 15, 12, 5],
                        [4, 9, 12, 9, 4],
                        [2, 4, 5, 4, 2]], dtype=np.int64)
TAN22_Q15 = 13573          # round(tan(22.5 deg) * 2^15)


def image_from_tokens(z, w_img, b_img, Hp: int, Wp: int, p: int):
    """z[B, N, D] -> image [B, Hp*p, Wp*p]: pixel (i, j) of patch n is
    w_img[i*p + j] . z[n] + b_img[i*p + j]."""
    z = np.asarray(z, F64)
    B = z.shape[0]
    px = z @ np.asarray(w_img, F64).T + np.asarray(b_img, F64)          # [B, N, p*p]
    return px.reshape(B, Hp, Wp, p, p).transpose(0, 1, 3, 2, 4).reshape(B, Hp * p, Wp * p)


def quantise_u8(img):
    """One sample's float32 field -> integers 0..255 (float32 arithmetic, the
    operation order of the docstring above)."""
    v = np.asarray(img, np.float32)
    mn, mx = v.min(), v.max()
    if not mx > mn:
        return np.zeros(v.shape, np.int64)
    scale = np.float32(255.0) / np.float32(mx - mn)
    q = np.floor((v - mn).astype(np.float32) * scale + np.float32(0.5)).astype(np.float32)
    return np.clip(q, 0, 255).astype(np.int64)


def _shift(a, dy: int, dx: int, fill=None):
    """b[y, x] = a[y + dy, x + dx]; outside: replicate the border (fill None) or a constant."""
    H, W = a.shape
    if fill is None:
        ys = np.clip(np.arange(H) + dy, 0, H - 1)
        xs = np.clip(np.arange(W) + dx, 0, W - 1)
        return a[np.ix_(ys, xs)]
    out = np.full_like(a, fill)
    y0, y1 = max(0, -dy), min(H, H - dy)
    x0, x1 = max(0, -dx), min(W, W - dx)
    if y1 > y0 and x1 > x0:
        out[y0:y1, x0:x1] = a[y0 + dy:y1 + dy, x0 + dx:x1 + dx]
    return out


def smooth(q):
    """5x5 integer smoothing with rounded division by the mask's sum, borders replicated."""
    q = np.asarray(q, np.int64)
    acc = np.zeros_like(q)
    for dy in range(-2, 3):
        for dx in range(-2, 3):
            acc += SMOOTH_MASK[dy + 2, dx + 2] * _shift(q, dy, dx)
    return (acc + 79) // 159


def sobel(sm):
    """3x3 Sobel derivatives (gx along columns, gy along rows), borders replicated."""
    gx = (_shift(sm, -1, 1) + 2 * _shift(sm, 0, 1) + _shift(sm, 1, 1)) - \
         (_shift(sm, -1, -1) + 2 * _shift(sm, 0, -1) + _shift(sm, 1, -1))
    gy = (_shift(sm, 1, -1) + 2 * _shift(sm, 1, 0) + _shift(sm, 1, 1)) - \
         (_shift(sm, -1, -1) + 2 * _shift(sm, -1, 0) + _shift(sm, -1, 1))
    return gx, gy


def sector(gx, gy):
    """Quantised gradient direction: 0 along x (|angle| < 22.5 deg from the x axis),
    2 along y, 1 main diagonal (derivatives of one sign), 3 the other diagonal."""
    ax, ay = np.abs(gx), np.abs(gy)
    horiz = (ay << 15) < ax * TAN22_Q15
    vert = (ay << 15) > ax * (TAN22_Q15 + (1 << 16))          # tan 67.5 = tan 22.5 + 2
    same = (gx ^ gy) >= 0
    return np.where(horiz, 0, np.where(vert, 2, np.where(same, 1, 3)))


def candidates(q, low: int, high: int):
    """(strong, weak): pixels that survive non-maximum suppression with magnitude
    above the high / the low threshold (strong is a subset of weak)."""
    gx, gy = sobel(smooth(q))
    mag = np.abs(gx) + np.abs(gy)
    sec = sector(gx, gy)
    step = {0: (0, 1), 1: (1, 1), 2: (1, 0), 3: (1, -1)}      # (dy, dx) towards the "next" neighbour
    prev = np.zeros_like(mag)
    nxt = np.zeros_like(mag)
    for k, (dy, dx) in step.items():
        prev = np.where(sec == k, _shift(mag, -dy, -dx, 0), prev)
        nxt = np.where(sec == k, _shift(mag, dy, dx, 0), nxt)
    keep = (mag > prev) & (mag >= nxt)
    return keep & (mag > high), keep & (mag > low)


def hysteresis(strong, weak):
    """Weak pixels connected to a strong one through weak pixels (8-neighbourhood)."""
    edges = strong.copy()
    while True:
        grown = edges.copy()
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                grown |= _shift(edges, dy, dx, False)
        grown &= weak
        if (grown == edges).all():
            return edges
        edges = grown


def canny_edges(q, low: int, high: int):
    """q: integer image 0..255 [H, W] -> boolean edge map."""
    strong, weak = candidates(q, low, high)
    return hysteresis(strong, weak)


def quadtree_leaves(edges, p: int, max_leaf: int, min_leaf: int, tau: float):
    """edges[H, W] (one sample) -> list of leaves (y0, x0, s) in patch units."""
    H, W = edges.shape
    Hp, Wp = H // p, W // p
    e = np.asarray(edges, np.int64)
    tau32 = np.float32(tau)
    leaves = []

    def visit(y0, x0, s):
        if y0 >= Hp or x0 >= Wp:
            return                                             # wholly in the padding
        inside = y0 + s <= Hp and x0 + s <= Wp
        cnt = int(e[y0 * p:(y0 + s) * p, x0 * p:(x0 + s) * p].sum())
        area = (s * p) * (s * p)
        if not inside or (s > min_leaf and np.float32(cnt) > np.float32(tau32 * np.float32(area))):
            h = s // 2
            visit(y0, x0, h)
            visit(y0, x0 + h, h)
            visit(y0 + h, x0, h)
            visit(y0 + h, x0 + h, h)
        else:
            leaves.append((y0, x0, s))

    for ry in range(0, Hp, max_leaf):
        for rx in range(0, Wp, max_leaf):
            visit(ry, rx, max_leaf)
    return leaves


def build(images, p: int, max_leaf: int, min_leaf: int, low: int, high: int, tau: float):
    """images[B, H, W] float32 -> dict with the leaf table of the batch:
    leaf_y0, leaf_x0, leaf_s [L]; sample_off [B + 1]; patch_leaf [B, Hp*Wp]
    (index into the batch-wide leaf list)."""
    images = np.asarray(images, np.float32)
    B, H, W = images.shape
    Hp, Wp = H // p, W // p
    ly, lx, ls, off = [], [], [], [0]
    patch_leaf = np.empty((B, Hp * Wp), np.int64)
    for b in range(B):
        leaves = quadtree_leaves(canny_edges(quantise_u8(images[b]), low, high), p, max_leaf, min_leaf, tau)
        for (y0, x0, s) in leaves:
            idx = len(ly)
            ly.append(y0); lx.append(x0); ls.append(s)
            for yy in range(y0, y0 + s):
                patch_leaf[b, yy * Wp + x0:yy * Wp + x0 + s] = idx
        off.append(len(ly))
    return dict(leaf_y0=np.array(ly, np.int64), leaf_x0=np.array(lx, np.int64), leaf_s=np.array(ls, np.int64),
                sample_off=np.array(off, np.int64), patch_leaf=patch_leaf)


def compress(z, table, Wp: int):
    """z[B, N, D] -> [L, D]: mean over each leaf's patches."""
    z = np.asarray(z, F64)
    L = len(table["leaf_s"])
    out = np.empty((L, z.shape[2]), F64)
    for b in range(z.shape[0]):
        for i in range(int(table["sample_off"][b]), int(table["sample_off"][b + 1])):
            y0, x0, s = int(table["leaf_y0"][i]), int(table["leaf_x0"][i]), int(table["leaf_s"][i])
            rows = [yy * Wp + xx for yy in range(y0, y0 + s) for xx in range(x0, x0 + s)]
            out[i] = z[b, rows, :].sum(axis=0) / float(s * s)
    return out


def decompress(Xc, table):
    """[L, D] -> [B, N, D]: every patch takes its leaf's token."""
    return np.asarray(Xc, F64)[table["patch_leaf"]]


def blocks_compressed(Xc, table, w, cfg):
    """All ViT blocks on the compressed tokens; attention stays inside a sample."""
    Xc = np.asarray(Xc, F64).copy()
    off = table["sample_off"]
    for b in range(len(off) - 1):
        X = Xc[off[b]:off[b + 1]]
        for layer in range(cfg.depth):
            X = ro.block_tokens(X, w, layer, cfg.heads)
        Xc[off[b]:off[b + 1]] = X
    return Xc


def forward_compressed(x, w, cfg, table):
    """Reslim forward with the compression module switched on (no tiling):
    embed, compress, blocks, decompress, final LayerNorm, head, + residual path."""
    x = np.asarray(x, F64)
    B, V, H, W = x.shape
    p, s, C = cfg.patch, cfg.scale, cfg.out_vars
    Hp, Wp = H // p, W // p
    z = ro.embed_tokens(x, w, p, cfg.heads, cfg.res_idx)
    Xc = blocks_compressed(compress(z, table, Wp), table, w, cfg)
    Xn = ro.layer_norm(decompress(Xc, table), w["lnf_g"], w["lnf_b"])
    y = ro.unpatchify(ro.head_project(Xn, w), Hp, Wp, C, p * s)
    for b in range(B):
        y[b] += ro.residual_path(x[b], w, s)
    return y


# ---------------------------------------------------------------------------
# Training side: gradients of the two linear maps and of a block on the leaves
# (chain rule; Table 2(b) of the paper times training with compression)
# ---------------------------------------------------------------------------
def compress_bwd(dZc, table, B: int, N: int):
    """Gradient of `compress`: the mean over a leaf hands 1/(s*s) of the leaf's
    gradient to each of its patches.  dZc[L, D] -> [B, N, D]."""
    dZc = np.asarray(dZc, F64)
    s2 = (np.asarray(table["leaf_s"], F64) ** 2)[:, None]
    return (dZc / s2)[np.asarray(table["patch_leaf"]).reshape(B, N)]


def decompress_bwd(dZ, table):
    """Gradient of `decompress`: a leaf collects the gradients of all patches that
    copied it.  dZ[B, N, D] -> [L, D]."""
    dZ = np.asarray(dZ, F64)
    out = np.zeros((len(table["leaf_s"]), dZ.shape[2]), F64)
    np.add.at(out, np.asarray(table["patch_leaf"]).reshape(-1), dZ.reshape(-1, dZ.shape[2]))
    return out


def block_compressed(Xc, table, w, layer: int, heads: int):
    """One ViT block on the leaves; attention stays inside a sample."""
    Xc = np.asarray(Xc, F64)
    out = np.empty_like(Xc)
    off = table["sample_off"]
    for b in range(len(off) - 1):
        out[off[b]:off[b + 1]] = ro.block_tokens(Xc[off[b]:off[b + 1]], w, layer, heads)
    return out


def block_compressed_bwd(Xc, table, w, layer: int, heads: int, d_out):
    """Gradient of `block_compressed`: (d_Xc, parameter gradients summed over samples)."""
    Xc = np.asarray(Xc, F64)
    d_out = np.asarray(d_out, F64)
    dX = np.empty_like(Xc)
    grads = None
    off = table["sample_off"]
    for b in range(len(off) - 1):
        dx, g = ro.block_tokens_bwd(Xc[off[b]:off[b + 1]], w, layer, heads, d_out[off[b]:off[b + 1]])
        dX[off[b]:off[b + 1]] = dx
        grads = g if grads is None else {k: grads[k] + g[k] for k in g}
    return dX, grads


# ---------------------------------------------------------------------------
# Compression combined with TILES (Table 3 of the paper runs "4x compression, 16 tiles")
# ---------------------------------------------------------------------------
# The paper does not say how the two combine.  Reading: TILES cuts the field into haloed
# boxes and downscales each box "separately" (Sec. 4.2), so each box is compressed
# separately too, exactly as a whole sample is in the untiled case: the 8-bit image, the
# edge map and the quad-tree of a tile are those of its haloed box cut out of the field
# (roots anchored at the box's first patch; a box that is no multiple of the root size is a
# ragged grid as above).  A leaf never straddles a box edge, halo patches are compressed
# with their box like any other patch, and after decompression the halo is discarded as in
# plain TILES: an interior patch takes the token of its leaf in the tile that owns it.
# parity unpinned against the paper; pinned by: one tile = forward_compressed, one patch
# per leaf = the plain tiled forward, literal form = batched form.
def build_tiles(images, p: int, tiles, max_leaf: int, min_leaf: int, low: int, high: int, tau: float, Wp: int):
    """images[B, H, W] float32, tiles from reslim_oracle.tiles_partition -> dict with the
    leaf table of the batch in GLOBAL patch coordinates: leaf_y0, leaf_x0, leaf_s [L];
    sample_off [B*T + 1], one entry per (sample, tile) sequence, sample-major;
    patch_leaf [B, Hp*Wp]: for each patch the leaf (batch-wide index) that holds it in the
    tile whose interior owns it."""
    images = np.asarray(images, np.float32)
    B, H, W = images.shape
    Hp = H // p
    ly, lx, ls, off = [], [], [], [0]
    patch_leaf = np.full((B, Hp * Wp), -1, np.int64)
    for b in range(B):
        for t in tiles:
            crop = images[b, t["Y0"] * p:t["Y1"] * p, t["X0"] * p:t["X1"] * p]
            leaves = quadtree_leaves(canny_edges(quantise_u8(crop), low, high), p, max_leaf, min_leaf, tau)
            for (y0, x0, s) in leaves:
                idx = len(ly)
                gy, gx = y0 + t["Y0"], x0 + t["X0"]
                ly.append(gy); lx.append(gx); ls.append(s)
                for yy in range(max(gy, t["y0"]), min(gy + s, t["y1"])):
                    for xx in range(max(gx, t["x0"]), min(gx + s, t["x1"])):
                        patch_leaf[b, yy * Wp + xx] = idx
            off.append(len(ly))
    assert (patch_leaf >= 0).all()
    return dict(leaf_y0=np.array(ly, np.int64), leaf_x0=np.array(lx, np.int64), leaf_s=np.array(ls, np.int64),
                sample_off=np.array(off, np.int64), patch_leaf=patch_leaf)


def compress_tiles(z, table, Wp: int, T: int):
    """z[B, N, D] -> [L, D]: mean over each leaf's patches; sequence q belongs to sample q // T."""
    z = np.asarray(z, F64)
    out = np.empty((len(table["leaf_s"]), z.shape[2]), F64)
    off = table["sample_off"]
    for q in range(len(off) - 1):
        b = q // T
        for i in range(int(off[q]), int(off[q + 1])):
            y0, x0, s = int(table["leaf_y0"][i]), int(table["leaf_x0"][i]), int(table["leaf_s"][i])
            rows = [yy * Wp + xx for yy in range(y0, y0 + s) for xx in range(x0, x0 + s)]
            out[i] = z[b, rows, :].sum(axis=0) / float(s * s)
    return out


def compress_tiles_bwd(dZc, table, B: int, N: int, Wp: int, T: int):
    """Gradient of `compress_tiles`: every leaf hands 1/(s*s) of its gradient to each of its
    patches; with tiles a patch lies in the leaves of every box whose haloed region holds it, so
    the contributions add up.  dZc[L, D] -> [B, N, D].  (`decompress` and `decompress_bwd` need
    no tiled form: they follow patch_leaf, which already names the owning tile's leaf.)"""
    dZc = np.asarray(dZc, F64)
    out = np.zeros((B, N, dZc.shape[1]), F64)
    off = table["sample_off"]
    for q in range(len(off) - 1):
        b = q // T
        for i in range(int(off[q]), int(off[q + 1])):
            y0, x0, s = int(table["leaf_y0"][i]), int(table["leaf_x0"][i]), int(table["leaf_s"][i])
            for yy in range(y0, y0 + s):
                for xx in range(x0, x0 + s):
                    out[b, yy * Wp + xx] += dZc[i] / float(s * s)
    return out


def forward_compressed_tiles(x, w, cfg, table):
    """Batched form of the tiled forward with compression: embed once, one leaf set per
    (sample, tile), blocks with attention inside a leaf set, each patch decompressed from
    the tile that owns it, final LayerNorm, head, residual path per tile."""
    x = np.asarray(x, F64)
    B, V, H, W = x.shape
    p, s, C = cfg.patch, cfg.scale, cfg.out_vars
    Hp, Wp = H // p, W // p
    ps = p * s
    tiles = ro.tiles_partition(Hp, Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)[0]
    z = ro.embed_tokens(x, w, p, cfg.heads, cfg.res_idx)
    Xc = blocks_compressed(compress_tiles(z, table, Wp, len(tiles)), table, w, cfg)
    Xn = ro.layer_norm(decompress(Xc, table), w["lnf_g"], w["lnf_b"])
    y = ro.unpatchify(ro.head_project(Xn, w), Hp, Wp, C, ps)
    for t in tiles:
        iy0, ix0 = (t["y0"] - t["Y0"]) * ps, (t["x0"] - t["X0"]) * ps
        hy, hx = (t["y1"] - t["y0"]) * ps, (t["x1"] - t["x0"]) * ps
        for b in range(B):
            r = ro.residual_path(x[b, :, t["Y0"] * p:t["Y1"] * p, t["X0"] * p:t["X1"] * p], w, s)
            y[b, :, t["y0"] * ps:t["y1"] * ps, t["x0"] * ps:t["x1"] * ps] += r[:, iy0:iy0 + hy, ix0:ix0 + hx]
    return y


def forward_compressed_tile_literal(x_b, image_b, w, cfg, tile: dict, Wp: int, max_leaf: int, min_leaf: int,
                                    low: int, high: int, tau: float):
    """Literal form for one tile of one sample: cut the haloed box out of the field (and out
    of the image the detector looks at), run the UNTILED compressed model on the cut with
    position rows taken at the global positions, discard the halo.  Returns the fine interior."""
    p, s, C = cfg.patch, cfg.scale, cfg.out_vars
    ps = p * s
    t = tile
    box = np.asarray(x_b, F64)[:, t["Y0"] * p:t["Y1"] * p, t["X0"] * p:t["X1"] * p]
    crop = np.asarray(image_b, np.float32)[t["Y0"] * p:t["Y1"] * p, t["X0"] * p:t["X1"] * p]
    hp, wp = t["Y1"] - t["Y0"], t["X1"] - t["X0"]
    table = build(crop[None], p, max_leaf, min_leaf, low, high, tau)
    pos_rows = np.array([y * Wp + xx for y in range(t["Y0"], t["Y1"]) for xx in range(t["X0"], t["X1"])])
    z = ro.embed_tokens(box[None], w, p, cfg.heads, cfg.res_idx, pos_rows=pos_rows)
    Xc = blocks_compressed(compress(z, table, wp), table, w, cfg)
    Xn = ro.layer_norm(decompress(Xc, table), w["lnf_g"], w["lnf_b"])
    y = ro.unpatchify(ro.head_project(Xn, w), hp, wp, C, ps)[0] + ro.residual_path(box, w, s)
    iy0, ix0 = (t["y0"] - t["Y0"]) * ps, (t["x0"] - t["X0"]) * ps
    return y[:, iy0:iy0 + (t["y1"] - t["y0"]) * ps, ix0:ix0 + (t["x1"] - t["x0"]) * ps]
