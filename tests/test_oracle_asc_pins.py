"""Pins for the adaptive-spatial-compression oracle (Sec. 4.1, "Adaptive Spatial
Compression"): every step is checked against something that is not the oracle
itself - a library routine, a closed form, a hand-derived picture or a brute
force on a tiny input.  CPU only."""
import math

import numpy as np
import pytest
from scipy import ndimage

from oracle import asc_oracle as A
from oracle import reslim_oracle as ro
O = ro
from paper_2505_04802_amd import workloads as WL


def _rand_u8(seed, H=40, W=56, smooth=2.0):
    r = np.random.default_rng(seed)
    f = ndimage.gaussian_filter(r.standard_normal((H, W)), smooth)
    return A.quantise_u8(f.astype(np.float32))


def test_quantise_range_and_special_cases():
    r = np.random.default_rng(0)
    v = r.standard_normal((16, 24)).astype(np.float32)
    q = A.quantise_u8(v)
    assert q.min() == 0 and q.max() == 255
    # affine in v up to the rounding: |q - exact| <= 0.5 + float32 slack
    exact = (v.astype(np.float64) - v.min()) * 255.0 / (float(v.max()) - float(v.min()))
    assert np.abs(q - exact).max() <= 0.5 + 1e-3
    assert (A.quantise_u8(np.full((4, 4), 3.5, np.float32)) == 0).all()      # constant field
    # monotone: ordering of the input is never reversed
    o = np.argsort(v.ravel())
    assert (np.diff(q.ravel()[o]) >= 0).all()


def test_smoothing_against_library_correlation():
    assert A.SMOOTH_MASK.sum() == 159 and (A.SMOOTH_MASK == A.SMOOTH_MASK.T).all()
    q = _rand_u8(1)
    ref = ndimage.correlate(q, A.SMOOTH_MASK, mode="nearest")
    assert (A.smooth(q) == (ref + 79) // 159).all()
    assert (A.smooth(np.full((9, 9), 200)) == 200).all()                     # a constant stays


def test_sobel_against_library():
    sm = A.smooth(_rand_u8(2))
    gx, gy = A.sobel(sm)
    assert (gx == ndimage.sobel(sm, axis=1, mode="nearest")).all()
    assert (gy == ndimage.sobel(sm, axis=0, mode="nearest")).all()
    ramp = np.tile(np.arange(12) * 3, (10, 1))                               # d/dx = 3 -> gx = 8 * 3 inside
    gx, gy = A.sobel(ramp)
    assert (gx[:, 1:-1] == 24).all() and (gy == 0).all()


def test_sector_against_atan2():
    r = np.random.default_rng(3)
    gx = r.integers(-1020, 1021, 20000)
    gy = r.integers(-1020, 1021, 20000)
    keep = (gx != 0) | (gy != 0)
    gx, gy = gx[keep], gy[keep]
    ang = np.degrees(np.arctan2(gy, gx)) % 180.0                             # direction modulo 180
    ref = np.select([(ang < 22.5) | (ang >= 157.5), ang < 67.5, ang < 112.5], [0, 1, 2], 3)
    near = np.abs(((ang - 22.5) % 45.0 + 22.5) % 45.0 - 22.5) < 0.01         # within 0.01 deg of a sector border
    near |= np.abs((ang - 22.5) % 45.0) < 0.01
    got = A.sector(gx, gy)
    assert (got[~near] == ref[~near]).all()
    # axis-aligned and exactly diagonal gradients
    assert A.sector(np.array([5]), np.array([0]))[0] == 0 and A.sector(np.array([0]), np.array([-7]))[0] == 2
    assert A.sector(np.array([4]), np.array([4]))[0] == 1 and A.sector(np.array([4]), np.array([-4]))[0] == 3


def test_step_edges_by_hand():
    """A vertical step gives one column of edge pixels, on the dark side of the step
    (the tie between the two columns next to the step goes to the left one); a
    horizontal step one row; an ideal diagonal step the two anti-diagonals next to
    it (they are not neighbours along the gradient, so both are maxima)."""
    q = np.zeros((32, 32), np.int64)
    q[:, 16:] = 255
    e = A.canny_edges(q, 50, 100)
    assert e.sum() == 32 and e[:, 15].all()
    e = A.canny_edges(q.T, 50, 100)
    assert e.sum() == 32 and e[15, :].all()
    yy, xx = np.mgrid[0:32, 0:32]
    e = A.canny_edges(((yy + xx) >= 32) * 255, 50, 100)
    inner = e[4:28, :]
    assert ((yy + xx)[4:28][inner] // 1 >= 31).all() and ((yy + xx)[4:28][inner] <= 32).all()
    assert (inner.sum(axis=1) == 2).all()
    assert A.canny_edges(np.full((20, 20), 77), 1, 2).sum() == 0             # nothing in a constant field


def test_thresholds_and_nms_definition_brute_force():
    q = _rand_u8(4, 24, 28, 1.5)
    gx, gy = A.sobel(A.smooth(q))
    mag = np.abs(gx) + np.abs(gy)
    low, high = int(np.quantile(mag, 0.5)), int(np.quantile(mag, 0.8))
    strong, weak = A.candidates(q, low, high)
    H, W = q.shape
    step = {0: (0, 1), 1: (1, 1), 2: (1, 0), 3: (1, -1)}
    for y in range(H):
        for x in range(W):
            ang = math.degrees(math.atan2(gy[y, x], gx[y, x])) % 180.0 if mag[y, x] else 0.0
            k = 0 if (ang < 22.5 or ang >= 157.5) else 1 if ang < 67.5 else 2 if ang < 112.5 else 3
            dy, dx = step[k]
            def m(yy, xx):
                return int(mag[yy, xx]) if 0 <= yy < H and 0 <= xx < W else 0
            keep = mag[y, x] > m(y - dy, x - dx) and mag[y, x] >= m(y + dy, x + dx)
            assert bool(weak[y, x]) == (keep and mag[y, x] > low), (y, x)
            assert bool(strong[y, x]) == (keep and mag[y, x] > high), (y, x)
    assert (weak | ~strong).all()


def test_hysteresis_against_connected_components():
    r = np.random.default_rng(5)
    weak = r.random((40, 50)) < 0.35
    strong = weak & (r.random((40, 50)) < 0.05)
    lab, n = ndimage.label(weak, structure=np.ones((3, 3), int))
    keep = np.unique(lab[strong])
    ref = np.isin(lab, keep[keep > 0])
    assert (A.hysteresis(strong, weak) == ref).all()
    # a weak pixel chain reaching a strong pixel survives, an isolated one does not
    w = np.zeros((5, 9), bool); w[2, 1:6] = True; w[0, 8] = True
    s = np.zeros_like(w); s[2, 1] = True
    out = A.hysteresis(s, w)
    assert out[2, 1:6].all() and not out[0, 8]


def _check_tree(edges, leaves, p, max_leaf, min_leaf, tau):
    H, W = edges.shape
    Hp, Wp = H // p, W // p
    cover = np.zeros((Hp, Wp), int)
    def dens_split(y0, x0, s):
        if y0 + s > Hp or x0 + s > Wp:
            return True                                         # sticks out of a ragged grid: always splits
        cnt = edges[y0 * p:(y0 + s) * p, x0 * p:(x0 + s) * p].sum()
        return s > min_leaf and np.float32(cnt) > np.float32(np.float32(tau) * np.float32((s * p) ** 2))
    for (y0, x0, s) in leaves:
        assert s >= 1 and s <= max_leaf and (s & (s - 1)) == 0 and y0 % s == 0 and x0 % s == 0
        assert y0 + s <= Hp and x0 + s <= Wp
        cover[y0:y0 + s, x0:x0 + s] += 1
        assert not dens_split(y0, x0, s)                        # a leaf does not split
        a = 2 * s
        while a <= max_leaf:                                    # every ancestor did
            assert dens_split(y0 // a * a, x0 // a * a, a)
            a *= 2
    assert (cover == 1).all()                                   # a partition of the patch grid


def test_quadtree_properties_and_extremes():
    r = np.random.default_rng(6)
    p, mx, mn = 2, 8, 1
    edges = ndimage.gaussian_filter(r.standard_normal((32, 48)), 3.0) > 0.12
    edges &= r.random(edges.shape) < 0.4
    for tau in (0.02, 0.08, 0.2):
        leaves = A.quadtree_leaves(edges, p, mx, mn, tau)
        _check_tree(edges, leaves, p, mx, mn, tau)
    none = A.quadtree_leaves(np.zeros((32, 48), bool), p, mx, mn, 0.05)
    assert none == [(y, x, 8) for y in (0, 8) for x in (0, 8, 16)]           # one leaf per root, row-major
    full = A.quadtree_leaves(np.ones((32, 48), bool), p, mx, mn, 0.05)
    assert len(full) == 16 * 24 and all(s == 1 for _, _, s in full)          # identity: one leaf per patch
    # depth-first NW, NE, SW, SE inside a root
    assert full[:4] == [(0, 0, 1), (0, 1, 1), (1, 0, 1), (1, 1, 1)]
    assert full[4] == (0, 2, 1) and full[8] == (2, 0, 1) and full[12] == (2, 2, 1) and full[16] == (0, 4, 1) and full[64] == (0, 8, 1)
    assert all(s >= 2 for _, _, s in A.quadtree_leaves(np.ones((32, 48), bool), p, mx, 2, 0.05))
    # a grid that is no multiple of the root size (18 x 30 patches, roots of 8): the paper's 90 x 180
    # patch grid is of this kind; nodes that stick out split, what lies inside follows the density rule
    ragged = edges[:36, :60]
    for tau in (0.02, 0.2, 2.0):
        leaves = A.quadtree_leaves(ragged, p, mx, mn, tau)
        _check_tree(ragged, leaves, p, mx, mn, tau)
    no_edges = A.quadtree_leaves(np.zeros((36, 60), bool), p, mx, mn, 0.05)
    assert sum(s * s for _, _, s in no_edges) == 18 * 30
    assert [l for l in no_edges if l[2] == 8] == [(y, x, 8) for y in (0, 8) for x in (0, 8, 16)]
    assert (16, 0, 2) in no_edges and (0, 24, 4) in no_edges and (16, 28, 2) in no_edges and all(s < 8 for y, x, s in no_edges if y >= 16 or x >= 24)


def test_compress_decompress_means_and_identity():
    r = np.random.default_rng(7)
    B, Hp, Wp, D, p = 2, 8, 16, 5, 2
    imgs = ndimage.gaussian_filter(r.standard_normal((B, Hp * p, Wp * p)), (0, 1.5, 1.5)).astype(np.float32)
    tab = A.build(imgs, p, 4, 1, 40, 90, 0.06)
    L = len(tab["leaf_s"])
    assert tab["sample_off"][0] == 0 and tab["sample_off"][-1] == L
    assert (tab["leaf_s"] ** 2).sum() == B * Hp * Wp
    z = r.standard_normal((B, Hp * Wp, D))
    zc = A.compress(z, tab, Wp)
    back = A.decompress(zc, tab)
    for b in range(B):
        for i in range(tab["sample_off"][b], tab["sample_off"][b + 1]):
            members = np.nonzero(tab["patch_leaf"][b] == i)[0]
            assert len(members) == tab["leaf_s"][i] ** 2
            np.testing.assert_allclose(zc[i], z[b, members].mean(axis=0), rtol=0, atol=1e-14)
            assert (back[b, members] == zc[i]).all()
    np.testing.assert_allclose(A.compress(np.ones_like(z), tab, Wp), 1.0, rtol=0, atol=1e-15)
    ident = A.build(imgs, p, 4, 4, 40, 90, 0.06)                              # min = max: uniform leaves of 4 x 4
    assert (ident["leaf_s"] == 4).all()


def test_forward_with_single_patch_leaves_is_the_uncompressed_model():
    """Switched off (every leaf one patch) the module is the identity: the
    compressed forward must reproduce the plain untiled forward."""
    cfg1 = WL.CONFIGS["c0"].with_(tiles_y=1, tiles_x=1, halo=0, batch=2)
    w = WL.make_weights(cfg1)
    x = WL.make_fields(cfg1)
    Hp, Wp = cfg1.H // cfg1.patch, cfg1.W // cfg1.patch
    ones = np.ones((cfg1.batch, cfg1.H, cfg1.W), bool)
    ly, lx, ls, off = [], [], [], [0]
    patch_leaf = np.empty((cfg1.batch, Hp * Wp), np.int64)
    for b in range(cfg1.batch):
        for (y0, x0, s) in A.quadtree_leaves(ones[b], cfg1.patch, 4, 1, 0.5):
            patch_leaf[b, y0 * Wp + x0] = len(ly)
            ly.append(y0); lx.append(x0); ls.append(s)
        off.append(len(ly))
    tab = dict(leaf_y0=np.array(ly), leaf_x0=np.array(lx), leaf_s=np.array(ls), sample_off=np.array(off), patch_leaf=patch_leaf)
    y_c = A.forward_compressed(x, w, cfg1, tab)
    y_ref = ro.reslim_forward(x, w, cfg1)
    assert ro.rel_l2(y_c, y_ref) < 1e-12


def test_image_from_tokens_layout():
    r = np.random.default_rng(8)
    B, Hp, Wp, D, p = 1, 3, 4, 6, 2
    z = r.standard_normal((B, Hp * Wp, D))
    w_img, b_img = r.standard_normal((p * p, D)), r.standard_normal(p * p)
    img = A.image_from_tokens(z, w_img, b_img, Hp, Wp, p)
    for n in (0, 5, 11):
        for i in range(p):
            for j in range(p):
                ref = float(w_img[i * p + j] @ z[0, n] + b_img[i * p + j])
                assert abs(img[0, (n // Wp) * p + i, (n % Wp) * p + j] - ref) < 1e-12


def test_gradients_of_compress_and_decompress_are_the_adjoint_maps():
    """compress and decompress are linear: their gradients must be the transposed
    maps, <A z, g> = <z, A^T g> for arbitrary z and g (to rounding)."""
    r = np.random.default_rng(11)
    B, Hp, Wp, D, p = 2, 8, 16, 4, 2
    imgs = ndimage.gaussian_filter(r.standard_normal((B, Hp * p, Wp * p)), (0, 1.5, 1.5)).astype(np.float32)
    tab = A.build(imgs, p, 4, 1, 40, 90, 0.06)
    L, N = len(tab["leaf_s"]), Hp * Wp
    assert 1 < L < B * N
    z, g_c = r.standard_normal((B, N, D)), r.standard_normal((L, D))
    assert abs((A.compress(z, tab, Wp) * g_c).sum() - (z * A.compress_bwd(g_c, tab, B, N)).sum()) < 1e-10
    zc, g = r.standard_normal((L, D)), r.standard_normal((B, N, D))
    assert abs((A.decompress(zc, tab) * g).sum() - (zc * A.decompress_bwd(g, tab)).sum()) < 1e-10
    # decompress after compress keeps leaf means: the composed gradient is the projection again
    np.testing.assert_allclose(A.compress(A.decompress(zc, tab), tab, Wp), zc, atol=1e-14)


def test_block_gradient_on_leaves_by_finite_differences():
    cfg = WL.CONFIGS["c0"].with_(tiles_y=1, tiles_x=1, halo=0, batch=2, embed_dim=32, heads=2, depth=1, H=16, W=16)
    w = {k: np.asarray(v, np.float64) for k, v in WL.make_weights(cfg, std=0.2).items()}
    r = np.random.default_rng(12)
    tab = dict(sample_off=np.array([0, 5, 12]), leaf_s=np.ones(12, np.int64))
    X, d_out = r.standard_normal((12, cfg.embed_dim)), r.standard_normal((12, cfg.embed_dim))
    dX, grads = A.block_compressed_bwd(X, tab, w, 0, cfg.heads, d_out)
    f = lambda X_, w_: float((A.block_compressed(X_, tab, w_, 0, cfg.heads) * d_out).sum())
    eps = 1e-6
    for (i, j) in ((0, 3), (4, 0), (5, 7), (11, 31)):           # both samples, first and last rows
        Xp, Xm = X.copy(), X.copy(); Xp[i, j] += eps; Xm[i, j] -= eps
        assert abs((f(Xp, w) - f(Xm, w)) / (2 * eps) - dX[i, j]) < 1e-6 * max(1.0, abs(dX[i, j]))
    for name, idx in (("w_qkv", (0, 5, 3)), ("b_fc1", (0, 7)), ("ln1_g", (0, 2)), ("w_fc2", (0, 3, 9))):
        wp, wm = dict(w), dict(w)
        wp[name] = w[name].copy(); wm[name] = w[name].copy()
        wp[name][idx] += eps; wm[name][idx] -= eps
        fd = (f(X, wp) - f(X, wm)) / (2 * eps)
        assert abs(fd - grads[name][idx[1:]]) < 1e-6 * max(1.0, abs(fd)), name
    # attention never crosses a sample: the gradient of sample 0's rows ignores sample 1's upstream gradient
    d2 = d_out.copy(); d2[5:] = 0.0
    dX2, _ = A.block_compressed_bwd(X, tab, w, 0, cfg.heads, d2)
    np.testing.assert_allclose(dX2[:5], dX[:5], atol=1e-14)
    assert np.abs(dX2[5:]).max() == 0.0


# ----------------------------------------------------------------- compression combined with TILES
def _tiled_case(seed=21, tiles_y=2, tiles_x=3, halo=1, H=24, W=40, depth=2):
    cfg = WL.ReslimConfig("asc_tiles", batch=2, in_vars=3, out_vars=2, H=H, W=W, scale=2, patch=2, embed_dim=16, heads=2,
                          mlp_ratio=2, depth=depth, tiles_y=tiles_y, tiles_x=tiles_x, halo=halo, dtype=0, seed=seed)
    w = WL.make_weights(cfg, std=0.3)
    x = WL.make_fields(cfg)
    tiles = O.tiles_partition(cfg.Hp, cfg.Wp, tiles_y, tiles_x, halo)[0]
    return cfg, w, x, tiles


PRM = dict(max_leaf=4, min_leaf=1, low=30, high=70, tau=0.08)


def test_tiled_table_is_a_partition_of_every_haloed_box():
    cfg, w, x, tiles = _tiled_case()
    tab = A.build_tiles(x[:, 0], cfg.patch, tiles, Wp=cfg.Wp, **PRM)
    off = tab["sample_off"]
    assert len(off) == cfg.batch * len(tiles) + 1 and off[0] == 0 and off[-1] == len(tab["leaf_s"])
    some_merged = False
    for q in range(len(off) - 1):
        b, t = q // len(tiles), tiles[q % len(tiles)]
        cover = np.zeros((cfg.Hp, cfg.Wp), int)
        for i in range(off[q], off[q + 1]):
            y0, x0, s = tab["leaf_y0"][i], tab["leaf_x0"][i], tab["leaf_s"][i]
            assert s & (s - 1) == 0 and (y0 - t["Y0"]) % s == 0 and (x0 - t["X0"]) % s == 0      # aligned to the box
            assert t["Y0"] <= y0 and y0 + s <= t["Y1"] and t["X0"] <= x0 and x0 + s <= t["X1"]   # never straddles it
            cover[y0:y0 + s, x0:x0 + s] += 1
            some_merged |= s > 1
        want = np.zeros_like(cover)
        want[t["Y0"]:t["Y1"], t["X0"]:t["X1"]] = 1
        assert (cover == want).all()
        # interior patches point at a leaf of their own tile that holds them
        for yy in range(t["y0"], t["y1"]):
            for xx in range(t["x0"], t["x1"]):
                i = tab["patch_leaf"][b, yy * cfg.Wp + xx]
                assert off[q] <= i < off[q + 1]
                assert tab["leaf_y0"][i] <= yy < tab["leaf_y0"][i] + tab["leaf_s"][i]
                assert tab["leaf_x0"][i] <= xx < tab["leaf_x0"][i] + tab["leaf_s"][i]
    assert some_merged and len(tab["leaf_s"]) < cfg.batch * sum(t["n_tok"] for t in tiles)


def test_tiled_compressed_forward_batched_equals_literal():
    """The table-driven form the library follows against the literal one: cut each haloed box
    out of the field, run the untiled compressed model on it, keep the interior."""
    cfg, w, x, tiles = _tiled_case()
    tab = A.build_tiles(x[:, 0], cfg.patch, tiles, Wp=cfg.Wp, **PRM)
    y = A.forward_compressed_tiles(x, w, cfg, tab)
    ps = cfg.patch * cfg.scale
    for b in range(cfg.batch):
        for t in tiles:
            lit = A.forward_compressed_tile_literal(x[b], x[b, 0], w, cfg, t, cfg.Wp, **PRM)
            np.testing.assert_allclose(y[b, :, t["y0"] * ps:t["y1"] * ps, t["x0"] * ps:t["x1"] * ps], lit, atol=1e-10)


def test_tiled_compressed_forward_special_cases():
    # one tile: the tiled functions ARE the untiled compressed forward
    cfg, w, x, tiles = _tiled_case(tiles_y=1, tiles_x=1, halo=3)
    tab1 = A.build_tiles(x[:, 0], cfg.patch, tiles, Wp=cfg.Wp, **PRM)
    tab0 = A.build(x[:, 0], cfg.patch, PRM["max_leaf"], PRM["min_leaf"], PRM["low"], PRM["high"], PRM["tau"])
    for k in tab0:
        assert np.array_equal(tab0[k], tab1[k]), k
    np.testing.assert_allclose(A.forward_compressed_tiles(x, w, cfg, tab1), A.forward_compressed(x, w, cfg, tab0), atol=1e-12)
    # one patch per leaf (thresholds nothing passes, minimum = maximum = 1): the plain tiled forward
    cfg, w, x, tiles = _tiled_case()
    tab = A.build_tiles(x[:, 0], cfg.patch, tiles, 1, 1, 30, 70, 0.08, Wp=cfg.Wp)
    assert len(tab["leaf_s"]) == cfg.batch * sum(t["n_tok"] for t in tiles) and (tab["leaf_s"] == 1).all()
    np.testing.assert_allclose(A.forward_compressed_tiles(x, w, cfg, tab), O.reslim_forward(x, w, cfg), atol=1e-12)
    # the order of leaves inside a (sample, tile) sequence is the tile-major token order in that case
    g = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)[1]
    n_h = len(g)
    rows = tab["leaf_y0"] * cfg.Wp + tab["leaf_x0"]
    assert np.array_equal(rows[:n_h], g) and np.array_equal(rows[n_h:], g)
    # tiles do not interact: changing the field inside one tile's interior, away from every halo,
    # leaves the other tiles' outputs untouched
    cfg, w, x, tiles = _tiled_case(tiles_y=1, tiles_x=2, halo=1, H=16, W=64)
    tab = A.build_tiles(x[:, 0], cfg.patch, tiles, Wp=cfg.Wp, **PRM)
    y = A.forward_compressed_tiles(x, w, cfg, tab)
    x2 = x.copy()
    x2[:, :, :, :8] += 1.0                                             # far inside tile 0 (its halo ends at column 34)
    tab2 = A.build_tiles(x2[:, 0], cfg.patch, tiles, Wp=cfg.Wp, **PRM)
    y2 = A.forward_compressed_tiles(x2, w, cfg, tab2)
    ps = cfg.patch * cfg.scale
    t1 = tiles[1]
    np.testing.assert_allclose(y2[..., t1["x0"] * ps:], y[..., t1["x0"] * ps:], atol=1e-12)
    assert np.abs(y2[..., :8 * cfg.scale] - y[..., :8 * cfg.scale]).max() > 1e-3


def test_tiled_compression_gradients_are_the_adjoint_maps():
    """The gradient maps under TILES against the forward maps they transpose (which the pins above
    hold): <A z, g> = <z, A^T g> for compression per box and for decompression from the owning tile;
    one tile: the untiled gradient; the halo's share: a patch in k boxes collects k contributions."""
    cfg, w, x, tiles = _tiled_case()
    T, N, D = len(tiles), cfg.Hp * cfg.Wp, 5
    tab = A.build_tiles(x[:, 0], cfg.patch, tiles, Wp=cfg.Wp, **PRM)
    L = len(tab["leaf_s"])
    r = np.random.default_rng(12)
    z, g_c = r.standard_normal((cfg.batch, N, D)), r.standard_normal((L, D))
    lhs = (A.compress_tiles(z, tab, cfg.Wp, T) * g_c).sum()
    assert abs(lhs - (z * A.compress_tiles_bwd(g_c, tab, cfg.batch, N, cfg.Wp, T)).sum()) < 1e-10
    zc, g = r.standard_normal((L, D)), r.standard_normal((cfg.batch, N, D))
    assert abs((A.decompress(zc, tab) * g).sum() - (zc * A.decompress_bwd(g, tab)).sum()) < 1e-10
    # leaves that only cover halo patches of their box receive nothing from decompression
    used = np.zeros(L, bool)
    used[np.unique(tab["patch_leaf"])] = True
    assert not used.all() and not A.decompress_bwd(g, tab)[~used].any()
    # all-ones leaf gradient: a patch gets 1 per box that holds it (the number of its tile-major copies)
    copies = np.bincount(O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)[1], minlength=N)
    ones = A.compress_tiles_bwd(np.ones((L, 1)) * (tab["leaf_s"][:, None] ** 2), tab, cfg.batch, N, cfg.Wp, T)
    # (scaled by s*s so that each leaf hands exactly 1 to each of its patches)
    assert np.array_equal(ones[0, :, 0], copies) and copies.max() > 1
    # one tile: the untiled map
    cfg1, w1, x1, tiles1 = _tiled_case(tiles_y=1, tiles_x=1, halo=3)
    tab1 = A.build_tiles(x1[:, 0], cfg1.patch, tiles1, Wp=cfg1.Wp, **PRM)
    g1 = r.standard_normal((len(tab1["leaf_s"]), D))
    np.testing.assert_allclose(A.compress_tiles_bwd(g1, tab1, cfg1.batch, cfg1.Hp * cfg1.Wp, cfg1.Wp, 1),
                               A.compress_bwd(g1, tab1, cfg1.batch, cfg1.Hp * cfg1.Wp), atol=1e-14)

