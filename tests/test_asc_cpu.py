"""Host side of adaptive spatial compression (Sec. 4.1): the library's quad-tree
builder against the oracle, bit for bit, on seeded synthetic fields; error paths.
No GPU involved: reslim_asc_build and reslim_asc_edges make no HIP call."""
import numpy as np
import pytest
from scipy import ndimage

from oracle import asc_oracle as A
from paper_2505_04802_amd import binding as B
from paper_2505_04802_amd import workloads as WL

KEYS = ("leaf_y0", "leaf_x0", "leaf_s", "sample_off", "patch_leaf")


def fields(seed, B_, H, W, smooth):
    r = np.random.default_rng(seed)
    return ndimage.gaussian_filter(r.standard_normal((B_, H, W)), (0, smooth, smooth)).astype(np.float32)


@pytest.mark.parametrize("seed,shape,patch,mx,mn,low,high,tau,smooth", [
    (0, (3, 64, 96), 2, 8, 1, 20, 60, 0.05, 2.0),
    (1, (2, 48, 80), 2, 8, 2, 10, 30, 0.02, 3.0),
    (2, (1, 32, 32), 4, 4, 1, 40, 90, 0.10, 1.0),
    (3, (2, 40, 56), 1, 8, 1, 30, 70, 0.08, 2.5),       # patch 1: 40 x 56 grid, roots of 8
    (4, (1, 96, 160), 2, 16, 1, 25, 50, 0.04, 4.0),
    (5, (2, 36, 60), 2, 8, 1, 20, 60, 0.05, 2.0),        # 18 x 30 patches: no multiple of the root size
    (6, (1, 180, 360), 2, 16, 2, 30, 70, 0.05, 3.0),     # the paper's 112 km grid: 90 x 180 patches
])
def test_builder_matches_oracle(seed, shape, patch, mx, mn, low, high, tau, smooth):
    imgs = fields(seed, *shape, smooth)
    got = B.reslim_asc_build(imgs, patch, mx, mn, low, high, tau)
    ref = A.build(imgs, patch, mx, mn, low, high, tau)
    for k in KEYS:
        assert np.asarray(got[k]).shape == np.asarray(ref[k]).shape, k
        assert (np.asarray(got[k]) == np.asarray(ref[k])).all(), k
    for b in range(shape[0]):
        e = B.reslim_asc_edges(imgs[b], low, high)
        assert (e.astype(bool) == A.canny_edges(A.quantise_u8(imgs[b]), low, high)).all()


def test_builder_on_the_workload_fields():
    """The synthetic fields of the benchmark workloads (random Fourier modes + noise)."""
    cfg = WL.CONFIGS["c0"].with_(batch=2)
    x = WL.make_fields(cfg)
    imgs = np.ascontiguousarray(x[:, 0])
    got = B.reslim_asc_build(imgs, cfg.patch, 8, 1, 30, 80, 0.05)
    ref = A.build(imgs, cfg.patch, 8, 1, 30, 80, 0.05)
    for k in KEYS:
        assert (np.asarray(got[k]) == np.asarray(ref[k])).all(), k
    assert got["sample_off"][-1] == len(got["leaf_s"]) < cfg.batch * cfg.n_tokens


def test_builder_extremes_and_errors():
    flat = np.full((1, 16, 32), 2.5, np.float32)                     # constant field: no edges, one leaf per root
    t = B.reslim_asc_build(flat, 2, 4, 1, 10, 20, 0.01)
    assert (t["leaf_s"] == 4).all() and len(t["leaf_s"]) == 2 * 4
    step = np.zeros((1, 16, 32), np.float32)
    step[:, :, 16:] = 1.0                                            # one vertical edge: fine leaves only along it
    t = B.reslim_asc_build(step, 2, 4, 1, 10, 20, 0.01)
    small = t["leaf_s"] == 1
    assert small.any() and (t["leaf_x0"][small] // 4 == 1).all() and (t["leaf_s"][t["leaf_x0"] >= 8] == 4).all()
    same = B.reslim_asc_build(step, 2, 4, 4, 10, 20, 0.01)           # min = max: uniform
    assert (same["leaf_s"] == 4).all()
    with pytest.raises(B.ReslimError):
        B.reslim_asc_build(step, 2, 3, 1, 10, 20, 0.01)              # not a power of two
    big = B.reslim_asc_build(step, 2, 16, 1, 10, 20, 0.01)           # 8 x 16 patches under roots of 16: they stick out and split
    assert (big["leaf_s"] ** 2).sum() == 8 * 16 and big["leaf_s"].max() == 8
    with pytest.raises(B.ReslimError):
        B.reslim_asc_build(step, 2, 4, 1, 30, 20, 0.01)              # low > high
    with pytest.raises(B.ReslimError):
        B.reslim_asc_build(step, 2, 4, 1, 10, 20, float("nan"))
    bad = step.copy()
    bad[0, 3, 3] = np.inf
    with pytest.raises(B.ReslimError):
        B.reslim_asc_build(bad, 2, 4, 1, 10, 20, 0.01)


def test_builder_matches_oracle_on_random_shapes():
    """Forty seeded draws of grid shape (mostly no multiple of the root size), patch
    size, leaf bounds, thresholds and field smoothness: identical tables."""
    r = np.random.default_rng(2024)
    for trial in range(40):
        patch = int(r.choice([1, 2, 4]))
        Hp, Wp = int(r.integers(3, 40)), int(r.integers(3, 56))
        mx = int(r.choice([1, 2, 4, 8, 16]))
        mn = int(r.choice([m for m in (1, 2, 4, 8, 16) if m <= mx]))
        low = int(r.integers(0, 80))
        high = low + int(r.integers(0, 120))
        tau = float(r.choice([0.0, 0.01, 0.05, 0.2, 1.0]))
        Bn = int(r.integers(1, 4))
        imgs = fields(1000 + trial, Bn, Hp * patch, Wp * patch, float(r.uniform(0.5, 4.0)))
        if trial % 7 == 0:
            imgs[0] = 1.0                                                  # a constant sample among the others
        got = B.reslim_asc_build(imgs, patch, mx, mn, low, high, tau)
        ref = A.build(imgs, patch, mx, mn, low, high, tau)
        for k in KEYS:
            assert np.array_equal(np.asarray(got[k]), np.asarray(ref[k])), (trial, k, Hp, Wp, patch, mx, mn, low, high, tau)


# ----------------------------------------------------------------- compression combined with TILES (host builder)
@pytest.mark.parametrize("seed,shape,patch,ty,tx,halo,mx,mn,low,high,tau,smooth", [
    (10, (2, 48, 80), 2, 2, 3, 1, 4, 1, 20, 60, 0.05, 2.0),
    (11, (1, 64, 64), 2, 4, 4, 2, 8, 1, 15, 40, 0.03, 3.0),
    (12, (3, 30, 44), 1, 3, 2, 3, 8, 2, 25, 70, 0.06, 1.5),       # boxes that are no multiple of the root size
    (13, (1, 180, 360), 2, 4, 4, 2, 16, 1, 30, 70, 0.05, 3.0),    # the paper's 112 km grid with its 16 tiles
    (14, (2, 32, 48), 2, 1, 1, 5, 8, 1, 20, 60, 0.05, 2.0),       # one tile: the untiled builder
])
def test_tiled_builder_matches_oracle(seed, shape, patch, ty, tx, halo, mx, mn, low, high, tau, smooth):
    from oracle import reslim_oracle as O
    imgs = fields(seed, *shape, smooth)
    Hp, Wp = shape[1] // patch, shape[2] // patch
    tiles = O.tiles_partition(Hp, Wp, ty, tx, halo)[0]
    got = B.reslim_asc_build_tiles(imgs, patch, ty, tx, halo, mx, mn, low, high, tau)
    ref = A.build_tiles(imgs, patch, tiles, mx, mn, low, high, tau, Wp=Wp)
    for k in KEYS:
        assert np.asarray(got[k]).shape == np.asarray(ref[k]).shape, k
        assert (np.asarray(got[k]) == np.asarray(ref[k])).all(), k
    if ty == tx == 1:
        one = B.reslim_asc_build(imgs, patch, mx, mn, low, high, tau)
        for k in KEYS:
            assert np.array_equal(one[k], got[k]), k


def test_tiled_builder_errors():
    imgs = fields(20, 1, 16, 24, 2.0)
    with pytest.raises(B.ReslimError):
        B.reslim_asc_build_tiles(imgs, 2, 9, 1, 1, 4, 1, 10, 20, 0.05)     # more tile rows than patch rows
    with pytest.raises(B.ReslimError):
        B.reslim_asc_build_tiles(imgs, 2, 2, 2, -1, 4, 1, 10, 20, 0.05)    # negative halo
    with pytest.raises(B.ReslimError):
        B.reslim_asc_build_tiles(imgs, 2, 2, 2, 1, 3, 1, 10, 20, 0.05)     # leaf bound not a power of two
