"""GPU parity of adaptive spatial compression (Sec. 4.1): image-space map,
leaf-mean compression and the whole forward on the leaves, through the C ABI,
against the CPU oracle on the same seeded inputs.  The leaf tables come from the
oracle's own builder (the library's builder is compared with it bit for bit in
the CPU tests), so no expected value depends on the GPU path.

Tolerances: fp32 path rel-L2 <= 1e-5, bf16 path <= 2e-2 (the forward's bars)."""
import numpy as np
import pytest
import torch

from oracle import asc_oracle as A
from oracle import reslim_oracle as O
from paper_2505_04802_amd import binding as B
from paper_2505_04802_amd import workloads as WL

pytestmark = pytest.mark.gpu
TOL = {0: 1e-5, 1: 2e-2}

ASC_F32 = WL.ReslimConfig("a32", batch=3, in_vars=3, out_vars=2, H=32, W=48, scale=2, patch=2,
                          embed_dim=48, heads=3, mlp_ratio=2, depth=2, tiles_y=1, tiles_x=1,
                          halo=0, dtype=0, seed=21)
ASC_BF16 = WL.ReslimConfig("abf", batch=2, in_vars=3, out_vars=3, H=64, W=96, scale=4, patch=2,
                           embed_dim=128, heads=2, mlp_ratio=4, depth=2, tiles_y=1, tiles_x=1,
                           halo=0, dtype=1, seed=22)       # dh = 64; up to 1536 tokens per sample before compression
ASC_BF16_DH128 = ASC_BF16.with_(name="abf128", embed_dim=256, heads=2, seed=23)
# grids that are no multiple of the root size (18 x 30 and 22 x 38 patches under roots of 8)
ASC_F32_RAGGED = ASC_F32.with_(name="a32r", H=36, W=60, seed=24)
ASC_BF16_RAGGED = ASC_BF16.with_(name="abfr", H=44, W=76, seed=25)


def cuda(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype)


def say(msg):
    print(msg, flush=True)


def table_for(cfg, x, max_leaf=8, min_leaf=1, tau=0.05):
    """Leaf table from the oracle's builder on the first input variable; thresholds at
    fixed quantiles of that field's own gradient magnitude so that the tree is mixed."""
    imgs = np.ascontiguousarray(x[:, 0])
    q = A.quantise_u8(imgs[0])
    gx, gy = A.sobel(A.smooth(q))
    mag = np.abs(gx) + np.abs(gy)
    low, high = int(np.quantile(mag, 0.6)), int(np.quantile(mag, 0.85))
    return A.build(imgs, cfg.patch, max_leaf, min_leaf, low, high, tau)


@pytest.mark.parametrize("cfg", [ASC_F32, ASC_BF16], ids=lambda c: c.name)
def test_image_and_compress_parity(cfg):
    say(f"asc image + compress {cfg.name}")
    r = np.random.default_rng(cfg.seed)
    D, N, p = cfg.embed_dim, cfg.n_tokens, cfg.patch
    z = r.standard_normal((cfg.batch, N, D)).astype(np.float32)
    w_img = (r.standard_normal((p * p, D)) / np.sqrt(D)).astype(np.float32)
    b_img = r.standard_normal(p * p).astype(np.float32)
    x = WL.make_fields(cfg)
    tab = table_for(cfg, x)
    L = len(tab["leaf_s"])
    say(f"  {cfg.batch * N} patches -> {L} leaves, per sample {np.diff(tab['sample_off']).tolist()}")
    assert L < cfg.batch * N and len(set(np.diff(tab["sample_off"]).tolist())) > 1      # compressed, ragged
    with B.Reslim(cfg, WL.make_weights(cfg)) as m:
        img = torch.full((cfg.batch, cfg.H, cfg.W), float("nan"), dtype=torch.float32, device="cuda")
        B.reslim_asc_image(m.ctx, cuda(z), cuda(w_img), cuda(b_img), img, cfg.batch)
        ref = A.image_from_tokens(z, w_img, b_img, cfg.Hp, cfg.Wp, p)
        err = O.rel_l2(img.cpu().numpy(), ref)
        say(f"  image rel-L2 {err:.3e}")
        assert err <= 1e-6
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            assert B.reslim_asc_plan_info(plan) == (L, int(np.diff(tab["sample_off"]).max()))
            zc = torch.full((L, D), float("nan"), dtype=torch.float32, device="cuda")
            B.reslim_asc_compress(m.ctx, plan, cuda(z), zc)
            err = O.rel_l2(zc.cpu().numpy(), A.compress(z, tab, cfg.Wp))
            say(f"  compress rel-L2 {err:.3e}")
            assert err <= 1e-6
        finally:
            B.reslim_asc_plan_destroy(plan)


@pytest.mark.parametrize("cfg", [ASC_F32, ASC_BF16, ASC_BF16_DH128, ASC_F32_RAGGED, ASC_BF16_RAGGED], ids=lambda c: c.name)
def test_compressed_forward_parity(cfg):
    say(f"asc forward {cfg.name}")
    w = WL.make_weights(cfg, std=0.05)
    x = WL.make_fields(cfg)
    tab = table_for(cfg, x)
    L = len(tab["leaf_s"])
    say(f"  {cfg.batch * cfg.n_tokens} patches -> {L} leaves, per sample {np.diff(tab['sample_off']).tolist()}")
    ref = A.forward_compressed(x, w, cfg, tab)
    with B.Reslim(cfg, w) as m:
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            y = torch.full((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), float("nan"),
                           dtype=torch.float32, device="cuda")
            B.reslim_asc_forward(m.ctx, plan, cuda(x), y, m.ws)
            out = y.cpu().numpy()
        finally:
            B.reslim_asc_plan_destroy(plan)
    assert np.isfinite(out).all()
    err = max(O.rel_l2(out[b, c], ref[b, c]) for b in range(cfg.batch) for c in range(cfg.out_vars))
    say(f"  max rel-L2 over planes {err:.3e}")
    assert err <= TOL[cfg.dtype]


def test_single_patch_leaves_reproduce_the_plain_forward():
    """Switched off (one patch per leaf) the module is the identity: the library's
    compressed forward and its plain forward agree, and both match the oracle."""
    cfg = ASC_F32
    w = WL.make_weights(cfg, std=0.05)
    x = WL.make_fields(cfg)
    ones = np.ones((cfg.batch, cfg.H, cfg.W), np.float32)
    r = np.random.default_rng(3)
    noise = r.standard_normal(ones.shape).astype(np.float32)          # white noise: edges everywhere
    tab = A.build(noise, cfg.patch, 8, 1, 0, 0, 0.0)
    if not (tab["leaf_s"] == 1).all():                                 # any patch without an edge pixel keeps its parent
        tab = A.build(noise, cfg.patch, 1, 1, 0, 0, 0.0)
    assert (tab["leaf_s"] == 1).all()
    ref = O.reslim_forward(x, w, cfg)
    with B.Reslim(cfg, w) as m:
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            y = torch.empty((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), dtype=torch.float32, device="cuda")
            B.reslim_asc_forward(m.ctx, plan, cuda(x), y, m.ws)
            plain = m.forward(cuda(x)).cpu().numpy()
        finally:
            B.reslim_asc_plan_destroy(plan)
    assert O.rel_l2(y.cpu().numpy(), ref) <= 1e-5 and O.rel_l2(plain, ref) <= 1e-5
    assert np.abs(y.cpu().numpy() - plain).max() <= 1e-5


def test_plan_errors():
    cfg = ASC_F32
    x = WL.make_fields(cfg)
    tab = table_for(cfg, x)
    w = WL.make_weights(cfg)
    with B.Reslim(cfg, w) as m:
        bad = dict(tab); bad["leaf_s"] = tab["leaf_s"].copy(); bad["leaf_s"][0] *= 2        # overlaps / leaves the grid
        with pytest.raises(B.ReslimError):
            B.reslim_asc_plan_create(m.ctx, cfg.batch, bad)
        bad = dict(tab); bad["patch_leaf"] = tab["patch_leaf"].copy(); bad["patch_leaf"][1, 5] += 1
        with pytest.raises(B.ReslimError):
            B.reslim_asc_plan_create(m.ctx, cfg.batch, bad)
        bad = dict(tab); bad["sample_off"] = tab["sample_off"].copy(); bad["sample_off"][1] += 1   # sample 0 takes a leaf of sample 1
        with pytest.raises(B.ReslimError):
            B.reslim_asc_plan_create(m.ctx, cfg.batch, bad)
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            with B.Reslim(cfg, w) as other:                                                  # a plan is tied to its context
                y = torch.empty((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), dtype=torch.float32, device="cuda")
                with pytest.raises(B.ReslimError):
                    B.reslim_asc_forward(other.ctx, plan, cuda(x), y, other.ws)
        finally:
            B.reslim_asc_plan_destroy(plan)
    tiled = cfg.with_(tiles_y=2, tiles_x=2, halo=1)
    with B.Reslim(tiled, WL.make_weights(tiled)) as m:
        with pytest.raises(B.ReslimError):
            B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)


def test_compressed_forward_at_the_benchmark_grid():
    """The benchmark's compression case: the c1 grid as one tile (8192 patches per
    sample) with its ~8x quad-tree parameters, two samples, whole output against the
    oracle; the library's host builder must give the oracle's table."""
    import bench
    cfg = WL.CONFIGS["c1"].with_(tiles_y=1, tiles_x=1, halo=0, batch=2)
    prm = bench.ASC_PARAMS[0]
    w = WL.make_weights(cfg)
    x = WL.make_fields(cfg)
    imgs = np.ascontiguousarray(x[:, 0])
    say("asc benchmark grid: building the table (oracle and library)")
    tab = A.build(imgs, cfg.patch, prm["max_leaf"], prm["min_leaf"], prm["canny_low"], prm["canny_high"], prm["tau"])
    lib = B.reslim_asc_build(imgs, cfg.patch, prm["max_leaf"], prm["min_leaf"], prm["canny_low"], prm["canny_high"], prm["tau"])
    for k in tab:
        assert (np.asarray(tab[k]) == np.asarray(lib[k])).all(), k
    L = len(tab["leaf_s"])
    say(f"  {cfg.batch * cfg.n_tokens} patches -> {L} leaves, per sample {np.diff(tab['sample_off']).tolist()}; oracle forward ...")
    ref = A.forward_compressed(x, w, cfg, tab)
    with B.Reslim(cfg, w) as m:
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            y = torch.full((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), float("nan"),
                           dtype=torch.float32, device="cuda")
            B.reslim_asc_forward(m.ctx, plan, cuda(x), y, m.ws)
            out = y.cpu().numpy()
        finally:
            B.reslim_asc_plan_destroy(plan)
    err = max(O.rel_l2(out[b, c], ref[b, c]) for b in range(cfg.batch) for c in range(cfg.out_vars))
    say(f"  max rel-L2 over planes {err:.3e}")
    assert np.isfinite(out).all() and err <= TOL[1]


@pytest.mark.parametrize("dtype", [0, 1], ids=["f32", "bf16"])
def test_degenerate_trees(dtype):
    """One sample whose whole grid is a single leaf (attention over one token) next to
    one that is split down to single patches, and a uniform tree with min = max."""
    cfg = WL.ReslimConfig("adeg", batch=2, in_vars=2, out_vars=2, H=32, W=32, scale=2, patch=2,
                          embed_dim=128, heads=2, mlp_ratio=2, depth=2, tiles_y=1, tiles_x=1,
                          halo=0, dtype=dtype, seed=31)
    w = WL.make_weights(cfg, std=0.05)
    x = WL.make_fields(cfg)
    r = np.random.default_rng(9)
    imgs = np.stack([np.full((cfg.H, cfg.W), 1.25, np.float32), r.standard_normal((cfg.H, cfg.W)).astype(np.float32)])
    for (mx, mn) in ((16, 1), (4, 4)):
        tab = A.build(imgs, cfg.patch, mx, mn, 0, 0, 0.0)
        counts = np.diff(tab["sample_off"]).tolist()
        say(f"asc degenerate {'bf16' if dtype else 'f32'} max {mx} min {mn}: leaves per sample {counts}")
        if mx == 16:
            assert counts[0] == 1 and counts[1] > 200
        ref = A.forward_compressed(x, w, cfg, tab)
        with B.Reslim(cfg, w) as m:
            plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
            try:
                y = torch.full((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), float("nan"),
                               dtype=torch.float32, device="cuda")
                B.reslim_asc_forward(m.ctx, plan, cuda(x), y, m.ws)
                out = y.cpu().numpy()
            finally:
                B.reslim_asc_plan_destroy(plan)
        err = max(O.rel_l2(out[b, c], ref[b, c]) for b in range(cfg.batch) for c in range(cfg.out_vars))
        say(f"  max rel-L2 over planes {err:.3e}")
        assert np.isfinite(out).all() and err <= TOL[dtype]


# ------------------------------------------------------------------ training on the leaves
def _u8(n):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("cfg", [ASC_F32, ASC_BF16], ids=lambda c: c.name)
def test_gradients_of_compress_and_decompress(cfg):
    r = np.random.default_rng(cfg.seed + 1)
    D, N = cfg.embed_dim, cfg.n_tokens
    tab = table_for(cfg, WL.make_fields(cfg))
    L = len(tab["leaf_s"])
    zc = r.standard_normal((L, D)).astype(np.float32)
    g = r.standard_normal((cfg.batch, N, D)).astype(np.float32)
    with B.Reslim(cfg, WL.make_weights(cfg)) as m:
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            full = torch.full((cfg.batch * N, D), float("nan"), dtype=torch.float32, device="cuda")
            B.reslim_asc_decompress(m.ctx, plan, cuda(zc), full)
            assert np.array_equal(full.cpu().numpy().reshape(cfg.batch, N, D), A.decompress(zc, tab).astype(np.float32))
            B.reslim_asc_compress_bwd(m.ctx, plan, cuda(zc), full)
            err = O.rel_l2(full.cpu().numpy().reshape(cfg.batch, N, D), A.compress_bwd(zc, tab, cfg.batch, N))
            say(f"  compress_bwd {cfg.name} rel-L2 {err:.3e}")
            assert err <= 1e-6
            dc = torch.full((L, D), float("nan"), dtype=torch.float32, device="cuda")
            B.reslim_asc_decompress_bwd(m.ctx, plan, cuda(g), dc)
            err = O.rel_l2(dc.cpu().numpy(), A.decompress_bwd(g, tab))
            say(f"  decompress_bwd {cfg.name} rel-L2 {err:.3e}")
            assert err <= 1e-6
        finally:
            B.reslim_asc_plan_destroy(plan)


@pytest.mark.parametrize("cfg", [ASC_F32, ASC_BF16, ASC_BF16_DH128], ids=lambda c: c.name)
def test_block_training_on_the_leaves(cfg):
    """Forward-for-training and backward of one block on a compressed batch (ragged
    per-sample leaf counts) against the oracle: output, input gradient, all twelve
    parameter gradients; a second backward gives the same bits."""
    say(f"asc block train {cfg.name}")
    w = WL.make_weights(cfg, std=0.1)
    tab = table_for(cfg, WL.make_fields(cfg))
    L, D, layer = len(tab["leaf_s"]), cfg.embed_dim, 1
    r = np.random.default_rng(cfg.seed + 2)
    x = r.standard_normal((L, D)).astype(np.float32)
    d_out = r.standard_normal((L, D)).astype(np.float32)
    ref_out = A.block_compressed(x, tab, w, layer, cfg.heads)
    ref_dx, ref_g = A.block_compressed_bwd(x, tab, w, layer, cfg.heads, d_out)
    with B.Reslim(cfg, w) as m:
        B.reslim_train_prepare(m.ctx)
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            sb, wb = B.reslim_asc_block_train_bytes(m.ctx, plan)
            saved, ws = _u8(sb), _u8(wb)
            x_dev, out = cuda(x), torch.full((L, D), float("nan"), dtype=torch.float32, device="cuda")
            B.reslim_asc_block_fwd_train(m.ctx, plan, layer, x_dev, out, saved, ws)
            err = O.rel_l2(out.cpu().numpy(), ref_out)
            say(f"  x_out rel-L2 {err:.3e}")
            assert err <= TOL[cfg.dtype]
            grads = {n: torch.full(np.shape(w[n][layer]), float("nan"), dtype=torch.float32, device="cuda") for n in B.BLOCK_PARAMS}
            dx = torch.full((L, D), float("nan"), dtype=torch.float32, device="cuda")
            B.reslim_asc_block_bwd(m.ctx, plan, layer, x_dev, saved, cuda(d_out), dx, grads, ws)
            torch.cuda.synchronize()
            err = O.rel_l2(dx.cpu().numpy(), ref_dx)
            say(f"  d_x rel-L2 {err:.3e}")
            assert err <= TOL[cfg.dtype]
            for n in B.BLOCK_PARAMS:
                err = O.rel_l2(grads[n].cpu().numpy(), ref_g[n])
                say(f"  d_{n} rel-L2 {err:.3e}")
                assert err <= TOL[cfg.dtype], n
            again = {n: torch.empty_like(grads[n]) for n in B.BLOCK_PARAMS}
            dx2 = torch.empty_like(dx)
            B.reslim_asc_block_bwd(m.ctx, plan, layer, x_dev, saved, cuda(d_out), dx2, again, ws)
            torch.cuda.synchronize()
            assert torch.equal(dx, dx2) and all(torch.equal(grads[n], again[n]) for n in B.BLOCK_PARAMS)
            # error paths: short buffers, a plan of another context
            lib = B.load()
            st = torch.cuda.current_stream().cuda_stream
            assert lib.reslim_asc_block_fwd_train(m.ctx, plan, layer, x_dev.data_ptr(), out.data_ptr(), saved.data_ptr(),
                                                  sb - 256, ws.data_ptr(), wb, st) == B.RESLIM_EWORKSPACE
            with B.Reslim(cfg, w) as other:
                B.reslim_train_prepare(other.ctx)
                assert lib.reslim_asc_block_fwd_train(other.ctx, plan, layer, x_dev.data_ptr(), out.data_ptr(),
                                                      saved.data_ptr(), sb, ws.data_ptr(), wb, st) == B.RESLIM_EINVAL
        finally:
            B.reslim_asc_plan_destroy(plan)


def test_compressed_forward_at_the_papers_grid():
    """Table 2(b)'s own workload: the 9.5M model on the 112 km grid ([180, 360, 23] in,
    90 x 180 patches, no multiple of the root size) as one tile, the benchmark's ~7x
    quad-tree; whole output against the oracle, library builder against the oracle's."""
    import bench
    cfg = WL.CONFIGS["m9m"].with_(tiles_y=1, tiles_x=1, halo=0)
    prm = bench.ASC_PARAMS_BY_WORKLOAD["m9m"][0]
    w = WL.make_weights(cfg)
    x = WL.make_fields(cfg)
    imgs = np.ascontiguousarray(x[:, 0])
    args = (cfg.patch, prm["max_leaf"], prm["min_leaf"], prm["canny_low"], prm["canny_high"], prm["tau"])
    tab = A.build(imgs, *args)
    lib = B.reslim_asc_build(imgs, *args)
    for k in tab:
        assert (np.asarray(tab[k]) == np.asarray(lib[k])).all(), k
    L = len(tab["leaf_s"])
    say(f"asc paper grid: {cfg.n_tokens} patches -> {L} leaves; oracle forward ...")
    assert 4 * L < cfg.n_tokens
    ref = A.forward_compressed(x, w, cfg, tab)
    with B.Reslim(cfg, w) as m:
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            y = torch.full((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), float("nan"),
                           dtype=torch.float32, device="cuda")
            B.reslim_asc_forward(m.ctx, plan, cuda(x), y, m.ws)
            out = y.cpu().numpy()
        finally:
            B.reslim_asc_plan_destroy(plan)
    err = max(O.rel_l2(out[b, c], ref[b, c]) for b in range(cfg.batch) for c in range(cfg.out_vars))
    say(f"  max rel-L2 over planes {err:.3e}")
    assert np.isfinite(out).all() and err <= TOL[1]


# ------------------------------------------------------------------ compression combined with TILES
from parity_checks import assert_parity

TILED_F32 = ASC_F32.with_(name="a32t", tiles_y=2, tiles_x=3, halo=1, seed=41)
TILED_BF16 = ASC_BF16.with_(name="abft", tiles_y=2, tiles_x=2, halo=2, seed=42)
TILED_BF16_RAGGED = ASC_BF16_RAGGED.with_(name="abftr", tiles_y=3, tiles_x=2, halo=3, seed=43)


def tiled_table_for(cfg, x, max_leaf=8, min_leaf=1, tau=0.05):
    tiles = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)[0]
    imgs = np.ascontiguousarray(x[:, 0])
    gx, gy = A.sobel(A.smooth(A.quantise_u8(imgs[0])))
    mag = np.abs(gx) + np.abs(gy)
    low, high = int(np.quantile(mag, 0.6)), int(np.quantile(mag, 0.85))
    return A.build_tiles(imgs, cfg.patch, tiles, max_leaf, min_leaf, low, high, tau, Wp=cfg.Wp), tiles, (low, high)


@pytest.mark.parametrize("cfg", [TILED_F32, TILED_BF16, TILED_BF16_RAGGED], ids=lambda c: c.name)
def test_tiled_compressed_forward_parity(cfg):
    """Every (sample, tile) pair compressed on its own haloed box, attention among the leaves of one
    box, interior patches decompressed from their own tile: whole output against the oracle; the
    library's host builder must give the oracle's table."""
    say(f"asc + tiles forward {cfg.name}")
    w = WL.make_weights(cfg, std=0.05)
    x = WL.make_fields(cfg)
    tab, tiles, (low, high) = tiled_table_for(cfg, x)
    lib = B.reslim_asc_build_tiles(np.ascontiguousarray(x[:, 0]), cfg.patch, cfg.tiles_y, cfg.tiles_x, cfg.halo, 8, 1, low, high, 0.05)
    for k in tab:
        assert np.array_equal(np.asarray(tab[k]), np.asarray(lib[k])), k
    L, n_h = len(tab["leaf_s"]), sum(t["n_tok"] for t in tiles)
    per_seq = np.diff(tab["sample_off"])
    say(f"  {cfg.batch * n_h} haloed patches -> {L} leaves, per (sample, tile) {per_seq.tolist()}")
    assert L < cfg.batch * n_h and len(set(per_seq.tolist())) > 1
    ref = A.forward_compressed_tiles(x, w, cfg, tab)
    with B.Reslim(cfg, w) as m:
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            assert B.reslim_asc_plan_info(plan) == (L, int(per_seq.max()))
            y = torch.full((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), float("nan"),
                           dtype=torch.float32, device="cuda")
            B.reslim_asc_forward(m.ctx, plan, cuda(x), y, m.ws)
            out = y.cpu().numpy()
            B.reslim_asc_forward(m.ctx, plan, cuda(x), y, m.ws)
            assert np.array_equal(out, y.cpu().numpy())               # same input, same bits
        finally:
            B.reslim_asc_plan_destroy(plan)
    assert_parity(out, ref, TOL[cfg.dtype], "tiled compressed forward", say)


def test_tiled_single_patch_leaves_reproduce_the_plain_tiled_forward():
    cfg = TILED_BF16
    w = WL.make_weights(cfg, std=0.05)
    x = WL.make_fields(cfg)
    tiles = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)[0]
    tab = A.build_tiles(np.ascontiguousarray(x[:, 0]), cfg.patch, tiles, 1, 1, 10, 20, 0.05, Wp=cfg.Wp)
    assert (tab["leaf_s"] == 1).all()
    with B.Reslim(cfg, w) as m:
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            y = torch.empty((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), dtype=torch.float32, device="cuda")
            B.reslim_asc_forward(m.ctx, plan, cuda(x), y, m.ws)
            plain = m.forward(cuda(x)).cpu().numpy()
        finally:
            B.reslim_asc_plan_destroy(plan)
    # the same rows through the same kernels: the leaf mean of one patch and the row maps are exact
    assert np.array_equal(y.cpu().numpy(), plain)
    assert_parity(plain, O.reslim_forward(x, w, cfg), TOL[1], "plain tiled forward", say)


def test_tiled_plan_errors():
    cfg = TILED_F32
    x = WL.make_fields(cfg)
    tab, tiles, _ = tiled_table_for(cfg, x)
    with B.Reslim(cfg, WL.make_weights(cfg)) as m:
        lib = B.load()
        # a leaf moved across its box edge, two leaves swapped between sequences, a hole, a wrong owner
        q1 = int(tab["sample_off"][1])
        bad = {k: np.array(v, copy=True) for k, v in tab.items()}
        bad["leaf_x0"][q1] -= int(bad["leaf_s"][q1])                     # first leaf of tile 1 pushed out of its box
        with pytest.raises(B.ReslimError):
            B.reslim_asc_plan_create(m.ctx, cfg.batch, bad)
        bad = {k: np.array(v, copy=True) for k, v in tab.items()}
        bad["leaf_y0"][0], bad["leaf_x0"][0] = bad["leaf_y0"][1], bad["leaf_x0"][1]
        bad["leaf_s"][0] = bad["leaf_s"][1]                              # leaf 0 duplicates leaf 1: overlap and hole
        with pytest.raises(B.ReslimError):
            B.reslim_asc_plan_create(m.ctx, cfg.batch, bad)
        bad = {k: np.array(v, copy=True) for k, v in tab.items()}
        t1 = tiles[1]
        g = t1["y0"] * cfg.Wp + t1["x0"]                                 # an interior patch of tile 1 ...
        bad["patch_leaf"][0, g] = 0                                      # ... decompressed from a leaf of tile 0
        with pytest.raises(B.ReslimError):
            B.reslim_asc_plan_create(m.ctx, cfg.batch, bad)
        one = A.build(np.ascontiguousarray(x[:, 0]), cfg.patch, 8, 1, 20, 60, 0.05)     # an untiled table
        with pytest.raises(B.ReslimError):
            B.reslim_asc_plan_create(m.ctx, cfg.batch, one)
        plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
        try:
            L, D = len(tab["leaf_s"]), cfg.embed_dim
            a = torch.zeros((L, D), dtype=torch.float32, device="cuda")
            b = torch.zeros((cfg.batch * cfg.n_tokens, D), dtype=torch.float32, device="cuda")
            B.reslim_asc_decompress(m.ctx, plan, a, b)
            # the two gradient maps under TILES against the oracle (fp32: the same sums in another order)
            r = np.random.default_rng(5)
            N, T = cfg.n_tokens, len(tiles)
            g_c = r.standard_normal((L, D)).astype(np.float32)
            B.reslim_asc_compress_bwd(m.ctx, plan, cuda(g_c), b)
            ref = A.compress_tiles_bwd(g_c, tab, cfg.batch, N, cfg.Wp, T)
            assert_parity(b.cpu().numpy().reshape(cfg.batch, N, D), ref, 1e-6, "compress_bwd under tiles", say, k_elem=1e-5)
            g = r.standard_normal((cfg.batch, N, D)).astype(np.float32)
            B.reslim_asc_decompress_bwd(m.ctx, plan, cuda(g.reshape(-1, D)), a)
            ref = A.decompress_bwd(g, tab)
            got = a.cpu().numpy()
            assert_parity(got[None], ref[None], 1e-6, "decompress_bwd under tiles", say, k_elem=1e-5)
            unused = np.setdiff1d(np.arange(L), np.unique(tab["patch_leaf"]))
            assert len(unused) and not got[unused].any()                  # leaves of halo patches alone receive nothing
            a2 = torch.full_like(a, float("nan"))
            B.reslim_asc_decompress_bwd(m.ctx, plan, cuda(g.reshape(-1, D)), a2)
            assert torch.equal(a, a2)                                     # deterministic
        finally:
            B.reslim_asc_plan_destroy(plan)
