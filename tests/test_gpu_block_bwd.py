"""GPU parity of the training side of a block (through the C ABI) against the CPU oracle's
chain rule in fp64: the LayerNorm gradient, the gradient of each of the four linear layers
(input gradient, weight gradient, bias gradient), and the whole block forward-for-training +
backward (input gradient and all twelve parameter gradients).

Tolerances: fp32 debug path <= 1e-5 (1e-4 for sums over many thousand tokens in fp32),
bf16 path <= 2e-2, max relative L2 per tensor (the bar of the benchmark definition)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import reslim_oracle as O
from paper_2505_04802_amd import binding as B
from paper_2505_04802_amd import workloads as WL
from parity_checks import GRAD_BF16, assert_parity
from test_gpu_parity import SMALL_F32, SMALL_BF16, SMALL_BF16_DH128, TOL, cuda, say, weights_for

pytestmark = pytest.mark.gpu
CFGS = [SMALL_F32, SMALL_BF16, SMALL_BF16_DH128]
# wide rows: from 1280 columns on a whole work-group takes a row of the LayerNorm gradient; 1280 and
# 2304 leave the last column group of a thread partly empty, 3072 and 8192 are the 1B and 10B widths
WIDE_LN = [SMALL_BF16_DH128.with_(name=f"w{d}", embed_dim=d, heads=h, depth=1, mlp_ratio=1, batch=1)
           for d, h in ((1280, 10), (2304, 18), (3072, 24), (8192, 32))]
WIDE_LN.append(SMALL_F32.with_(name="w2304_f32", embed_dim=2304, heads=18, depth=1, mlp_ratio=1, batch=1))
WIDE_BLOCK = [SMALL_BF16_DH128.with_(name="w3072_block", embed_dim=3072, heads=24, depth=1, batch=1),
              SMALL_BF16_DH128.with_(name="w8192_block", embed_dim=8192, heads=32, depth=1, mlp_ratio=1, batch=1)]


def u8(n):
    return torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")


def rnd(shape, seed, bf16):
    a = np.random.default_rng([seed, 7]).standard_normal(shape, dtype=np.float32)
    return WL.round_to_bf16(a) if bf16 else a


@pytest.mark.parametrize("cfg", CFGS + WIDE_LN, ids=lambda c: c.name)
def test_layernorm_bwd_parity(cfg):
    D, bf = cfg.embed_dim, cfg.dtype == 1
    rows = 1237 if D <= 4096 else 4099              # several slabs of rows and a ragged last one
    x = rnd((rows, D), 1, False) * 1.5 + 0.3
    dy = rnd((rows, D), 2, bf)
    res = rnd((rows, D), 3, False)
    gam = (1 + 0.2 * rnd((D,), 4, False)).astype(np.float32)
    ref_dx, ref_dg, ref_db = O.layer_norm_bwd(x, gam, dy)
    with B.Reslim(cfg, weights_for(cfg)) as m:
        dx = torch.empty((rows, D), dtype=torch.float32, device="cuda")
        dg, db = (torch.empty(D, dtype=torch.float32, device="cuda") for _ in range(2))
        ws = u8(1024 * 2 * D * 4)
        B.reslim_layernorm_bwd(m.ctx, cuda(x), cuda(dy, m.act_dtype), cuda(gam), cuda(res), dx, dg, db, rows, ws)
        torch.cuda.synchronize()
        errs = {}
        for name, got, ref in (("dx", dx, ref_dx + res), ("dgamma", dg, ref_dg), ("dbeta", db, ref_db)):
            errs[name] = O.rel_l2(got.cpu().numpy(), ref)
            say(f"  layernorm_bwd {cfg.name} {name} rel-L2 {errs[name]:.3e}")
        # fp32 arithmetic on both paths; dy is the only bf16 input
        assert max(errs.values()) <= 1e-5, (errs, np.where(np.abs(dg.cpu().numpy() - ref_dg) > 1e-3)[0][:8])
        B.reslim_layernorm_bwd(m.ctx, cuda(x), cuda(dy, m.act_dtype), cuda(gam), None, dx, dg, db, rows, ws)
        assert O.rel_l2(dx.cpu().numpy(), ref_dx) <= 1e-5


@pytest.mark.parametrize("cfg", CFGS, ids=lambda c: c.name)
@pytest.mark.parametrize("which", [0, 1, 2, 3])
def test_linear_bwd_parity(cfg, which):
    D, R, bf = cfg.embed_dim, cfg.embed_dim * cfg.mlp_ratio, cfg.dtype == 1
    n_in, n_out = (R if which == 3 else D), (3 * D, D, R, D)[which]
    name = ("w_qkv", "w_proj", "w_fc1", "w_fc2")[which]
    rows = 1000 + 37 * which                        # not a multiple of the token block of the kernels
    w = weights_for(cfg, std=0.1)
    x, dy = rnd((rows, n_in), 10 + which, bf), rnd((rows, n_out), 20 + which, bf)
    ref_dx, ref_dw, ref_db = O.linear_bwd(x, w[name][1], dy)
    with B.Reslim(cfg, w) as m:
        B.reslim_train_prepare(m.ctx)
        dx = torch.empty((rows, n_in), dtype=m.act_dtype, device="cuda")
        dw = torch.full((n_out, n_in), float("nan"), dtype=torch.float32, device="cuda")
        db = torch.empty(n_out, dtype=torch.float32, device="cuda")
        ws = u8(B.reslim_linear_bwd_workspace_bytes(m.ctx, which, rows))
        B.reslim_linear_bwd(m.ctx, 1, which, cuda(x, m.act_dtype), cuda(dy, m.act_dtype), dx, dw, db, rows, ws)
        torch.cuda.synchronize()
        for nm, got, ref, tol in (("dx", dx, ref_dx, TOL[cfg.dtype]), ("dw", dw, ref_dw, 1e-5), ("db", db, ref_db, 1e-5)):
            # dw, db: exact products of the given inputs, fp32 sums
            assert_parity(got.float().cpu().numpy(), ref, tol, f"linear_bwd {cfg.name} {name} {nm}", say)


@pytest.mark.parametrize("cfg", CFGS + WIDE_BLOCK, ids=lambda c: c.name)
def test_block_train_parity(cfg):
    """Forward-for-training and backward of one block on the tile-major stream."""
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    D, layer = cfg.embed_dim, cfg.depth - 1
    # wide weights: softmaxes and GELUs far from linear (scaled down with the width, so that the
    # pre-activations keep that spread)
    w = weights_for(cfg, std=0.1 if D <= 256 else 0.1 * (256.0 / D) ** 0.5)
    x = rnd((cfg.batch, n_h, D), 30, False)
    d_out = rnd((cfg.batch, n_h, D), 31, False)
    ref_out = O.reslim_block(x, tiles, w, layer, cfg.heads)
    ref_dx, ref_g = O.reslim_block_bwd(x, tiles, w, layer, cfg.heads, d_out)
    with B.Reslim(cfg, w) as m:
        B.reslim_train_prepare(m.ctx)
        sb, wb = B.reslim_block_train_bytes(m.ctx, cfg.batch)
        saved, ws = u8(sb), u8(wb)
        x_dev, out = cuda(x), torch.empty((cfg.batch, n_h, D), dtype=torch.float32, device="cuda")
        B.reslim_block_fwd_train(m.ctx, layer, x_dev, out, saved, cfg.batch, ws)
        assert_parity(out.cpu().numpy(), ref_out, TOL[cfg.dtype], f"block_fwd_train {cfg.name}", say)
        plain = m.block(layer, x_dev.clone()).cpu().numpy()          # the inference entry point on the same input
        assert O.rel_l2(out.cpu().numpy(), plain) <= TOL[cfg.dtype]
        grads = {n: torch.full(np.shape(w[n][layer]), float("nan"), dtype=torch.float32, device="cuda") for n in B.BLOCK_PARAMS}
        dx = torch.empty_like(out)
        B.reslim_block_bwd(m.ctx, layer, x_dev, saved, cuda(d_out), dx, grads, cfg.batch, ws)
        torch.cuda.synchronize()
        extra = GRAD_BF16 if cfg.dtype else {}
        assert_parity(dx.cpu().numpy(), ref_dx, TOL[cfg.dtype], f"block_bwd {cfg.name} d_x", say, **extra)
        for n in B.BLOCK_PARAMS:
            assert_parity(grads[n].cpu().numpy(), ref_g[n], TOL[cfg.dtype], f"block_bwd {cfg.name} d_{n}", say, **extra)
        # determinism: a second backward gives the same bits
        again = {n: torch.empty_like(grads[n]) for n in B.BLOCK_PARAMS}
        dx2 = torch.empty_like(dx)
        B.reslim_block_bwd(m.ctx, layer, x_dev, saved, cuda(d_out), dx2, again, cfg.batch, ws)
        torch.cuda.synchronize()
        assert torch.equal(dx, dx2) and all(torch.equal(grads[n], again[n]) for n in B.BLOCK_PARAMS)


def test_block_train_c1_full_size():
    """The block shape bench.py times (c1: 42,560 tile-major tokens, D = 512, 8 heads, 16 tiles with
    halo): forward-for-training and backward of one block against the oracle on ALL tokens (the
    parameter gradients are sums over every token, so nothing can be sampled; the fp64 oracle
    takes about 15 s for this)."""
    cfg = WL.CONFIGS["c1"].with_(depth=1)
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    D = cfg.embed_dim
    w = WL.make_weights(cfg, std=0.05)
    x = rnd((cfg.batch, n_h, D), 40, False)
    d_out = rnd((cfg.batch, n_h, D), 41, False)
    with B.Reslim(cfg, w) as m:
        B.reslim_train_prepare(m.ctx)
        sb, wb = B.reslim_block_train_bytes(m.ctx, cfg.batch)
        saved, ws = u8(sb), u8(wb)
        x_dev = cuda(x)
        out, dx = (torch.empty((cfg.batch, n_h, D), dtype=torch.float32, device="cuda") for _ in range(2))
        grads = {n: torch.full(np.shape(w[n][0]), float("nan"), dtype=torch.float32, device="cuda") for n in B.BLOCK_PARAMS}
        B.reslim_block_fwd_train(m.ctx, 0, x_dev, out, saved, cfg.batch, ws)
        B.reslim_block_bwd(m.ctx, 0, x_dev, saved, cuda(d_out), dx, grads, cfg.batch, ws)
        torch.cuda.synchronize()
        got_out, got_dx = out.cpu().numpy(), dx.cpu().numpy()
        got_g = {n: grads[n].cpu().numpy() for n in B.BLOCK_PARAMS}
    say("  oracle ...")
    ref_out = O.reslim_block(x, tiles, w, 0, cfg.heads)
    ref_dx, ref_g = O.reslim_block_bwd(x, tiles, w, 0, cfg.heads, d_out)
    for name, got, ref in [("x_out", got_out, ref_out), ("d_x", got_dx, ref_dx)] + [("d_" + n, got_g[n], ref_g[n]) for n in B.BLOCK_PARAMS]:
        assert_parity(got, ref, 2e-2, f"c1 block train {name}", say, **({} if name == "x_out" else GRAD_BF16))


def test_training_entry_point_errors_and_tiny_tiles():
    """Error codes (no launch happens): training calls before reslim_train_prepare, null buffers,
    short or misaligned buffers, bad layer; then a tile grid as fine as the patch grid (one-token
    tiles with halo: every softmax has 1 .. 9 keys) through the whole block gradient."""
    cfg = SMALL_BF16
    with B.Reslim(cfg, weights_for(cfg)) as m:
        lib = B.load()
        st = torch.cuda.current_stream().cuda_stream
        n_h, D = m.n_h, cfg.embed_dim
        x = torch.zeros((cfg.batch, n_h, D), dtype=torch.float32, device="cuda")
        out, dx = torch.empty_like(x), torch.empty_like(x)
        sb, wb = B.reslim_block_train_bytes(m.ctx, cfg.batch)
        saved, ws = u8(sb), u8(wb)
        args = (x.data_ptr(), out.data_ptr(), saved.data_ptr(), sb, cfg.batch, ws.data_ptr(), wb, st)
        assert lib.reslim_block_fwd_train(m.ctx, 0, *args) == B.RESLIM_EINVAL
        assert b"reslim_train_prepare" in lib.reslim_last_error(m.ctx)
        B.reslim_train_prepare(m.ctx)
        B.reslim_train_prepare(m.ctx)                                  # idempotent
        assert lib.reslim_block_fwd_train(m.ctx, cfg.depth, *args) == B.RESLIM_EINVAL
        assert lib.reslim_block_fwd_train(m.ctx, 0, x.data_ptr(), x.data_ptr(), *args[2:]) == B.RESLIM_EINVAL      # aliased
        assert lib.reslim_block_fwd_train(m.ctx, 0, x.data_ptr(), out.data_ptr(), saved.data_ptr(), sb - 256, cfg.batch,
                                          ws.data_ptr(), wb, st) == B.RESLIM_EWORKSPACE
        assert lib.reslim_block_fwd_train(m.ctx, 0, x.data_ptr(), out.data_ptr(), saved.data_ptr(), sb, cfg.batch,
                                          ws.data_ptr() + 16, wb - 16, st) == B.RESLIM_EWORKSPACE
        assert lib.reslim_block_fwd_train(m.ctx, 0, x.data_ptr(), out.data_ptr(), saved.data_ptr(), sb, 0,
                                          ws.data_ptr(), wb, st) == B.RESLIM_ESHAPE
        g = B.BlockGradsC()                                            # all twelve pointers null
        assert lib.reslim_block_bwd(m.ctx, 0, x.data_ptr(), saved.data_ptr(), sb, out.data_ptr(), dx.data_ptr(),
                                    ctypes.byref(g), cfg.batch, ws.data_ptr(), wb, st) == B.RESLIM_EINVAL
        assert lib.tiles_attention_bwd(m.ctx, None, None, None, None, None, cfg.batch, ws.data_ptr(), wb, st) == B.RESLIM_EINVAL
        assert lib.reslim_linear_bwd(m.ctx, 0, 4, x.data_ptr(), x.data_ptr(), None, x.data_ptr(), x.data_ptr(), 8,
                                     ws.data_ptr(), wb, st) == B.RESLIM_EINVAL
        assert lib.reslim_layernorm_bwd(m.ctx, x.data_ptr(), x.data_ptr(), x.data_ptr(), None, dx.data_ptr(), dx.data_ptr(),
                                        dx.data_ptr(), 8, ws.data_ptr(), 64, st) == B.RESLIM_EWORKSPACE
    tiny = SMALL_BF16.with_(name="tinytiles", H=8, W=12, tiles_y=4, tiles_x=6, halo=1, batch=1)
    tiles, _, _, n_h = O.tiles_partition(tiny.Hp, tiny.Wp, tiny.tiles_y, tiny.tiles_x, tiny.halo)
    w = weights_for(tiny, std=0.1)
    x, d_out = rnd((1, n_h, tiny.embed_dim), 50, False), rnd((1, n_h, tiny.embed_dim), 51, False)
    ref_dx, ref_g = O.reslim_block_bwd(x, tiles, w, 0, tiny.heads, d_out)
    with B.Reslim(tiny, w) as m:
        B.reslim_train_prepare(m.ctx)
        sb, wb = B.reslim_block_train_bytes(m.ctx, 1)
        saved, ws = u8(sb), u8(wb)
        x_dev = cuda(x)
        out, dx = (torch.empty((1, n_h, tiny.embed_dim), dtype=torch.float32, device="cuda") for _ in range(2))
        grads = {n: torch.empty(np.shape(w[n][0]), dtype=torch.float32, device="cuda") for n in B.BLOCK_PARAMS}
        B.reslim_block_fwd_train(m.ctx, 0, x_dev, out, saved, 1, ws)
        B.reslim_block_bwd(m.ctx, 0, x_dev, saved, cuda(d_out), dx, grads, 1, ws)
        torch.cuda.synchronize()
        errs = {"d_x": O.rel_l2(dx.cpu().numpy(), ref_dx)}
        errs.update({n: O.rel_l2(grads[n].cpu().numpy(), ref_g[n]) for n in B.BLOCK_PARAMS})
    say(f"  tiny tiles (n_t = {sorted(set(t['n_tok'] for t in tiles))}): worst rel-L2 {max(errs.values()):.3e}")
    assert max(errs.values()) <= 2e-2, errs


def test_block_grads_unscale_and_overflow_flag():
    """Dynamic gradient scaling: a backward on an upstream gradient multiplied by S, unscaled by 1/S,
    equals the unscaled backward (S a power of two: exact in bf16 and fp32); an infinity planted in
    one gradient sets the flag, a clean set leaves it alone."""
    cfg = SMALL_BF16
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    D, S = cfg.embed_dim, 4096.0
    w = weights_for(cfg, std=0.1)
    x, d_out = rnd((cfg.batch, n_h, D), 60, False), rnd((cfg.batch, n_h, D), 61, False)
    with B.Reslim(cfg, w) as m:
        B.reslim_train_prepare(m.ctx)
        sb, wb = B.reslim_block_train_bytes(m.ctx, cfg.batch)
        saved, ws = u8(sb), u8(wb)
        x_dev = cuda(x)
        out, dx = (torch.empty((cfg.batch, n_h, D), dtype=torch.float32, device="cuda") for _ in range(2))
        g1 = {n: torch.empty(np.shape(w[n][0]), dtype=torch.float32, device="cuda") for n in B.BLOCK_PARAMS}
        g2 = {n: torch.empty_like(g1[n]) for n in B.BLOCK_PARAMS}
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.reslim_block_fwd_train(m.ctx, 0, x_dev, out, saved, cfg.batch, ws)
        B.reslim_block_bwd(m.ctx, 0, x_dev, saved, cuda(d_out), dx, g1, cfg.batch, ws)
        B.reslim_block_bwd(m.ctx, 0, x_dev, saved, cuda(d_out * np.float32(S)), dx, g2, cfg.batch, ws)
        B.reslim_block_grads_unscale(m.ctx, g2, 1.0 / S, flag)
        torch.cuda.synchronize()
        assert int(flag.item()) == 0
        ref, found = O.grads_unscale({n: g2[n].cpu().numpy() * S for n in B.BLOCK_PARAMS}, S)
        assert not found
        for n in B.BLOCK_PARAMS:
            assert O.rel_l2(g2[n].cpu().numpy(), g1[n].cpu().numpy()) <= 1e-6, n      # same bits up to fp32 sums of scaled terms
            assert np.allclose(g2[n].cpu().numpy(), ref[n], rtol=1e-6, atol=0)
        g2["w_fc1"][3, 5] = float("inf")
        B.reslim_block_grads_unscale(m.ctx, g2, 0.5, flag)
        torch.cuda.synchronize()
        assert int(flag.item()) == 1
        assert O.grads_unscale({n: g2[n].cpu().numpy() for n in B.BLOCK_PARAMS}, 1.0)[1]
        lib = B.load()
        g = B.BlockGradsC(**{n: g2[n].data_ptr() for n in B.BLOCK_PARAMS})
        assert lib.reslim_block_grads_unscale(m.ctx, ctypes.byref(g), 0.0, flag.data_ptr(), None) == B.RESLIM_EINVAL
