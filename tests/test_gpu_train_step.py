"""GPU parity of one whole training step's gradients (through the C ABI) against the CPU oracle's
chain rule in fp64 (oracle/train_oracle.py, pinned to PyTorch autograd on the CPU): the loss
gradient, the back end (head, residual path, final LayerNorm, halo rows), the front end (gather
transposed, aggregation, tokenisation) stage by stage from the oracle's intermediates, then
reslim_train_step_grads end to end with the loss scaled (Sec. 4.4) and unscaled again.

Tolerances: fp32 path <= 1e-5 (1e-4 where fp32 sums run over many thousand terms), bf16 path
<= 2e-2 per tensor, with the row and element bounds of parity_checks for gradients."""
import numpy as np
import pytest
import torch

from oracle import reslim_oracle as O
from oracle import train_oracle as TO
from paper_2505_04802_amd import binding as B
from paper_2505_04802_amd import workloads as WL
from parity_checks import GRAD_BF16, assert_parity

pytestmark = pytest.mark.gpu

TRAIN_F32 = WL.ReslimConfig("tr32", batch=2, in_vars=3, out_vars=2, H=24, W=40, scale=2, patch=2, embed_dim=48, heads=3,
                            mlp_ratio=2, depth=2, tiles_y=2, tiles_x=3, halo=1, dtype=0, seed=51, res_idx=1)
TRAIN_BF16 = WL.ReslimConfig("trbf", batch=2, in_vars=3, out_vars=3, H=44, W=60, scale=4, patch=2, embed_dim=128, heads=2,
                             mlp_ratio=4, depth=2, tiles_y=2, tiles_x=2, halo=2, dtype=1, seed=52)          # head width 192
TRAIN_BF16_DH128 = TRAIN_BF16.with_(name="trbf128", embed_dim=256, heads=2, in_vars=5, out_vars=4, seed=53)   # head width 256
# the headline workload's residual-path geometry (scale 8, 16 variables: 16 outputs per pass of the weight-gradient
# kernel, 20-column runs) and a scale above it (whole-row runs), both small enough for the oracle
TRAIN_S8 = WL.ReslimConfig("trs8", batch=1, in_vars=16, out_vars=16, H=8, W=16, scale=8, patch=2, embed_dim=32, heads=2,
                           mlp_ratio=2, depth=1, tiles_y=2, tiles_x=2, halo=1, dtype=0, seed=54)
TRAIN_S16 = WL.ReslimConfig("trs16", batch=2, in_vars=3, out_vars=2, H=6, W=8, scale=16, patch=2, embed_dim=32, heads=2,
                            mlp_ratio=2, depth=1, tiles_y=1, tiles_x=2, halo=1, dtype=0, seed=55)
FRONT = ("w_pe", "b_pe", "var_emb", "agg_q0", "agg_wq", "agg_bq", "agg_wk", "agg_bk", "agg_wv", "agg_bv", "agg_wo", "agg_bo",
         "pos_emb", "res_emb")
BACK = ("lnf_g", "lnf_b", "w_head", "b_head", "w_res", "b_res")


def say(m):
    print(m, flush=True)


def cuda(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype)


def u8(n):
    return torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")


def case(cfg, std):
    w = WL.make_weights(cfg, std=std)
    if cfg.out_vars < cfg.in_vars:
        w["out_var_idx"] = np.arange(cfg.in_vars - 1, cfg.in_vars - 1 - cfg.out_vars, -1).astype(np.int32)
    x = WL.make_fields(cfg)
    r = np.random.default_rng(cfg.seed + 7)
    sH, sW = cfg.H * cfg.scale, cfg.W * cfg.scale
    target = r.standard_normal((cfg.batch, cfg.out_vars, sH, sW)).astype(np.float32)
    lat_w = O.lat_weights(sH, -70.0, 80.0).astype(np.float32)
    return w, x, target, lat_w


def grad_buffers(w, names):
    return {n: torch.full(np.shape(w[n]), float("nan"), dtype=torch.float32, device="cuda") for n in names}


def check_grads(got, ref, names, cfg, what, zero_ok=("agg_bk",)):
    tol = 1e-4 if cfg.dtype == 0 else 2e-2
    extra = GRAD_BF16 if cfg.dtype else dict(k_elem=1e-3, row_tol=1e-4)
    scale = max(np.abs(ref[n]).max() for n in names)
    for n in names:
        a = got[n].cpu().numpy()
        assert np.isfinite(a).all(), n
        if n in zero_ok:        # exactly zero in exact arithmetic: both sides hold rounding noise
            assert np.abs(a).max() <= 1e-3 * scale and np.abs(ref[n]).max() <= 1e-9 * scale, n
            continue
        if n == "res_emb":      # rows the forward did not read are exactly zero
            other = [i for i in range(cfg.n_res) if i != cfg.res_idx]
            assert not a[other].any() and not ref[n][other].any()
            assert_parity(a[cfg.res_idx], ref[n][cfg.res_idx], tol, f"{what} d_{n}", say, **extra)
            continue
        assert_parity(a, ref[n], tol, f"{what} d_{n}", say, **extra)


@pytest.mark.parametrize("shape", [(2, 3, 37, 53), (1, 2, 64, 300), (1, 1, 1, 9), (1, 1, 70, 1), (4, 8, 512, 1024)], ids=str)
def test_loss_gradient_parity(shape):
    r = np.random.default_rng([9, shape[2], shape[3]])
    pred = r.standard_normal(shape).astype(np.float32)
    pred[..., : shape[3] // 2] = np.round(pred[..., : shape[3] // 2] * 2) / 2        # many equal neighbours: sign(0) = 0 matters
    target = r.standard_normal(shape).astype(np.float32)
    lw = O.lat_weights(shape[2], -80.0, 85.0).astype(np.float32)
    ref = TO.bayes_loss_bwd(pred, target, lw, 0.25) * 8.0
    d = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    B.reslim_bayes_loss_bwd(cuda(pred), cuda(target), cuda(lw), 0.25, 8.0, d)
    assert_parity(d.cpu().numpy(), ref, 1e-5, f"loss gradient {shape}", say, k_elem=1e-4)


@pytest.mark.parametrize("cfg", [TRAIN_F32, TRAIN_BF16, TRAIN_BF16_DH128, TRAIN_S8, TRAIN_S16], ids=lambda c: c.name)
def test_model_ends_stage_by_stage(cfg):
    """Each end of the model from the ORACLE's intermediates, so errors do not compound."""
    w, x, target, lat_w = case(cfg, 0.1)
    say(f"train stages {cfg.name}: oracle ...")
    loss, g_ref, inter = TO.reslim_loss_and_grads(x, target, w, cfg, lat_w, 0.5)
    with B.Reslim(cfg, w) as m:
        B.reslim_train_prepare_model(m.ctx, w)
        B.reslim_train_prepare_model(m.ctx, w)                          # idempotent
        xd = cuda(x)
        # back end
        g = grad_buffers(w, BACK)
        d_tok = torch.full((cfg.batch, m.n_h, cfg.embed_dim), float("nan"), dtype=torch.float32, device="cuda")
        ws = u8(B.reslim_head_bwd_workspace_bytes(m.ctx, cfg.batch))
        B.reslim_head_bwd(m.ctx, xd, cuda(inter["tokens_out"]), cuda(inter["d_y"]), d_tok, g, cfg.batch, ws)
        torch.cuda.synchronize()
        tol = 1e-5 if cfg.dtype == 0 else 2e-2
        assert_parity(d_tok.cpu().numpy(), inter["d_tokens_out"], tol, "d_tokens after the last block", say,
                      **(GRAD_BF16 if cfg.dtype else {}))
        tiles, gather_idx, interior_src, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
        halo_rows = np.setdiff1d(np.arange(n_h), np.asarray(interior_src))
        assert len(halo_rows) and not d_tok.cpu().numpy()[:, halo_rows].any()       # the halo's outputs are discarded
        check_grads(g, g_ref, BACK, cfg, "back end")
        # front end
        g = grad_buffers(w, FRONT)
        ws = u8(B.reslim_embed_bwd_workspace_bytes(m.ctx, cfg.batch))
        B.reslim_embed_bwd(m.ctx, xd, cuda(inter["d_tokens_in"]), g, cfg.batch, ws)
        torch.cuda.synchronize()
        check_grads(g, g_ref, FRONT, cfg, "front end")
        g2 = grad_buffers(w, FRONT)
        B.reslim_embed_bwd(m.ctx, xd, cuda(inter["d_tokens_in"]), g2, cfg.batch, ws)
        torch.cuda.synchronize()
        assert all(torch.equal(g[n], g2[n]) for n in FRONT)                         # deterministic


def run_step(m, cfg, w, x, target, lat_w, tv, scale):
    saved_b, ws_b = B.reslim_train_step_bytes(m.ctx, cfg.batch)
    saved, ws = u8(saved_b), u8(ws_b)
    g = grad_buffers(w, B.MODEL_PARAMS)
    y = torch.full((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), float("nan"), dtype=torch.float32, device="cuda")
    loss3 = torch.zeros(3, dtype=torch.float64, device="cuda")
    B.reslim_train_step_grads(m.ctx, cuda(x), cuda(target), cuda(lat_w), tv, scale, y, loss3, g, cfg.batch, saved, ws)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.reslim_grads_unscale(m.ctx, g, 1.0 / scale, flag)
    torch.cuda.synchronize()
    return g, y.cpu().numpy(), loss3.cpu().numpy(), int(flag.item())


@pytest.mark.parametrize("cfg", [TRAIN_F32, TRAIN_BF16, TRAIN_BF16_DH128, TRAIN_S8, TRAIN_S16], ids=lambda c: c.name)
def test_train_step_parity(cfg):
    """Forward, loss and every one of the 32 gradients end to end, the loss scaled by 1024 and the
    gradients unscaled again; a second call gives the same bits."""
    w, x, target, lat_w = case(cfg, 0.1)
    say(f"train step {cfg.name}: oracle ...")
    loss, g_ref, inter = TO.reslim_loss_and_grads(x, target, w, cfg, lat_w, 0.5)
    with B.Reslim(cfg, w) as m:
        B.reslim_train_prepare_model(m.ctx, w)
        g, y, loss3, flag = run_step(m, cfg, w, x, target, lat_w, 0.5, 1024.0)
        assert flag == 0
        tol = 1e-5 if cfg.dtype == 0 else 2e-2
        assert_parity(y, inter["y"], tol, "prediction", say)
        for a, b_ in zip(loss3, loss):
            assert abs(a - b_) <= (1e-5 if cfg.dtype == 0 else 2e-2) * abs(b_), (loss3, loss)
        check_grads(g, g_ref, B.MODEL_PARAMS, cfg, "step")
        g2, y2, loss3_2, _ = run_step(m, cfg, w, x, target, lat_w, 0.5, 1024.0)
        assert np.array_equal(y, y2) and np.array_equal(loss3, loss3_2)
        assert all(torch.equal(g[n], g2[n]) for n in B.MODEL_PARAMS)
        # a non-finite value in any of the 32 tensors raises the flag of the unscale pass
        for name in ("w_pe", "b_fc1", "b_res"):
            g2[name].view(-1)[-1] = float("inf")
            flag = torch.zeros(1, dtype=torch.int32, device="cuda")
            B.reslim_grads_unscale(m.ctx, g2, 0.5, flag)
            torch.cuda.synchronize()
            assert int(flag.item()) == 1, name
            g2[name].view(-1)[-1] = 0.0


def test_train_step_c1_one_sample():
    """The c1 workload's model and tiling (D = 512, 8 heads, 6 blocks, 16 tiles with halo) on one
    of its four samples (the fp64 oracle of one sample's step takes about a minute)."""
    cfg = WL.CONFIGS["c1"].with_(batch=1)
    w, x, target, lat_w = case(cfg, 0.05)
    with B.Reslim(cfg, w) as m:
        B.reslim_train_prepare_model(m.ctx, w)
        g, y, loss3, flag = run_step(m, cfg, w, x, target, lat_w, 0.5, 256.0)
    say("c1 train step: oracle ...")
    loss, g_ref, inter = TO.reslim_loss_and_grads(x, target, w, cfg, lat_w, 0.5)
    assert flag == 0
    assert_parity(y, inter["y"], 2e-2, "prediction", say)
    assert abs(loss3[0] - loss[0]) <= 2e-2 * abs(loss[0])
    check_grads(g, g_ref, B.MODEL_PARAMS, cfg, "c1 step")


def test_train_step_errors():
    cfg = TRAIN_F32
    w, x, target, lat_w = case(cfg, 0.1)
    with B.Reslim(cfg, w) as m:
        lib = B.load()
        ws = u8(1 << 20)
        g = B.GradsC()
        import ctypes
        d = torch.zeros(8, device="cuda")
        # before reslim_train_prepare_model
        assert lib.reslim_embed_bwd(m.ctx, d.data_ptr(), d.data_ptr(), ctypes.byref(B._grads_c(grad_buffers(w, FRONT))), cfg.batch,
                                    ws.data_ptr(), ws.numel(), None) == B.RESLIM_EINVAL
        B.reslim_train_prepare_model(m.ctx, w)
        assert lib.reslim_embed_bwd(m.ctx, d.data_ptr(), d.data_ptr(), ctypes.byref(g), cfg.batch, ws.data_ptr(), ws.numel(), None) == B.RESLIM_EINVAL   # null gradients
        assert lib.reslim_embed_bwd(m.ctx, d.data_ptr(), d.data_ptr(), ctypes.byref(B._grads_c(grad_buffers(w, FRONT))), cfg.batch,
                                    ws.data_ptr(), 256, None) == B.RESLIM_EWORKSPACE
        assert lib.reslim_bayes_loss_bwd(None, d.data_ptr(), d.data_ptr(), 1, 1, 2, 4, 1.0, 1.0, d.data_ptr(), None) == B.RESLIM_EINVAL
    bad = TRAIN_BF16.with_(scale=2)                                    # head width 3 * 16 = 48: no multiple of 64
    wb = WL.make_weights(bad)
    with B.Reslim(bad, wb) as m:
        with pytest.raises(B.ReslimError):
            B.reslim_train_prepare_model(m.ctx, wb)
