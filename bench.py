#!/usr/bin/env python3
"""Benchmark of the Reslim+TILES forward on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

A step is one pass of the whole forward (embed, all blocks, head, residual path,
stitch) over one batch of synthetic fields already resident in HBM.  Prints ONE
JSON line: whole-job tokens/s (unique coarse tokens, halo copies not counted), the
roofline position of the dominant kernel measured with HIP events on the launch
stream, and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_FP32_VECTOR_TFLOPS = 157.3  # MI355X fp32 vector (packed); plain fp32 instructions reach half of it
ALU_BOUND = ("embed_agg",)      # kernels whose time is plain fp32 vector arithmetic, not HBM or MFMA

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (see
# profiles/), keyed by (workload, kernel label); None where not measured.
# Source: profiles/forward_and_train_block_c1_all_kernels.md (fetched + written, scaled by the copy kernel).
# FC2 and the projection share one kernel symbol in every profile: no separate figure for them.
MEASURED_TRAFFIC = {
    ("c1", "gemm_fc1"): 140.5e6 + 167.6e6,
    ("c1", "tiles_attention"): 203.8e6,            # both kernel symbols (five launches of six, the last block's one), weighted
    ("c1", "gemm_qkv"): 98.2e6 + 130.7e6,
    ("c1", "layernorm"): 84.7e6 + 42.3e6,
    # profiles/forward_and_train_block_c2_all_kernels.md
    ("c2", "gemm_fc1"): 1961.5e6 + 1300.5e6,
    ("c2", "gemm_qkv"): 1504.2e6 + 991.7e6,
    ("c2", "tiles_attention"): 2321.4e6,           # both kernel symbols, weighted 11 : 1
    ("c2", "layernorm"): 651.8e6 + 325.9e6,
    # profiles/forward_c3_all_kernels.md
    ("c3", "gemm_fc1"): 4749.4e6 + 3155.6e6,
    ("c3", "gemm_qkv"): 3812.2e6 + 2477.3e6,
    ("c3", "tiles_attention"): 8763.7e6,          # both kernel symbols (seven launches of eight, the last block's one), weighted
    ("c3", "layernorm"): 1580.0e6 + 791.1e6,
    ("c3", "residual_unpatchify"): 4860.3e6 + 4246.7e6,
    ("c3", "gemm_head"): 3278.1e6 + 4252.4e6,
}


def train_block(B, torch, model, cfg, K, verbose):
    """Times reslim_block_fwd_train + reslim_block_bwd of block 0 on synthetic N(0,1) streams."""
    D, R = cfg.embed_dim, cfg.embed_dim * cfg.mlp_ratio
    B.reslim_train_prepare(model.ctx)
    sb, wb = B.reslim_block_train_bytes(model.ctx, cfg.batch)
    saved = torch.empty(sb, dtype=torch.uint8, device="cuda")
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cpu").manual_seed(0)
    x = torch.randn((cfg.batch, model.n_h, D), generator=g).cuda()
    d_out = torch.randn((cfg.batch, model.n_h, D), generator=g).cuda()
    out, dx = torch.empty_like(x), torch.empty_like(x)
    shapes = {"ln1_g": (D,), "ln1_b": (D,), "w_qkv": (3 * D, D), "b_qkv": (3 * D,), "w_proj": (D, D), "b_proj": (D,),
              "ln2_g": (D,), "ln2_b": (D,), "w_fc1": (R, D), "b_fc1": (R,), "w_fc2": (D, R), "b_fc2": (D,)}
    grads = {n: torch.empty(s, dtype=torch.float32, device="cuda") for n, s in shapes.items()}
    fwd = lambda: B.reslim_block_fwd_train(model.ctx, 0, x, out, saved, cfg.batch, ws)
    bwd = lambda: B.reslim_block_bwd(model.ctx, 0, x, saved, d_out, dx, grads, cfg.batch, ws)
    res = {}
    for label, fn in (("fwd_train", fwd), ("bwd", bwd)):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            fn()
        torch.cuda.synchronize()
        res[label + "_ms"] = round((time.perf_counter() - t0) / K * 1e3, 4)
    B.reslim_profile_enable(model.ctx, 32 * K)
    for _ in range(K):
        fwd()
        bwd()
    torch.cuda.synchronize()
    agg = {}
    for name, ms, flop, nbytes in B.reslim_profile_read(model.ctx):
        a = agg.setdefault(name, dict(calls=0, ms=0.0, flop=0.0, bytes=0.0))
        a["calls"] += 1
        a["ms"] += ms
        a["flop"] += flop
        a["bytes"] += nbytes
    B.reslim_profile_enable(model.ctx, 0)
    ks = []
    for name, a in agg.items():
        sec = a["ms"] * 1e-3
        ks.append(dict(kernel=name, launches=a["calls"] // K, ms=round(a["ms"] / K, 5),
                       tflops=round(a["flop"] / sec / 1e12, 2) if a["flop"] else None, gbs=round(a["bytes"] / sec / 1e9, 1)))
    ks.sort(key=lambda k: -k["ms"])
    flop = sum(a["flop"] for a in agg.values()) / K
    res["tflops"] = round(flop / ((res["fwd_train_ms"] + res["bwd_ms"]) * 1e-3) / 1e12, 2)
    res["haloed_tokens_per_s"] = round(cfg.batch * model.n_h / ((res["fwd_train_ms"] + res["bwd_ms"]) * 1e-3), 1)
    res["kernels"] = ks
    if verbose:
        for k in ks:
            print("train_block " + json.dumps(k), file=sys.stderr)
    return res


def train_step(B, torch, np, model, cfg, w, x_host, K, verbose):
    """Times reslim_train_step_grads: forward keeping intermediates, Bayesian loss, backward through the whole
    model (all 32 parameter gradients), the loss scaled by 1024 (Sec. 4.4) and the gradients unscaled again."""
    B.reslim_train_prepare_model(model.ctx, w)
    sb, wb = B.reslim_train_step_bytes(model.ctx, cfg.batch)
    saved = torch.empty(sb, dtype=torch.uint8, device="cuda")
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    sH, sW = cfg.H * cfg.scale, cfg.W * cfg.scale
    x = torch.from_numpy(x_host).cuda()
    g = torch.Generator(device="cuda").manual_seed(1)
    target = torch.randn((cfg.batch, cfg.out_vars, sH, sW), generator=g, device="cuda")
    lat = np.cos(np.deg2rad(-90.0 + (np.arange(sH) + 0.5) * 180.0 / sH))
    lat_w = torch.from_numpy((lat / lat.mean()).astype(np.float32)).cuda()
    y = torch.empty_like(target)
    loss3 = torch.zeros(3, dtype=torch.float64, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    grads = {n: torch.empty(np.shape(w[n]), dtype=torch.float32, device="cuda") for n in B.MODEL_PARAMS}

    def step():
        B.reslim_train_step_grads(model.ctx, x, target, lat_w, 1.0, 1024.0, y, loss3, grads, cfg.batch, saved, ws)
        B.reslim_grads_unscale(model.ctx, grads, 1.0 / 1024.0, flag)

    for _ in range(2):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / K * 1e3
    B.reslim_profile_enable(model.ctx, 4096)
    step()
    torch.cuda.synchronize()
    agg = {}
    for name, kms, flop, nbytes in B.reslim_profile_read(model.ctx):
        a = agg.setdefault(name, dict(calls=0, ms=0.0, flop=0.0, bytes=0.0))
        a["calls"] += 1
        a["ms"] += kms
        a["flop"] += flop
        a["bytes"] += nbytes
    B.reslim_profile_enable(model.ctx, 0)
    ks = [dict(kernel=n, launches=a["calls"], ms=round(a["ms"], 5),
               tflops=round(a["flop"] / (a["ms"] * 1e-3) / 1e12, 2) if a["flop"] and a["ms"] > 0 else None,
               gbs=round(a["bytes"] / (a["ms"] * 1e-3) / 1e9, 1) if a["ms"] > 0 else None) for n, a in agg.items()]
    ks.sort(key=lambda k: -k["ms"])
    # the training forward runs every block on every token (the inference forward's counts do not apply)
    D, Rm = cfg.embed_dim, cfg.embed_dim * cfg.mlp_ratio
    gflop = 2.0 * cfg.batch * model.n_h * D * (4.0 * D + 2.0 * Rm) * cfg.depth
    tiles = B.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)[0]
    aflop = 4.0 * sum(float(t["n_tok"]) ** 2 for t in tiles) * D * cfg.depth * cfg.batch
    hflop = 2.0 * cfg.batch * cfg.n_tokens * D * cfg.out_vars * (cfg.patch * cfg.scale) ** 2
    flop = 3.0 * (gflop + hflop) + 3.5 * aflop          # forward + input and weight gradients; attention gradient 2.5 x forward
    if verbose:
        for k in ks:
            print("train_step " + json.dumps(k), file=sys.stderr)
    return dict(ms_per_step=round(ms, 4), unique_tokens_per_s=round(cfg.batch * cfg.n_tokens / (ms * 1e-3), 1),
                tflops=round(flop / (ms * 1e-3) / 1e12, 2), mfma_frac=round(flop / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                loss=[float(v) for v in loss3.cpu()], found_inf=int(flag.item()), saved_gb=round(sb / 1e9, 2),
                workspace_gb=round(wb / 1e9, 2), kernels=ks)


# Adaptive spatial compression (Sec. 4.1; Table 2(b) quotes speed-ups at 8x / 16x / 32x compression
# on one tile): the workload's grid untiled, quad-trees from the library's host builder on the
# first input variable.  Parameters chosen so that the c1 fields compress about 8x and 22x, and the
# smoother (more pixels per wavelength) fields of the paper's 112 km grid about 7x and 40x.
ASC_PARAMS = [dict(max_leaf=16, min_leaf=1, canny_low=70, canny_high=140, tau=0.05),
              dict(max_leaf=16, min_leaf=1, canny_low=80, canny_high=160, tau=0.05)]
ASC_PARAMS_BY_WORKLOAD = {"m9m": [dict(max_leaf=16, min_leaf=1, canny_low=50, canny_high=100, tau=0.05),
                                  dict(max_leaf=16, min_leaf=1, canny_low=60, canny_high=120, tau=0.05)]}


def asc_leg(B, torch, np, cfg, w, x_host, K):
    """Forward time with and without compression on the untiled grid (extra measurement, not `value`)."""
    one = cfg.with_(tiles_y=1, tiles_x=1, halo=0)
    res = {"workload": f"{cfg.name} grid, one tile: B={one.batch}, {one.n_tokens} patches per sample", "cases": []}
    with B.Reslim(one, w) as m:
        x = torch.from_numpy(x_host).cuda()
        y = torch.empty((one.batch, one.out_vars, one.H * one.scale, one.W * one.scale), dtype=torch.float32, device="cuda")

        def timed(fn):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(K):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / K * 1e3

        res["plain_ms"] = round(timed(lambda: B.reslim_forward(m.ctx, x, y, one.batch, m.ws)), 4)
        # one block's training step (forward-for-training + backward) on N(0,1) rows, plain and on the leaves
        B.reslim_train_prepare(m.ctx)
        D, R = one.embed_dim, one.embed_dim * one.mlp_ratio
        shapes = {"ln1_g": (D,), "ln1_b": (D,), "w_qkv": (3 * D, D), "b_qkv": (3 * D,), "w_proj": (D, D), "b_proj": (D,),
                  "ln2_g": (D,), "ln2_b": (D,), "w_fc1": (R, D), "b_fc1": (R,), "w_fc2": (D, R), "b_fc2": (D,)}
        grads = {n: torch.empty(sh, dtype=torch.float32, device="cuda") for n, sh in shapes.items()}
        gen = torch.Generator().manual_seed(7)

        def train_step_ms(rows, fwd, bwd, sb, wb):
            saved = torch.empty(max(sb, 256), dtype=torch.uint8, device="cuda")
            wsb = torch.empty(max(wb, 256), dtype=torch.uint8, device="cuda")
            xi = torch.randn((rows, D), generator=gen).cuda()
            do = torch.randn((rows, D), generator=gen).cuda()
            xo, dxi = torch.empty_like(xi), torch.empty_like(xi)

            def step():
                fwd(xi, xo, saved, wsb)
                bwd(xi, saved, do, dxi, wsb)
            return timed(step)

        sb, wb = B.reslim_block_train_bytes(m.ctx, one.batch)
        res["plain_train_block_ms"] = round(train_step_ms(
            one.batch * m.n_h,
            lambda xi, xo, sv, wk: B.reslim_block_fwd_train(m.ctx, 0, xi, xo, sv, one.batch, wk),
            lambda xi, sv, do, dxi, wk: B.reslim_block_bwd(m.ctx, 0, xi, sv, do, dxi, grads, one.batch, wk), sb, wb), 4)
        imgs = np.ascontiguousarray(x_host[:, 0])
        for prm in ASC_PARAMS_BY_WORKLOAD.get(cfg.name, ASC_PARAMS):
            t0 = time.perf_counter()
            tab = B.reslim_asc_build(imgs, one.patch, prm["max_leaf"], prm["min_leaf"], prm["canny_low"], prm["canny_high"], prm["tau"])
            build_ms = (time.perf_counter() - t0) * 1e3
            plan = B.reslim_asc_plan_create(m.ctx, one.batch, tab)
            L = len(tab["leaf_s"])
            try:
                ms = timed(lambda: B.reslim_asc_forward(m.ctx, plan, x, y, m.ws))
                sb, wb = B.reslim_asc_block_train_bytes(m.ctx, plan)
                tms = train_step_ms(
                    L, lambda xi, xo, sv, wk: B.reslim_asc_block_fwd_train(m.ctx, plan, 0, xi, xo, sv, wk),
                    lambda xi, sv, do, dxi, wk: B.reslim_asc_block_bwd(m.ctx, plan, 0, xi, sv, do, dxi, grads, wk), sb, wb)
            finally:
                B.reslim_asc_plan_destroy(plan)
            res["cases"].append(dict(params=prm, leaves=L, compression=round(one.batch * one.n_tokens / L, 2),
                                     leaves_per_sample=np.diff(tab["sample_off"]).tolist(), ms=round(ms, 4),
                                     speedup=round(res["plain_ms"] / ms, 2), train_block_ms=round(tms, 4),
                                     train_block_speedup=round(res["plain_train_block_ms"] / tms, 2),
                                     host_builder_ms=round(build_ms, 2)))
    # compression combined with TILES (Table 3 of the paper runs "4x compression, 16 tiles"): the workload's own
    # tiling, every (sample, tile) pair compressed on its haloed box
    if cfg.tiles_y * cfg.tiles_x > 1:
        res["tiled"] = {"workload": f"{cfg.name}: {cfg.tiles_y}x{cfg.tiles_x} tiles, halo {cfg.halo}", "cases": []}
        with B.Reslim(cfg, w) as m:
            x = torch.from_numpy(x_host).cuda()
            y = torch.empty((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), dtype=torch.float32, device="cuda")

            def timed(fn):
                for _ in range(2):
                    fn()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(K):
                    fn()
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) / K * 1e3

            plain = timed(lambda: B.reslim_forward(m.ctx, x, y, cfg.batch, m.ws))
            res["tiled"]["plain_ms"] = round(plain, 4)
            for prm in ASC_PARAMS_BY_WORKLOAD.get(cfg.name, ASC_PARAMS):
                t0 = time.perf_counter()
                tab = B.reslim_asc_build_tiles(imgs, cfg.patch, cfg.tiles_y, cfg.tiles_x, cfg.halo, prm["max_leaf"], prm["min_leaf"],
                                               prm["canny_low"], prm["canny_high"], prm["tau"])
                build_ms = (time.perf_counter() - t0) * 1e3
                plan = B.reslim_asc_plan_create(m.ctx, cfg.batch, tab)
                try:
                    ms = timed(lambda: B.reslim_asc_forward(m.ctx, plan, x, y, m.ws))
                finally:
                    B.reslim_asc_plan_destroy(plan)
                L = len(tab["leaf_s"])
                res["tiled"]["cases"].append(dict(params=prm, leaves=L, haloed_patches=cfg.batch * m.n_h,
                                                  compression=round(cfg.batch * m.n_h / L, 2), ms=round(ms, 4),
                                                  speedup=round(plain / ms, 2), host_builder_ms=round(build_ms, 2)))
    return res


def measure(B, torch, cfg, w, x_host, K, W, verbose, want_train, note, want_step=False):
    """W warm-up + K timed forwards of one workload, then the same K steps again with every launch
    bracketed by HIP events on the launch stream.  Returns (result dict, open model)."""
    model = B.Reslim(cfg, w)
    x = torch.from_numpy(x_host).cuda()
    y = torch.empty((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), dtype=torch.float32, device="cuda")
    for _ in range(W):
        model.forward(x, y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        model.forward(x, y)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / K * 1e3
    tokens = cfg.batch * cfg.n_tokens

    # ---- per-kernel durations (kept out of the headline timing above)
    launches_per_step = 3 + 7 * cfg.depth + 3
    B.reslim_profile_enable(model.ctx, launches_per_step * K)
    for _ in range(K):
        model.forward(x, y)
    torch.cuda.synchronize()
    recs = B.reslim_profile_read(model.ctx)
    B.reslim_profile_enable(model.ctx, 0)
    agg = {}
    for name, ms, flop, nbytes in recs:
        a = agg.setdefault(name, dict(calls=0, ms=0.0, flop=0.0, bytes=0.0))
        a["calls"] += 1
        a["ms"] += ms
        a["flop"] += flop
        a["bytes"] += nbytes
    kernels = []
    for name, a in agg.items():
        # per launch, averaged over the launches of that name (the last block's are smaller: it runs
        # its projection and MLP on the rows the tiles own)
        a["flop"] /= a["calls"]
        a["bytes"] /= a["calls"]
        avg = a["ms"] / a["calls"]
        tfl = a["flop"] / (avg * 1e-3) / 1e12 if a["flop"] else None
        gbs = a["bytes"] / (avg * 1e-3) / 1e9
        kernels.append(dict(kernel=name, launches_per_step=a["calls"] // K, avg_ms=round(avg, 5),
                            ms_per_step=round(a["ms"] / K, 5),
                            tflops=round(tfl, 2) if tfl else None, gbs=round(gbs, 1),
                            bound="alu" if name in ALU_BOUND else "mfma" if tfl else "hbm",
                            frac=round(tfl / (PEAK_FP32_VECTOR_TFLOPS if name in ALU_BOUND else PEAK_BF16_TFLOPS), 4) if tfl
                            else round(gbs / PEAK_HBM_GBS, 4)))
    kernels.sort(key=lambda k: -k["ms_per_step"])
    dom = kernels[0]
    a = agg[dom["kernel"]]
    avg_s = a["ms"] / a["calls"] * 1e-3
    if a["flop"] > 0:
        achieved = a["flop"] / avg_s / 1e12
        alu = dom["kernel"] in ALU_BOUND
        peak = PEAK_FP32_VECTOR_TFLOPS if alu else PEAK_BF16_TFLOPS
        roof = dict(bound="alu" if alu else "mfma", kernel=dom["kernel"], achieved=round(achieved, 2), peak=peak,
                    unit="TFLOP/s", frac=round(achieved / peak, 4),
                    traffic=MEASURED_TRAFFIC.get((cfg.name, dom["kernel"])), avg_launch_ms=round(avg_s * 1e3, 5),
                    flop_per_launch=a["flop"])
    else:
        achieved = a["bytes"] / avg_s / 1e9
        roof = dict(bound="hbm", kernel=dom["kernel"], achieved=round(achieved, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(achieved / PEAK_HBM_GBS, 4), traffic=MEASURED_TRAFFIC.get((cfg.name, dom["kernel"])),
                    avg_launch_ms=round(avg_s * 1e3, 5), bytes_per_launch=a["bytes"])
    gflop, aflop, hflop = B.reslim_flop_counts(model.ctx, cfg.batch)
    tflops = (gflop + aflop + hflop) / (dt / K) / 1e12
    if verbose:
        for k in kernels:
            print(cfg.name + " " + json.dumps(k), file=sys.stderr)
    res = {
        "value": round(tokens / (dt / K), 1), "ms_per_step": round(ms_per_step, 4),
        "dtype": "bf16" if cfg.dtype else "f32",
        "config": {"workload": f"{cfg.name}: B={cfg.batch} V={cfg.in_vars} {cfg.H}x{cfg.W} x{cfg.scale} -> "
                               f"{cfg.H * cfg.scale}x{cfg.W * cfg.scale}, p={cfg.patch} D={cfg.embed_dim} "
                               f"heads={cfg.heads} r={cfg.mlp_ratio} L={cfg.depth} tiles={cfg.tiles_y}x{cfg.tiles_x} "
                               f"halo={cfg.halo}",
                   "unique_tokens": tokens, "haloed_tokens": cfg.batch * model.n_h},
        "tflops": round(tflops, 2), "mfma_frac": round(tflops / PEAK_BF16_TFLOPS, 4),
        "haloed_tokens_per_s": round(cfg.batch * model.n_h / (dt / K), 1),
        "roofline": roof, "kernels": kernels,
    }
    # ---- extra, outside `value`: one block's training forward + backward at the same shape
    # (gradient of tile attention, input- and weight-gradient GEMMs, LayerNorm / GELU gradients)
    res["train_block"] = train_block(B, torch, model, cfg, K, verbose) if want_train and cfg.depth > 0 else None
    del x, y
    torch.cuda.empty_cache()
    res["train_step"] = None
    if want_step and cfg.dtype == 1 and cfg.depth > 0:
        import numpy as np
        note(f"{cfg.name}: whole training step (forward, loss, all gradients)")
        res["train_step"] = train_step(B, torch, np, model, cfg, w, x_host, max(2, K // 4), verbose)
    model.close()
    x = y = None
    del x, y
    torch.cuda.empty_cache()
    return res


def cpu_oracle(cfg, w, x_host):
    """The CPU oracle, as it stands, on a bounded sample of the workload (about 10-30 s of host work)."""
    from oracle import reslim_oracle as O
    if cfg.name in ("c0", "c1"):
        t0 = time.perf_counter()
        O.reslim_forward(x_host[:1], w, cfg)
        ct = time.perf_counter() - t0
        cpu_tokens, sample = cfg.n_tokens, f"1 of {cfg.batch} samples, full forward"
    else:   # whole tiles through the whole stack, scaled by tiles (tiles never interact, Sec. 4.2)
        tiles = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)[0]
        T = len(tiles)
        picks = [0, cfg.tiles_x // 2, T // 2 + cfg.tiles_x // 2] if cfg.embed_dim <= 1024 else [T // 2 + cfg.tiles_x // 2]
        cpu_tokens, ct = 0, 0.0
        for i in picks:
            t = tiles[i]
            t0 = time.perf_counter()
            O.forward_tile(x_host[0], w, cfg, t, cfg.Wp)
            ct += time.perf_counter() - t0
            cpu_tokens += (t["y1"] - t["y0"]) * (t["x1"] - t["x0"])
        sample = (f"tiles {picks} (corner, edge, interior) of the {T} tiles of one sample, full stack; "
                  f"unique tokens of those tiles / their time (extrapolation linear in tiles)")
    cores = int(os.environ["OMP_NUM_THREADS"]) if os.environ.get("OMP_NUM_THREADS") else os.cpu_count()
    return dict(value=round(cpu_tokens / ct, 1), unit="tokens/s", cores=cores, kind="oracle", sample=sample,
                seconds=round(ct, 2))


HEADLINE = "c3"      # the largest of the five benchmark workloads that one GPU holds: the headline is quoted on it
OTHERS = ("c0", "c1", "c2", "c4")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default=HEADLINE,
                    help="workload the line is quoted on (c0..c4, or m9m / m126m / m1b / m10b: the paper's model sizes); "
                         "default: c3, the largest of the five benchmark workloads")
    ap.add_argument("--others", default=None,
                    help="comma-separated workloads measured as well and reported under `other_workloads` "
                         "(default: c0,c1,c2,c4 when --config is c3, else none; 'none' switches them off)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (developer runs)")
    ap.add_argument("--gemm-tile", type=int, default=-1, help="pin the bf16 GEMM kernel (2 = 128x128 tiles, 3 = persistent 256x256), -1 = heuristic")
    ap.add_argument("--kernels", action="store_true", help="also print the per-kernel table to stderr")
    ap.add_argument("--no-train-block", action="store_true",
                    help="skip the extra (untimed in `value`) measurement of one block's training forward + backward")
    ap.add_argument("--no-train-step", action="store_true",
                    help="skip the extra measurement of reslim_train_step_grads (whole-model training step)")
    ap.add_argument("--no-asc", action="store_true",
                    help="skip the extra measurement of the forward with adaptive spatial compression (run for c0, c1 and m9m only)")
    ap.add_argument("--asc-only", action="store_true",
                    help="developer runs (profiles): only the compression measurement, printed as its own JSON object")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch the library's plain copy kernel on 1 GiB five times (yardstick for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (tiles are batched on one MI355X); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2505_04802_amd import binding as B
    from paper_2505_04802_amd import workloads as WL

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path", file=sys.stderr)
        return 2
    note = lambda m: print("bench.py: " + m, file=sys.stderr, flush=True)
    if args.others is None:
        others = OTHERS if args.config == HEADLINE else ()
    else:
        others = tuple(n for n in args.others.split(",") if n and n != "none")
    K, W = args.steps, args.warmup
    B.reslim_debug_set_gemm_tile(args.gemm_tile)

    def inputs(cfg):
        note(f"{cfg.name}: generating weights and fields on the host")
        big = cfg.depth * cfg.embed_dim ** 2 > 1 << 28
        return WL.make_weights(cfg, progress=note if big else None), WL.make_fields(cfg)

    cfg = WL.CONFIGS[args.config]
    w, x_host = inputs(cfg)
    if args.asc_only:
        if args.copy_probe:
            a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            b = torch.empty_like(a)
            for _ in range(5):
                B.reslim_debug_copy(a, b)
            torch.cuda.synchronize()
            del a, b
        print(json.dumps(asc_leg(B, torch, np, cfg, w, x_host, K)))
        return 0
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            B.reslim_debug_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst
    note(f"{cfg.name}: {W} warm-up + {K} timed steps, then {K} steps with per-launch events")
    head = measure(B, torch, cfg, w, x_host, K, W, args.kernels, not args.no_train_block, note, not args.no_train_step)

    # ---- extra, outside `value`: the untiled grid with and without adaptive spatial compression
    asc = None
    if not args.no_asc and cfg.name in ("c0", "c1", "m9m"):
        asc = asc_leg(B, torch, np, cfg, w, x_host, K)

    # ---- the CPU oracle on a bounded sample of the headline workload
    cpu = None
    if not args.no_cpu_baseline:
        note(f"{cfg.name}: CPU oracle on a sample of the workload")
        cpu = cpu_oracle(cfg, w, x_host)
    del w, x_host

    # ---- the other benchmark workloads, same procedure, reported beside the headline
    other = {}
    for name in others:
        ocfg = WL.CONFIGS[name]
        ow, ox = inputs(ocfg)
        note(f"{name}: {W} warm-up + {K} timed steps, then {K} steps with per-launch events")
        r = measure(B, torch, ocfg, ow, ox, K, W, args.kernels, False, note, name == "c1" and not args.no_train_step)
        if name == "c1" and not args.no_asc:
            r["asc"] = asc_leg(B, torch, np, ocfg, ow, ox, K)
        other[name] = r
        del ow, ox

    out = {
        "metric": "Reslim+TILES fwd tokens/s", "value": head["value"], "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"],
        "data": "synthetic", "config": head["config"],
        "tflops": head["tflops"], "mfma_frac": head["mfma_frac"], "haloed_tokens_per_s": head["haloed_tokens_per_s"],
        "roofline": head["roofline"], "cpu_baseline": cpu, "kernels": head["kernels"],
        "train_block": head["train_block"], "train_step": head["train_step"], "asc": asc, "other_workloads": other,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
