"""GPU parity: the HIP library (through the C ABI) against the CPU oracle on the
same seeded inputs, element by element.

Tolerances (max relative L2 over planes, the bar the benchmark definition sets):
    fp32 debug path  <= 1e-5
    bf16 path        <= 2e-2
Tile partitioning is compared bit-exact in test_abi_cpu.py (host function)."""
import numpy as np
import pytest
import torch

from oracle import reslim_oracle as O
from paper_2505_04802_amd import binding as B
from paper_2505_04802_amd import workloads as WL
from parity_checks import assert_parity

pytestmark = pytest.mark.gpu
TOL = {0: 1e-5, 1: 2e-2}


def cuda(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def say(msg):
    print(msg, flush=True)


def rel(a, ref):
    a = np.asarray(a, np.float64).ravel()
    ref = np.asarray(ref, np.float64).ravel()
    return float(np.linalg.norm(a - ref) / max(np.linalg.norm(ref), 1e-300))


# small shapes that still span several MFMA tiles, several key blocks and ragged tails
SMALL_F32 = WL.ReslimConfig("s32", batch=2, in_vars=3, out_vars=2, H=20, W=28, scale=2, patch=2,
                            embed_dim=48, heads=3, mlp_ratio=2, depth=2, tiles_y=2, tiles_x=3,
                            halo=1, dtype=0, seed=11)
SMALL_BF16 = WL.ReslimConfig("sbf", batch=2, in_vars=3, out_vars=3, H=44, W=60, scale=4, patch=2,
                             embed_dim=128, heads=2, mlp_ratio=4, depth=2, tiles_y=2, tiles_x=2,
                             halo=2, dtype=1, seed=12)       # dh = 64, n_t = 13*17 .. -> 221..285 tokens
SMALL_BF16_DH128 = SMALL_BF16.with_(name="sbf128", embed_dim=256, heads=2, H=40, W=48, tiles_y=1, tiles_x=2,
                                    halo=3, seed=13)        # dh = 128, n_t = 20*15 = 300
SMALL_BF16_DH256 = SMALL_BF16.with_(name="sbf256", embed_dim=512, heads=2, H=36, W=52, tiles_y=2, tiles_x=1,
                                    halo=2, seed=14)        # dh = 256 (the 10B model's head size), n_t = 11*26 = 286


def weights_for(cfg, std=0.02):
    w = WL.make_weights(cfg, std=std)
    if cfg.out_vars < cfg.in_vars:          # exercise a non-identity variable selection
        w["out_var_idx"] = np.arange(cfg.in_vars - 1, cfg.in_vars - 1 - cfg.out_vars, -1).astype(np.int32)
    return w


# ------------------------------------------------------------------ tile attention
@pytest.mark.parametrize("cfg", [SMALL_F32, SMALL_BF16, SMALL_BF16_DH128, SMALL_BF16_DH256], ids=lambda c: c.name)
@pytest.mark.parametrize("peaked", [False, True])
def test_tiles_attention_parity(cfg, peaked):
    say(f"attention parity {cfg.name} peaked={peaked}")
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    qkv = WL.make_qkv(cfg.batch * n_h, cfg.embed_dim, seed=5, peaked=peaked, bf16=cfg.dtype == 1)
    qkv = qkv.reshape(cfg.batch, n_h, 3 * cfg.embed_dim)
    ref = O.tiles_attention(qkv, tiles, cfg.heads)
    with B.Reslim(cfg, weights_for(cfg)) as m:
        assert m.n_h == n_h
        out = m.attention(cuda(qkv, m.act_dtype)).float().cpu().numpy()
    assert_parity(out, ref, TOL[cfg.dtype], "attention output", say)
    if cfg.dtype == 1:      # element-wise: bf16 output rounding + bf16 P, well inside 3e-2 absolute for |v| ~ 1
        assert np.abs(out - ref).max() <= 3e-2
    # the same call with the log-sum-exp output (what the gradient needs)
    with B.Reslim(cfg, weights_for(cfg)) as m:
        q_dev = cuda(qkv, m.act_dtype)
        out2 = torch.empty((cfg.batch, n_h, cfg.embed_dim), dtype=m.act_dtype, device="cuda")
        lse = torch.full((cfg.batch, cfg.heads, n_h), float("nan"), dtype=torch.float32, device="cuda")
        B.tiles_attention_fwd_lse(m.ctx, q_dev, out2, lse, cfg.batch)
        assert np.array_equal(out2.float().cpu().numpy(), out)
        lse_ref = O.tiles_attention_lse(qkv, tiles, cfg.heads)
        d = np.abs(lse.cpu().numpy() - lse_ref).max()
        say(f"  lse max abs error {d:.3e}")
        assert d <= (2e-2 if cfg.dtype == 1 else 1e-4)      # an absolute error of the LOG of the denominator


def test_tiles_attention_special_cases_bf16():
    """Degenerate inputs with known answers: q = 0 gives the tile's column mean of v,
    constant v is reproduced, and one tile over the whole grid is global attention."""
    cfg = SMALL_BF16.with_(tiles_y=1, tiles_x=1, halo=5, batch=1)
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, 1, 1, 5)
    D = cfg.embed_dim
    qkv = WL.make_qkv(n_h, D, seed=6).reshape(1, n_h, 3 * D)
    with B.Reslim(cfg, weights_for(cfg)) as m:
        assert m.n_h == cfg.n_tokens
        z = qkv.copy(); z[..., :D] = 0
        out = m.attention(cuda(z, torch.bfloat16)).float().cpu().numpy()
        assert np.abs(out - z[0, :, 2 * D:].mean(0)).max() <= 1e-2
        cst = qkv.copy(); cst[..., 2 * D:] = WL.round_to_bf16(np.linspace(-2, 2, D, dtype=np.float32))
        out = m.attention(cuda(cst, torch.bfloat16)).float().cpu().numpy()
        assert np.abs(out - cst[0, 0, 2 * D:]).max() <= 2e-2
        out = m.attention(cuda(qkv, torch.bfloat16)).float().cpu().numpy()
        ref = O.self_attention(qkv[0, :, :D], qkv[0, :, D:2 * D], qkv[0, :, 2 * D:], cfg.heads)
        assert O.rel_l2(out[0], ref) <= 2e-2


# ------------------------------------------------------------------ kernels the heuristics do not pick at small sizes
@pytest.fixture
def kernel_hooks():
    """The two process-wide tuning hooks, restored to the built-in choice whatever the test does."""
    yield B
    B.reslim_debug_set_gemm_tile(-1)
    B.reslim_debug_set_attention_variant(0)


@pytest.mark.parametrize("tile", [2, 3, 102], ids=["tiles128", "persistent256", "tiles128_columns_fastest"])
@pytest.mark.parametrize("cfg", [SMALL_BF16, SMALL_BF16.with_(name="sbf_d64", embed_dim=64, heads=1, mlp_ratio=3)],
                         ids=lambda c: c.name)
def test_forced_gemm_kernels_on_small_ragged_shapes(kernel_hooks, cfg, tile):
    """Each bf16 GEMM kernel forced on shapes the heuristic would give to another one: about a
    thousand rows (no multiple of 128 or 256), outputs 128, 384 and 512 columns wide (64, 192 at
    embed dim 64: no multiple of 256, so the persistent kernel's column guard and its half-empty
    tiles run), contraction lengths 64 .. 512.  One block from the oracle's input, every epilogue
    (q-scaled bf16, residual add, GELU), then the head GEMM through the whole forward."""
    say(f"forced GEMM kernel {tile} on {cfg.name}")
    w = weights_for(cfg, std=0.1)
    x = WL.make_fields(cfg)
    y_ref, inter = O.reslim_forward(x, w, cfg, return_intermediates=True)
    with B.Reslim(cfg, w) as m:
        kernel_hooks.reslim_debug_set_gemm_tile(tile)
        prev = inter["tokens"]
        for l in range(cfg.depth):
            t = cuda(prev.astype(np.float32))
            m.block(l, t)
            assert_parity(t.cpu().numpy(), inter[f"block{l}"], TOL[1], f"block{l}", say)
            prev = inter[f"block{l}"]
        assert_parity(m.forward(cuda(x)).cpu().numpy(), y_ref, TOL[1], "forward", say)
        kernel_hooks.reslim_debug_set_gemm_tile(-1)
        t = cuda(inter["tokens"].astype(np.float32))
        m.block(0, t)
        assert_parity(t.cpu().numpy(), inter["block0"], TOL[1], "block0, built-in choice", say)


@pytest.mark.parametrize("variant", [0, 1], ids=["keys64_x3", "keys128_x2"])
@pytest.mark.parametrize("peaked", [False, True])
def test_attention_launch_shapes_dh64(kernel_hooks, variant, peaked):
    """Both launch shapes of the head-dimension-64 kernel (64-key blocks with three work-groups per
    compute unit, 128-key blocks with two) on ragged tiles (221 .. 285 tokens: the last key block
    is masked in both), normal and peaked logits."""
    cfg = SMALL_BF16
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    qkv = WL.make_qkv(cfg.batch * n_h, cfg.embed_dim, seed=15, peaked=peaked).reshape(cfg.batch, n_h, 3 * cfg.embed_dim)
    ref = O.tiles_attention(qkv, tiles, cfg.heads)
    with B.Reslim(cfg, weights_for(cfg)) as m:
        kernel_hooks.reslim_debug_set_attention_variant(variant)
        out = m.attention(cuda(qkv, m.act_dtype)).float().cpu().numpy()
    assert_parity(out, ref, TOL[1], f"attention variant {variant} peaked={peaked}", say)
    assert np.abs(out - ref).max() <= 3e-2


@pytest.mark.parametrize("cfg", [SMALL_BF16, SMALL_BF16_DH128, SMALL_BF16_DH256], ids=lambda c: c.name)
@pytest.mark.parametrize("octet", [0, 1], ids=["first_octets", "second_octets"])
def test_attention_large_logits_in_one_key_octet(cfg, octet):
    """The running reference logit of a query must see all of its keys.  Here the keys whose
    position in the tile falls in one half of each group of 16 (positions 16 j + 8 octet .. + 7)
    carry logits 184 binary orders of magnitude above the others: a reference taken from the
    other keys alone makes exp2(logit - reference) overflow to infinity, so any finite output
    that matches the oracle shows that the maximum covers both halves.  (The bf16 kernel keeps
    the two halves of a group in lanes l and l + 32 and exchanges their maxima.)  The inputs are
    rounded to bf16 before either side sees them."""
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    D, dh = cfg.embed_dim, cfg.embed_dim // cfg.heads
    qkv = (0.25 * WL.make_qkv(cfg.batch * n_h, D, seed=21)).reshape(cfg.batch, n_h, 3 * D).astype(np.float32)
    for t in tiles:
        pos = np.arange(t["n_tok"])
        big = np.where((pos % 16) // 8 == octet, 16.0, -16.0).astype(np.float32)
        r = slice(t["tok_off"], t["tok_off"] + t["n_tok"])
        for g in range(cfg.heads):
            qkv[:, r, g * dh] = 8.0 * np.sqrt(dh)          # q . k / sqrt(dh) = 8 * (+-16) = +-128
            qkv[:, r, D + g * dh] = big[None, :]
    qkv = WL.round_to_bf16(qkv)
    ref = O.tiles_attention(qkv, tiles, cfg.heads)
    with B.Reslim(cfg, weights_for(cfg)) as m:
        out = m.attention(cuda(qkv, m.act_dtype)).float().cpu().numpy()
    assert np.isfinite(out).all(), "overflow: the reference logit missed the large keys"
    assert_parity(out, ref, TOL[1], f"attention {cfg.name}, large logits in octet {octet}", say)


# ------------------------------------------------------------------ embed / block / head
@pytest.mark.parametrize("cfg", [SMALL_F32, SMALL_BF16, SMALL_BF16_DH128, SMALL_BF16_DH256], ids=lambda c: c.name)
def test_stage_by_stage_parity(cfg):
    """Every entry point against the oracle's intermediate of the same name; the
    weights are spread wide (std 0.1) so softmaxes and GELUs are far from linear."""
    say(f"stage parity {cfg.name}")
    w = weights_for(cfg, std=0.1)
    x = WL.make_fields(cfg)
    y_ref, inter = O.reslim_forward(x, w, cfg, return_intermediates=True)
    tol = TOL[cfg.dtype]
    with B.Reslim(cfg, w) as m:
        xd = cuda(x)
        tok = m.embed(xd)
        assert_parity(tok.cpu().numpy(), inter["tokens"], tol, "embed", say)
        # each block from the ORACLE's input, so errors do not compound in this check
        prev = inter["tokens"]
        for l in range(cfg.depth):
            t = cuda(prev.astype(np.float32))
            m.block(l, t)
            assert_parity(t.cpu().numpy(), inter[f"block{l}"], tol, f"block{l}", say)
            prev = inter[f"block{l}"]
        y = m.head(xd, cuda(prev.astype(np.float32))).cpu().numpy()
        assert_parity(y, y_ref, tol, "head", say)
        # the main path alone: the fp32 difference of two sums cancels digits, hence the wider fp32 bound
        assert_parity(y - inter["residual"], inter["y_main"], tol if cfg.dtype else 1e-4, "head (main path only)", say)
        # whole forward
        y = m.forward(xd).cpu().numpy()
        assert_parity(y, y_ref, tol, "forward", say)
        y2 = m.forward(xd).cpu().numpy()
        assert np.array_equal(y, y2)                 # same input, same bits


@pytest.mark.parametrize("cfg", [SMALL_BF16, SMALL_BF16_DH128, SMALL_BF16_DH256, WL.CONFIGS["c1"]], ids=lambda c: c.name)
def test_forward_equals_its_entry_points_chained(cfg):
    """The whole forward runs its last block on the rows the tiles own (halo tokens serve that
    block's attention as keys and values only) and lets its first block read the embedding
    through the gather list instead of a gathered copy; the entry points chained gather first and
    run every block on every token.  Row by row the arithmetic is the same, so the outputs agree
    bit for bit."""
    say(f"forward vs chained entry points {cfg.name}")
    w = weights_for(cfg, std=0.1)
    x = WL.make_fields(cfg)
    with B.Reslim(cfg, w) as m:
        assert m.n_h > cfg.Hp * cfg.Wp, "the case needs halo tokens"
        xd = cuda(x)
        tok = m.embed(xd)
        for l in range(cfg.depth):
            m.block(l, tok)
        y_chain = m.head(xd, tok).cpu().numpy()
        y = m.forward(xd).cpu().numpy()
    assert np.array_equal(y, y_chain)


def test_forward_equals_its_entry_points_chained_with_128_key_blocks(kernel_hooks):
    """The same identity with the other launch shape of the head-dimension-64 kernel (128-key
    blocks, two work-groups per compute unit), whose stitched form no other test reaches."""
    cfg = SMALL_BF16
    w = weights_for(cfg, std=0.1)
    x = WL.make_fields(cfg)
    y_ref = O.reslim_forward(x, w, cfg)
    with B.Reslim(cfg, w) as m:
        kernel_hooks.reslim_debug_set_attention_variant(1)
        xd = cuda(x)
        tok = m.embed(xd)
        for l in range(cfg.depth):
            m.block(l, tok)
        y_chain = m.head(xd, tok).cpu().numpy()
        y = m.forward(xd).cpu().numpy()
    assert np.array_equal(y, y_chain)
    assert_parity(y, y_ref, TOL[1], "forward, 128-key blocks", say)


@pytest.mark.parametrize("cfg", [SMALL_BF16, SMALL_F32, WL.CONFIGS["c1"]], ids=lambda c: c.name)
def test_flop_counts_are_the_sum_of_the_launch_records(cfg):
    """reslim_flop_counts (the numerator of the bench line's TFLOP/s) against the per-launch
    records of one forward: block GEMMs, tile attention and head GEMM each add up exactly."""
    w = weights_for(cfg)
    with B.Reslim(cfg, w) as m:
        xd = cuda(WL.make_fields(cfg))
        B.reslim_profile_enable(m.ctx, 256)
        m.forward(xd)
        torch.cuda.synchronize()
        recs = B.reslim_profile_read(m.ctx)
        B.reslim_profile_enable(m.ctx, 0)
        gflop, aflop, hflop = B.reslim_flop_counts(m.ctx, cfg.batch)
    by = {}
    for name, _, flop, _ in recs:
        by[name] = by.get(name, 0.0) + flop
    # embed (2 launches) + gather + 7 per block + head (3); the gather is folded into the first
    # block when the forward keeps a patch-order stream for its last block (bf16, halo tokens, >= 2 blocks)
    folded = cfg.dtype == 1 and cfg.depth >= 2 and m.n_h > cfg.Hp * cfg.Wp
    assert len(recs) == 3 + 7 * cfg.depth + 3 - (1 if folded else 0)
    assert ("gather" in by) == (not folded)
    assert np.isclose(by["gemm_qkv"] + by["gemm_proj"] + by["gemm_fc1"] + by["gemm_fc2"], gflop, rtol=1e-12)
    assert np.isclose(by["tiles_attention"], aflop, rtol=1e-12)
    assert np.isclose(by["gemm_head"], hflop, rtol=1e-12)


def test_forward_c0_fp32():
    cfg = WL.CONFIGS["c0"]
    w, x = WL.make_weights(cfg), WL.make_fields(cfg)
    ref, inter = O.reslim_forward(x, w, cfg, return_intermediates=True)
    with B.Reslim(cfg, w) as m:
        y = m.forward(cuda(x)).cpu().numpy()
    assert_parity(y, ref, 1e-5, "c0 forward", say)
    assert_parity(y - inter["residual"], inter["y_main"], 1e-4, "c0 main path", say)


def test_forward_c1_bf16_full_size():
    """The benchmark configuration at full size, in the launch configuration the
    benchmark times (batch 4, one forward), whole output against the oracle."""
    cfg = WL.CONFIGS["c1"]
    w, x = WL.make_weights(cfg), WL.make_fields(cfg)
    say("c1: oracle forward (float64, host) ...")
    ref, inter = O.reslim_forward(x, w, cfg, return_intermediates=True)
    with B.Reslim(cfg, w) as m:
        y = m.forward(cuda(x)).cpu().numpy()
    assert_parity(y, ref, 2e-2, "c1 forward", say)
    assert_parity(y - inter["residual"], inter["y_main"], 2e-2, "c1 main path", say)


def _sampled_tile_parity(cfg, tile_ids, batch_item=0, w=None):
    """Full-size forward on the GPU; the oracle recomputes single tiles through the
    whole stack (exact: tiles never interact, Sec. 4.2) and their interiors are compared."""
    w = WL.make_weights(cfg) if w is None else w
    x = WL.make_fields(cfg)
    tiles, _, _, _ = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    with B.Reslim(cfg, w) as m:
        y = m.forward(cuda(x))
        torch.cuda.synchronize()
        ps = cfg.patch * cfg.scale
        worst = 0.0
        for ti in tile_ids:
            t = tiles[ti]
            got = y[batch_item, :, t["y0"] * ps:t["y1"] * ps, t["x0"] * ps:t["x1"] * ps].cpu().numpy()
            ref = O.forward_tile(x[batch_item], w, cfg, t, cfg.Wp)
            e = assert_parity(got, ref, 2e-2, f"{cfg.name} tile {ti} (n_t={t['n_tok']})", say)
            worst = max(worst, e)
    assert worst <= 2e-2


def test_forward_c2_sampled_tiles():
    cfg = WL.CONFIGS["c2"]
    _sampled_tile_parity(cfg, [0, 3, 27, 63], batch_item=1)       # corner, edge, interior, far corner


def test_forward_c3_sampled_tiles():
    cfg = WL.CONFIGS["c3"]
    _sampled_tile_parity(cfg, [0, 8, 136, 255])


def test_forward_c4_sampled_tiles():
    """Corner (2244 tokens), interior (2448) and the LAST tile, whose rows end inside a 256-row tile
    of the persistent matrix kernel (37,520 rows in all) at contraction lengths 4096 and 16384."""
    cfg = WL.CONFIGS["c4"]
    _sampled_tile_parity(cfg, [0, 5, 15])


@pytest.mark.parametrize("name,tile_ids", [("m9m", [0, 5, 15]), ("m126m", [0, 6]), ("m1b", [0, 7, 10, 15])])
def test_forward_paper_model_sizes_sampled_tiles(name, tile_ids):
    """The paper's 9.5M / 126M / 1B model sizes (Sec. 5) on the [180,360,23] -> [720,1440,3]
    task, 16 tiles: more input than output variables, head dimensions 64 and 128."""
    _sampled_tile_parity(WL.CONFIGS[name], tile_ids)


def test_forward_10b_width_one_block_sampled_tile():
    """The 10B model's width (embed dim 8192, 32 heads of dimension 256) with ONE of its 11
    blocks, so the oracle stays within a minute; the blocks are copies of the same kernels."""
    _sampled_tile_parity(WL.CONFIGS["m10b"].with_(name="m10b_L1", depth=1), [9])


def test_forward_10b_model_at_its_real_depth_sampled_tile():
    """The 10B model of Sec. 5 at all 11 blocks (17.7 GB of bf16 weights on the device) on one tile
    through the whole stack.  Drawing 35 GB of truncated normals takes many minutes on the host, so
    one block is drawn with the seeded generator and the other ten are that block's tensors rolled
    along their output axis by a different amount each (every block distinct, every value already a
    bf16 number): layer offsets beyond 2^31 elements and the error growth over the real depth are
    what this checks."""
    one = WL.CONFIGS["m10b"].with_(name="m10b_L1", depth=1)
    cfg = WL.CONFIGS["m10b"]
    say("m10b: weights of one block ...")
    w = dict(WL.make_weights(one))
    for name in O.BLOCK_PARAMS:
        base = w[name][0]
        w[name] = np.stack([np.roll(base, 37 * l + 5 * l * l, axis=0) for l in range(cfg.depth)])
    assert not np.array_equal(w["w_fc1"][3], w["w_fc1"][7])
    say("m10b: forward with 11 blocks, then the oracle on tile 6 ...")
    _sampled_tile_parity(cfg, [6], w=w)


# ------------------------------------------------------------------ Bayesian loss (Sec. 4.1)
@pytest.mark.parametrize("shape", [(4, 8, 512, 1024), (2, 3, 37, 53), (1, 2, 33, 1027), (1, 1, 1, 1), (1, 1, 1, 9),
                                   (1, 1, 70, 1), (3, 1, 64, 2048)], ids=str)
def test_bayes_loss_parity(shape):
    """fp32 element arithmetic, fp64 accumulation: agrees with the fp64 oracle to 1e-5 relative
    (a sum of n fp32-rounded terms of one sign carries about 6e-8 relative error per term)."""
    rng = np.random.default_rng([5, shape[2], shape[3]])
    pred = rng.normal(size=shape).astype(np.float32)
    target = (pred + 0.3 * rng.normal(size=shape)).astype(np.float32)
    lw = O.lat_weights(shape[2], -80.0, 85.0).astype(np.float32)
    ref = O.bayes_loss(pred, target, lw, tv_weight=0.25)
    out = torch.zeros(3, dtype=torch.float64, device="cuda")
    ws = torch.empty(max(B.reslim_bayes_loss_workspace_bytes(*shape), 8), dtype=torch.uint8, device="cuda")
    p, t, l = cuda(pred), cuda(target), cuda(lw)
    B.reslim_bayes_loss_fwd(p, t, l, 0.25, out, ws)
    got = out.cpu().numpy()
    say(f"bayes loss {shape}: got {got}, oracle {np.array(ref)}")
    for g, r in zip(got, ref):
        assert abs(g - r) <= 1e-5 * abs(r) + 1e-12
    out2 = torch.zeros(3, dtype=torch.float64, device="cuda")
    B.reslim_bayes_loss_fwd(p, t, l, 0.25, out2, ws)
    assert torch.equal(out, out2)                                   # deterministic
    if pred.size >= 1 << 24:                                        # report the achieved bandwidth at full size
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            B.reslim_bayes_loss_fwd(p, t, l, 0.25, out2, ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 20
        say(f"bayes loss {shape}: {ms:.4f} ms per call, {2 * pred.nbytes / ms / 1e6:.0f} GB/s of algorithmic bytes (pred + target once)")
    small = torch.empty(8, dtype=torch.uint8, device="cuda")
    if B.reslim_bayes_loss_workspace_bytes(*shape) > 8:
        with pytest.raises(B.ReslimError):
            B.reslim_bayes_loss_fwd(p, t, l, 0.25, out, small)


# ------------------------------------------------------------------ edge cases
def test_edge_cases_and_errors():
    cfg = SMALL_BF16
    w = weights_for(cfg)
    with B.Reslim(cfg, w) as m:
        lib = B.load()
        x = cuda(WL.make_fields(cfg))
        y = torch.empty((cfg.batch, cfg.out_vars, cfg.H * 4, cfg.W * 4), device="cuda")
        ws = m.ws
        st = torch.cuda.current_stream().cuda_stream
        # empty batch, missing / short / misaligned workspace, bad layer: codes, no launch
        assert lib.reslim_forward(m.ctx, x.data_ptr(), y.data_ptr(), 0, ws.data_ptr(), ws.numel(), st) == B.RESLIM_ESHAPE
        assert lib.reslim_forward(m.ctx, x.data_ptr(), y.data_ptr(), 2, None, 0, st) == B.RESLIM_EWORKSPACE
        assert lib.reslim_forward(m.ctx, x.data_ptr(), y.data_ptr(), 2, ws.data_ptr(), 1024, st) == B.RESLIM_EWORKSPACE
        assert lib.reslim_forward(m.ctx, x.data_ptr(), y.data_ptr(), 2, ws.data_ptr() + 16, ws.numel() - 16, st) == B.RESLIM_EWORKSPACE
        assert lib.reslim_block_fwd(m.ctx, cfg.depth, x.data_ptr(), 2, ws.data_ptr(), ws.numel(), st) == B.RESLIM_EINVAL
        assert b"layer" in lib.reslim_last_error(m.ctx)
        assert lib.reslim_forward(m.ctx, None, y.data_ptr(), 2, ws.data_ptr(), ws.numel(), st) == B.RESLIM_EINVAL
        # batch 1 of a batch-2 context equals item 0 of the batch-2 result
        y2 = m.forward(x).cpu().numpy()
        y1 = m.forward(x[:1].contiguous()).cpu().numpy()
        assert np.array_equal(y1[0], y2[0])
    # one tile with a halo wider than the grid, and a tile grid as fine as the patch grid
    for kw in (dict(tiles_y=1, tiles_x=1, halo=50), dict(H=8, W=8, tiles_y=4, tiles_x=4, halo=1, batch=1)):
        c2 = cfg.with_(**kw)
        w2, x2 = weights_for(c2, 0.1), WL.make_fields(c2)
        ref = O.reslim_forward(x2, w2, c2)
        with B.Reslim(c2, w2) as m:
            e = O.rel_l2(m.forward(cuda(x2)).cpu().numpy(), ref)
        say(f"  edge {kw}: rel-L2 {e:.3e}")
        assert e <= 2e-2


def test_forward_is_capturable_in_a_hip_graph():
    """reslim_forward only enqueues kernels on the caller's stream (no allocation, no
    memset, no synchronisation), so a caller may record it into a HIP graph.  Every
    replay, with new inputs in the captured buffers and eager work in between, must
    reproduce the eager result bit for bit."""
    cfg = SMALL_BF16
    w = weights_for(cfg)
    r = np.random.default_rng(5)
    xs = [WL.make_fields(cfg)] + [r.standard_normal((cfg.batch, cfg.in_vars, cfg.H, cfg.W)).astype(np.float32) for _ in range(2)]
    with B.Reslim(cfg, w) as m:
        x = cuda(xs[0], torch.float32)
        y = torch.empty((cfg.batch, cfg.out_vars, cfg.H * cfg.scale, cfg.W * cfg.scale), dtype=torch.float32, device="cuda")
        B.reslim_forward(m.ctx, x, y, cfg.batch, m.ws)                 # warm-up outside the capture
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            B.reslim_forward(m.ctx, x, y, cfg.batch, m.ws)
        torch.cuda.synchronize()
        for i, xi in enumerate(xs + xs[:1]):
            say(f"graph replay {i}")
            x.copy_(cuda(xi, torch.float32))
            y.fill_(float("nan"))
            g.replay()
            torch.cuda.synchronize()
            got = y.clone()
            B.reslim_forward(m.ctx, x, y, cfg.batch, m.ws)             # the program's own eager work between replays
            torch.cuda.synchronize()
            assert torch.isfinite(got).all() and torch.equal(got, y)
        assert O.rel_l2(y.cpu().numpy(), O.reslim_forward(xs[0], w, cfg)) <= TOL[1]


def test_create_refuses_a_head_the_bf16_epilogues_cannot_store():
    """out_vars * (patch * scale)^2 must be a multiple of 8 on the bf16 path (16-byte
    row pieces in the GEMM epilogues); the fp32 path takes the same shape."""
    cfg = SMALL_BF16.with_(scale=1, out_vars=1, in_vars=3)            # head width 4
    with pytest.raises(B.ReslimError):
        B.Reslim(cfg, weights_for(cfg))
    ok = cfg.with_(dtype=0, embed_dim=48, heads=3)
    w = weights_for(ok)
    x = WL.make_fields(ok)
    with B.Reslim(ok, w) as m:
        y = m.forward(cuda(x, torch.float32)).cpu().numpy()
    assert O.rel_l2(y, O.reslim_forward(x, w, ok)) <= TOL[0]
