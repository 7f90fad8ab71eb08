"""GPU parity of the gradient of tile-local attention (tiles_attention_bwd through the
C ABI) against the CPU oracle's chain rule in fp64, on the same seeded inputs.

Tolerances: fp32 debug path <= 1e-5, bf16 path <= 2e-2 (max relative L2 of each of the
three gradients, the bar of the benchmark definition).  The oracle computes its own
forward in fp64; the library is given its own forward's output and log-sum-exp."""
import numpy as np
import pytest
import torch

from oracle import reslim_oracle as O
from paper_2505_04802_amd import binding as B
from paper_2505_04802_amd import workloads as WL
from parity_checks import GRAD_BF16, assert_parity
from test_gpu_parity import SMALL_F32, SMALL_BF16, SMALL_BF16_DH128, SMALL_BF16_DH256, TOL, cuda, say, weights_for

pytestmark = pytest.mark.gpu


def _inputs(cfg, n_h, peaked, seed=5):
    bf = cfg.dtype == 1
    qkv = WL.make_qkv(cfg.batch * n_h, cfg.embed_dim, seed=seed, peaked=peaked, bf16=bf)
    d_out = WL.make_qkv(cfg.batch * n_h, cfg.embed_dim, seed=seed + 100, bf16=bf)[:, :cfg.embed_dim]
    return (qkv.reshape(cfg.batch, n_h, 3 * cfg.embed_dim),
            np.ascontiguousarray(d_out).reshape(cfg.batch, n_h, cfg.embed_dim))


def _run(m, qkv, d_out):
    q_dev, g_dev = cuda(qkv, m.act_dtype), cuda(d_out, m.act_dtype)
    out, lse = m.attention_with_lse(q_dev)
    d_qkv = m.attention_bwd(q_dev, out, lse, g_dev)
    torch.cuda.synchronize()
    return d_qkv.float().cpu().numpy()


@pytest.mark.parametrize("cfg", [SMALL_F32, SMALL_BF16, SMALL_BF16_DH128, SMALL_BF16_DH256], ids=lambda c: c.name)
@pytest.mark.parametrize("peaked", [False, True])
def test_tiles_attention_bwd_parity(cfg, peaked):
    say(f"attention gradient parity {cfg.name} peaked={peaked}")
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    qkv, d_out = _inputs(cfg, n_h, peaked)
    ref = O.tiles_attention_bwd(qkv, d_out, tiles, cfg.heads)
    with B.Reslim(cfg, weights_for(cfg)) as m:
        got = _run(m, qkv, d_out)
    assert np.isfinite(got).all()
    D = cfg.embed_dim
    for name, sl in (("dq", slice(0, D)), ("dk", slice(D, 2 * D)), ("dv", slice(2 * D, 3 * D))):
        assert_parity(got[..., sl], ref[..., sl], TOL[cfg.dtype], name, say, **(GRAD_BF16 if cfg.dtype else {}))


def test_tiles_attention_bwd_special_cases():
    """Known answers: a zero upstream gradient gives a zero gradient; with constant v the
    output does not depend on q or k, so dq = dk = 0 and dv_j = sum_i P_ij dO_i;
    one tile over the whole grid is the gradient of global attention."""
    cfg = SMALL_BF16.with_(tiles_y=1, tiles_x=1, halo=5, batch=1)
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, 1, 1, 5)
    D = cfg.embed_dim
    qkv, d_out = _inputs(cfg, n_h, False, seed=6)
    with B.Reslim(cfg, weights_for(cfg)) as m:
        assert m.n_h == cfg.n_tokens
        got = _run(m, qkv, np.zeros_like(d_out))
        assert not got.any()
        cst = qkv.copy()
        cst[..., 2 * D:] = WL.round_to_bf16(np.linspace(-2, 2, D, dtype=np.float32))
        got = _run(m, cst, d_out)
        ref = O.tiles_attention_bwd(cst, d_out, tiles, cfg.heads)
        scale = np.abs(ref[..., 2 * D:]).max()
        assert np.abs(got[..., :2 * D]).max() <= 2e-2 * scale      # exact answer 0; bf16 rounding of O leaks a little
        assert O.rel_l2(got[..., 2 * D:], ref[..., 2 * D:]) <= 2e-2
        got = _run(m, qkv, d_out)
        dq, dk, dv = O.self_attention_bwd(qkv[0, :, :D], qkv[0, :, D:2 * D], qkv[0, :, 2 * D:], d_out[0], cfg.heads)
        assert O.rel_l2(got[0], np.concatenate([dq, dk, dv], axis=1)) <= 2e-2


def test_tiles_attention_bwd_ragged_and_tiny_tiles():
    """Tiles of 1 x 1 .. few patches (fewer tokens than one streamed block, one wave
    partly idle) and a tile size that leaves ragged ends on both sides."""
    for cfg in (SMALL_BF16.with_(name="tiny", H=8, W=12, tiles_y=4, tiles_x=6, halo=0, batch=1),
                SMALL_BF16.with_(name="ragged", H=46, W=66, tiles_y=1, tiles_x=2, halo=1, batch=1),
                SMALL_F32.with_(name="tiny32", H=8, W=12, tiles_y=4, tiles_x=6, halo=0, batch=1)):
        tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
        say(f"  {cfg.name}: n_t = {sorted(set(t['n_tok'] for t in tiles))}")
        qkv, d_out = _inputs(cfg, n_h, False, seed=8)
        ref = O.tiles_attention_bwd(qkv, d_out, tiles, cfg.heads)
        with B.Reslim(cfg, weights_for(cfg)) as m:
            got = _run(m, qkv, d_out)
        assert_parity(got, ref, TOL[cfg.dtype], cfg.name, say, **(GRAD_BF16 if cfg.dtype else {}))


FULL_SIZE = [("c1", ((0, 0), (1, 5), (3, 15), (2, 10))),      # dh 64: the shape bench.py times
             ("c4", ((0, 0), (0, 9))),                          # dh 128, 2448 tokens per interior tile
             ("m10b", ((0, 5), (0, 15)))]                       # dh 256 (the 10B model's heads)


@pytest.mark.parametrize("name,pairs", FULL_SIZE, ids=[n for n, _ in FULL_SIZE])
def test_tiles_attention_bwd_full_size_sampled_tiles(name, pairs):
    """Full-size shapes (c1: 4 x 16 tiles x 8 heads, 612..720 tokens per tile; c4 and the 10B
    model: one sample, 16 tiles, 32 heads of dimension 128 / 256): the oracle recomputes sampled
    (sample, tile) pairs (exact: tiles do not interact), and two properties are checked over the
    whole output: sum_i dq_i . q_i = sum_j dk_j . k_j per (sample, tile, head) (both equal
    sum_ij dS_ij S_ij), and determinism."""
    cfg = WL.CONFIGS[name]
    tiles, _, _, n_h = O.tiles_partition(cfg.Hp, cfg.Wp, cfg.tiles_y, cfg.tiles_x, cfg.halo)
    qkv, d_out = _inputs(cfg, n_h, False, seed=9)
    D, dh = cfg.embed_dim, cfg.embed_dim // cfg.heads
    one = cfg.with_(depth=1, mlp_ratio=1)   # the attention entry points do not use the block weights
    with B.Reslim(one, WL.make_weights(one)) as m:
        got = _run(m, qkv, d_out)
        again = _run(m, qkv, d_out)
    assert np.array_equal(got, again)
    for b, t in pairs:
        tl = tiles[t]
        r = slice(tl["tok_off"], tl["tok_off"] + tl["n_tok"])
        dq, dk, dv = O.self_attention_bwd(qkv[b, r, :D], qkv[b, r, D:2 * D], qkv[b, r, 2 * D:], d_out[b, r], cfg.heads)
        for gname, a, ref in (("dq", got[b, r, :D], dq), ("dk", got[b, r, D:2 * D], dk), ("dv", got[b, r, 2 * D:], dv)):
            assert_parity(a, ref, 2e-2, f"{name} sample {b} tile {t} {gname}", say, **GRAD_BF16)
    worst = 0.0
    for tl in tiles:
        r = slice(tl["tok_off"], tl["tok_off"] + tl["n_tok"])
        q64, g64 = qkv[:, r].astype(np.float64), got[:, r].astype(np.float64)
        r = slice(None)
        a = (g64[:, r, :D] * q64[:, r, :D]).reshape(cfg.batch, -1, cfg.heads, dh).sum(axis=(1, 3))
        c = (g64[:, r, D:2 * D] * q64[:, r, D:2 * D]).reshape(cfg.batch, -1, cfg.heads, dh).sum(axis=(1, 3))
        n = np.sqrt((g64[:, r, :D] ** 2).reshape(cfg.batch, -1, cfg.heads, dh).sum(axis=(1, 3)) *
                    (q64[:, r, :D] ** 2).reshape(cfg.batch, -1, cfg.heads, dh).sum(axis=(1, 3)))
        worst = max(worst, float((np.abs(a - c) / n).max()))
    say(f"  trace identity, worst normalised gap {worst:.3e}")
    assert worst <= 2e-2
