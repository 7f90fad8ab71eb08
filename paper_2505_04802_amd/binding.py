"""Thin ctypes binding over libreslim.so (declarations: include/reslim.h).

Argument marshalling only -- every step of the forward runs in the library's HIP
kernels.  PyTorch is used for device memory and the current stream.  There is no
CPU fallback: a missing library or a missing GPU raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libreslim.so")

RESLIM_OK, RESLIM_EINVAL, RESLIM_ESHAPE, RESLIM_ENOMEM, RESLIM_EHIP, RESLIM_EWORKSPACE = 0, -1, -2, -3, -4, -5
RESLIM_F32, RESLIM_BF16 = 0, 1

_CONFIG_FIELDS = ["in_vars", "out_vars", "H", "W", "scale", "patch", "embed_dim", "heads", "mlp_ratio",
                  "depth", "tiles_y", "tiles_x", "halo", "res_idx", "n_res", "dtype"]
_WEIGHT_FIELDS = ["w_pe", "b_pe", "var_emb", "agg_q0", "agg_wq", "agg_bq", "agg_wk", "agg_bk", "agg_wv",
                  "agg_bv", "agg_wo", "agg_bo", "pos_emb", "res_emb", "ln1_g", "ln1_b", "w_qkv", "b_qkv",
                  "w_proj", "b_proj", "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2", "lnf_g", "lnf_b",
                  "w_head", "b_head", "w_res", "b_res", "out_var_idx"]

EXPORTS = ["tiles_partition", "reslim_create", "reslim_destroy", "reslim_last_error",
           "reslim_tokens_per_sample", "reslim_workspace_bytes", "reslim_embed_fwd", "tiles_attention_fwd",
           "reslim_block_fwd", "reslim_head_fwd", "reslim_forward", "reslim_flop_counts",
           "reslim_debug_set_gemm_tile", "reslim_profile_enable", "reslim_profile_reset", "reslim_profile_read",
           "reslim_debug_copy", "reslim_debug_set_attention_variant",
           "reslim_bayes_loss_workspace_bytes", "reslim_bayes_loss_fwd", "reslim_bayes_loss_static_max_groups",
           "reslim_bayes_loss_fwd_static", "tiles_attention_fwd_lse",
           "tiles_attention_bwd_workspace_bytes", "tiles_attention_bwd",
           "reslim_train_prepare", "reslim_layernorm_bwd", "reslim_linear_bwd_workspace_bytes", "reslim_linear_bwd",
           "reslim_block_train_bytes", "reslim_block_fwd_train", "reslim_block_bwd",
           "reslim_block_grads_unscale", "reslim_grad_scale_update",
           "reslim_train_prepare_model", "reslim_bayes_loss_bwd", "reslim_head_bwd_workspace_bytes", "reslim_head_bwd",
           "reslim_embed_bwd_workspace_bytes", "reslim_embed_bwd", "reslim_train_step_bytes", "reslim_train_step_grads",
           "reslim_grads_unscale",
           "reslim_asc_build", "reslim_asc_build_tiles", "reslim_asc_edges", "reslim_asc_plan_create", "reslim_asc_plan_destroy",
           "reslim_asc_plan_info", "reslim_asc_image", "reslim_asc_compress", "reslim_asc_forward",
           "reslim_asc_decompress", "reslim_asc_compress_bwd", "reslim_asc_decompress_bwd",
           "reslim_asc_block_train_bytes", "reslim_asc_block_fwd_train", "reslim_asc_block_bwd"]


class ReslimConfigC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in _CONFIG_FIELDS]


class ReslimWeightsC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WEIGHT_FIELDS]


class TileDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("y0", "y1", "x0", "x1", "Y0", "Y1", "X0", "X1")] + \
               [("tok_off", C.c_int64), ("n_tok", C.c_int32), ("_pad", C.c_int32)]


BLOCK_PARAMS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj", "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


class BlockGradsC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in BLOCK_PARAMS]


MODEL_PARAMS = ("w_pe", "b_pe", "var_emb", "agg_q0", "agg_wq", "agg_bq", "agg_wk", "agg_bk", "agg_wv", "agg_bv", "agg_wo", "agg_bo",
                "pos_emb", "res_emb") + BLOCK_PARAMS + ("lnf_g", "lnf_b", "w_head", "b_head", "w_res", "b_res")


class GradsC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in MODEL_PARAMS]


class ProfileRecord(C.Structure):
    _fields_ = [("name", C.c_char_p), ("ms", C.c_float), ("flop", C.c_double), ("bytes", C.c_double)]


class ReslimError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libreslim error {code}: {msg}")
        self.code = code


_lib: Optional[C.CDLL] = None


def load() -> C.CDLL:
    """dlopen the library and set the prototypes.  Needs no GPU."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python __graft_entry__.py` (hipcc, gfx950) first")
    lib = C.CDLL(LIB_PATH)
    for name in EXPORTS:
        if not hasattr(lib, name):
            raise ImportError(f"{LIB_PATH} does not export {name}")
    vp, i32, i64p, szp = C.c_void_p, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_size_t)
    lib.tiles_partition.argtypes = [i32, i32, i32, i32, i32, C.POINTER(TileDesc), vp, vp, i64p]
    lib.reslim_create.argtypes = [C.POINTER(ReslimConfigC), C.POINTER(ReslimWeightsC), C.POINTER(vp)]
    lib.reslim_destroy.argtypes = [vp]
    lib.reslim_destroy.restype = None
    lib.reslim_last_error.argtypes = [vp]
    lib.reslim_last_error.restype = C.c_char_p
    lib.reslim_tokens_per_sample.argtypes = [vp, i64p]
    lib.reslim_workspace_bytes.argtypes = [vp, i32, szp]
    lib.reslim_embed_fwd.argtypes = [vp, vp, vp, i32, vp, C.c_size_t, vp]
    lib.tiles_attention_fwd.argtypes = [vp, vp, vp, i32, vp]
    lib.tiles_attention_fwd_lse.argtypes = [vp, vp, vp, vp, i32, vp]
    lib.tiles_attention_bwd_workspace_bytes.argtypes = [vp, i32, szp]
    lib.tiles_attention_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, C.c_size_t, vp]
    lib.reslim_block_fwd.argtypes = [vp, i32, vp, i32, vp, C.c_size_t, vp]
    lib.reslim_block_grads_unscale.argtypes = [vp, C.POINTER(BlockGradsC), C.c_float, vp, vp]
    lib.reslim_grad_scale_update.argtypes = [C.POINTER(C.c_float), C.POINTER(i32), i32, C.c_float, C.c_float, i32]
    lib.reslim_train_prepare.argtypes = [vp]
    lib.reslim_train_prepare_model.argtypes = [vp, C.POINTER(ReslimWeightsC)]
    lib.reslim_bayes_loss_bwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, C.c_float, C.c_float, vp, vp]
    lib.reslim_head_bwd_workspace_bytes.argtypes = [vp, i32, szp]
    lib.reslim_embed_bwd_workspace_bytes.argtypes = [vp, i32, szp]
    lib.reslim_head_bwd.argtypes = [vp, vp, vp, vp, vp, C.POINTER(GradsC), i32, vp, C.c_size_t, vp]
    lib.reslim_embed_bwd.argtypes = [vp, vp, vp, C.POINTER(GradsC), i32, vp, C.c_size_t, vp]
    lib.reslim_train_step_bytes.argtypes = [vp, i32, szp, szp]
    lib.reslim_train_step_grads.argtypes = [vp, vp, vp, vp, C.c_float, C.c_float, vp, vp, C.POINTER(GradsC), i32, vp, C.c_size_t,
                                            vp, C.c_size_t, vp]
    lib.reslim_grads_unscale.argtypes = [vp, C.POINTER(GradsC), C.c_float, vp, vp]
    lib.reslim_layernorm_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, C.c_int64, vp, C.c_size_t, vp]
    lib.reslim_linear_bwd_workspace_bytes.argtypes = [vp, i32, i32, szp]
    lib.reslim_linear_bwd.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, i32, vp, C.c_size_t, vp]
    lib.reslim_block_train_bytes.argtypes = [vp, i32, szp, szp]
    lib.reslim_block_fwd_train.argtypes = [vp, i32, vp, vp, vp, C.c_size_t, i32, vp, C.c_size_t, vp]
    lib.reslim_block_bwd.argtypes = [vp, i32, vp, vp, C.c_size_t, vp, vp, C.POINTER(BlockGradsC), i32, vp, C.c_size_t, vp]
    lib.reslim_head_fwd.argtypes = [vp, vp, vp, vp, i32, vp, C.c_size_t, vp]
    lib.reslim_forward.argtypes = [vp, vp, vp, i32, vp, C.c_size_t, vp]
    dp = C.POINTER(C.c_double)
    lib.reslim_flop_counts.argtypes = [vp, i32, dp, dp, dp]
    lib.reslim_profile_enable.argtypes = [vp, i32]
    lib.reslim_profile_reset.argtypes = [vp]
    lib.reslim_profile_read.argtypes = [vp, C.POINTER(ProfileRecord), i32, C.POINTER(i32)]
    lib.reslim_debug_copy.argtypes = [vp, vp, C.c_size_t, vp]
    lib.reslim_bayes_loss_workspace_bytes.argtypes = [i32, i32, i32, i32, C.POINTER(C.c_size_t)]
    lib.reslim_bayes_loss_fwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, C.c_float, vp, vp, C.c_size_t, vp]
    lib.reslim_bayes_loss_static_max_groups.argtypes = [C.POINTER(C.c_int64)]
    lib.reslim_bayes_loss_fwd_static.argtypes = [vp, vp, vp, i32, i32, i32, i32, C.c_float, vp, vp]
    lib.reslim_asc_build.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, i32, C.c_float, vp, vp, vp, vp, vp, C.POINTER(C.c_int64)]
    lib.reslim_asc_build_tiles.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, i32, i32, C.c_float, vp, vp, vp, vp, vp,
                                           C.POINTER(C.c_int64)]
    lib.reslim_asc_edges.argtypes = [vp, i32, i32, i32, i32, vp]
    lib.reslim_asc_plan_create.argtypes = [vp, i32, vp, vp, vp, C.c_int64, vp, C.c_int64, vp, C.POINTER(vp)]
    lib.reslim_asc_plan_destroy.argtypes = [vp]
    lib.reslim_asc_plan_destroy.restype = None
    lib.reslim_asc_plan_info.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(i32)]
    lib.reslim_asc_image.argtypes = [vp, vp, vp, vp, vp, i32, vp]
    lib.reslim_asc_compress.argtypes = [vp, vp, vp, vp, vp]
    lib.reslim_asc_forward.argtypes = [vp, vp, vp, vp, vp, C.c_size_t, vp]
    for nm in ("reslim_asc_decompress", "reslim_asc_compress_bwd", "reslim_asc_decompress_bwd"):
        getattr(lib, nm).argtypes = [vp, vp, vp, vp, vp]
    lib.reslim_asc_block_train_bytes.argtypes = [vp, vp, szp, szp]
    lib.reslim_asc_block_fwd_train.argtypes = [vp, vp, i32, vp, vp, vp, C.c_size_t, vp, C.c_size_t, vp]
    lib.reslim_asc_block_bwd.argtypes = [vp, vp, i32, vp, vp, C.c_size_t, vp, vp, C.POINTER(BlockGradsC), vp, C.c_size_t, vp]
    lib.reslim_debug_set_gemm_tile.argtypes = [i32]
    lib.reslim_debug_set_gemm_tile.restype = None
    lib.reslim_debug_set_attention_variant.argtypes = [i32]
    lib.reslim_debug_set_attention_variant.restype = None
    for name in EXPORTS:
        if name not in ("reslim_destroy", "reslim_last_error", "reslim_debug_set_gemm_tile",
                        "reslim_debug_set_attention_variant", "reslim_asc_plan_destroy"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int, ctx=None):
    if rc != RESLIM_OK:
        msg = load().reslim_last_error(ctx)
        raise ReslimError(rc, msg.decode() if msg else "")


# ------------------------------------------------------------------ plain calls
def tiles_partition(Hp: int, Wp: int, Ty: int, Tx: int, halo: int):
    """Returns (tiles: list of dict, gather_idx: int32[n_h], interior_src: int32[Hp*Wp], n_h)."""
    lib = load()
    n_h = C.c_int64(0)
    _check(lib.tiles_partition(Hp, Wp, Ty, Tx, halo, None, None, None, C.byref(n_h)))
    tiles = (TileDesc * (Ty * Tx))()
    gather = np.empty(n_h.value, np.int32)
    isrc = np.empty(Hp * Wp, np.int32)
    _check(lib.tiles_partition(Hp, Wp, Ty, Tx, halo, tiles, gather.ctypes.data, isrc.ctypes.data, None))
    names = ("y0", "y1", "x0", "x1", "Y0", "Y1", "X0", "X1", "tok_off", "n_tok")
    return [{n: int(getattr(t, n)) for n in names} for t in tiles], gather, isrc, int(n_h.value)


def reslim_debug_set_attention_variant(variant: int) -> None:
    load().reslim_debug_set_attention_variant(variant)


def reslim_debug_set_gemm_tile(choice: int) -> None:
    load().reslim_debug_set_gemm_tile(choice)


def reslim_create(cfg, weights: Dict[str, np.ndarray]) -> int:
    """cfg: object with the reslim_config fields; weights: name -> contiguous fp32 array."""
    lib = load()
    cc = ReslimConfigC(**{n: int(getattr(cfg, n)) for n in _CONFIG_FIELDS})
    keep = []
    wc = ReslimWeightsC()
    for n in _WEIGHT_FIELDS:
        a = np.ascontiguousarray(weights[n], dtype=np.int32 if n == "out_var_idx" else np.float32)
        keep.append(a)
        setattr(wc, n, a.ctypes.data)
    ctx = C.c_void_p()
    _check(lib.reslim_create(C.byref(cc), C.byref(wc), C.byref(ctx)))
    return ctx.value


def reslim_destroy(ctx: int) -> None:
    load().reslim_destroy(ctx)


def reslim_tokens_per_sample(ctx: int) -> int:
    v = C.c_int64()
    _check(load().reslim_tokens_per_sample(ctx, C.byref(v)), ctx)
    return v.value


def reslim_workspace_bytes(ctx: int, batch: int) -> int:
    v = C.c_size_t()
    _check(load().reslim_workspace_bytes(ctx, batch, C.byref(v)), ctx)
    return v.value


def reslim_flop_counts(ctx: int, batch: int):
    g, a, h = C.c_double(), C.c_double(), C.c_double()
    _check(load().reslim_flop_counts(ctx, batch, C.byref(g), C.byref(a), C.byref(h)), ctx)
    return g.value, a.value, h.value


def reslim_debug_copy(src, dst, stream=None) -> None:
    """Plain copy kernel src -> dst (same-size torch CUDA tensors); the profilers' bandwidth yardstick."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(load().reslim_debug_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream_ptr(stream)))


def reslim_bayes_loss_workspace_bytes(batch: int, n_vars: int, Hf: int, Wf: int) -> int:
    n = C.c_size_t(0)
    _check(load().reslim_bayes_loss_workspace_bytes(batch, n_vars, Hf, Wf, C.byref(n)))
    return int(n.value)


def reslim_bayes_loss_fwd(pred, target, lat_w, tv_weight: float, out3, workspace, stream=None) -> None:
    """pred, target: fp32 CUDA tensors [B, K, Hf, Wf]; lat_w: fp32 CUDA [Hf]; out3: float64 CUDA [3]
    (total, data term, prior term); workspace: CUDA byte buffer of reslim_bayes_loss_workspace_bytes."""
    b, k, hf, wf = pred.shape
    _check(load().reslim_bayes_loss_fwd(pred.data_ptr(), target.data_ptr(), lat_w.data_ptr(), b, k, hf, wf,
                                        float(tv_weight), out3.data_ptr(), workspace.data_ptr(),
                                        workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


def reslim_bayes_loss_static_max_groups() -> int:
    n = C.c_int64(0)
    _check(load().reslim_bayes_loss_static_max_groups(C.byref(n)))
    return int(n.value)


def reslim_bayes_loss_fwd_static(pred, target, lat_w, tv_weight: float, out3, stream=None) -> None:
    """reslim_bayes_loss_fwd without a workspace: the partial sums use the library's fixed device array."""
    b, k, hf, wf = pred.shape
    _check(load().reslim_bayes_loss_fwd_static(pred.data_ptr(), target.data_ptr(), lat_w.data_ptr(), b, k, hf, wf,
                                               float(tv_weight), out3.data_ptr(), _stream_ptr(stream)))


def reslim_profile_enable(ctx: int, max_records: int) -> None:
    _check(load().reslim_profile_enable(ctx, max_records), ctx)


def reslim_profile_reset(ctx: int) -> None:
    _check(load().reslim_profile_reset(ctx), ctx)


def reslim_profile_read(ctx: int):
    """[(label, ms, flop, bytes)] of the launches since the last reset (waits for them)."""
    lib = load()
    n = C.c_int32()
    _check(lib.reslim_profile_read(ctx, None, 0, C.byref(n)), ctx)
    recs = (ProfileRecord * max(n.value, 1))()
    _check(lib.reslim_profile_read(ctx, recs, n.value, C.byref(n)), ctx)
    return [(recs[i].name.decode(), float(recs[i].ms), recs[i].flop, recs[i].bytes) for i in range(n.value)]


def _stream_ptr(stream=None) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def reslim_embed_fwd(ctx, x, tokens, batch, workspace, stream=None):
    _check(load().reslim_embed_fwd(ctx, x.data_ptr(), tokens.data_ptr(), batch, workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_ptr(stream)), ctx)


def tiles_attention_fwd_lse(ctx, qkv, out, lse, batch, stream=None):
    _check(load().tiles_attention_fwd_lse(ctx, qkv.data_ptr(), out.data_ptr(), lse.data_ptr(), batch, _stream_ptr(stream)), ctx)


def tiles_attention_bwd_workspace_bytes(ctx, batch) -> int:
    out = C.c_size_t(0)
    _check(load().tiles_attention_bwd_workspace_bytes(ctx, batch, C.byref(out)), ctx)
    return out.value


def tiles_attention_bwd(ctx, qkv, out, lse, d_out, d_qkv, batch, workspace, stream=None):
    _check(load().tiles_attention_bwd(ctx, qkv.data_ptr(), out.data_ptr(), lse.data_ptr(), d_out.data_ptr(),
                                      d_qkv.data_ptr(), batch, workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream_ptr(stream)), ctx)


def tiles_attention_fwd(ctx, qkv, out, batch, stream=None):
    _check(load().tiles_attention_fwd(ctx, qkv.data_ptr(), out.data_ptr(), batch, _stream_ptr(stream)), ctx)


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def reslim_train_prepare(ctx):
    _check(load().reslim_train_prepare(ctx), ctx)


def reslim_train_prepare_model(ctx, weights: Dict[str, np.ndarray]) -> None:
    keep = []
    wc = ReslimWeightsC()
    for n in _WEIGHT_FIELDS:
        a = np.ascontiguousarray(weights[n], dtype=np.int32 if n == "out_var_idx" else np.float32)
        keep.append(a)
        setattr(wc, n, a.ctypes.data)
    _check(load().reslim_train_prepare_model(ctx, C.byref(wc)), ctx)


def _grads_c(grads) -> "GradsC":
    """grads: name -> fp32 CUDA tensor; names that are absent become null pointers."""
    return GradsC(**{n: (grads[n].data_ptr() if n in grads else None) for n in MODEL_PARAMS})


def reslim_bayes_loss_bwd(pred, target, lat_w, tv_weight: float, upstream: float, d_pred, stream=None) -> None:
    b, k, hf, wf = pred.shape
    _check(load().reslim_bayes_loss_bwd(pred.data_ptr(), target.data_ptr(), lat_w.data_ptr(), b, k, hf, wf, float(tv_weight),
                                        float(upstream), d_pred.data_ptr(), _stream_ptr(stream)))


def reslim_head_bwd_workspace_bytes(ctx, batch: int) -> int:
    n = C.c_size_t(0)
    _check(load().reslim_head_bwd_workspace_bytes(ctx, batch, C.byref(n)), ctx)
    return int(n.value)


def reslim_embed_bwd_workspace_bytes(ctx, batch: int) -> int:
    n = C.c_size_t(0)
    _check(load().reslim_embed_bwd_workspace_bytes(ctx, batch, C.byref(n)), ctx)
    return int(n.value)


def reslim_head_bwd(ctx, x, tokens, d_y, d_tokens, grads, batch: int, workspace, stream=None) -> None:
    g = _grads_c(grads)
    _check(load().reslim_head_bwd(ctx, x.data_ptr(), tokens.data_ptr(), d_y.data_ptr(), d_tokens.data_ptr(), C.byref(g), batch,
                                  workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream)), ctx)


def reslim_embed_bwd(ctx, x, d_tokens, grads, batch: int, workspace, stream=None) -> None:
    g = _grads_c(grads)
    _check(load().reslim_embed_bwd(ctx, x.data_ptr(), d_tokens.data_ptr(), C.byref(g), batch, workspace.data_ptr(),
                                   _nbytes(workspace), _stream_ptr(stream)), ctx)


def reslim_train_step_bytes(ctx, batch: int):
    a, b = C.c_size_t(0), C.c_size_t(0)
    _check(load().reslim_train_step_bytes(ctx, batch, C.byref(a), C.byref(b)), ctx)
    return int(a.value), int(b.value)


def reslim_train_step_grads(ctx, x, target, lat_w, tv_weight: float, loss_scale: float, y, loss3, grads, batch: int, saved,
                            workspace, stream=None) -> None:
    g = _grads_c(grads)
    _check(load().reslim_train_step_grads(ctx, x.data_ptr(), target.data_ptr(), lat_w.data_ptr(), float(tv_weight), float(loss_scale),
                                          y.data_ptr(), loss3.data_ptr(), C.byref(g), batch, saved.data_ptr(), _nbytes(saved),
                                          workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream)), ctx)


def reslim_grads_unscale(ctx, grads, inv_scale: float, found_inf, stream=None) -> None:
    g = _grads_c(grads)
    _check(load().reslim_grads_unscale(ctx, C.byref(g), float(inv_scale), found_inf.data_ptr(), _stream_ptr(stream)), ctx)


def reslim_layernorm_bwd(ctx, x, dy, gamma, res, dx, dgamma, dbeta, rows, workspace, stream=None):
    _check(load().reslim_layernorm_bwd(ctx, x.data_ptr(), dy.data_ptr(), gamma.data_ptr(),
                                       res.data_ptr() if res is not None else None, dx.data_ptr(), dgamma.data_ptr(),
                                       dbeta.data_ptr(), rows, workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream)), ctx)


def reslim_linear_bwd_workspace_bytes(ctx, which, rows) -> int:
    out = C.c_size_t(0)
    _check(load().reslim_linear_bwd_workspace_bytes(ctx, which, rows, C.byref(out)), ctx)
    return out.value


def reslim_linear_bwd(ctx, layer, which, x, dy, dx, dw, db, rows, workspace, stream=None):
    _check(load().reslim_linear_bwd(ctx, layer, which, x.data_ptr(), dy.data_ptr(), dx.data_ptr() if dx is not None else None,
                                    dw.data_ptr(), db.data_ptr(), rows, workspace.data_ptr(), _nbytes(workspace),
                                    _stream_ptr(stream)), ctx)


def reslim_block_train_bytes(ctx, batch):
    a, b = C.c_size_t(0), C.c_size_t(0)
    _check(load().reslim_block_train_bytes(ctx, batch, C.byref(a), C.byref(b)), ctx)
    return a.value, b.value


def reslim_block_fwd_train(ctx, layer, x_in, x_out, saved, batch, workspace, stream=None):
    _check(load().reslim_block_fwd_train(ctx, layer, x_in.data_ptr(), x_out.data_ptr(), saved.data_ptr(), _nbytes(saved),
                                         batch, workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream)), ctx)


def reslim_block_bwd(ctx, layer, x_in, saved, d_x_out, d_x_in, grads, batch, workspace, stream=None):
    """grads: dict name -> fp32 CUDA tensor for every name in BLOCK_PARAMS (written)."""
    g = BlockGradsC(**{n: grads[n].data_ptr() for n in BLOCK_PARAMS})
    _check(load().reslim_block_bwd(ctx, layer, x_in.data_ptr(), saved.data_ptr(), _nbytes(saved), d_x_out.data_ptr(),
                                   d_x_in.data_ptr(), C.byref(g), batch, workspace.data_ptr(), _nbytes(workspace),
                                   _stream_ptr(stream)), ctx)


def reslim_block_grads_unscale(ctx, grads, inv_scale, found_inf, stream=None):
    """grads: dict of fp32 CUDA tensors (BLOCK_PARAMS), scaled in place; found_inf: int32 CUDA tensor of one element."""
    g = BlockGradsC(**{n: grads[n].data_ptr() for n in BLOCK_PARAMS})
    _check(load().reslim_block_grads_unscale(ctx, C.byref(g), inv_scale, found_inf.data_ptr(), _stream_ptr(stream)), ctx)


def reslim_grad_scale_update(scale, tracker, found_inf, growth=2.0, backoff=0.5, interval=2000):
    """Host function: returns the new (scale, tracker)."""
    s, t = C.c_float(scale), C.c_int32(tracker)
    _check(load().reslim_grad_scale_update(C.byref(s), C.byref(t), int(bool(found_inf)), growth, backoff, interval))
    return s.value, t.value


def reslim_block_fwd(ctx, layer, x_inout, batch, workspace, stream=None):
    _check(load().reslim_block_fwd(ctx, layer, x_inout.data_ptr(), batch, workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_ptr(stream)), ctx)


def reslim_head_fwd(ctx, x, tokens, y, batch, workspace, stream=None):
    _check(load().reslim_head_fwd(ctx, x.data_ptr(), tokens.data_ptr(), y.data_ptr(), batch, workspace.data_ptr(),
                                  workspace.numel() * workspace.element_size(), _stream_ptr(stream)), ctx)


def reslim_forward(ctx, x, y, batch, workspace, stream=None):
    _check(load().reslim_forward(ctx, x.data_ptr(), y.data_ptr(), batch, workspace.data_ptr(),
                                 workspace.numel() * workspace.element_size(), _stream_ptr(stream)), ctx)


# ------------------------------------------------------------------ adaptive spatial compression
def reslim_asc_build(images: np.ndarray, patch: int, max_leaf: int, min_leaf: int, canny_low: int, canny_high: int,
                     tau: float) -> Dict[str, np.ndarray]:
    """Host function.  images: fp32 [B, H, W].  Returns the leaf table as int32 arrays:
    leaf_y0, leaf_x0, leaf_s [L], sample_off [B + 1], patch_leaf [B, Hp*Wp]."""
    images = np.ascontiguousarray(images, np.float32)
    B, H, W = images.shape
    cap = max(B * (H // max(patch, 1)) * (W // max(patch, 1)), 1)
    ly, lx, ls = (np.zeros(cap, np.int32) for _ in range(3))
    off = np.zeros(B + 1, np.int32)
    pl = np.zeros(cap, np.int32)
    n = C.c_int64(0)
    _check(load().reslim_asc_build(images.ctypes.data, B, H, W, patch, max_leaf, min_leaf, canny_low, canny_high, tau,
                                   ly.ctypes.data, lx.ctypes.data, ls.ctypes.data, off.ctypes.data, pl.ctypes.data,
                                   C.byref(n)))
    L = int(n.value)
    return dict(leaf_y0=ly[:L].copy(), leaf_x0=lx[:L].copy(), leaf_s=ls[:L].copy(), sample_off=off,
                patch_leaf=pl.reshape(B, -1))


def reslim_asc_build_tiles(images: np.ndarray, patch: int, tiles_y: int, tiles_x: int, halo: int, max_leaf: int, min_leaf: int,
                           canny_low: int, canny_high: int, tau: float) -> Dict[str, np.ndarray]:
    """Host function: reslim_asc_build per (sample, tile) on the tile's haloed box.  Returns the table of
    reslim_asc_build with leaf coordinates on the whole grid and sample_off [B * T + 1] (one entry per
    (sample, tile) sequence)."""
    images = np.ascontiguousarray(images, np.float32)
    B, H, W = images.shape
    Hp, Wp = H // max(patch, 1), W // max(patch, 1)
    n_h = C.c_int64(0)
    if Hp >= 1 and Wp >= 1 and tiles_y >= 1 and tiles_x >= 1:
        _check(load().tiles_partition(Hp, Wp, tiles_y, tiles_x, halo, (TileDesc * (tiles_y * tiles_x))(), None, None, C.byref(n_h)))
    cap = max(B * int(n_h.value), 1)
    ly, lx, ls = (np.zeros(cap, np.int32) for _ in range(3))
    off = np.zeros(B * max(tiles_y * tiles_x, 1) + 1, np.int32)
    pl = np.zeros(max(B * Hp * Wp, 1), np.int32)
    n = C.c_int64(0)
    _check(load().reslim_asc_build_tiles(images.ctypes.data, B, H, W, patch, tiles_y, tiles_x, halo, max_leaf, min_leaf,
                                         canny_low, canny_high, tau, ly.ctypes.data, lx.ctypes.data, ls.ctypes.data,
                                         off.ctypes.data, pl.ctypes.data, C.byref(n)))
    L = int(n.value)
    return dict(leaf_y0=ly[:L].copy(), leaf_x0=lx[:L].copy(), leaf_s=ls[:L].copy(), sample_off=off,
                patch_leaf=pl.reshape(B, -1))


def reslim_asc_edges(image: np.ndarray, canny_low: int, canny_high: int) -> np.ndarray:
    image = np.ascontiguousarray(image, np.float32)
    H, W = image.shape
    out = np.zeros((H, W), np.uint8)
    _check(load().reslim_asc_edges(image.ctypes.data, H, W, canny_low, canny_high, out.ctypes.data))
    return out


def reslim_asc_plan_create(ctx, batch: int, table: Dict[str, np.ndarray]) -> int:
    arrs = {k: np.ascontiguousarray(table[k], np.int32) for k in ("leaf_y0", "leaf_x0", "leaf_s", "sample_off", "patch_leaf")}
    out = C.c_void_p(None)
    _check(load().reslim_asc_plan_create(ctx, batch, arrs["leaf_y0"].ctypes.data, arrs["leaf_x0"].ctypes.data,
                                         arrs["leaf_s"].ctypes.data, len(arrs["leaf_s"]), arrs["sample_off"].ctypes.data,
                                         len(arrs["sample_off"]) - 1, arrs["patch_leaf"].ctypes.data, C.byref(out)), ctx)
    return out.value


def reslim_asc_plan_destroy(plan) -> None:
    load().reslim_asc_plan_destroy(plan)


def reslim_asc_plan_info(plan):
    n, m = C.c_int64(0), C.c_int32(0)
    _check(load().reslim_asc_plan_info(plan, C.byref(n), C.byref(m)))
    return int(n.value), int(m.value)


def reslim_asc_image(ctx, tokens, w_img, b_img, image, batch, stream=None):
    _check(load().reslim_asc_image(ctx, tokens.data_ptr(), w_img.data_ptr(), b_img.data_ptr(), image.data_ptr(), batch,
                                   _stream_ptr(stream)), ctx)


def reslim_asc_compress(ctx, plan, tokens, tokens_c, stream=None):
    _check(load().reslim_asc_compress(ctx, plan, tokens.data_ptr(), tokens_c.data_ptr(), _stream_ptr(stream)), ctx)


def reslim_asc_forward(ctx, plan, x, y, workspace, stream=None):
    _check(load().reslim_asc_forward(ctx, plan, x.data_ptr(), y.data_ptr(), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream_ptr(stream)), ctx)


def reslim_asc_decompress(ctx, plan, tokens_c, tokens, stream=None):
    _check(load().reslim_asc_decompress(ctx, plan, tokens_c.data_ptr(), tokens.data_ptr(), _stream_ptr(stream)), ctx)


def reslim_asc_compress_bwd(ctx, plan, d_tokens_c, d_tokens, stream=None):
    _check(load().reslim_asc_compress_bwd(ctx, plan, d_tokens_c.data_ptr(), d_tokens.data_ptr(), _stream_ptr(stream)), ctx)


def reslim_asc_decompress_bwd(ctx, plan, d_tokens, d_tokens_c, stream=None):
    _check(load().reslim_asc_decompress_bwd(ctx, plan, d_tokens.data_ptr(), d_tokens_c.data_ptr(), _stream_ptr(stream)), ctx)


def reslim_asc_block_train_bytes(ctx, plan):
    a, b = C.c_size_t(0), C.c_size_t(0)
    _check(load().reslim_asc_block_train_bytes(ctx, plan, C.byref(a), C.byref(b)), ctx)
    return int(a.value), int(b.value)


def reslim_asc_block_fwd_train(ctx, plan, layer, x_in, x_out, saved, workspace, stream=None):
    _check(load().reslim_asc_block_fwd_train(ctx, plan, layer, x_in.data_ptr(), x_out.data_ptr(), saved.data_ptr(),
                                             _nbytes(saved), workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream)), ctx)


def reslim_asc_block_bwd(ctx, plan, layer, x_in, saved, d_x_out, d_x_in, grads, workspace, stream=None):
    g = BlockGradsC(**{n: grads[n].data_ptr() for n in BLOCK_PARAMS})
    _check(load().reslim_asc_block_bwd(ctx, plan, layer, x_in.data_ptr(), saved.data_ptr(), _nbytes(saved),
                                       d_x_out.data_ptr(), d_x_in.data_ptr(), C.byref(g), workspace.data_ptr(),
                                       _nbytes(workspace), _stream_ptr(stream)), ctx)


# ------------------------------------------------------------------ convenience holder
class Reslim:
    """Owns a reslim_ctx and a workspace tensor; methods take/return torch CUDA tensors."""

    def __init__(self, cfg, weights, max_batch: Optional[int] = None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("libreslim needs a GPU: there is no CPU path")
        self.cfg = cfg
        self.ctx = reslim_create(cfg, weights)
        self.n_h = reslim_tokens_per_sample(self.ctx)
        self.max_batch = max_batch or cfg.batch
        self.ws = torch.empty(reslim_workspace_bytes(self.ctx, self.max_batch), dtype=torch.uint8, device="cuda")
        assert self.ws.data_ptr() % 256 == 0
        self.act_dtype = torch.bfloat16 if cfg.dtype == RESLIM_BF16 else torch.float32

    def close(self):
        if self.ctx:
            import torch
            torch.cuda.synchronize()
            reslim_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def _batch(self, t):
        b = t.shape[0]
        assert b <= self.max_batch and t.is_cuda and t.is_contiguous()
        return b

    def embed(self, x):
        import torch
        b = self._batch(x)
        tok = torch.empty((b, self.n_h, self.cfg.embed_dim), dtype=torch.float32, device="cuda")
        reslim_embed_fwd(self.ctx, x, tok, b, self.ws)
        return tok

    def attention(self, qkv):
        import torch
        b = self._batch(qkv)
        assert qkv.dtype == self.act_dtype and qkv.shape[1:] == (self.n_h, 3 * self.cfg.embed_dim)
        out = torch.empty((b, self.n_h, self.cfg.embed_dim), dtype=self.act_dtype, device="cuda")
        tiles_attention_fwd(self.ctx, qkv, out, b)
        return out

    def attention_with_lse(self, qkv):
        """Forward that also returns the log-sum-exp [b, heads, n_h] the gradient needs."""
        import torch
        b = self._batch(qkv)
        assert qkv.dtype == self.act_dtype and qkv.shape[1:] == (self.n_h, 3 * self.cfg.embed_dim)
        out = torch.empty((b, self.n_h, self.cfg.embed_dim), dtype=self.act_dtype, device="cuda")
        lse = torch.empty((b, self.cfg.heads, self.n_h), dtype=torch.float32, device="cuda")
        tiles_attention_fwd_lse(self.ctx, qkv, out, lse, b)
        return out, lse

    def attention_bwd(self, qkv, out, lse, d_out):
        """Gradient of the tile attention with respect to qkv."""
        import torch
        b = self._batch(qkv)
        assert qkv.dtype == self.act_dtype and d_out.dtype == self.act_dtype and out.dtype == self.act_dtype
        assert qkv.shape[1:] == (self.n_h, 3 * self.cfg.embed_dim) and d_out.shape == out.shape == (b, self.n_h, self.cfg.embed_dim)
        assert all(t.is_contiguous() for t in (qkv, out, lse, d_out))
        ws = torch.empty(max(tiles_attention_bwd_workspace_bytes(self.ctx, b), 256), dtype=torch.uint8, device="cuda")
        d_qkv = torch.empty_like(qkv)
        tiles_attention_bwd(self.ctx, qkv, out, lse, d_out, d_qkv, b, ws)
        return d_qkv

    def block(self, layer, tokens):
        b = self._batch(tokens)
        assert tokens.dtype.is_floating_point and tokens.element_size() == 4
        reslim_block_fwd(self.ctx, layer, tokens, b, self.ws)
        return tokens

    def head(self, x, tokens):
        import torch
        b = self._batch(x)
        c = self.cfg
        y = torch.empty((b, c.out_vars, c.H * c.scale, c.W * c.scale), dtype=torch.float32, device="cuda")
        reslim_head_fwd(self.ctx, x, tokens, y, b, self.ws)
        return y

    def forward(self, x, y=None):
        import torch
        b = self._batch(x)
        c = self.cfg
        if y is None:
            y = torch.empty((b, c.out_vars, c.H * c.scale, c.W * c.scale), dtype=torch.float32, device="cuda")
        reslim_forward(self.ctx, x, y, b, self.ws)
        return y
