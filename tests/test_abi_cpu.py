"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, its host-side partition is bit-exact against the oracle, and argument
errors are reported as codes (no compute call is made here)."""
import ctypes as C
import itertools
import os
import re

import numpy as np
import pytest

from oracle import reslim_oracle as O
from paper_2505_04802_amd import binding as B
from paper_2505_04802_amd import workloads as WL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    header = open(os.path.join(ROOT, "include", "reslim.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:reslim|tiles)_[a-z0-9_]+)\s*\(", header))
    assert {"reslim_create", "tiles_partition", "tiles_attention_fwd", "reslim_block_fwd", "reslim_forward"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert declared <= set(B.EXPORTS)


def _same_partition(Hp, Wp, Ty, Tx, h):
    tiles, g, src, n_h = B.tiles_partition(Hp, Wp, Ty, Tx, h)
    rt, rg, rs, rn = O.tiles_partition(Hp, Wp, Ty, Tx, h)
    assert n_h == rn and tiles == rt
    assert g.dtype == np.int32 and np.array_equal(g, rg) and np.array_equal(src, rs)


def test_partition_bit_exact_small_grids():
    for Hp, Wp in [(1, 1), (3, 5), (7, 12), (12, 9)]:
        for Ty, Tx, h in itertools.product(range(1, 5), range(1, 5), range(0, 4)):
            if Ty <= Hp and Tx <= Wp:
                _same_partition(Hp, Wp, Ty, Tx, h)


@pytest.mark.parametrize("name", ["c0", "c1", "c2", "c3", "c4"])
def test_partition_bit_exact_benchmark_configs(name):
    c = WL.CONFIGS[name]
    _same_partition(c.Hp, c.Wp, c.tiles_y, c.tiles_x, c.halo)


def test_partition_rejects_bad_arguments():
    lib = B.load()
    n = C.c_int64()
    for args in [(4, 4, 5, 1, 0), (4, 4, 1, 5, 0), (4, 4, 1, 1, -1), (0, 4, 1, 1, 0), (4, 4, 0, 1, 0)]:
        assert lib.tiles_partition(*args, None, None, None, C.byref(n)) == B.RESLIM_ESHAPE
        assert b"tiles_partition" in lib.reslim_last_error(None)


def test_create_rejects_bad_configs_before_touching_the_gpu():
    base = WL.CONFIGS["c0"]
    w = WL.make_weights(base)
    for kw, code in [(dict(H=33), B.RESLIM_ESHAPE), (dict(heads=3), B.RESLIM_ESHAPE),
                     (dict(out_vars=3), B.RESLIM_ESHAPE), (dict(res_idx=5), B.RESLIM_ESHAPE),
                     (dict(dtype=7), B.RESLIM_EINVAL), (dict(dtype=1), B.RESLIM_ESHAPE),   # dh = 32 on the bf16 path
                     (dict(dtype=1, heads=2, scale=1, out_vars=1), B.RESLIM_ESHAPE),          # bf16 head narrower than 8 columns
                     (dict(scale=0), B.RESLIM_ESHAPE)]:
        with pytest.raises(B.ReslimError) as e:
            B.reslim_create(base.with_(**kw), w)
        assert e.value.code == code, kw
    lib = B.load()
    assert lib.reslim_create(None, None, None) == B.RESLIM_EINVAL
    assert lib.reslim_workspace_bytes(None, 1, None) == B.RESLIM_EINVAL
    assert lib.reslim_forward(None, None, None, 1, None, 0, None) == B.RESLIM_EINVAL


def test_grad_scale_update_host_rule_matches_oracle():
    """reslim_grad_scale_update is host arithmetic (no GPU): the same sequence of overflow flags through
    the library and through the oracle's restatement of the rule (itself pinned to PyTorch's GradScaler)."""
    from oracle import reslim_oracle as O
    seq = [0, 0, 1, 0, 0, 0, 0, 1, 1, 0, 0, 0, 0, 0, 0, 0]
    a = b = (65536.0, 0)
    for f in seq:
        a = B.reslim_grad_scale_update(a[0], a[1], f, 2.0, 0.5, 3)
        b = O.grad_scale_update(b[0], b[1], bool(f), 2.0, 0.5, 3)
        assert a == b
    lib = B.load()
    import ctypes as C
    s, t = C.c_float(1.0), C.c_int32(0)
    assert lib.reslim_grad_scale_update(None, C.byref(t), 0, 2.0, 0.5, 3) == B.RESLIM_EINVAL
    assert lib.reslim_grad_scale_update(C.byref(s), C.byref(t), 0, 0.5, 0.5, 3) == B.RESLIM_EINVAL      # growth < 1
    assert lib.reslim_grad_scale_update(C.byref(s), C.byref(t), 0, 2.0, 0.0, 3) == B.RESLIM_EINVAL      # backoff <= 0
    assert lib.reslim_grad_scale_update(C.byref(s), C.byref(t), 0, 2.0, 0.5, 0) == B.RESLIM_EINVAL
