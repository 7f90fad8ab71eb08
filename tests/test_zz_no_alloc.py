"""The loss entry point that allocates nothing (reslim_bayes_loss_fwd_static) against the entry
point with a caller-owned workspace (reslim_bayes_loss_fwd), through the C ABI.

Both run the same two kernels with the same launch shape, so the results must be bit-identical;
the oracle comparison of the loss itself lives in test_gpu_parity.py.  Two calls in a row, the
second on a smaller input: the fixed array keeps the first call's partial sums and the second
call must not see them."""
import numpy as np
import pytest
import torch

from oracle import reslim_oracle as O
from paper_2505_04802_amd import binding as B

pytestmark = pytest.mark.gpu


def _inputs(shape, seed):
    rng = np.random.default_rng([41, seed])
    pred = rng.normal(size=shape).astype(np.float32)
    target = (pred + 0.3 * rng.normal(size=shape)).astype(np.float32)
    lw = O.lat_weights(shape[2], -80.0, 85.0).astype(np.float32)
    return pred, target, lw


def _both(shape, seed):
    pred, target, lw = _inputs(shape, seed)
    p, t, l = (torch.from_numpy(a).cuda() for a in (pred, target, lw))
    ws = torch.empty(max(B.reslim_bayes_loss_workspace_bytes(*shape), 8), dtype=torch.uint8, device="cuda")
    ref = torch.zeros(3, dtype=torch.float64, device="cuda")
    got = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    B.reslim_bayes_loss_fwd(p, t, l, 0.25, ref, ws)
    B.reslim_bayes_loss_fwd_static(p, t, l, 0.25, got)
    torch.cuda.synchronize()
    return got.cpu().numpy(), ref.cpu().numpy(), O.bayes_loss(pred, target, lw, tv_weight=0.25)


def test_static_loss_two_calls_second_smaller():
    print("static loss: first call (3, 4, 203, 2051), then (1, 2, 37, 53)", flush=True)
    for seed, shape in enumerate([(3, 4, 203, 2051), (1, 2, 37, 53)]):
        got, ref, oracle = _both(shape, seed)
        print(f"static loss {shape}: static {got}, workspace {ref}, oracle {np.array(oracle)}", flush=True)
        assert np.array_equal(got, ref)                     # same kernels, same order of additions
        for g, r in zip(got, oracle):
            assert abs(g - r) <= 1e-5 * abs(r) + 1e-12      # the bar of test_bayes_loss_parity


def test_static_loss_limit_and_arguments():
    max_groups = B.reslim_bayes_loss_static_max_groups()
    assert max_groups == 1 << 18
    p = torch.zeros((1, 1, 8, 8), dtype=torch.float32, device="cuda")
    l = torch.ones(8, dtype=torch.float32, device="cuda")
    out = torch.zeros(3, dtype=torch.float64, device="cuda")
    lib = B.load()
    # one work-group per 8 rows x 1024 columns of a plane: 65535 planes x 5 strips is beyond the array;
    # the size check comes before any launch, so the (too small) buffers are never touched
    rc = lib.reslim_bayes_loss_fwd_static(p.data_ptr(), p.data_ptr(), l.data_ptr(), 65535, 1, 40, 8, 0.25, out.data_ptr(), None)
    assert rc == B.RESLIM_EWORKSPACE
    assert lib.reslim_bayes_loss_fwd_static(None, p.data_ptr(), l.data_ptr(), 1, 1, 8, 8, 0.25, out.data_ptr(), None) == B.RESLIM_EINVAL
    assert lib.reslim_bayes_loss_fwd_static(p.data_ptr(), p.data_ptr(), l.data_ptr(), 1, 1, 0, 8, 0.25, out.data_ptr(), None) == B.RESLIM_EINVAL
