"""The allocation-free dense-gradient entry point against the allocating one, through the C ABI: two
calls in a row on one GPU, the second on a smaller problem, so whatever the first call left in the
library's fixed scratch array must not show in the second."""
import numpy as np
import pytest
import torch

from oracle import rng
from paper_1902_01064_amd import hop, inputs

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _case(d, B, rows, seed, loss):
    ws = inputs.hidden_w(seed, d)
    X, y = inputs.dense_svm_data(seed, 0, rows, d, ws)
    w = (inputs.initial_params(seed, d, 0.01) + 0.02 * ws / np.sqrt(d)).contiguous()
    ridx = torch.from_numpy(rng.batch_rows(seed, 0, 3, B, rows).astype(np.int32))
    return [t.to(DEV) for t in (X, y, w, ridx)] + [B, d, loss]


def _run(case, static):
    X, y, w, ridx, B, d, loss = case
    st = torch.cuda.current_stream().cuda_stream
    g = torch.full((d + 8,), 7.0, dtype=torch.float32, device=DEV)
    coef = torch.full((B + 8,), 7.0, dtype=torch.float32, device=DEV)
    args = (X.data_ptr(), y.data_ptr(), w.data_ptr(), ridx.data_ptr(), B, d, 1e-3, g.data_ptr(), coef.data_ptr())
    if static:
        hop.hop_svm_grad_dense_static(*args, st, loss)
    else:
        scratch = torch.empty(hop.hop_grad_scratch_floats(d, B), dtype=torch.float32, device=DEV)
        hop.hop_svm_grad_dense(*args, scratch.data_ptr(), st, loss)
    torch.cuda.synchronize()
    return g.cpu().numpy(), coef.cpu().numpy()


def test_static_entry_point_equals_the_allocating_one_twice_in_a_row():
    hop.load()
    big = _case(16384 * 3 + 4, 200, 300, 11, hop.HOP_LOSS_HINGE)       # 4 column segments x 200 samples
    small = _case(1022, 37, 64, 12, hop.HOP_LOSS_LOG)                  # 1 segment, ragged d, other loss
    want = [_run(c, False) for c in (big, small)]
    got = [_run(c, True) for c in (big, small)]                        # back to back, the smaller one second
    for (g0, c0), (g1, c1), case in zip(want, got, (big, small)):
        B, d = case[4], case[5]
        assert np.array_equal(g0.view(np.uint32), g1.view(np.uint32))          # same kernels: bit for bit
        assert np.array_equal(c0.view(np.uint32), c1.view(np.uint32))
        assert (g1[d:] == 7.0).all() and (c1[B:] == 7.0).all()                 # nothing written past the ends
        assert np.isfinite(g1[:d]).all() and np.abs(g1[:d]).max() > 0


def test_static_entry_point_refuses_what_does_not_fit():
    case = _case(16384 * 70, 1000, 8, 13, hop.HOP_LOSS_HINGE)           # 70 segments x 1000 samples > 65536
    X, y, w, ridx, B, d, loss = case
    g = torch.zeros(d, dtype=torch.float32, device=DEV)
    coef = torch.zeros(B, dtype=torch.float32, device=DEV)
    with pytest.raises(hop.HopError) as e:
        hop.hop_svm_grad_dense_static(X.data_ptr(), y.data_ptr(), w.data_ptr(), ridx.data_ptr(), B, d, 1e-3,
                                      g.data_ptr(), coef.data_ptr(), torch.cuda.current_stream().cuda_stream, loss)
    assert e.value.code == hop.HOP_ERR_ARENA_TOO_SMALL
    torch.cuda.synchronize()
    assert float(g.abs().max()) == 0.0                                  # nothing was launched
