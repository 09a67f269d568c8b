"""CaffeNet's fully connected layers run through the convolution entry points: a fully connected
layer on a C x H x W input is a convolution whose kernel covers the whole input (fc6: 256 x 6 x 6
-> 4096, kernel 6, one output pixel), and on a vector a 1 x 1 convolution on a 1 x 1 image (fc7,
fc8).  Lowering is then trivial (one position per image: the lowered matrix is the flattened input)
and the multiply phase is the layer.  Batch 256 as in the full-stack configuration; every pass,
AUTO lowering; sampled outputs against the oracle."""
import numpy as np
import pytest

import oracle
from paper_1504_04343_amd import synth
from gpu_util import TOL_F32, desc_of, gpu_backward_data, gpu_backward_weights, gpu_forward, layer, odims

pytestmark = pytest.mark.gpu

FC = [
    layer("fc6", 256, 256, 6, 6, 4096, 6, 1, 0, 1, "relu_normal", 0.005, 0.1),
    layer("fc7", 256, 4096, 1, 1, 4096, 1, 1, 0, 1, "relu_normal", 0.005, 0.1),
    layer("fc8", 256, 4096, 1, 1, 1000, 1, 1, 0, 1, "relu_normal", 0.01, 0.1),
]


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1504_04343_amd import binding
    return binding


@pytest.mark.parametrize("L", FC, ids=[L.name for L in FC])
def test_fully_connected_as_convolution(B, L):
    assert (L.Hout, L.Wout) == (1, 1)
    x, w, b, dy = synth.make_x(L, 2), synth.make_w(L, 2), synth.make_bias(L, 2), synth.make_dy(L, 2)
    od = odims(oracle, L)
    for lowering in (B.LOWER_AUTO, 1):
        idx = synth.sample_indices(L.N * L.O, 2000, 1)
        want = oracle.conv_forward_at(od, x, w, b, idx)
        got = gpu_forward(B, L, x, w, b, lowering).ravel()[idx]
        assert np.abs(got - want).max() / np.abs(want).max() <= TOL_F32, ("forward", lowering)
        idx = synth.sample_indices(L.N * L.C * L.H * L.W, 2000, 2)
        want = oracle.conv_backward_data_at(od, w, dy, idx)
        got = gpu_backward_data(B, L, w, dy, lowering).ravel()[idx]
        assert np.abs(got - want).max() / np.abs(want).max() <= TOL_F32, ("backward-data", lowering)
        idx = synth.sample_indices(L.O * L.C * L.K * L.K, 2000, 3)
        want = oracle.conv_backward_weights_at(od, x, dy, idx)
        dw, db = gpu_backward_weights(B, L, x, dy, lowering)
        assert np.abs(dw.ravel()[idx] - want).max() / np.abs(want).max() <= TOL_F32, ("backward-weights", lowering)
        db_want = dy.astype(np.float64).sum(axis=(0, 2, 3))
        assert np.abs(db - db_want).max() / np.abs(db_want).max() <= TOL_F32
