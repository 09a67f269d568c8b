"""GPU parity at the benchmark's full sizes (CaffeNet conv1-5, batch 256, the launch
configuration bench.py times: AUTO lowering, default workspace), on sampled outputs that the
oracle computes one by one."""
import numpy as np
import pytest

import oracle
from paper_1504_04343_amd import synth
from gpu_util import (TOL_F32, desc_of, gpu_backward_data, gpu_backward_weights, gpu_forward,
                      odims, rel_err)

pytestmark = pytest.mark.gpu

LAYERS = synth.caffenet(256)


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_1504_04343_amd import binding
    return binding


def scale_of(vals):
    return float(np.abs(vals).max())


@pytest.mark.parametrize("L", LAYERS, ids=[L.name for L in LAYERS])
def test_full_size_layer_forward_backward_sampled(B, L):
    print("full-size", L.name, flush=True)
    x, w, dy = synth.make_x(L), synth.make_w(L), synth.make_dy(L)
    bias = (np.random.default_rng(11).standard_normal(L.O) * 0.1).astype(np.float32)
    od = odims(oracle, L)

    y = gpu_forward(B, L, x, w, bias, B.LOWER_AUTO)
    idx = synth.sample_indices(y.size, 4000, 1)
    want = oracle.conv_forward_at(od, x, w, bias, idx)
    assert np.abs(y.ravel()[idx] - want).max() / scale_of(want) <= TOL_F32
    assert np.isfinite(y).all()
    del y

    dx = gpu_backward_data(B, L, w, dy, B.LOWER_AUTO)
    idx = synth.sample_indices(dx.size, 4000, 2)
    want = oracle.conv_backward_data_at(od, w, dy, idx)
    assert np.abs(dx.ravel()[idx] - want).max() / scale_of(want) <= TOL_F32
    assert np.isfinite(dx).all()
    del dx

    dw, db = gpu_backward_weights(B, L, x, dy, B.LOWER_AUTO)
    idx = synth.sample_indices(dw.size, 96, 3)
    want = oracle.conv_backward_weights_at(od, x, dy, idx)
    assert np.abs(dw.ravel()[idx] - want).max() / scale_of(want) <= TOL_F32
    assert np.isfinite(dw).all()
    # dbias is a plain sum: fp64 numpy sum is its definition
    want_db = dy.astype(np.float64).sum(axis=(0, 2, 3))
    assert rel_err(db, want_db) <= TOL_F32


BIG = [L.with_batch(1024) for L in LAYERS if L.name in ("conv1", "conv3")]


@pytest.mark.parametrize("L", BIG, ids=[L.name + "_b1024" for L in BIG])
def test_batch_1024_sampled(B, L):
    """The larger batch of the full-stack configuration.  conv1's lowered matrices (4.5 GB at this
    batch) exceed the default workspace, so its backward passes run in several chunks."""
    print("batch-1024", L.name, flush=True)
    x, w, dy = synth.make_x(L), synth.make_w(L), synth.make_dy(L)
    od = odims(oracle, L)
    y = gpu_forward(B, L, x, w, None, B.LOWER_AUTO)
    idx = synth.sample_indices(y.size, 1500, 1)
    want = oracle.conv_forward_at(od, x, w, None, idx)
    assert np.abs(y.ravel()[idx] - want).max() / scale_of(want) <= TOL_F32
    del y
    dx = gpu_backward_data(B, L, w, dy, B.LOWER_AUTO)
    idx = synth.sample_indices(dx.size, 1500, 2)
    want = oracle.conv_backward_data_at(od, w, dy, idx)
    assert np.abs(dx.ravel()[idx] - want).max() / scale_of(want) <= TOL_F32
    del dx
    dw, db = gpu_backward_weights(B, L, x, dy, B.LOWER_AUTO)
    idx = synth.sample_indices(dw.size, 24, 3)
    want = oracle.conv_backward_weights_at(od, x, dy, idx)
    assert np.abs(dw.ravel()[idx] - want).max() / scale_of(want) <= TOL_F32
    assert rel_err(db, dy.astype(np.float64).sum(axis=(0, 2, 3))) <= TOL_F32


@pytest.mark.parametrize("L", [LAYERS[1], LAYERS[2]], ids=["conv2_bf16", "conv3_bf16"])
def test_full_size_bf16_variant_sampled(B, L):
    """bf16 operands, fp32 accumulate, AUTO lowering, against the fp64 oracle on unrounded inputs."""
    from gpu_util import TOL_BF16
    print("full-size bf16", L.name, flush=True)
    x, w, dy = synth.make_x(L), synth.make_w(L), synth.make_dy(L)
    od = odims(oracle, L)
    P = B.PREC_BF16_IN_F32_ACC
    y = gpu_forward(B, L, x, w, None, B.LOWER_AUTO, P)
    idx = synth.sample_indices(y.size, 2000, 1)
    want = oracle.conv_forward_at(od, x, w, None, idx)
    assert np.abs(y.ravel()[idx] - want).max() / scale_of(want) <= TOL_BF16
    del y
    dx = gpu_backward_data(B, L, w, dy, B.LOWER_AUTO, P)
    idx = synth.sample_indices(dx.size, 2000, 2)
    want = oracle.conv_backward_data_at(od, w, dy, idx)
    assert np.abs(dx.ravel()[idx] - want).max() / scale_of(want) <= TOL_BF16
    del dx
    dw, _ = gpu_backward_weights(B, L, x, dy, B.LOWER_AUTO, P)
    idx = synth.sample_indices(dw.size, 48, 3)
    want = oracle.conv_backward_weights_at(od, x, dy, idx)
    assert np.abs(dw.ravel()[idx] - want).max() / scale_of(want) <= TOL_BF16
