"""Seeded random small geometries: every pass, every layout the library accepts for the shape
(AUTO, Types 1-3, FUSED), against the oracle.  Meant to hit the corner cases of the index logic
(windows in the padding, strides that do not divide, chunks of positions that span images, odd
channel counts per group) that the hand-picked shapes may miss."""
import numpy as np
import pytest

import oracle
from paper_1504_04343_amd import synth
from gpu_util import (TOL_F32, gpu_backward_data, gpu_backward_weights, gpu_forward, layer, odims,
                      rel_err)

pytestmark = pytest.mark.gpu


def random_layers(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        g = int(rng.choice([1, 1, 2, 3]))
        C = g * int(rng.integers(1, 9))
        O = g * int(rng.integers(1, 12))
        K = int(rng.integers(1, 6))
        s = int(rng.integers(1, 4))
        p = int(rng.integers(0, K + 1))
        H = int(rng.integers(1, 21))
        W = int(rng.integers(1, 21))
        if H + 2 * p < K or W + 2 * p < K:
            continue
        N = int(rng.integers(1, 7))
        out.append(layer("rnd%d" % len(out), N, C, H, W, O, K, s, p, g))
    return out


def random_wide_layers(count, seed):
    """More channels per group (the fused kernels stage them 16 at a time) and more images."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        g = int(rng.choice([1, 2]))
        C = g * int(rng.integers(17, 72))
        O = g * int(rng.integers(8, 150))
        K = int(rng.choice([2, 3, 3, 5]))
        s = int(rng.choice([1, 1, 2]))
        p = int(rng.integers(0, K))
        H = int(rng.integers(K, 30))
        W = int(rng.integers(K, 30))
        N = int(rng.integers(2, 13))
        out.append(layer("wide%d" % len(out), N, C, H, W, O, K, s, p, g))
    return out


LAYERS = random_layers(36, 2024) + random_wide_layers(16, 99)


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_1504_04343_amd import binding
    return binding


@pytest.mark.parametrize("L", LAYERS, ids=[
    "%s_N%d_C%d_%dx%d_O%d_K%d_s%d_p%d_g%d" % (L.name, L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad,
                                               L.groups) for L in LAYERS])
def test_random_shape_all_layouts(B, L):
    x, w = synth.make_x(L, 7), synth.make_w(L, 7)
    b, dy = synth.make_bias(L, 7), synth.make_dy(L, 7)
    od = odims(oracle, L)
    y_want = oracle.conv_forward(od, x, w, b)
    dx_want = oracle.conv_backward_data(od, w, dy)
    dw_want, db_want = oracle.conv_backward_weights(od, x, dy)
    ran = 0
    for lowering in (B.LOWER_AUTO, 1, 2, 3, B.LOWER_FUSED):
        for name, call, want in (
                ("forward", lambda: gpu_forward(B, L, x, w, b, lowering), y_want),
                ("backward_data", lambda: gpu_backward_data(B, L, w, dy, lowering), dx_want),
                ("backward_weights", lambda: gpu_backward_weights(B, L, x, dy, lowering), None)):
            try:
                got = call()
            except B.CctError as e:
                assert e.code == B.EUNSUPPORTED and lowering == B.LOWER_FUSED, (name, lowering, e)
                continue
            ran += 1
            if want is None:
                dw, db = got
                assert rel_err(dw, dw_want) <= TOL_F32, (name, lowering)
                assert rel_err(db, db_want) <= TOL_F32, (name, lowering)
            else:
                assert np.isfinite(got).all(), (name, lowering)
                assert rel_err(got, want) <= TOL_F32, (name, lowering)
    assert ran >= 12      # AUTO and the three materialised layouts always run
