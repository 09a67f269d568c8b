"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar: lowering maps bit-exact; fp32 outputs max|gpu-oracle|/max|oracle| <= 1e-4; bf16-operand
variant <= 2e-2.  Small cases are compared element by element (they still span several GEMM
tiles and ragged tails); the full-size CaffeNet layers at batch 256 are compared on sampled
outputs that the oracle computes one by one."""
import numpy as np
import pytest

import oracle
from paper_1504_04343_amd import synth
from gpu_util import (TOL_BF16, TOL_F32, desc_of, dev, gpu_backward_data, gpu_backward_weights,
                      gpu_forward, layer, odims, rel_err)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1504_04343_amd import binding
    return binding


# name, N, C, H, W, O, K, s, p, g
SMALL = [
    layer("cfg1", 4, 3, 32, 32, 16, 5, 1, 2, 1),                 # BASELINE config 1
    layer("ragged", 3, 5, 17, 13, 7, 3, 1, 1, 1),                # H != W, odd everything
    layer("stride2_floor", 2, 4, 10, 10, 6, 3, 2, 0, 2),         # floor in Hout, groups
    layer("conv1_like", 2, 3, 67, 67, 96, 11, 4, 0, 1),          # K=363 tail, M=96 tile
    layer("conv2_like", 2, 96, 27, 27, 256, 5, 1, 2, 2),         # groups 2, M=128
    layer("conv3_like", 3, 64, 13, 13, 384, 3, 1, 1, 1),         # M spans 3 tiles
    layer("wide_m", 2, 8, 9, 9, 200, 3, 1, 1, 1),                # M=200: ragged M tile
    layer("k1", 2, 40, 12, 12, 24, 1, 1, 0, 1),                  # 1x1: all layouts coincide
    layer("pad_gt_k", 1, 2, 6, 6, 3, 2, 1, 3, 1),                # windows entirely in the padding
    layer("stride3_g3", 2, 6, 14, 11, 9, 4, 3, 1, 3),
    layer("single_pixel_out", 2, 3, 5, 5, 4, 5, 1, 0, 1),        # Hout = Wout = 1
    layer("long_k", 1, 352, 6, 6, 8, 3, 1, 1, 1),                # 3168 patch rows: beyond the fused kernel's LDS tap table
    layer("depthwise", 2, 8, 9, 9, 8, 3, 1, 1, 8),               # groups = C = O: one channel per group
    layer("tiny", 1, 1, 1, 1, 1, 1, 1, 0, 1),                    # everything is 1
]
IDS = [L.name for L in SMALL]


def inputs(L, seed=0):
    return synth.make_x(L, seed), synth.make_w(L, seed), synth.make_bias(L, seed), synth.make_dy(L, seed)


# ------------------------------------------------------------------ lowering maps, bit-exact
@pytest.mark.parametrize("L", SMALL, ids=IDS)
@pytest.mark.parametrize("lowering", [1, 2, 3])
def test_lowering_map_bit_exact(B, L, lowering):
    import torch
    x = synth.make_x(L, 1)
    d = desc_of(B, L)
    rows, cols, _ = B.cct_lowered_shape(d, lowering)
    ld = B.cct_lowered_ld(d, lowering)
    dhat = torch.full((L.groups * cols, ld), float("nan"), device="cuda")
    B.cct_lower(d, lowering, dev(x), dhat)
    torch.cuda.synchronize()
    got = dhat.cpu().numpy()[:, :rows].reshape(L.groups, cols, rows)
    want = oracle.lower_data(odims(oracle, L), lowering, x)          # (groups, rows, cols)
    assert oracle.lowered_shape(odims(oracle, L), lowering)[:2] == (rows, cols)
    assert got.tobytes() == np.ascontiguousarray(want.transpose(0, 2, 1)).tobytes()


def test_lowering_map_names_its_source(B):
    """Input whose value encodes its own linear index (per image, < 2^24)."""
    import torch
    L = layer("idx", 2, 3, 19, 23, 4, 5, 2, 2, 1)
    per = L.C * L.H * L.W
    x = np.tile(np.arange(1, per + 1, dtype=np.float32), L.N).reshape(L.N, L.C, L.H, L.W)
    d = desc_of(B, L)
    for lowering in (1, 2, 3):
        rows, cols, _ = B.cct_lowered_shape(d, lowering)
        dhat = torch.zeros((cols, B.cct_lowered_ld(d, lowering)), device="cuda")
        B.cct_lower(d, lowering, dev(x), dhat)
        got = dhat.cpu().numpy()[:, :rows]
        want = oracle.lower_data(odims(oracle, L), lowering, x)[0].T
        assert np.array_equal(got, want)
        assert not np.signbit(got[got == 0]).any()


# ------------------------------------------------------------------ forward
@pytest.mark.parametrize("L", SMALL, ids=IDS)
@pytest.mark.parametrize("lowering", [1, 2, 3, 4])
def test_forward_matches_oracle(B, L, lowering):
    x, w, b, _ = inputs(L)
    want = oracle.conv_forward(odims(oracle, L), x, w, b)
    got = gpu_forward(B, L, x, w, b, lowering)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= TOL_F32


@pytest.mark.parametrize("L", SMALL[:6], ids=IDS[:6])
def test_forward_auto_and_no_bias(B, L):
    x, w, _, _ = inputs(L, 3)
    want = oracle.conv_forward(odims(oracle, L), x, w, None)
    got = gpu_forward(B, L, x, w, None, B.LOWER_AUTO)
    assert rel_err(got, want) <= TOL_F32


@pytest.mark.parametrize("lowering", [1, 2, 3, 4])
@pytest.mark.parametrize("chunk", [1, 3])
def test_forward_chunked_batch(B, lowering, chunk):
    """A small workspace makes the library lower and multiply the batch in several chunks
    (Sec. 2.2 trades memory for batch size); the result must not change."""
    L = layer("chunked", 7, 6, 15, 15, 10, 3, 1, 1, 2)
    x, w, b, _ = inputs(L, 5)
    want = oracle.conv_forward(odims(oracle, L), x, w, b)
    got = gpu_forward(B, L, x, w, b, lowering, chunk=chunk)
    assert rel_err(got, want) <= TOL_F32
    assert np.array_equal(got, gpu_forward(B, L, x, w, b, lowering))   # same bits as one chunk


def test_forward_is_deterministic(B):
    L = SMALL[4]
    x, w, b, _ = inputs(L)
    a = gpu_forward(B, L, x, w, b, 1)
    assert a.tobytes() == gpu_forward(B, L, x, w, b, 1).tobytes()


# ------------------------------------------------------------------ backward
FUSED_BWDD_UNSUPPORTED = {"stride2_floor", "pad_gt_k", "stride3_g3"}
STRIDED = [
    layer("s2_k3", 3, 16, 15, 17, 32, 3, 2, 1, 1),               # U = 2: 4 residue classes, 4 taps each
    layer("s2_k5_g2", 2, 8, 21, 19, 64, 5, 2, 2, 2),             # U = 3, groups, 32 kernels per group
    layer("s3_k7", 2, 5, 29, 23, 16, 7, 3, 0, 1),                # U = 3, unpadded, (H - K) % s != 0
    layer("s4_k11_p1", 2, 3, 51, 47, 48, 11, 4, 1, 1),           # conv1-like with padding
    layer("s2_k4_deep", 2, 4, 18, 14, 80, 4, 2, 1, 1),           # 5 channel groups of 16 kernels
]


def test_backward_data_fused_strided_without_overlap_is_unsupported(B):
    """K <= stride leaves one tap per residue class (a 1x1 sub-kernel): not a fused form."""
    for L in (layer("s2_k2", 2, 6, 12, 12, 16, 2, 2, 0, 1), layer("s3_k2", 1, 4, 14, 14, 16, 2, 3, 0, 1)):
        _, w, _, dy = inputs(L)
        with pytest.raises(B.CctError) as e:
            gpu_backward_data(B, L, w, dy, B.LOWER_FUSED)
        assert e.value.code == B.EUNSUPPORTED
        want = oracle.conv_backward_data(odims(oracle, L), w, dy)     # AUTO still runs them
        assert rel_err(gpu_backward_data(B, L, w, dy, B.LOWER_AUTO), want) <= TOL_F32


@pytest.mark.parametrize("L", STRIDED, ids=[L.name for L in STRIDED])
def test_backward_data_fused_strided_matches_oracle(B, L):
    """Backward-data of strided layers through the fused kernel (s*s residue classes of dx as one
    stride-1 convolution of dy, written back depth-to-space)."""
    _, w, _, dy = inputs(L, 7)
    want = oracle.conv_backward_data(odims(oracle, L), w, dy)
    got = gpu_backward_data(B, L, w, dy, B.LOWER_FUSED)
    assert np.isfinite(got).all()                   # NaN prefill: every pixel was written
    assert rel_err(got, want) <= TOL_F32
    assert np.array_equal(got, gpu_backward_data(B, L, w, dy, B.LOWER_FUSED, chunk=1))


@pytest.mark.parametrize("L", SMALL, ids=IDS)
@pytest.mark.parametrize("lowering", [1, 2, 3, 4])
def test_backward_data_matches_oracle(B, L, lowering):
    _, w, _, dy = inputs(L)
    # the fused backward-data pass is a stride-1 convolution of dy: with the flipped kernels at
    # stride 1 (pad <= K-1), with the s*s residue sub-kernels at stride s when the kernels fill
    # groups of 16; anything else has no fused form and must say so before launching anything
    if lowering == 4 and L.name in FUSED_BWDD_UNSUPPORTED:
        with pytest.raises(B.CctError) as e:
            gpu_backward_data(B, L, w, dy, lowering)
        assert e.value.code == B.EUNSUPPORTED
        return
    want = oracle.conv_backward_data(odims(oracle, L), w, dy)
    got = gpu_backward_data(B, L, w, dy, lowering)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= TOL_F32


# The fused backward-weights pass stages the input rows of 32 positions in LDS; shapes where they
# do not fit (and 1x1 kernels) gather the lowered rows inside the split-K GEMM instead, which needs
# an unpadded layer.  A padded layer whose rows do not fit has no fused form.
FUSED_BWDW_UNSUPPORTED = {"stride3_g3"}
BWDW_EXTRA = [
    layer("many_images", 37, 20, 9, 7, 40, 3, 1, 1, 2),          # 2331 positions: several splits
    layer("tiny_planes", 50, 4, 4, 4, 5, 2, 1, 0, 1),            # 9 positions per image: a chunk spans 4 or 5 images
    layer("stride2_pad", 9, 6, 15, 15, 10, 3, 2, 1, 2),
    layer("k7_s3", 5, 3, 30, 26, 12, 7, 3, 2, 1),
]


@pytest.mark.parametrize("L", SMALL + BWDW_EXTRA, ids=IDS + [L.name for L in BWDW_EXTRA])
@pytest.mark.parametrize("lowering", [1, 2, 3, 4])
def test_backward_weights_matches_oracle(B, L, lowering):
    x, _, _, dy = inputs(L)
    if lowering == 4 and L.name in FUSED_BWDW_UNSUPPORTED:
        with pytest.raises(B.CctError) as e:
            gpu_backward_weights(B, L, x, dy, lowering)
        assert e.value.code == B.EUNSUPPORTED
        return
    dw_want, db_want = oracle.conv_backward_weights(odims(oracle, L), x, dy)
    dw, db = gpu_backward_weights(B, L, x, dy, lowering)
    assert np.isfinite(dw).all() and np.isfinite(db).all()
    assert rel_err(dw, dw_want) <= TOL_F32
    assert rel_err(db, db_want) <= TOL_F32


@pytest.mark.parametrize("chunk", [1, 3])
def test_backward_chunked_batch(B, chunk):
    L = layer("chunked", 7, 6, 15, 15, 10, 3, 2, 1, 2)
    x, w, _, dy = inputs(L, 5)
    od = odims(oracle, L)
    assert rel_err(gpu_backward_data(B, L, w, dy, 1, chunk=chunk), oracle.conv_backward_data(od, w, dy)) <= TOL_F32
    dw_want, db_want = oracle.conv_backward_weights(od, x, dy)
    for lowering in (1, 4):
        dw, db = gpu_backward_weights(B, L, x, dy, lowering, chunk=chunk)
        assert rel_err(dw, dw_want) <= TOL_F32 and rel_err(db, db_want) <= TOL_F32, lowering


@pytest.mark.parametrize("chunk", [1, 3])
def test_backward_data_type2_gather_chunked(B, chunk):
    """Type 2 at stride 1 gathers dR^ from dy inside the GEMM; chunks must not change the bits."""
    L = layer("chunked_s1", 7, 6, 15, 15, 10, 3, 1, 1, 2)
    _, w, _, dy = inputs(L, 5)
    want = oracle.conv_backward_data(odims(oracle, L), w, dy)
    got = gpu_backward_data(B, L, w, dy, 2, chunk=chunk)
    assert rel_err(got, want) <= TOL_F32
    assert np.array_equal(got, gpu_backward_data(B, L, w, dy, 2))


def test_backward_weights_without_dbias_and_deterministic(B):
    L = SMALL[4]
    x, _, _, dy = inputs(L)
    a, none = gpu_backward_weights(B, L, x, dy, 1, want_dbias=False)
    assert none is None
    b, _ = gpu_backward_weights(B, L, x, dy, 1)
    assert a.tobytes() == b.tobytes()          # fixed-order split-K reduction: same bits run to run


# ------------------------------------------------------------------ bf16-operand variant
@pytest.mark.parametrize("L", [SMALL[0], SMALL[3], SMALL[4], SMALL[5]], ids=[IDS[0], IDS[3], IDS[4], IDS[5]])
@pytest.mark.parametrize("lowering", [1, 2, 3])
def test_bf16_variant(B, L, lowering):
    x, w, b, dy = inputs(L)
    od = odims(oracle, L)
    got = gpu_forward(B, L, x, w, b, lowering, B.PREC_BF16_IN_F32_ACC)
    assert rel_err(got, oracle.conv_forward(od, x, w, b)) <= TOL_BF16
    got = gpu_backward_data(B, L, w, dy, lowering, B.PREC_BF16_IN_F32_ACC)
    assert rel_err(got, oracle.conv_backward_data(od, w, dy)) <= TOL_BF16
    dw_want, db_want = oracle.conv_backward_weights(od, x, dy)
    dw, db = gpu_backward_weights(B, L, x, dy, lowering, B.PREC_BF16_IN_F32_ACC)
    assert rel_err(dw, dw_want) <= TOL_BF16
    assert rel_err(db, db_want) <= TOL_F32          # dbias is summed from the fp32 dy


# ------------------------------------------------------------------ trade-off sweep shapes (Appendix A)
SWEEP = [L.with_batch(4) for L in synth.tradeoff_sweep()]


@pytest.mark.parametrize("L", SWEEP, ids=[L.name for L in SWEEP])
def test_tradeoff_sweep_shapes_all_layouts(B, L):
    """The #input/#output-channel sweep of the lowering trade-off study, at a small batch: every
    layout and the selector's pick give the oracle's result."""
    x, w, b, _ = inputs(L, 2)
    idx = synth.sample_indices(L.N * L.O * L.Hout * L.Wout, 3000, 4)
    want = oracle.conv_forward_at(odims(oracle, L), x, w, b, idx)
    scale = np.abs(want).max()
    for lowering in (1, 2, 3, B.LOWER_FUSED, B.LOWER_AUTO):
        got = gpu_forward(B, L, x, w, b, lowering).ravel()[idx]
        assert np.abs(got - want).max() / scale <= TOL_F32, lowering


# ------------------------------------------------------------------ error paths on the device entry points
def test_unsupported_and_workspace_errors(B):
    import torch
    L = SMALL[0]
    x, w, b, dy = inputs(L)
    d = desc_of(B, L, 1)
    y = torch.empty((L.N, L.O, L.Hout, L.Wout), device="cuda")
    with pytest.raises(B.CctError) as e:
        B.cct_conv_forward(d, dev(x), dev(w), dev(b), y, torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.code == B.EWORKSPACE
    with pytest.raises(ValueError):
        B.cct_conv_forward(d, dev(x)[:2], dev(w), dev(b), y, B.alloc_workspace(d, 0))
    # the fused bf16 kernel needs whole groups of 16 channels (this layer has 3), and there is no
    # fused backward-weights pass for a padded layer whose input rows do not fit in LDS
    df = desc_of(B, L, B.LOWER_FUSED, B.PREC_BF16_IN_F32_ACC)
    with pytest.raises(B.CctError) as e:
        B.cct_conv_workspace_bytes(df, B.PASS_FORWARD)
    assert e.value.code == B.EUNSUPPORTED
    with pytest.raises(B.CctError) as e:
        B.cct_conv_workspace_bytes(desc_of(B, SMALL[9], B.LOWER_FUSED), B.PASS_BACKWARD_WEIGHTS)
    assert e.value.code == B.EUNSUPPORTED
    df = desc_of(B, L, B.LOWER_FUSED)
    with pytest.raises(B.CctError) as e:
        B.cct_lowered_shape(df, B.LOWER_FUSED)
    assert e.value.code == B.EINVAL
