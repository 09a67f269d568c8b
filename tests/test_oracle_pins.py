"""Pins for the CPU oracle: everything here is fixed by the paper or by mathematics,
never by the oracle itself and never by the HIP path."""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import Dims

RNG = np.random.default_rng(1234)


def rnd(*shape):
    return RNG.standard_normal(shape).astype(np.float32)


def ints(*shape, lo=-3, hi=4):
    return RNG.integers(lo, hi, size=shape).astype(np.float32)


# ---------------------------------------------------------------- brute force, by hand
def test_hand_computed_3x3_by_2x2():
    # eq. (1): R[r,c] = sum D[r+r', c+c'] K[r', c'], n=3, k=2, m=n-k+1=2
    x = np.array([[[[1, 2, 3], [4, 5, 6], [7, 8, 10]]]], np.float32)
    w = np.array([[[[1, -1], [2, 3]]]], np.float32)
    want = np.array([[1 - 2 + 8 + 15, 2 - 3 + 10 + 18], [4 - 5 + 14 + 24, 5 - 6 + 16 + 30]], float)
    got = oracle.conv_forward(Dims(1, 1, 3, 3, 1, 2), x, w)
    assert got.shape == (1, 1, 2, 2)
    assert np.array_equal(got[0, 0], want)


def test_hand_computed_two_groups_integer():
    # N=1, C=2, O=2, groups=2, 2x2 input, 1x1... use K=2 pad=0 -> single output per channel
    x = np.array([[[[1, 2], [3, 4]], [[5, 6], [7, 8]]]], np.float32)
    w = np.array([[[[1, 0], [0, 1]]], [[[2, 1], [1, 2]]]], np.float32)  # O=2, Cg=1
    b = np.array([10, -10], np.float32)
    got = oracle.conv_forward(Dims(1, 2, 2, 2, 2, 2, groups=2), x, w, b)
    # group 0: channel 0 only: 1+4+10 ; group 1: channel 1 only: 10+6+7+16-10
    assert np.array_equal(got.ravel(), np.array([15.0, 29.0]))


def test_hand_computed_channel_sum():
    # two input channels, one group: the sum over i in eq. (1) runs over both
    x = np.array([[[[1, 2], [3, 4]], [[5, 6], [7, 8]]]], np.float32)
    w = np.array([[[[1, 1], [1, 1]], [[1, 0], [0, -1]]]], np.float32)
    got = oracle.conv_forward(Dims(1, 2, 2, 2, 1, 2), x, w)
    assert got.ravel()[0] == (1 + 2 + 3 + 4) + (5 - 8)


# ---------------------------------------------------------------- 1x1 conv == matrix product
@pytest.mark.parametrize("N,C,O,H,W", [(2, 5, 7, 4, 3), (1, 8, 2, 5, 5)])
def test_1x1_is_matmul(N, C, O, H, W):
    x, w = rnd(N, C, H, W), rnd(O, C, 1, 1)
    got = oracle.conv_forward(Dims(N, C, H, W, O, 1), x, w)
    want = np.einsum("oc,nchw->nohw", w[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- delta kernel (no flip) + padding
@pytest.mark.parametrize("i0,j0", [(0, 0), (0, 2), (2, 1), (1, 1)])
def test_delta_kernel_shifts_input(i0, j0):
    H, W, K, p = 6, 7, 3, 1
    x = rnd(2, 1, H, W)
    w = np.zeros((1, 1, K, K), np.float32)
    w[0, 0, i0, j0] = 1
    got = oracle.conv_forward(Dims(2, 1, H, W, 1, K, 1, p), x, w)
    xp = np.pad(x.astype(np.float64), ((0, 0), (0, 0), (p, p), (p, p)))
    # cross-correlation: y[r,c] = x[r + i0 - p, c + j0 - p]; a flipped kernel would shift the other way
    want = xp[:, :, i0:i0 + H, j0:j0 + W]
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- all-ones closed form
@pytest.mark.parametrize("H,W,K,s,p,g", [(7, 9, 3, 1, 1, 1), (10, 10, 3, 2, 0, 2), (11, 8, 5, 2, 2, 1),
                                         (9, 9, 4, 3, 1, 3)])
def test_all_ones_counts_in_range_taps(H, W, K, s, p, g):
    C, O = 6, 6
    d = Dims(2, C, H, W, O, K, s, p, g)
    got = oracle.conv_forward(d, np.ones((2, C, H, W), np.float32), np.ones((O, C // g, K, K), np.float32))
    ho, wo = (H + 2 * p - K) // s + 1, (W + 2 * p - K) // s + 1
    assert got.shape == (2, O, ho, wo)
    rows = np.array([sum(0 <= r * s + i - p < H for i in range(K)) for r in range(ho)])
    cols = np.array([sum(0 <= c * s + j - p < W for j in range(K)) for c in range(wo)])
    want = (C // g) * np.outer(rows, cols)
    assert np.array_equal(got, np.broadcast_to(want, got.shape))


def test_floor_in_output_size_last_row_unused():
    # H=10, K=3, s=2, p=0 -> Hout = floor(7/2)+1 = 4; input row 9 never read
    d = Dims(1, 1, 10, 10, 1, 3, 2, 0)
    assert oracle.output_dims(d) == (4, 4)
    x = rnd(1, 1, 10, 10)
    w = rnd(1, 1, 3, 3)
    y0 = oracle.conv_forward(d, x, w)
    x2 = x.copy()
    x2[:, :, 9, :] = 99
    x2[:, :, :, 9] = -99
    assert np.array_equal(oracle.conv_forward(d, x2, w), y0)


# ---------------------------------------------------------------- structural identities
def test_pad_equals_explicit_zero_padding():
    N, C, H, W, O, K, s, p = 2, 3, 6, 5, 4, 3, 2, 2
    x, w, b = rnd(N, C, H, W), rnd(O, C, K, K), rnd(O)
    a = oracle.conv_forward(Dims(N, C, H, W, O, K, s, p), x, w, b)
    xp = np.pad(x, ((0, 0), (0, 0), (p, p), (p, p)))
    bb = oracle.conv_forward(Dims(N, C, H + 2 * p, W + 2 * p, O, K, s, 0), xp, w, b)
    assert np.array_equal(a, bb)


def test_stride_equals_subsampled_stride1():
    N, C, H, W, O, K, s, p = 1, 2, 11, 9, 3, 3, 3, 1
    x, w = rnd(N, C, H, W), rnd(O, C, K, K)
    a = oracle.conv_forward(Dims(N, C, H, W, O, K, s, p), x, w)
    full = oracle.conv_forward(Dims(N, C, H, W, O, K, 1, p), x, w)
    assert np.array_equal(a, full[:, :, ::s, ::s][:, :, :a.shape[2], :a.shape[3]])


def test_groups_equal_independent_convs():
    N, C, H, W, O, K, g = 2, 6, 5, 5, 4, 3, 2
    x, w, b = rnd(N, C, H, W), rnd(O, C // g, K, K), rnd(O)
    a = oracle.conv_forward(Dims(N, C, H, W, O, K, 1, 1, g), x, w, b)
    parts = []
    for q in range(g):
        xs = np.ascontiguousarray(x[:, q * 3:(q + 1) * 3])
        parts.append(oracle.conv_forward(Dims(N, 3, H, W, 2, K, 1, 1, 1), xs,
                                         np.ascontiguousarray(w[q * 2:(q + 1) * 2]),
                                         np.ascontiguousarray(b[q * 2:(q + 1) * 2])))
    assert np.array_equal(a, np.concatenate(parts, axis=1))


def test_linearity_and_bias():
    d = Dims(2, 3, 6, 6, 4, 3, 1, 1)
    x1, x2, w = ints(2, 3, 6, 6), ints(2, 3, 6, 6), ints(4, 3, 3, 3)
    b = ints(4)
    f = lambda x, bias=None: oracle.conv_forward(d, x, w, bias)
    assert np.array_equal(f(x1 + 2 * x2), f(x1) + 2 * f(x2))        # small integers: exact
    assert np.array_equal(f(x1, b), f(x1) + b.astype(np.float64)[None, :, None, None])


# ---------------------------------------------------------------- library routines as special cases
def test_against_scipy_correlate2d():
    from scipy.signal import correlate2d
    x, w = rnd(1, 1, 9, 8), rnd(1, 1, 4, 4)
    got = oracle.conv_forward(Dims(1, 1, 9, 8, 1, 4), x, w)[0, 0]
    want = correlate2d(x[0, 0].astype(np.float64), w[0, 0].astype(np.float64), mode="valid")
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


CASES = [
    # N, C, H, W, O, K, s, p, g
    (2, 3, 8, 8, 4, 3, 1, 1, 1),
    (1, 4, 9, 7, 6, 3, 2, 0, 2),
    (2, 6, 11, 11, 3, 5, 2, 2, 3),
    (1, 3, 23, 23, 8, 11, 4, 0, 1),
    (3, 2, 5, 6, 2, 1, 1, 0, 1),
    (1, 2, 7, 7, 2, 2, 3, 1, 1),
    (2, 4, 6, 6, 4, 4, 2, 3, 2),
]


@pytest.mark.parametrize("case", CASES)
def test_against_torch_conv2d_fp64_with_autograd(case):
    """torch's CPU conv2d in fp64 and its autograd are an independent implementation of the
    Caffe-style layer (stride, zero pad, groups, bias) and of its gradients."""
    import torch
    import torch.nn.functional as F
    N, C, H, W, O, K, s, p, g = case
    d = Dims(N, C, H, W, O, K, s, p, g)
    x, w, b = rnd(N, C, H, W), rnd(O, C // g, K, K), rnd(O)
    ho, wo = oracle.output_dims(d)
    dy = rnd(N, O, ho, wo)
    tx = torch.from_numpy(x).double().requires_grad_()
    tw = torch.from_numpy(w).double().requires_grad_()
    tb = torch.from_numpy(b).double().requires_grad_()
    ty = F.conv2d(tx, tw, tb, stride=s, padding=p, groups=g)
    ty.backward(torch.from_numpy(dy).double())
    np.testing.assert_allclose(oracle.conv_forward(d, x, w, b), ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_backward_data(d, w, dy), tx.grad.numpy(), rtol=1e-11, atol=1e-12)
    dw, db = oracle.conv_backward_weights(d, x, dy)
    np.testing.assert_allclose(dw, tw.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- the paper's printed formulas
def paper_vec(a):
    """vec() of a k x k x d (or k x d, or d) slice; any fixed flattening works as long as the data
    and kernel sides use the same one (the printed Z_{5i+j} for a 5x2 slice cannot be right)."""
    return np.asarray(a, np.float64).reshape(-1)


def paper_type1(D, Ks):
    n, k = D.shape[0], Ks[0].shape[0]
    m = n - k + 1
    Dh = np.zeros((m * m, k * k * D.shape[2]))
    for r in range(m):
        for c in range(m):
            Dh[c * m + r, :] = paper_vec(D[r:r + k, c:c + k, :])           # D^[cm+r,:] = vec(D[r:r+k,c:c+k,:])
    out = []
    for Kt in Ks:
        Rh = Dh @ paper_vec(Kt)                                             # K^ = vec(K)
        R = np.zeros((m, m))
        for r in range(m):
            for c in range(m):
                R[r, c] = Rh[c * m + r]                                     # trivial reshape
        out.append(R)
    return out


def paper_type3(D, Ks):
    n, k, dd = D.shape[0], Ks[0].shape[0], D.shape[2]
    m = n - k + 1
    Dh = np.zeros((n * n, dd))
    for r in range(n):
        for c in range(n):
            Dh[c * n + r, :] = paper_vec(D[r, c, :])                        # D^[cn+r,:] = vec(D[r,c,:])
    out = []
    for Kt in Ks:
        Kh = np.zeros((dd, k * k))
        for i in range(k):
            for j in range(k):
                Kh[:, i * k + j] = paper_vec(Kt[i, j, :])                   # K^[:,ik+j] = vec(K[i,j,:])
        Rh = Dh @ Kh
        R = np.zeros((m, m))
        for r in range(m):
            for c in range(m):
                R[r, c] = sum(Rh[(c + j) * n + r + i, i * k + j] for i in range(k) for j in range(k))
        out.append(R)
    return out


def paper_type2(D, Ks):
    n, k, dd = D.shape[0], Ks[0].shape[0], D.shape[2]
    m = n - k + 1
    Dh = np.zeros((n * n, k * dd))
    for r in range(n):
        for c in range(m):                                                  # columns with a full window
            Dh[c * n + r, :] = paper_vec(D[r, c:c + k, :])                  # D^[cn+r,:] = vec(D[r,c:c+k,:])
    out = []
    for Kt in Ks:
        Kh = np.zeros((k * dd, k))
        for i in range(k):
            Kh[:, i] = paper_vec(Kt[i, :, :])                               # K^[:,i] = vec(K[i,:,:])
        Rh = Dh @ Kh
        R = np.zeros((m, m))
        for r in range(m):
            for c in range(m):
                R[r, c] = sum(Rh[c * n + r + j, j] for j in range(k))       # R[r,c] = sum_j R^[cn+r+j, j]
        out.append(R)
    return out


@pytest.mark.parametrize("n,k,dd,o", [(5, 2, 3, 2), (6, 3, 2, 3), (4, 4, 1, 1)])
def test_paper_printed_lowerings_equal_direct(n, k, dd, o):
    """Types 1-3 exactly as printed in Sec. 2.1 (channel-last tensors, rows cm+r / cn+r, the
    printed lifting sums) all reproduce eq. (1), and all agree with the oracle's direct loop."""
    D = ints(n, n, dd)
    Ks = [ints(k, k, dd) for _ in range(o)]
    x = np.ascontiguousarray(D.transpose(2, 0, 1))[None]                    # NCHW
    w = np.ascontiguousarray(np.stack([Kt.transpose(2, 0, 1) for Kt in Ks]))
    direct = oracle.conv_forward(Dims(1, dd, n, n, o, k), x, w)[0]
    for fn in (paper_type1, paper_type2, paper_type3):
        got = fn(D, Ks)
        for t in range(o):
            assert np.array_equal(got[t], direct[t]), fn.__name__


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("lowering", [1, 2, 3])
def test_oracle_lowered_route_equals_direct(case, lowering):
    N, C, H, W, O, K, s, p, g = case
    d = Dims(N, C, H, W, O, K, s, p, g)
    x, w, b = ints(N, C, H, W), ints(O, C // g, K, K), ints(O)
    assert np.array_equal(oracle.conv_forward_lowered(d, lowering, x, w, b), oracle.conv_forward(d, x, w, b))


def test_lowering_is_a_pure_copy_with_positive_zero_padding():
    d = Dims(2, 2, 5, 5, 2, 3, 2, 1, 1)
    x = (np.arange(2 * 2 * 5 * 5, dtype=np.float32) + 1).reshape(2, 2, 5, 5)   # value names its source
    for t in (1, 2, 3):
        dh = oracle.lower_data(d, t, x)
        vals = set(np.unique(dh).tolist())
        assert vals <= set(x.ravel().tolist()) | {0.0}
        assert not np.signbit(dh[dh == 0]).any()
    d1 = oracle.lower_data(d, 1, x)[0]
    # row (n=1, r=1, c=2), col (ci=1, i=2, j=0): x[1,1, 1*2+2-1, 2*2+0-1]
    assert d1[(1 * 3 + 1) * 3 + 2, (1 * 3 + 2) * 3 + 0] == x[1, 1, 3, 3]
    # top-left window starts in the padding: (i=0,*) and (*,j=0) are zero
    assert d1[0, 0] == 0 and d1[0, 4] == x[0, 0, 0, 0]


def test_type2_and_type3_lowered_entries_written_out_by_hand():
    """Sec. 2.1: a Type-2 row holds, for one input row and one output column, the K pixels of the
    horizontal window of every channel; a Type-3 row holds the channels of one input pixel.  The
    entries below are worked out by hand from those two sentences for a grouped, strided, padded
    layer, with x[n,c,h,w] = 1000 n + 100 c + 10 h + w + 1 so that a value names its source."""
    N, C, H, W, O, K, s, p, g = 2, 4, 5, 6, 2, 3, 2, 1, 2
    d = Dims(N, C, H, W, O, K, s, p, g)
    x = np.zeros((N, C, H, W), np.float32)
    for n, c, h, w in itertools.product(range(N), range(C), range(H), range(W)):
        x[n, c, h, w] = 1000 * n + 100 * c + 10 * h + w + 1
    assert oracle.output_dims(d) == (3, 3)                       # (5+2-3)//2+1 = 3, (6+2-3)//2+1 = 3
    Wout, Cg = 3, 2

    d2 = oracle.lower_data(d, 2, x)                              # (groups, N*H*Wout, Cg*K)
    assert d2.shape == (2, N * H * Wout, Cg * K)
    # group 0, image 1, input row h=4, output column c=2: window columns c*s+j-p = 3,4,5
    row = (1 * H + 4) * Wout + 2
    assert d2[0, row].tolist() == [1044, 1045, 1046,             # channel 0: x[1,0,4,3..5]
                                   1144, 1145, 1146]             # channel 1: x[1,1,4,3..5]
    # group 1 (channels 2,3), image 0, row h=0, column c=0: window columns -1,0,1 -> first is padding
    row = (0 * H + 0) * Wout + 0
    assert d2[1, row].tolist() == [0, 201, 202, 0, 301, 302]
    # a middle column, c=1: window columns 1,2,3; every input row appears, also odd ones (h=3)
    row = (0 * H + 3) * Wout + 1
    assert d2[0, row].tolist() == [32, 33, 34, 132, 133, 134]
    # a wrong row order (c-major instead of h-major) would put x[.,.,1,*] here, not x[.,.,0,*]
    assert d2[0, 1].tolist() == [2, 3, 4, 102, 103, 104]          # (h=0, c=1)
    assert d2[0, Wout].tolist() == [0, 11, 12, 0, 111, 112]       # (h=1, c=0)

    d3 = oracle.lower_data(d, 3, x)                              # (groups, N*H*W, Cg)
    assert d3.shape == (2, N * H * W, Cg)
    assert d3[0, (1 * H + 2) * W + 5].tolist() == [1026, 1126]    # pixel (n=1,h=2,w=5), channels 0,1
    assert d3[1, (0 * H + 4) * W + 0].tolist() == [241, 341]      # pixel (n=0,h=4,w=0), channels 2,3
    assert d3[0, 1].tolist() == [2, 102]                          # (h=0,w=1): w runs fastest
    assert d3[0, W].tolist() == [11, 111]                         # (h=1,w=0)
    # Type 3 is a pure transpose of x: every entry, rebuilt without the oracle
    want3 = x.reshape(N, g, Cg, H * W).transpose(1, 0, 3, 2).reshape(g, N * H * W, Cg)
    assert np.array_equal(d3, want3)
    # Type 2, every entry, from the sentence above with explicit zero padding of the columns
    xp = np.pad(x, ((0, 0), (0, 0), (0, 0), (p, p)))
    want2 = np.zeros((g, N * H * Wout, Cg * K), np.float32)
    for q, n, h, c, ci, j in itertools.product(range(g), range(N), range(H), range(Wout), range(Cg), range(K)):
        want2[q, (n * H + h) * Wout + c, ci * K + j] = xp[n, q * Cg + ci, h, c * s + j]
    assert np.array_equal(d2, want2)


# ---------------------------------------------------------------- shape laws
def test_shape_laws_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "caffenet_shapes.txt")
    seen = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        C, H, O, K, s, p, g, hout = map(int, f[1:9])
        want = list(map(int, f[9:15]))
        d = Dims(1, C, H, H, O, K, s, p, g)
        assert oracle.output_dims(d) == (hout, hout)
        got = []
        for t in (1, 2, 3):
            rows, cols, rcols = oracle.lowered_shape(d, t)
            got += [rows, cols]
            assert rcols == (O // g) * K ** (t - 1)
        assert got == want, f[0]
        seen += 1
    assert seen == 5


def test_m_equals_n_minus_k_plus_1():
    for n, k in itertools.product((5, 13, 27), (1, 3, 5)):
        assert oracle.output_dims(Dims(1, 1, n, n, 1, k)) == (n - k + 1, n - k + 1)


def test_lowered_matrix_grows_linearly_with_batch():
    # Sec. 2.2: a batch of b images makes the lowered matrix b times larger
    for t in (1, 2, 3):
        r1 = oracle.lowered_shape(Dims(1, 4, 9, 9, 4, 3, 1, 1), t)
        r8 = oracle.lowered_shape(Dims(8, 4, 9, 9, 4, 3, 1, 1), t)
        assert r8[0] == 8 * r1[0] and r8[1:] == r1[1:]


# ---------------------------------------------------------------- backward passes
@pytest.mark.parametrize("case", CASES)
def test_adjoint_identities(case):
    N, C, H, W, O, K, s, p, g = case
    d = Dims(N, C, H, W, O, K, s, p, g)
    x, w = ints(N, C, H, W), ints(O, C // g, K, K)
    ho, wo = oracle.output_dims(d)
    dy = ints(N, O, ho, wo)
    lhs = float((dy.astype(np.float64) * oracle.conv_forward(d, x, w)).sum())
    assert lhs == float((oracle.conv_backward_data(d, w, dy) * x).sum())
    dw, db = oracle.conv_backward_weights(d, x, dy)
    assert lhs == float((dw * w).sum())
    assert np.array_equal(db, dy.astype(np.float64).sum(axis=(0, 2, 3)))


def test_finite_differences_of_inner_product():
    """L(x,w,b) = <dy, y> is linear in each argument, so a central difference with a dyadic step on
    dyadic data is exact: every gradient entry must match with zero error."""
    d = Dims(2, 2, 5, 4, 2, 3, 2, 1, 1)
    x, w, b = ints(2, 2, 5, 4), ints(2, 2, 3, 3), ints(2)
    ho, wo = oracle.output_dims(d)
    dy = ints(2, 2, ho, wo).astype(np.float32)
    L = lambda x_, w_, b_: float((dy.astype(np.float64) * oracle.conv_forward(d, x_, w_, b_)).sum())
    dx = oracle.conv_backward_data(d, w, dy)
    dw, db = oracle.conv_backward_weights(d, x, dy)
    h = np.float32(0.5)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        assert (L(xp, w, b) - L(xm, w, b)) / (2 * float(h)) == dx[idx]
    for idx in np.ndindex(*w.shape):
        wp, wm = w.copy(), w.copy()
        wp[idx] += h
        wm[idx] -= h
        assert (L(x, wp, b) - L(x, wm, b)) / (2 * float(h)) == dw[idx]
    for o in range(2):
        bp, bm = b.copy(), b.copy()
        bp[o] += h
        bm[o] -= h
        assert (L(x, w, bp) - L(x, w, bm)) / (2 * float(h)) == db[o]


# ---------------------------------------------------------------- sampled entry points == full ones
def test_sampled_entry_points_match_full():
    d = Dims(2, 4, 7, 6, 4, 3, 2, 1, 2)
    x, w, b = rnd(2, 4, 7, 6), rnd(4, 2, 3, 3), rnd(4)
    ho, wo = oracle.output_dims(d)
    dy = rnd(2, 4, ho, wo)
    y = oracle.conv_forward(d, x, w, b)
    idx = np.arange(y.size)[::3]
    assert np.array_equal(oracle.conv_forward_at(d, x, w, b, idx), y.ravel()[idx])
    dx = oracle.conv_backward_data(d, w, dy)
    idx = np.arange(dx.size)[::5]
    assert np.array_equal(oracle.conv_backward_data_at(d, w, dy, idx), dx.ravel()[idx])
    dw, _ = oracle.conv_backward_weights(d, x, dy)
    idx = np.arange(dw.size)[::2]
    assert np.array_equal(oracle.conv_backward_weights_at(d, x, dy, idx), dw.ravel()[idx])
    with pytest.raises(ValueError):
        oracle.conv_forward_at(d, x, w, b, np.array([y.size]))


def test_rejects_bad_shapes():
    with pytest.raises(ValueError):
        oracle.output_dims(Dims(1, 3, 4, 4, 2, 3, 1, 0, 2))      # C % groups != 0
    with pytest.raises(ValueError):
        oracle.output_dims(Dims(1, 1, 2, 2, 1, 3))               # kernel larger than padded input


# ---------------------------------------------------------------- ReLU and max pooling (the layers between the convolutions)
def test_relu_by_hand():
    x = np.array([-2.0, -0.0, 0.0, 0.5, 3.0], np.float32)
    dy = np.array([10.0, 20.0, 30.0, 40.0, 50.0], np.float32)
    assert oracle.relu_forward(x).tolist() == [0.0, 0.0, 0.0, 0.5, 3.0]
    assert oracle.relu_backward(x, dy).tolist() == [0.0, 0.0, 0.0, 40.0, 50.0]


def test_maxpool_output_size_law():
    P = oracle.PoolDims
    assert oracle.pool_output_dims(P(1, 1, 55, 55, 3, 2)) == (27, 27)      # CaffeNet pool1
    assert oracle.pool_output_dims(P(1, 1, 27, 27, 3, 2)) == (13, 13)      # pool2
    assert oracle.pool_output_dims(P(1, 1, 13, 13, 3, 2)) == (6, 6)        # pool5
    assert oracle.pool_output_dims(P(1, 1, 6, 7, 3, 2)) == (3, 3)          # ceil: (6-3)/2 = 1.5 -> 2, +1
    assert oracle.pool_output_dims(P(1, 1, 4, 4, 2, 2, 1)) == (3, 3)       # padded: windows start at -1, 1, 3
    assert oracle.pool_output_dims(P(1, 1, 5, 5, 3, 1)) == (3, 3)


def test_maxpool_by_hand_with_overlapping_windows_and_ceil_clipping():
    # 4 x 5 plane, 3 x 3 windows, stride 2: Hout = ceil(1/2)+1 = 2, Wout = ceil(2/2)+1 = 2;
    # the second row / column of windows is clipped at the border
    x = np.array([[1, 2, 3, 4, 5],
                  [6, 9, 8, 7, 0],
                  [3, 3, 3, 3, 3],
                  [9, 1, 1, 1, 2]], np.float32).reshape(1, 1, 4, 5)
    d = oracle.PoolDims(1, 1, 4, 5, 3, 2)
    y, am = oracle.maxpool_forward(d, x)
    # windows: rows 0-2 x cols 0-2 -> 9 at (1,1); rows 0-2 x cols 2-4 -> 8 at (1,2);
    #          rows 2-3 x cols 0-2 -> 9 at (3,0); rows 2-3 x cols 2-4 -> 3, first at (2,2)
    assert y.reshape(2, 2).tolist() == [[9, 8], [9, 3]]
    assert am.reshape(2, 2).tolist() == [[1 * 5 + 1, 1 * 5 + 2], [3 * 5 + 0, 2 * 5 + 2]]
    dy = np.array([[1, 10], [100, 1000]], np.float32).reshape(1, 1, 2, 2)
    want = np.zeros((4, 5), np.float32)
    want[1, 1], want[1, 2], want[3, 0], want[2, 2] = 1, 10, 100, 1000
    assert np.array_equal(oracle.maxpool_backward(d, dy, am)[0, 0], want)


def test_maxpool_tie_goes_to_first_in_scan_order_and_overlaps_add():
    d = oracle.PoolDims(1, 1, 5, 5, 3, 2)                       # windows start at 0, 2: pixel (2,2) is in all four
    x = np.zeros((1, 1, 5, 5), np.float32)
    y, am = oracle.maxpool_forward(d, x)
    assert am.reshape(2, 2).tolist() == [[0, 2], [10, 12]]      # top-left pixel of every window
    x[0, 0, 2, 2] = 1.0
    y, am = oracle.maxpool_forward(d, x)
    assert (am == 12).all() and (y == 1).all()
    dx = oracle.maxpool_backward(d, np.array([1, 2, 4, 8], np.float32).reshape(1, 1, 2, 2), am)
    assert dx[0, 0, 2, 2] == 15 and dx.sum() == 15


@pytest.mark.parametrize("N,C,H,W,K,s,p", [(2, 3, 55, 55, 3, 2, 0), (1, 4, 27, 27, 3, 2, 0), (2, 2, 9, 11, 2, 2, 0),
                                           (1, 3, 10, 7, 3, 1, 1), (1, 2, 8, 8, 3, 2, 1)])
def test_maxpool_against_torch_cpu_on_tie_free_data(N, C, H, W, K, s, p):
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(77)
    x = rng.permutation(N * C * H * W).astype(np.float32).reshape(N, C, H, W)    # all values distinct
    d = oracle.PoolDims(N, C, H, W, K, s, p)
    y, am = oracle.maxpool_forward(d, x)
    tx = torch.from_numpy(x).requires_grad_()
    ty, tidx = F.max_pool2d(tx, K, s, p, ceil_mode=True, return_indices=True)
    assert tuple(ty.shape) == y.shape
    assert np.array_equal(y, ty.detach().numpy())
    assert np.array_equal(am, tidx.numpy().astype(np.int32))
    dy = rng.standard_normal(y.shape).astype(np.float32)
    ty.backward(torch.from_numpy(dy))
    np.testing.assert_allclose(oracle.maxpool_backward(d, dy, am), tx.grad.numpy(), rtol=1e-6, atol=1e-6)


def test_relu_against_torch_cpu():
    import torch
    x = rnd(3, 4, 5, 6)
    dy = rnd(3, 4, 5, 6)
    tx = torch.from_numpy(x).requires_grad_()
    ty = torch.relu(tx)
    ty.backward(torch.from_numpy(dy))
    assert np.array_equal(oracle.relu_forward(x), ty.detach().numpy())
    assert np.array_equal(oracle.relu_backward(x, dy), tx.grad.numpy())


# ------------------------------------------------------------------ local response normalisation
def test_lrn_by_hand_three_channels():
    """size 3, alpha 3, beta 1, k 1 on one pixel with channels (1, 2, 3): the sums of squares over
    the windows are 1+4, 1+4+9, 4+9, so scale = 1 + (3/3)*(5, 14, 13) = (6, 15, 14) and y = x/scale."""
    d = oracle.LrnDims(1, 3, 1, 1, size=3, alpha=3.0, beta=1.0, k=1.0)
    x = np.array([1.0, 2.0, 3.0], np.float32).reshape(1, 3, 1, 1)
    y = oracle.lrn_forward(d, x).ravel()
    np.testing.assert_allclose(y, [1 / 6, 2 / 15, 3 / 14], rtol=1e-7)
    # backward by hand for dy = (1, 0, 0): dx0 = 1/6 - 2*x0*(x0/36) = 1/6 - 1/18, dx1 = -2*x1*(x0/36),
    # dx2 = 0 (channel 0 is outside the window of channel 2)
    dx = oracle.lrn_backward(d, x, np.array([1.0, 0.0, 0.0], np.float32).reshape(1, 3, 1, 1)).ravel()
    np.testing.assert_allclose(dx, [1 / 6 - 2 * 1 * (1 / 36), -2 * 2 * (1 / 36), 0.0], rtol=1e-6, atol=1e-9)


def test_lrn_constant_tensor_closed_form_and_edge_channels():
    """On a constant tensor v the window of an inner channel holds `size` squares, that of an edge
    channel fewer (zero padding across channels): y = v * (k + alpha/size * m * v^2)^-beta."""
    d = oracle.LrnDims(2, 7, 3, 2, size=5, alpha=0.5, beta=0.75, k=2.0)
    v = 1.5
    y = oracle.lrn_forward(d, np.full((2, 7, 3, 2), v, np.float32))
    counts = [3, 4, 5, 5, 5, 4, 3]
    for c, m in enumerate(counts):
        want = v * (2.0 + 0.5 / 5 * m * v * v) ** -0.75
        np.testing.assert_allclose(y[:, c], want, rtol=1e-6)


def test_lrn_size_one_is_a_pointwise_power_law():
    d = oracle.LrnDims(1, 4, 2, 2, size=1, alpha=2.0, beta=0.5, k=1.0)
    x = np.random.default_rng(3).standard_normal((1, 4, 2, 2)).astype(np.float32)
    want = x.astype(np.float64) * (1.0 + 2.0 * x.astype(np.float64) ** 2) ** -0.5
    np.testing.assert_allclose(oracle.lrn_forward(d, x), want, rtol=1e-6)


@pytest.mark.parametrize("N,C,H,W,size", [(2, 9, 4, 3, 5), (1, 5, 2, 2, 3), (2, 3, 3, 3, 5)])
def test_lrn_against_torch_cpu(N, C, H, W, size):
    import torch
    d = oracle.LrnDims(N, C, H, W, size=size, alpha=0.3, beta=0.75, k=1.0)
    rng = np.random.default_rng(5)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32) * 2
    dy = rng.standard_normal((N, C, H, W)).astype(np.float32)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = torch.nn.functional.local_response_norm(tx, size, alpha=0.3, beta=0.75, k=1.0)
    ty.backward(torch.tensor(dy, dtype=torch.float64))
    np.testing.assert_allclose(oracle.lrn_forward(d, x), ty.detach().numpy(), rtol=2e-6, atol=1e-7)
    np.testing.assert_allclose(oracle.lrn_backward(d, x, dy), tx.grad.numpy(), rtol=2e-5, atol=1e-6)


def test_lrn_backward_is_the_derivative_of_forward():
    """Central differences in fp64 on the oracle's own forward formula written out in numpy."""
    d = oracle.LrnDims(1, 6, 1, 2, size=5, alpha=0.8, beta=0.75, k=1.0)
    rng = np.random.default_rng(8)
    x = rng.standard_normal((1, 6, 1, 2))
    dy = rng.standard_normal((1, 6, 1, 2))

    def f(xx):
        out = np.zeros_like(xx)
        for c in range(6):
            lo, hi = max(0, c - 2), min(6, c + 3)
            scale = 1.0 + 0.8 / 5 * (xx[:, lo:hi] ** 2).sum(axis=1)
            out[:, c] = xx[:, c] * scale ** -0.75
        return out
    want = np.zeros_like(x)
    h = 1e-6
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        want[idx] = ((f(xp) - f(xm)) * dy).sum() / (2 * h)
    got = oracle.lrn_backward(d, x.astype(np.float32), dy.astype(np.float32))
    np.testing.assert_allclose(got, want, rtol=2e-4, atol=2e-6)


# ---- dropout and the softmax loss ------------------------------------------------------------

def test_dropout_identity_zero_and_torch_cpu():
    """mask of ones with scale 1 is the identity, a zero mask gives zeros; torch's CPU dropout
    fixes the scale 1/(1-p): its output names the mask it drew, and the oracle on that mask must
    give torch's output."""
    import torch
    rng = np.random.default_rng(3)
    x = rng.standard_normal(1000).astype(np.float32) + 3.0          # no zeros in x
    ones = np.ones(1000, np.uint8)
    assert np.array_equal(oracle.dropout(x, ones, 1.0), x)
    assert np.array_equal(oracle.dropout(x, np.zeros(1000, np.uint8), 2.0), np.zeros(1000, np.float32))
    torch.manual_seed(5)
    for p in (0.5, 0.25):
        ty = torch.nn.functional.dropout(torch.from_numpy(x).double(), p=p, training=True).numpy()
        mask = (ty != 0).astype(np.uint8)
        assert 0 < mask.sum() < 1000
        np.testing.assert_allclose(oracle.dropout(x, mask, 1.0 / (1.0 - p)), ty, rtol=1e-7)


def test_dropout_backward_is_the_adjoint():
    """<dropout(x), dy> == <x, dropout(dy)> exactly on small dyadic values."""
    rng = np.random.default_rng(4)
    x = rng.integers(-8, 9, 500).astype(np.float32) / 4
    dy = rng.integers(-8, 9, 500).astype(np.float32) / 8
    mask = (rng.random(500) < 0.5).astype(np.uint8)
    lhs = (oracle.dropout(x, mask, 2.0).astype(np.float64) * dy).sum()
    rhs = (x.astype(np.float64) * oracle.dropout(dy, mask, 2.0)).sum()
    assert lhs == rhs


def test_softmax_loss_hand_cases():
    # two classes, scores (0, ln 3): probabilities 1/4 and 3/4
    x = np.array([[0.0, np.log(3.0)]], np.float32)
    prob, loss = oracle.softmax_loss_forward(x, [1])
    np.testing.assert_allclose(prob, [[0.25, 0.75]], rtol=1e-6)
    np.testing.assert_allclose(loss, -np.log(0.75), rtol=1e-6)
    prob, loss = oracle.softmax_loss_forward(x, [0])
    np.testing.assert_allclose(loss, np.log(4.0), rtol=1e-6)
    np.testing.assert_allclose(oracle.softmax_loss_backward(prob, [0]), [[-0.75, 0.75]], rtol=1e-6)
    # uniform scores: prob = 1/C whatever the level, loss = log C; the mean runs over the images
    for C, level in ((10, 0.0), (1000, 50.0), (7, -200.0)):
        x = np.full((3, C), level, np.float32)
        prob, loss = oracle.softmax_loss_forward(x, [0, C - 1, C // 2])
        np.testing.assert_allclose(prob, 1.0 / C, rtol=1e-6)
        np.testing.assert_allclose(loss, np.log(C), rtol=1e-9)
    # one certain image and one uniform one: the loss is their mean
    x = np.array([[100.0, 0.0, 0.0, 0.0], [1.0, 1.0, 1.0, 1.0]], np.float32)
    _, loss = oracle.softmax_loss_forward(x, [0, 2])
    np.testing.assert_allclose(loss, 0.5 * np.log(4.0), rtol=1e-9)
    with pytest.raises(ValueError):
        oracle.softmax_loss_forward(x, [0, 4])                       # label out of range


def test_softmax_shift_invariance_and_rows_sum_to_one():
    rng = np.random.default_rng(6)
    x = (rng.integers(-128, 129, (5, 33)) / 8.0).astype(np.float32)     # multiples of 1/8
    label = rng.integers(0, 33, 5)
    p0, l0 = oracle.softmax_loss_forward(x, label)
    p1, l1 = oracle.softmax_loss_forward(x + np.float32(64.0), label)    # exact shift in fp32
    np.testing.assert_allclose(p0, p1, rtol=1e-6)
    np.testing.assert_allclose(l0, l1, rtol=1e-6)
    np.testing.assert_allclose(p0.astype(np.float64).sum(axis=1), 1.0, rtol=1e-6)
    # scores far apart: the losing probabilities underflow, the loss stays finite
    x = np.array([[0.0, 200.0]], np.float32)
    prob, loss = oracle.softmax_loss_forward(x, [0])
    assert prob[0, 0] == 0.0 and np.isfinite(loss)
    np.testing.assert_allclose(loss, 200.0, rtol=1e-9)


@pytest.mark.parametrize("N,C", [(4, 10), (7, 1000), (1, 3)])
def test_softmax_loss_against_torch_cpu(N, C):
    import torch
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((N, C)) * 3).astype(np.float32)
    label = rng.integers(0, C, N)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tl = torch.nn.functional.cross_entropy(tx, torch.from_numpy(label), reduction="mean")
    tl.backward()
    prob, loss = oracle.softmax_loss_forward(x, label)
    np.testing.assert_allclose(prob, torch.softmax(tx.detach(), dim=1).numpy(), rtol=1e-6, atol=1e-12)
    np.testing.assert_allclose(loss, tl.item(), rtol=1e-9)
    np.testing.assert_allclose(oracle.softmax_loss_backward(prob, label), tx.grad.numpy(), rtol=1e-5, atol=1e-8)


def test_softmax_loss_backward_is_the_derivative_of_the_loss():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((3, 6)).astype(np.float32)
    label = [5, 0, 2]
    prob, _ = oracle.softmax_loss_forward(x, label)
    got = oracle.softmax_loss_backward(prob, label)
    h = np.float32(2.0 ** -7)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd = (oracle.softmax_loss_forward(xp, label)[1] - oracle.softmax_loss_forward(xm, label)[1]) / (2.0 * float(h))
        np.testing.assert_allclose(got[idx], fd, rtol=2e-3, atol=2e-5)
