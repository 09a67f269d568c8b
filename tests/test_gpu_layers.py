"""GPU parity of the ReLU, max-pooling and local-response-normalisation entry points against the
CPU oracle: values, argmax indices and ReLU gradients bit-exact; pooling gradients (a sum of at
most four fp32 terms against the oracle's fp64 sum) within 1e-6; normalisation (fp32 powf against
fp64) within 1e-5 of the largest value."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_1504_04343_amd import binding
    return binding


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("n", [1, 3, 4, 1023, 4096, 1 << 20, (1 << 20) + 5])
def test_relu_forward_backward_bit_exact(B, n):
    import torch
    rng = np.random.default_rng(n)
    x = rng.standard_normal(n).astype(np.float32)
    x[::7] = 0.0
    x[1::11] = -0.0
    dy = rng.standard_normal(n).astype(np.float32)
    tx, tdy = dev(x), dev(dy)
    y = torch.full_like(tx, float("nan"))
    dx = torch.full_like(tx, float("nan"))
    B.cct_relu_forward(tx, y)
    B.cct_relu_backward(tx, tdy, dx)
    torch.cuda.synchronize()
    assert y.cpu().numpy().tobytes() == oracle.relu_forward(x).tobytes()
    assert dx.cpu().numpy().tobytes() == oracle.relu_backward(x, dy).tobytes()
    # the mask may be taken from the output instead of the input, and both calls work in place
    B.cct_relu_backward(y, tdy, tdy)
    B.cct_relu_forward(tx, tx)
    torch.cuda.synchronize()
    assert tdy.cpu().numpy().tobytes() == oracle.relu_backward(x, dy).tobytes()
    assert tx.cpu().numpy().tobytes() == oracle.relu_forward(x).tobytes()


def test_relu_on_a_misaligned_view(B):
    import torch
    x = np.random.default_rng(5).standard_normal(1001).astype(np.float32)
    base = dev(np.concatenate([[0.0], x]).astype(np.float32))
    tx = base[1:]                                   # 4 bytes past a 16-byte boundary
    y = torch.empty(1001, device="cuda")
    B.cct_relu_forward(tx, y)
    torch.cuda.synchronize()
    assert y.cpu().numpy().tobytes() == oracle.relu_forward(x).tobytes()


POOLS = [
    # N, C, H, W, K, s, p
    (2, 3, 55, 55, 3, 2, 0),      # CaffeNet pool1 geometry
    (3, 5, 27, 27, 3, 2, 0),      # pool2
    (2, 4, 13, 13, 3, 2, 0),      # pool5
    (1, 2, 6, 7, 3, 2, 0),        # ceil: clipped last windows
    (2, 3, 9, 11, 2, 2, 0),
    (1, 3, 10, 7, 3, 1, 1),       # padded, overlapping
    (2, 2, 8, 8, 3, 2, 1),
    (1, 1, 1, 1, 1, 1, 0),
    (1, 2, 5, 4, 5, 3, 2),
    (5, 7, 13, 13, 3, 2, 0),      # 35 planes: the backward pass takes 24 per workgroup, then 11
    (1, 2, 300, 290, 3, 2, 0),    # planes too large for the backward pass's LDS staging
]


@pytest.mark.parametrize("case", POOLS)
@pytest.mark.parametrize("relu_input", [False, True], ids=["normal", "relu_ties"])
def test_maxpool_forward_backward(B, case, relu_input):
    import torch
    N, C, H, W, K, s, p = case
    rng = np.random.default_rng(sum(case))
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    if relu_input:
        x = np.maximum(x, 0)                        # about half zeros: windows with tied maxima
    od = oracle.PoolDims(N, C, H, W, K, s, p)
    d = B.make_pool_desc(N, C, H, W, K, s, p)
    assert B.cct_pool_output_dims(d) == oracle.pool_output_dims(od)
    ho, wo = B.cct_pool_output_dims(d)
    y = torch.full((N, C, ho, wo), float("nan"), device="cuda")
    am = torch.full((N, C, ho, wo), -7, dtype=torch.int32, device="cuda")
    B.cct_maxpool_forward(d, dev(x), y, am)
    y2 = torch.full_like(y, float("nan"))
    B.cct_maxpool_forward(d, dev(x), y2)            # argmax is optional
    want_y, want_am = oracle.maxpool_forward(od, x)
    torch.cuda.synchronize()
    assert y.cpu().numpy().tobytes() == want_y.tobytes()
    assert y2.cpu().numpy().tobytes() == want_y.tobytes()
    assert np.array_equal(am.cpu().numpy(), want_am)
    dy = rng.standard_normal((N, C, ho, wo)).astype(np.float32)
    dx = torch.full((N, C, H, W), float("nan"), device="cuda")
    B.cct_maxpool_backward(d, dev(dy), am, dx)
    torch.cuda.synchronize()
    want_dx = oracle.maxpool_backward(od, dy, want_am)
    got = dx.cpu().numpy()
    assert np.isfinite(got).all()
    assert np.abs(got - want_dx).max() <= 1e-6 * max(1.0, np.abs(want_dx).max())


@pytest.mark.parametrize("name,C,H", [("pool1", 96, 55), ("pool2", 256, 27)])
def test_maxpool_full_size_batch_256(B, name, C, H):
    """CaffeNet's pool1 / pool2 at batch 256 on post-ReLU data, every element."""
    import torch
    print("full-size", name, flush=True)
    N = 256
    rng = np.random.default_rng(3)
    x = np.maximum(rng.standard_normal((N, C, H, H), dtype=np.float32), np.float32(0))
    od = oracle.PoolDims(N, C, H, H, 3, 2, 0)
    d = B.make_pool_desc(N, C, H, H, 3, 2, 0)
    ho, wo = B.cct_pool_output_dims(d)
    y = torch.empty((N, C, ho, wo), device="cuda")
    am = torch.empty((N, C, ho, wo), dtype=torch.int32, device="cuda")
    tx = dev(x)
    B.cct_maxpool_forward(d, tx, y, am)
    want_y, want_am = oracle.maxpool_forward(od, x)
    torch.cuda.synchronize()
    assert y.cpu().numpy().tobytes() == want_y.tobytes()
    assert np.array_equal(am.cpu().numpy(), want_am)
    dy = rng.standard_normal((N, C, ho, wo), dtype=np.float32)
    dx = torch.empty_like(tx)
    B.cct_maxpool_backward(d, dev(dy), am, dx)
    torch.cuda.synchronize()
    want_dx = oracle.maxpool_backward(od, dy, want_am)
    assert np.abs(dx.cpu().numpy() - want_dx).max() <= 1e-6 * np.abs(want_dx).max()


def test_pool_rejects_bad_descriptors(B):
    for bad in (dict(N=0), dict(K=0), dict(stride=0), dict(pad=3), dict(pad=-1), dict(H=0)):
        kw = dict(N=1, C=1, H=5, W=5, K=3, stride=2, pad=0)
        kw.update(bad)
        with pytest.raises(B.CctError) as e:
            B.cct_pool_output_dims(B.make_pool_desc(**kw))
        assert e.value.code == B.EINVAL


# ------------------------------------------------------------------ local response normalisation
LRN_CASES = [
    # N, C, H, W, size, alpha, beta, k
    (2, 9, 5, 7, 5, 0.3, 0.75, 1.0),          # strong normalisation, odd sizes
    (3, 3, 4, 4, 5, 1e-2, 0.75, 2.0),         # fewer channels than the window
    (1, 1, 3, 3, 3, 0.5, 0.5, 1.0),           # one channel
    (2, 16, 6, 5, 1, 2.0, 0.5, 1.0),          # size 1: pointwise
    (2, 20, 3, 3, 9, 0.1, 1.25, 1.0),         # widest compiled window
    (1, 40, 13, 13, 7, 1e-3, 0.75, 1.0),
]


@pytest.mark.parametrize("case", LRN_CASES, ids=["c%d_s%d" % (c[1], c[4]) for c in LRN_CASES])
def test_lrn_forward_backward(B, case):
    """fp32 powf against the fp64 oracle: 1e-5 of the largest value (the bar of the fp32 path is 1e-4)."""
    import torch
    N, C, H, W, size, alpha, beta, k = case
    rng = np.random.default_rng(size * 100 + C)
    x = (rng.standard_normal((N, C, H, W)) * 3).astype(np.float32)
    dy = rng.standard_normal((N, C, H, W)).astype(np.float32)
    od = oracle.LrnDims(N, C, H, W, size, alpha, beta, k)
    d = B.make_lrn_desc(N, C, H, W, size, alpha, beta, k)
    tx, tdy = dev(x), dev(dy)
    y = torch.full_like(tx, float("nan"))
    dx = torch.full_like(tx, float("nan"))
    B.cct_lrn_forward(d, tx, y)
    B.cct_lrn_backward(d, tx, tdy, dx)
    torch.cuda.synchronize()
    want_y, want_dx = oracle.lrn_forward(od, x), oracle.lrn_backward(od, x, dy)
    assert np.abs(y.cpu().numpy() - want_y).max() <= 1e-5 * np.abs(want_y).max()
    assert np.abs(dx.cpu().numpy() - want_dx).max() <= 1e-5 * np.abs(want_dx).max()


@pytest.mark.parametrize("name,C,H", [("norm1", 96, 27), ("norm2", 256, 13)])
def test_lrn_caffenet_layers_batch_256(B, name, C, H):
    """CaffeNet's two normalisation layers at batch 256 on post-ReLU, post-pooling like data,
    every element against the oracle."""
    import torch
    N = 256
    rng = np.random.default_rng(C)
    x = np.maximum(rng.standard_normal((N, C, H, H)) * 20, 0).astype(np.float32)   # activations of tens
    dy = rng.standard_normal((N, C, H, H)).astype(np.float32)
    od = oracle.LrnDims(N, C, H, H)
    d = B.make_lrn_desc(N, C, H, H)
    tx, tdy = dev(x), dev(dy)
    y, dx = torch.empty_like(tx), torch.empty_like(tx)
    B.cct_lrn_forward(d, tx, y)
    B.cct_lrn_backward(d, tx, tdy, dx)
    torch.cuda.synchronize()
    want_y, want_dx = oracle.lrn_forward(od, x), oracle.lrn_backward(od, x, dy)
    assert np.abs(y.cpu().numpy() - want_y).max() <= 1e-5 * np.abs(want_y).max(), name
    assert np.abs(dx.cpu().numpy() - want_dx).max() <= 1e-5 * np.abs(want_dx).max(), name


def test_lrn_rejects_bad_descriptors(B):
    import torch
    t = torch.zeros((1, 4, 2, 2), device="cuda")
    for bad, code in ((dict(size=4), B.EINVAL), (dict(size=11), B.EUNSUPPORTED), (dict(k=0.0), B.EINVAL),
                      (dict(alpha=-1.0), B.EINVAL)):
        kw = dict(size=5, alpha=1e-4, beta=0.75, k=1.0)
        kw.update(bad)
        with pytest.raises(B.CctError) as e:
            B.cct_lrn_forward(B.make_lrn_desc(1, 4, 2, 2, **kw), t, torch.empty_like(t))
        assert e.value.code == code, bad


@pytest.mark.parametrize("n,ratio", [(1, 0.5), (1001, 0.5), (256 * 4096, 0.5), (70001, 0.25)])
def test_dropout_forward_backward_bit_exact(B, n, ratio):
    """One fp32 product per kept element: the oracle's fp64 product with the same fp32 scale rounds
    to the same bits."""
    import torch
    rng = np.random.default_rng(n)
    x = rng.standard_normal(n).astype(np.float32)
    dy = rng.standard_normal(n).astype(np.float32)
    mask = (rng.random(n) >= ratio).astype(np.uint8)
    scale = float(np.float32(1.0 / (1.0 - ratio)))
    tm = torch.from_numpy(mask).cuda()
    y = torch.full((n,), float("nan"), device="cuda")
    dx = torch.full((n,), float("nan"), device="cuda")
    B.cct_dropout_forward(dev(x), tm, scale, y)
    B.cct_dropout_backward(dev(dy), tm, scale, dx)
    torch.cuda.synchronize()
    assert y.cpu().numpy().tobytes() == oracle.dropout(x, mask, scale).tobytes()
    assert dx.cpu().numpy().tobytes() == oracle.dropout(dy, mask, scale).tobytes()
    with pytest.raises(B.CctError) as e:
        B.cct_dropout_forward(dev(x), tm, 0.0, y)
    assert e.value.code == B.EINVAL


@pytest.mark.parametrize("N,C,spread", [(256, 1000, 3.0), (7, 10, 1.0), (1, 1, 1.0), (33, 300, 30.0),
                                        (5, 2049, 0.1)])
def test_softmax_loss_forward_backward(B, N, C, spread):
    """fp32 expf / logf against the fp64 oracle; the backward pass on the GPU's own fp32 prob is one
    subtraction and one product per element."""
    import torch
    rng = np.random.default_rng(N * 7 + C)
    x = (rng.standard_normal((N, C)) * spread).astype(np.float32)
    label = rng.integers(0, C, N).astype(np.int32)
    tx, tl = dev(x), torch.from_numpy(label).cuda()
    prob = torch.full((N, C), float("nan"), device="cuda")
    il = torch.full((N,), float("nan"), device="cuda")
    loss = torch.full((1,), float("nan"), device="cuda")
    B.cct_softmax_loss_forward(tx, tl, prob, il, loss)
    dx = torch.full((N, C), float("nan"), device="cuda")
    B.cct_softmax_loss_backward(prob, tl, dx)
    torch.cuda.synchronize()
    want_prob, want_loss = oracle.softmax_loss_forward(x, label)
    got_prob = prob.cpu().numpy()
    assert np.abs(got_prob - want_prob).max() <= 1e-5 * want_prob.max()
    assert abs(float(loss.item()) - want_loss) <= 1e-5 * max(abs(want_loss), 1.0)
    _, one = oracle.softmax_loss_forward(x[:1], label[:1])
    assert abs(float(il[0].item()) - one) <= 1e-5 * max(abs(one), 1.0)
    want_dx = oracle.softmax_loss_backward(got_prob, label)          # from the prob the GPU consumed
    assert np.abs(dx.cpu().numpy() - want_dx).max() <= 1e-6 * np.abs(want_dx).max()
    # same bits on a second run (fixed-order sums)
    prob2, il2, loss2 = torch.empty_like(prob), torch.empty_like(il), torch.empty_like(loss)
    B.cct_softmax_loss_forward(tx, tl, prob2, il2, loss2)
    torch.cuda.synchronize()
    assert torch.equal(prob, prob2) and torch.equal(loss, loss2)


def test_softmax_loss_label_out_of_range_gives_nan_not_a_fault(B):
    import torch
    x = torch.zeros((3, 5), device="cuda")
    label = torch.tensor([0, 7, -1], dtype=torch.int32, device="cuda")
    prob, il, loss = torch.empty_like(x), torch.empty(3, device="cuda"), torch.empty(1, device="cuda")
    B.cct_softmax_loss_forward(x, label, prob, il, loss)
    dx = torch.empty_like(x)
    B.cct_softmax_loss_backward(prob, label, dx)
    torch.cuda.synchronize()
    assert bool(torch.isnan(il[1])) and bool(torch.isnan(il[2])) and bool(torch.isnan(loss[0]))
    assert abs(float(il[0]) - np.log(5.0)) < 1e-5
    assert torch.allclose(dx[1], torch.full((5,), 0.2 / 3, device="cuda"))
