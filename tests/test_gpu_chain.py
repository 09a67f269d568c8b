"""The full-stack configuration run as a real chain on the GPU: conv1 -> ReLU -> pool -> norm ->
conv2 -> ReLU -> pool -> norm -> conv3 -> ReLU -> conv4 -> ReLU -> conv5 at batch 256, fp32, AUTO
lowering, then the gradient back through the same layers (normalisation, pooling argmax, ReLU
masks), with backward-weights at every convolution.  Every layer is one of the library's own
entry points.

Parity is gated per layer, teacher-forced: each convolution's outputs are compared, on sampled
elements the oracle computes one by one, with the oracle applied to the exact fp32 tensors that
the GPU layer consumed.  The end-to-end drift (the GPU chain against the oracle's own chain on the
first images) is printed and only loosely bounded."""
import numpy as np
import pytest

import oracle
from paper_1504_04343_amd import synth
from gpu_util import TOL_BF16, TOL_F32, desc_of, odims

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_1504_04343_amd import binding
    return binding


def host(t):
    return t.detach().cpu().numpy()


def check(name, got, want, idx, tol):
    err = float(np.abs(got.ravel()[idx] - want).max() / np.abs(want).max())
    print("  %-28s sampled rel err %.2e" % (name, err), flush=True)
    assert err <= tol, (name, err)


@pytest.mark.parametrize("N,precision", [(256, 0), (1024, 0), (256, 1)], ids=["b256_f32", "b1024_f32", "b256_bf16"])
def test_caffenet_conv_stack_as_a_chain(B, N, precision):
    import torch
    tol = TOL_F32 if precision == 0 else TOL_BF16
    layers = synth.caffenet(N)
    pool_after = {"conv1": (96, 55), "conv2": (256, 27)}       # 3x3 stride-2 max pooling
    W = {L.name: torch.from_numpy(synth.make_w(L)).cuda() for L in layers}
    bias = {L.name: torch.from_numpy((np.random.default_rng(40 + i).standard_normal(L.O) * 0.1)
                                     .astype(np.float32)).cuda() for i, L in enumerate(layers)}
    x = torch.from_numpy(synth.make_x(layers[0])).cuda()        # U[-1,1] images
    acts = {}
    ns = 1500 if N == 256 else 600

    # ---------------- forward chain ----------------
    for L in layers:
        print("forward", L.name, "batch", N, flush=True)
        d = desc_of(B, L, B.LOWER_AUTO, precision)
        y = torch.full((N, L.O, L.Hout, L.Wout), float("nan"), device="cuda")
        B.cct_conv_forward(d, x, W[L.name], bias[L.name], y, B.alloc_workspace(d, B.PASS_FORWARD))
        torch.cuda.synchronize()
        idx = synth.sample_indices(y.numel(), ns, 1)
        want = oracle.conv_forward_at(odims(oracle, L), host(x), host(W[L.name]), host(bias[L.name]), idx)
        check(L.name + " forward", host(y), want, idx, tol)
        rec = dict(x=x, y=y)
        if L.name != "conv5":
            a = torch.empty_like(y)
            B.cct_relu_forward(y, a)
            rec["relu"] = a
            if L.name in pool_after:
                C, H = pool_after[L.name]
                pd = B.make_pool_desc(N, C, H, H, 3, 2, 0)
                ho, wo = B.cct_pool_output_dims(pd)
                pooled = torch.empty((N, C, ho, wo), device="cuda")
                am = torch.empty((N, C, ho, wo), dtype=torch.int32, device="cuda")
                B.cct_maxpool_forward(pd, a, pooled, am)
                ld = B.make_lrn_desc(N, C, ho, wo)                # CaffeNet: size 5, alpha 1e-4, beta 0.75
                normed = torch.empty_like(pooled)
                B.cct_lrn_forward(ld, pooled, normed)
                rec.update(pd=pd, am=am, ld=ld, pooled=pooled)
                x = normed
            else:
                x = a
        acts[L.name] = rec

    # ---------------- end-to-end drift on the first images (reported, loosely bounded) ----------------
    if N == 256:
        k = 4
        ox = synth.make_x(layers[0])[:k]
        for L in layers:
            Lk = L.with_batch(k)
            oy = oracle.conv_forward(odims(oracle, Lk), ox, host(W[L.name]), host(bias[L.name])).astype(np.float32)
            if L.name != "conv5":
                oa = oracle.relu_forward(oy)
                if L.name in pool_after:
                    C, H = pool_after[L.name]
                    oa, _ = oracle.maxpool_forward(oracle.PoolDims(k, C, H, H, 3, 2, 0), oa)
                    oa = oracle.lrn_forward(oracle.LrnDims(k, C, oa.shape[2], oa.shape[3]), oa)
                ox = oa
        got = host(acts["conv5"]["y"][:k])
        drift = float(np.abs(got - oy).max() / np.abs(oy).max())
        print("  end-to-end drift of conv5's output over %d images: %.2e" % (k, drift), flush=True)
        assert drift <= 50 * tol

    # ---------------- backward chain ----------------
    last = layers[-1]
    g = torch.from_numpy(synth.make_dy(last)).cuda()            # gradient at conv5's output, N(0,1)
    for L in reversed(layers):
        print("backward", L.name, flush=True)
        rec = acts[L.name]
        d = desc_of(B, L, B.LOWER_AUTO, precision)
        od = odims(oracle, L)
        hx, hg, hw = host(rec["x"]), host(g), host(W[L.name])
        dw = torch.full_like(W[L.name], float("nan"))
        db = torch.full_like(bias[L.name], float("nan"))
        B.cct_conv_backward_weights(d, rec["x"], g, dw, db, B.alloc_workspace(d, B.PASS_BACKWARD_WEIGHTS))
        dx = torch.full_like(rec["x"], float("nan"))
        B.cct_conv_backward_data(d, W[L.name], g, dx, B.alloc_workspace(d, B.PASS_BACKWARD_DATA))
        torch.cuda.synchronize()
        idx = synth.sample_indices(dw.numel(), 48 if N == 256 else 16, 3)
        check(L.name + " backward-weights", host(dw), oracle.conv_backward_weights_at(od, hx, hg, idx), idx, tol)
        dbw = hg.astype(np.float64).sum(axis=(0, 2, 3))
        assert np.abs(host(db) - dbw).max() / np.abs(dbw).max() <= TOL_F32
        idx = synth.sample_indices(dx.numel(), ns, 2)
        check(L.name + " backward-data", host(dx), oracle.conv_backward_data_at(od, hw, hg, idx), idx, tol)
        if L.name == "conv1":
            break
        prev = acts[layers[layers.index(L) - 1].name]
        g = dx                                                   # gradient at the previous layer's (pooled) activation
        if "pd" in prev:
            gp = torch.empty_like(prev["pooled"])
            B.cct_lrn_backward(prev["ld"], prev["pooled"], g, gp)
            up = torch.empty_like(prev["relu"])
            B.cct_maxpool_backward(prev["pd"], gp, prev["am"], up)
            g = up
        gy = torch.empty_like(prev["y"])
        B.cct_relu_backward(prev["y"], g, gy)
        g = gy
        assert bool(torch.isfinite(g).all())


def test_caffenet_classifier_head_as_a_chain(B):
    """The layers after pool5 as a real chain at their CaffeNet sizes, batch 64: fc6 -> ReLU -> dropout
    -> fc7 -> ReLU -> dropout -> fc8 -> softmax loss, and the gradient back to pool5's output.  Every
    layer is teacher-forced against the oracle on the exact fp32 tensors the GPU layer consumed."""
    import torch
    from gpu_util import layer
    N = 64
    fcs = [layer("fc6", N, 256, 6, 6, 4096, 6, 1, 0, 1, "relu_normal", 0.005, 0.1),
           layer("fc7", N, 4096, 1, 1, 4096, 1, 1, 0, 1, "relu_normal", 0.005, 0.1),
           layer("fc8", N, 4096, 1, 1, 1000, 1, 1, 0, 1, "relu_normal", 0.01, 0.1)]
    rng = np.random.default_rng(11)
    W = {L.name: torch.from_numpy(synth.make_w(L, 3)).cuda() for L in fcs}
    bias = {L.name: torch.from_numpy(synth.make_bias(L, 3)).cuda() for L in fcs}
    masks = {n: torch.from_numpy((rng.random((N, 4096, 1, 1)) >= 0.5).astype(np.uint8)).cuda()
             for n in ("fc6", "fc7")}
    label_h = rng.integers(0, 1000, N).astype(np.int32)
    label = torch.from_numpy(label_h).cuda()
    x = torch.from_numpy(synth.make_x(fcs[0], 3)).cuda()
    ins, pre = {}, {}
    for L in fcs:                                                   # ---- forward
        print("forward", L.name, flush=True)
        d = desc_of(B, L)
        ins[L.name] = x
        y = torch.full((N, L.O, 1, 1), float("nan"), device="cuda")
        B.cct_conv_forward(d, x, W[L.name], bias[L.name], y, B.alloc_workspace(d, B.PASS_FORWARD))
        torch.cuda.synchronize()
        want = oracle.conv_forward(odims(oracle, L), host(x), host(W[L.name]), host(bias[L.name]))
        check(L.name + " forward", host(y), want.ravel(), np.arange(y.numel()), TOL_F32)
        pre[L.name] = y
        if L.name != "fc8":
            a, o = torch.empty_like(y), torch.empty_like(y)
            B.cct_relu_forward(y, a)
            B.cct_dropout_forward(a, masks[L.name], 2.0, o)
            torch.cuda.synchronize()
            assert host(a).tobytes() == oracle.relu_forward(host(y)).tobytes()
            assert host(o).tobytes() == oracle.dropout(host(a), host(masks[L.name]), 2.0).tobytes()
            x = o.view(N, 4096, 1, 1)
    scores = pre["fc8"].view(N, 1000)
    prob, il, loss = torch.empty_like(scores), torch.empty(N, device="cuda"), torch.empty(1, device="cuda")
    B.cct_softmax_loss_forward(scores, label, prob, il, loss)
    g = torch.full((N, 1000), float("nan"), device="cuda")
    B.cct_softmax_loss_backward(prob, label, g)
    torch.cuda.synchronize()
    want_prob, want_loss = oracle.softmax_loss_forward(host(scores), label_h)
    assert np.abs(host(prob) - want_prob).max() <= 1e-5 * want_prob.max()
    assert abs(float(loss.item()) - want_loss) <= 1e-5 * want_loss
    print("  loss %.5f (oracle %.5f; log 1000 = %.5f)" % (float(loss.item()), want_loss, np.log(1000.0)), flush=True)
    want_g = oracle.softmax_loss_backward(host(prob), label_h)
    assert np.abs(host(g) - want_g).max() <= 1e-6 * np.abs(want_g).max()
    g = g.view(N, 1000, 1, 1)
    for L in reversed(fcs):                                         # ---- backward
        print("backward", L.name, flush=True)
        d = desc_of(B, L)
        if L.name != "fc8":
            ga, gy = torch.empty_like(pre[L.name]), torch.empty_like(pre[L.name])
            B.cct_dropout_backward(g.view_as(ga), masks[L.name], 2.0, ga)
            B.cct_relu_backward(pre[L.name], ga, gy)
            torch.cuda.synchronize()
            assert host(ga).tobytes() == oracle.dropout(host(g).reshape(ga.shape), host(masks[L.name]), 2.0).tobytes()
            assert host(gy).tobytes() == oracle.relu_backward(host(pre[L.name]), host(ga)).tobytes()
            g = gy
        dw, db = torch.empty_like(W[L.name]), torch.empty_like(bias[L.name])
        B.cct_conv_backward_weights(d, ins[L.name], g, dw, db, B.alloc_workspace(d, B.PASS_BACKWARD_WEIGHTS))
        gx = torch.full_like(ins[L.name], float("nan"))
        B.cct_conv_backward_data(d, W[L.name], g, gx, B.alloc_workspace(d, B.PASS_BACKWARD_DATA))
        torch.cuda.synchronize()
        idx = synth.sample_indices(dw.numel(), 3000, 2)
        want = oracle.conv_backward_weights_at(odims(oracle, L), host(ins[L.name]), host(g), idx)
        check(L.name + " backward-weights", host(dw), want, idx, TOL_F32)
        want = oracle.conv_backward_data(odims(oracle, L), host(W[L.name]), host(g))
        check(L.name + " backward-data", host(gx), want.ravel(), np.arange(gx.numel()), TOL_F32)
        g = gx
