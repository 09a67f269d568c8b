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
