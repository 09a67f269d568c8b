"""Shared helpers of the GPU parity tests: upload seeded inputs, call the C ABI through the
binding, bring results back as numpy.  No arithmetic of the method lives here."""
import numpy as np

from paper_1504_04343_amd import synth

TOL_F32 = 1e-4      # max |gpu - oracle| / max |oracle|, fp32 path
TOL_BF16 = 2e-2     # same metric, bf16-operand path


def rel_err(got, want):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    denom = np.abs(want).max()
    if denom == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - want).max() / denom)


def desc_of(B, L, lowering=0, precision=0):
    return B.make_desc(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups, lowering, precision)


def odims(oracle, L):
    return oracle.Dims(L.N, L.C, L.H, L.W, L.O, L.K, L.stride, L.pad, L.groups)


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def workspace(B, d, pass_, chunk=None):
    return B.alloc_workspace(d, pass_, chunk)


def gpu_forward(B, L, x, w, bias, lowering=0, precision=0, chunk=None):
    import torch
    d = desc_of(B, L, lowering, precision)
    y = torch.full((L.N, L.O, L.Hout, L.Wout), float("nan"), device="cuda")
    ws = workspace(B, d, B.PASS_FORWARD, chunk)
    B.cct_conv_forward(d, dev(x), dev(w), None if bias is None else dev(bias), y, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def gpu_backward_data(B, L, w, dy, lowering=0, precision=0, chunk=None):
    import torch
    d = desc_of(B, L, lowering, precision)
    dx = torch.full((L.N, L.C, L.H, L.W), float("nan"), device="cuda")
    ws = workspace(B, d, B.PASS_BACKWARD_DATA, chunk)
    B.cct_conv_backward_data(d, dev(w), dev(dy), dx, ws)
    torch.cuda.synchronize()
    return dx.cpu().numpy()


def gpu_backward_weights(B, L, x, dy, lowering=0, precision=0, chunk=None, want_dbias=True):
    import torch
    d = desc_of(B, L, lowering, precision)
    dw = torch.full((L.O, L.C // L.groups, L.K, L.K), float("nan"), device="cuda")
    db = torch.full((L.O,), float("nan"), device="cuda") if want_dbias else None
    ws = workspace(B, d, B.PASS_BACKWARD_WEIGHTS, chunk)
    B.cct_conv_backward_weights(d, dev(x), dev(dy), dw, db, ws)
    torch.cuda.synchronize()
    return dw.cpu().numpy(), (None if db is None else db.cpu().numpy())


def layer(name, N, C, H, W, O, K, s=1, p=0, g=1, x_dist="uniform", w_std=0.05, bias_std=0.1):
    return synth.Layer(name, N, C, H, W, O, K, s, p, g, x_dist, w_std, bias_std)
