"""The automatic lowering optimizer has no reference to pin against (the paper gives neither a
formula nor thresholds), so it is graded by regret: the layout it picks must not be much slower
than the fastest layout measured in the same run, and on the channel-ratio sweep of Appendix A
the measured winner must move from Type 1 to Type 3 as #input/#output channels grows."""
import pytest

from paper_1504_04343_amd import synth
from gpu_util import desc_of, dev

pytestmark = pytest.mark.gpu
REGRET = 0.10      # picked layout may be at most 10 % slower than the best measured one


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_1504_04343_amd import binding
    return binding


def time_pass(B, L, lowering, pass_, reps=7):
    import torch
    d = desc_of(B, L, lowering)
    x, w, b = dev(synth.make_x(L)), dev(synth.make_w(L)), dev(synth.make_bias(L))
    dy = dev(synth.make_dy(L))
    y, dx, dw, db = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w), torch.empty_like(b)
    ws = B.alloc_workspace(d, pass_)

    def run():
        if pass_ == B.PASS_FORWARD:
            B.cct_conv_forward(d, x, w, b, y, ws)
        elif pass_ == B.PASS_BACKWARD_DATA:
            B.cct_conv_backward_data(d, w, dy, dx, ws)
        else:
            B.cct_conv_backward_weights(d, x, dy, dw, db, ws)

    run()
    run()
    torch.cuda.synchronize()
    times = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    return sorted(times)[len(times) // 2]          # median


def measured(B, L, pass_=0):
    d = desc_of(B, L)
    costs = {}
    for t in (1, 2, 3, 4):
        try:
            costs[t] = B.cct_lowering_cost(d, pass_, t)
            B.cct_conv_workspace_bytes(desc_of(B, L, t), pass_)     # raises when unsupported
        except B.CctError:
            costs.pop(t, None)
    cheapest = min(costs.values())
    # layouts the model prices at more than 5x the cheapest are not worth running (conv1 Type 3)
    return {t: time_pass(B, L, t, pass_) for t, c in costs.items() if c <= 5 * cheapest}


@pytest.mark.parametrize("pass_", [0, 1, 2], ids=["forward", "backward_data", "backward_weights"])
@pytest.mark.parametrize("L", synth.caffenet(256), ids=lambda L: L.name)
def test_regret_on_caffenet_layers(B, L, pass_):
    times = measured(B, L, pass_)
    pick = B.cct_pick_lowering(desc_of(B, L), pass_)
    assert pick in times
    assert times[pick] <= (1 + REGRET) * min(times.values()), (pick, times)


def test_measured_winner_follows_channel_ratio(B):
    sweep = [L for L in synth.tradeoff_sweep() if L.K == 3]           # batch 128, as the study names it
    winners = {}
    for L in sweep:
        times = measured(B, L)
        winners[(L.C, L.O)] = min(times, key=times.get)
        pick = B.cct_pick_lowering(desc_of(B, L), B.PASS_FORWARD)
        assert times[pick] <= (1 + REGRET) * min(times.values()), (L.name, pick, times)
    assert winners[(16, 512)] in (1, 4)             # few input, many output channels: Type 1 (or its fusion)
    assert winners[(1024, 32)] in (2, 3)            # many input, few output channels: not Type 1
    assert winners[(512, 16)] in (2, 3)
