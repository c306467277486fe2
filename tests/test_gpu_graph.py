"""The step allocates nothing and does not synchronise, so it can be recorded into a HIP
graph: a captured step, replayed several times on fresh inputs with eager work and
synchronisations between the replays, gives the bits of the eager step every time.
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests.test_gpu_parity import RESNET_BF16_SMALL, _make

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("net", [wl.network(1, B=96, name="standard_96"), RESNET_BF16_SMALL,
                                 wl.network(6, B=64, name="full_64"),
                                 wl.network(2, B=70, name="standard_bf16_70")], ids=lambda n: n["name"])
def test_captured_step_replays_bitwise(torch_cuda, net):
    torch = torch_cuda
    pol, _ = _make(torch, net)
    d = pol.device
    B = net["B"]

    def inputs(t):
        meas = wl.measurements(net, t, B)
        return (torch.from_numpy(wl.observations(net, t, B)).to(d), torch.from_numpy(wl.initial_state(net, B)).to(d),
                torch.from_numpy(wl.done_mask(net, t, B)).to(d), None if meas is None else torch.from_numpy(meas).to(d))

    obs, state, done, meas = inputs(0)
    out = pol.alloc_outputs(B)
    side = torch.cuda.Stream(device=d)
    with torch.cuda.stream(side):      # warm-up outside the capture
        pol.step(obs, state, done, 1, 0, out=out, stream=side, meas=meas)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pol.step(obs, state, done, 1, 0, out=out, stream=torch.cuda.current_stream(d), meas=meas)
    for t in range(1, 4):
        o2, s2, d2, m2 = inputs(t)
        eager = pol.step(o2, s2, d2, 1, 0, meas=m2)       # eager work between the replays
        torch.cuda.synchronize()
        obs.copy_(o2)
        state.copy_(s2)
        done.copy_(d2)
        if meas is not None:
            meas.copy_(m2)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in ("actions", "logp", "value", "h_out", "logits"):
            assert torch.equal(out[k], eager[k]), (t, k)
    pol.close()


def test_captured_pass_over_trajectories_replays_bitwise(torch_cuda):
    """The learner's forward pass (1 + T + 1 + the encoder's launches, nothing allocated) recorded
    once and replayed on fresh trajectories: the eager call's bits every time."""
    torch = torch_cuda
    net = wl.network(6, name="full_unrolled", p_done=0.1)
    T, N = 6, 8
    pol, _ = _make(torch, net, max_batch=T * N)
    d = pol.device

    def inputs(shift):
        obs, h0, done, meas = wl.trajectory_inputs(net, T + shift, N)
        return [torch.from_numpy(np.ascontiguousarray(a[shift:] if a.shape[0] == T + shift else a)).to(d)
                for a in (obs, h0, done, meas)]

    obs, h0, done, meas = inputs(0)
    out = pol.unroll(obs, h0, done, meas=meas)
    side = torch.cuda.Stream(device=d)
    side.wait_stream(torch.cuda.current_stream(d))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pol.unroll(obs, h0, done, out=out, stream=torch.cuda.current_stream(d), meas=meas)
    for shift in range(1, 4):
        o2, _, d2, m2 = inputs(shift)
        eager = pol.unroll(o2, h0, d2, meas=m2)           # eager work between the replays
        torch.cuda.synchronize()
        obs.copy_(o2)
        done.copy_(d2)
        meas.copy_(m2)
        for v in out.values():
            v.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in ("logits", "value", "h_seq"):
            assert torch.equal(out[k], eager[k]), (shift, k)
    pol.close()
