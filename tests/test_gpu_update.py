"""Weight updates through the C ABI (paper, Sec. 3.3: the policy workers take the learner's
new parameters after every learner step): after sf_policy_update_weights a policy computes
exactly what a policy created with the new parameters computes, matches the oracle with
those parameters, and the switch is ordered by the stream with no host synchronisation.
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests import parity
from tests.test_gpu_parity import RESNET_BF16_SMALL, _make, _to_np
from tests.test_gpu_core import NETS

pytestmark = pytest.mark.gpu

CASES = [wl.network(0), wl.network(1, B=70, name="standard_small"),
         wl.network(2, B=37, name="standard_bf16_small"), RESNET_BF16_SMALL, NETS[5], NETS[3]]


def _step(torch, pol, net, t, seed=1):
    d = pol.device
    B = net["B"]
    obs, state, done = wl.observations(net, t, B), wl.initial_state(net, B), wl.done_mask(net, t, B)
    meas = wl.measurements(net, t, B)
    out = pol.step(torch.from_numpy(obs).to(d), torch.from_numpy(state).to(d), torch.from_numpy(done).to(d),
                   seed, t, meas=None if meas is None else torch.from_numpy(meas).to(d))
    return out, (obs, state, done, meas)


@pytest.mark.parametrize("net", CASES, ids=lambda n: n["name"])
def test_updated_policy_equals_a_fresh_one_and_the_oracle(torch_cuda, ref, net):
    torch = torch_cuda
    w0, w1 = wl.weights(net), wl.weights(net, seed=4242)
    pol, _ = _make(torch, net)
    before, _ = _step(torch, pol, net, 0)
    torch.cuda.synchronize()
    before = _to_np(before)
    pol.update_weights(w1)
    after, (obs, state, done, meas) = _step(torch, pol, net, 0)
    torch.cuda.synchronize()
    after = _to_np(after)
    from paper_2006_11751_amd import binding
    fresh = binding.Policy(net, w1, max_batch=net["B"])
    want, _ = _step(torch, fresh, net, 0)
    torch.cuda.synchronize()
    want = _to_np(want)
    for k in ("actions", "logp", "value", "h_out", "logits"):
        assert np.array_equal(after[k], want[k]), k
    assert not np.array_equal(after["logits"], before["logits"])
    o = ref.policy_step(net, w1, obs, state, done, 1, 0, meas=meas)
    parity.check_against_oracle(net, after, o, ref, 1, 0)
    # and back again
    pol.update_weights(w0)
    again, _ = _step(torch, pol, net, 0)
    torch.cuda.synchronize()
    again = _to_np(again)
    for k in ("actions", "logp", "value", "h_out", "logits"):
        assert np.array_equal(again[k], before[k]), k
    fresh.close()
    pol.close()


def test_updates_are_ordered_by_the_stream_without_host_synchronisation(torch_cuda):
    torch = torch_cuda
    net = wl.network(1, B=256, name="standard_256")
    w = [wl.weights(net), wl.weights(net, seed=777)]
    pol, _ = _make(torch, net)
    d = pol.device
    B = net["B"]
    obs = torch.from_numpy(wl.observations(net, 0, B)).to(d)
    state = torch.from_numpy(wl.initial_state(net, B)).to(d)
    done = torch.from_numpy(wl.done_mask(net, 0, B)).to(d)
    side = torch.cuda.Stream(device=d)
    torch.cuda.synchronize()
    outs = []
    with torch.cuda.stream(side):
        for i in range(6):                      # step(w0) update(w1) step(w1) update(w0) step(w0) ...
            out = pol.alloc_outputs(B)
            pol.step(obs, state, done, 1, 0, out=out, stream=side)
            outs.append(out)
            pol.update_weights(w[(i + 1) % 2], stream=side)
    side.synchronize()
    outs = [_to_np(o) for o in outs]
    for i in range(2, 6):
        for k in ("actions", "logp", "value", "h_out", "logits"):
            assert np.array_equal(outs[i][k], outs[i % 2][k]), (i, k)
    assert not np.array_equal(outs[0]["logits"], outs[1]["logits"])
    pol.close()


def test_update_rejects_missing_tensors(torch_cuda):
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    net = wl.network(0)
    pol, w = _make(torch, net)
    ws, keep = binding.make_weights(w)
    ws.fc_w = None
    with pytest.raises(binding.SfError) as e:
        binding.sf_policy_update_weights(pol.handle, ws, None)
    assert e.value.code == binding.SF_ERR_ARG
    assert binding.load_library().sf_policy_update_weights(None, None, None) == binding.SF_ERR_ARG
    pol.close()


@pytest.mark.parametrize("net", [wl.network(1, B=70, name="standard_small"), RESNET_BF16_SMALL], ids=lambda n: n["name"])
def test_rejected_update_leaves_the_old_parameters_in_place(torch_cuda, net):
    """The whole parameter set is packed and checked before the first copy is enqueued: an update
    whose LAST tensors are bad (a NaN in the value head's bias; for the fp16 encoder a weight beyond
    the fp16 range in the FC layer) fails with SF_ERR_ARG and the next step still computes the old
    policy's bits, although every earlier tensor of the update differed from the old one."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    pol, w0 = _make(torch, net)
    before, _ = _step(torch, pol, net, 0)
    torch.cuda.synchronize()
    before = _to_np(before)
    bad = []
    w1 = wl.weights(net, seed=777)
    w1["v_b"] = w1["v_b"].copy()
    w1["v_b"][0] = np.nan
    bad.append(w1)
    if net["dtype"] == "bf16" and net["encoder"] == "resnet":
        w2 = wl.weights(net, seed=778)
        w2["fc_w"] = w2["fc_w"].copy()
        w2["fc_w"][1, 5] = 1.0e5
        bad.append(w2)
    for w in bad:
        with pytest.raises(binding.SfError) as e:
            pol.update_weights(w)
        assert e.value.code == binding.SF_ERR_ARG
        after, _ = _step(torch, pol, net, 0)
        torch.cuda.synchronize()
        after = _to_np(after)
        for k in ("actions", "logp", "value", "h_out", "logits"):
            assert np.array_equal(after[k], before[k]), k
    # a good update still goes through afterwards
    pol.update_weights(wl.weights(net, seed=779))
    ok, _ = _step(torch, pol, net, 0)
    torch.cuda.synchronize()
    assert not np.array_equal(_to_np(ok)["logits"], before["logits"])
    pol.close()
