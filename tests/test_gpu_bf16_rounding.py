"""bf16 configurations define their parameters as the nearest bf16 values (ties to even) of
what the caller passes.  Every other bf16 test hands over parameters that are already rounded,
on which the library's own rounding is the identity; here the parameters arrive as drawn
(fp32), with exact ties and values one fp32 step either side of a tie planted in every tensor.
The result must equal, bit for bit, that of a policy created from parameters rounded
beforehand by the input generator, and must match the oracle run on those rounded parameters.
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests import parity
from tests.test_gpu_parity import RESNET_BF16_SMALL, STD_BF16_SMALL, _gpu_step

pytestmark = pytest.mark.gpu


def _plant_ties(w, seed):
    """In every tensor, overwrite a tenth of the entries' low 16 bits with 0x8000 (an exact tie
    between two bf16 neighbours; the kept upper half is odd or even as drawn), 0x7FFF or 0x8001."""
    rng = np.random.default_rng(seed)
    out = {}
    for k, v in w.items():
        def plant(a):
            a = np.array(a, dtype=np.float32, copy=True)
            bits = a.view(np.uint32).ravel()
            n = max(3, bits.size // 10)
            idx = rng.choice(bits.size, size=min(n, bits.size), replace=False)
            low = rng.choice(np.array([0x8000, 0x7FFF, 0x8001], np.uint32), size=idx.size)
            bits[idx] = (bits[idx] & np.uint32(0xFFFF0000)) | low
            return a
        out[k] = [plant(a) for a in v] if isinstance(v, list) else plant(v)
    return out


@pytest.mark.parametrize("net", [STD_BF16_SMALL, RESNET_BF16_SMALL,
                                 wl.network(2, B=19, name="lstm_bf16", rnn_type="lstm")],
                         ids=lambda n: n["name"])
def test_unrounded_parameters(torch_cuda, ref, net):
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    w_raw = _plant_ties(wl.weights(net, seed=2024, rounded=False), seed=5)
    w_rounded = wl.round_weights_to_bf16(w_raw)
    changed = sum(int(np.sum(a != b)) for a, b in zip(w_raw["conv_w"], w_rounded["conv_w"]))
    assert changed > 0 and not np.array_equal(w_raw["fc_w"], w_rounded["fc_w"])
    B = net["B"]
    obs, h_in, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    pol = binding.Policy(net, w_raw)
    g = _gpu_step(torch, pol, obs, h_in, done, 7, 1)
    pol.close()
    pre = binding.Policy(net, w_rounded)
    g2 = _gpu_step(torch, pre, obs, h_in, done, 7, 1)
    pre.close()
    for k in g:
        assert np.array_equal(g[k], g2[k]), k
    o = ref.policy_step(net, w_rounded, obs, h_in, done, 7, 1)
    print(net["name"], parity.check_against_oracle(net, g, o, ref, 7, 1))


def test_update_with_unrounded_parameters(torch_cuda, ref):
    """The same through a weight update."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    net = STD_BF16_SMALL
    B = net["B"]
    obs, h_in, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    w_raw = _plant_ties(wl.weights(net, seed=2025, rounded=False), seed=6)
    pol = binding.Policy(net, wl.weights(net))
    pol.update_weights(w_raw)
    g = _gpu_step(torch, pol, obs, h_in, done, 7, 1)
    pol.close()
    o = ref.policy_step(net, wl.round_weights_to_bf16(w_raw), obs, h_in, done, 7, 1)
    parity.check_against_oracle(net, g, o, ref, 7, 1)
