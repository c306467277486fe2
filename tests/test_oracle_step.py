"""Pins for the oracle's whole step: an independent PyTorch fp64 composition,
the reset rule, row independence, the prefix property, purity and the
multi-head bookkeeping (paper, App. "VizDoom experiments", action-space table).
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2006_11751_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def torch_step(net, w, obs, h_in, done):
    """The network written with PyTorch CPU fp64 ops (third opinion)."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).double()
    x = (torch.from_numpy(obs).double() - float(np.float32(net["obs_sub"]))) * float(np.float32(net["obs_mul"]))
    if net["encoder"] == "conv":
        for (co, k, s, p), cw, cb in zip(net["convs"], w["conv_w"], w["conv_b"]):
            x = F.relu(F.conv2d(x, t(cw), t(cb), stride=s, padding=p))
    else:
        i = 0
        conv = lambda x, i: F.conv2d(x, t(w["conv_w"][i]), t(w["conv_b"][i]), padding=1)
        for _ in net["stages"]:
            x = F.max_pool2d(conv(x, i), 3, 2, 1)
            i += 1
            for _ in range(net["blocks_per_stage"]):
                x = x + conv(F.relu(conv(F.relu(x), i)), i + 1)
                i += 2
        x = F.relu(x)
    f = F.relu(F.linear(x.flatten(1), t(w["fc_w"]), t(w["fc_b"])))
    h = t(h_in) * (1.0 - torch.from_numpy(done.astype(np.float64)))[:, None]
    cell = torch.nn.GRUCell(net["fc"], net["rnn"]).double()
    with torch.no_grad():
        cell.weight_ih.copy_(t(w["rnn_w_ih"]))
        cell.weight_hh.copy_(t(w["rnn_w_hh"]))
        cell.bias_ih.copy_(t(w["rnn_b_ih"]))
        cell.bias_hh.copy_(t(w["rnn_b_hh"]))
        hn = cell(f, h)
        logits = F.linear(hn, t(w["pi_w"]), t(w["pi_b"]))
        value = F.linear(hn, t(w["v_w"])[None], t(w["v_b"]))[:, 0]
    return hn.numpy(), logits.numpy(), value.numpy()


def _inputs(net, B, t=0):
    return (wl.observations(net, t, B), wl.initial_state(net, B), wl.done_mask(net, t, B))


SMALL_RESNET = dict(name="resnet_small", B=3, obs=(3, 18, 24), encoder="resnet", stages=[4, 6, 6],
                    blocks_per_stage=2, fc=16, rnn=12, heads=[5], dtype="fp32", p_done=0.3, steps=1,
                    obs_sub=0.0, obs_mul=wl.OBS_MUL, index=4)
SMALL_STD = dict(name="std_small", B=3, obs=(3, 72, 128), encoder="conv",
                 convs=[(4, 8, 4, 0), (6, 4, 2, 0), (8, 3, 2, 0)], fc=24, rnn=20, heads=[3, 3, 2, 11],
                 dtype="fp32", p_done=0.4, steps=1, obs_sub=3.0, obs_mul=0.01, index=3)


@pytest.mark.parametrize("net", [wl.network(0), SMALL_STD, SMALL_RESNET], ids=lambda n: n["name"])
def test_step_matches_torch_composition(ref, net):
    B = net["B"]
    w = wl.weights(net)
    obs, h_in, done = _inputs(net, B)
    done[0], done[1] = 1, 0
    out = ref.policy_step(net, w, obs, h_in, done, 1, 0)
    hn, logits, value = torch_step(net, w, obs, h_in, done)
    np.testing.assert_allclose(out["h_out"], hn, rtol=2e-7, atol=1e-7)
    np.testing.assert_allclose(out["logits"], logits, rtol=2e-7, atol=1e-7)
    np.testing.assert_allclose(out["value"], value, rtol=2e-7, atol=1e-7)
    # joint log-probability = sum over heads of log-softmax at the sampled action
    off = 0
    lp = np.zeros(B)
    for k, A in enumerate(net["heads"]):
        ls = torch.log_softmax(torch.from_numpy(out["logits"][:, off:off + A]).double(), dim=1).numpy()
        a = out["actions"][:, k]
        assert np.all((0 <= a) & (a < A))
        lp += ls[np.arange(B), a]
        off += A
    np.testing.assert_allclose(out["logp"], lp, rtol=2e-7, atol=1e-7)


def test_step_actions_are_per_head_samples_of_its_logits(ref):
    net = SMALL_STD
    w = wl.weights(net)
    obs, h_in, done = _inputs(net, 3)
    out = ref.policy_step(net, w, obs, h_in, done, 5, 9)
    for b in range(3):
        off = 0
        for k, A in enumerate(net["heads"]):
            a, _, mg = ref.head_sample(out["logits"][b, off:off + A], 5, b, 9, k)
            assert a == out["actions"][b, k] and mg == out["margin"][b, k]
            off += A


def test_done_resets_incoming_state(ref):
    net = wl.network(0)
    w = wl.weights(net)
    obs, h_in, _ = _inputs(net, 8)
    done = np.array([1, 0, 1, 0, 1, 0, 0, 1], np.uint8)
    a = ref.policy_step(net, w, obs, h_in, done, 1, 0)
    # rows with done=1 do not depend on h_in and equal the zero-state result bit for bit
    h2 = h_in.copy()
    h2[done == 1] = 123.0
    b = ref.policy_step(net, w, obs, h2, done, 1, 0)
    h0 = h_in.copy()
    h0[done == 1] = 0.0
    c = ref.policy_step(net, w, obs, h0, np.zeros(8, np.uint8), 1, 0)
    for key in ("h_out", "logits", "value", "logp", "actions"):
        assert np.array_equal(a[key], b[key]) and np.array_equal(a[key], c[key])
    # the reset is applied before the cell: the new state of a reset row is not zero
    assert np.all(np.abs(a["h_out"][done == 1]).max(axis=1) > 0)
    # rows with done=0 do depend on h_in
    h3 = h_in.copy()
    h3[done == 0] += 0.5
    d = ref.policy_step(net, w, obs, h3, done, 1, 0)
    assert not np.array_equal(a["h_out"][1], d["h_out"][1])
    assert np.array_equal(a["h_out"][0], d["h_out"][0])
    # any non-zero byte counts as done
    done255 = done * 255
    e = ref.policy_step(net, w, obs, h_in, done255.astype(np.uint8), 1, 0)
    assert np.array_equal(a["h_out"], e["h_out"])


def test_rows_independent_prefix_and_purity(ref):
    net = wl.network(0)
    w = wl.weights(net)
    obs, h_in, done = _inputs(net, 8)
    a = ref.policy_step(net, w, obs, h_in, done, 1, 3)
    again = ref.policy_step(net, w, obs, h_in, done, 1, 3)
    for key in a:
        assert np.array_equal(a[key], again[key])
    perm = np.array([3, 0, 7, 1, 6, 2, 5, 4])
    p = ref.policy_step(net, w, obs[perm], h_in[perm], done[perm], 1, 3)
    for key in ("h_out", "logits", "value"):
        assert np.array_equal(p[key], a[key][perm])
    # the sampler's env word is the row index, so actions follow the row, not the data:
    # row r of the permuted call equals head_sample(logits of data perm[r], env = r)
    for r in range(8):
        act, _, _ = ref.head_sample(a["logits"][perm[r]], 1, r, 3, 0)
        assert act == p["actions"][r, 0]
    pre = ref.policy_step(net, w, obs[:5], h_in[:5], done[:5], 1, 3)
    for key in a:
        assert np.array_equal(pre[key], a[key][:5])
    # step and seed reach the sampler only
    s2 = ref.policy_step(net, w, obs, h_in, done, 1, 4)
    assert np.array_equal(s2["logits"], a["logits"]) and not np.array_equal(s2["margin"], a["margin"])
    empty = ref.policy_step(net, w, obs[:0], h_in[:0], done[:0], 1, 3)
    assert empty["actions"].shape == (0, 1)


def test_observation_normalisation_is_affine_in_the_byte(ref):
    # one 1x1 "image", 1x1 conv with weight 1: the encoder output is relu((u8 - sub) * mul)
    net = dict(name="pix", B=4, obs=(1, 1, 1), encoder="conv", convs=[(1, 1, 1, 0)], fc=1, rnn=1,
               heads=[2], dtype="fp32", p_done=0.0, obs_sub=16.0, obs_mul=0.125, index=0)
    w = wl.weights(net)
    w["conv_w"][0][:] = 1.0
    w["conv_b"][0][:] = 0.0
    w["fc_w"][:] = 1.0
    w["fc_b"][:] = 0.0
    # make the GRU pass f through: z -> 0 (h' = n), r irrelevant, n = tanh(f): invert with atanh
    w["rnn_w_ih"][:] = np.array([[0.0], [0.0], [1.0]], np.float32)
    w["rnn_w_hh"][:] = 0.0
    w["rnn_b_ih"][:] = np.array([0.0, -80.0, 0.0], np.float32)
    w["rnn_b_hh"][:] = 0.0
    obs = np.array([0, 16, 20, 24], np.uint8).reshape(4, 1, 1, 1)
    out = ref.policy_step(net, w, obs, np.zeros((4, 1), np.float32), np.zeros(4, np.uint8), 1, 0)
    want = np.tanh(np.maximum((obs.reshape(4).astype(np.float64) - 16.0) * 0.125, 0.0))
    np.testing.assert_allclose(out["h_out"][:, 0], want, rtol=1e-6, atol=1e-30)


def test_default_normalisation_constant():
    assert np.float32(wl.OBS_MUL).view(np.uint32) == 0x3B808081
    assert wl.network(1)["obs_sub"] == 0.0


def test_full_action_space_bookkeeping(ref):
    sizes = {}
    with open(os.path.join(GOLDEN, "vizdoom_action_heads.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                name, n = line.split()
                sizes[name] = int(n)
    total = sizes.pop("total_joint_actions")
    heads = list(sizes.values())
    assert len(heads) == 7 and int(np.prod(heads)) == total == 12096
    net = dict(SMALL_STD, heads=heads)
    w = wl.weights(net)
    obs, h_in, done = _inputs(net, 6)
    out = ref.policy_step(net, w, obs, h_in, done, 1, 0)
    assert out["logits"].shape == (6, sum(heads)) and out["actions"].shape == (6, 7)
    assert np.all(out["actions"] >= 0) and np.all(out["actions"] < np.array(heads)[None])
    # over many steps every head visits every one of its actions: 12096 joint actions reachable
    seen = [set() for _ in heads]
    for step in range(300):
        o = ref.policy_step(net, w, obs, h_in, done, 1, step, want_logits=False, want_margin=False)
        for k in range(7):
            seen[k].update(o["actions"][:, k].tolist())
    assert [len(s) for s in seen] == heads


def test_shapes_of_the_benchmark_configurations(ref):
    # encoder output sizes that follow from no-padding floor-division convolutions
    assert [wl.flat_size(wl.network(i)) for i in range(5)] == [576, 2304, 2304, 2304, 4608]
    assert [ref.flat_size(wl.network(i)) for i in range(5)] == [576, 2304, 2304, 2304, 4608]


def test_weight_recipe():
    net = wl.network(1)
    w = wl.weights(net)
    assert w["conv_w"][0].shape == (32, 3, 8, 8) and w["fc_w"].shape == (512, 2304)
    assert w["rnn_w_ih"].shape == (1536, 512) and w["pi_w"].shape == (7, 512) and w["v_w"].shape == (512,)
    assert abs(w["fc_w"].var() * 2304 - 1) < 0.01 and abs(w["rnn_w_hh"].var() * 512 - 1) < 0.01
    assert np.abs(w["fc_b"]).max() > 0
    wb = wl.weights(wl.network(2))
    for a in [wb["fc_w"], wb["conv_w"][1], wb["v_b"]]:
        assert np.all(a.view(np.uint32) & 0xFFFF == 0)
    # ties-to-even rounding
    x = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20], np.float32)
    assert np.array_equal(wl.round_to_bf16(x), np.array([1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7], np.float32))
