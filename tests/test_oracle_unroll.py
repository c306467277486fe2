"""Pins for the oracle's forward pass over trajectories (paper, Sec. 3.1: the learner unrolls
the recurrent core over the T steps of a trajectory): PyTorch's fp64 sequence modules
(torch.nn.GRU / torch.nn.LSTM over the whole sequence) as the independent library routine, the
episode-start rule (a done restarts the trajectory from a zero state at that step), causality,
independence of the trajectories, and T = 1 against the single step.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2006_11751_amd import workloads as wl
from tests.test_oracle_core import SMALL_FULL, SMALL_FULL_LSTM, SMALL_LSTM
from tests.test_oracle_step import SMALL_STD

_t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).double()


def torch_unroll(net, w, obs, meas, h0):
    """Encoder on all T*N frames, then the sequence module over [T, N, features]; no episode
    starts.  Returns h [T,N,H], final c [N,H] or None, logits, value."""
    T, N = obs.shape[:2]
    x = (torch.from_numpy(obs.reshape((T * N,) + obs.shape[2:])).double() - float(np.float32(net["obs_sub"]))) \
        * float(np.float32(net["obs_mul"]))
    for (co, k, s, p), cw, cb in zip(net["convs"], w["conv_w"], w["conv_b"]):
        x = F.relu(F.conv2d(x, _t(cw), _t(cb), stride=s, padding=p))
    f = F.relu(F.linear(x.flatten(1), _t(w["fc_w"]), _t(w["fc_b"])))
    if net.get("meas_dim", 0):
        m = _t(meas.reshape(T * N, -1))
        for mw, mb in zip(w["meas_w"], w["meas_b"]):
            m = F.relu(F.linear(m, _t(mw), _t(mb)))
        f = torch.cat([f, m], dim=1)
    f = f.reshape(T, N, -1)
    H = net["rnn"]
    lstm = net.get("rnn_type", "gru") == "lstm"
    with torch.no_grad():
        core = (torch.nn.LSTM if lstm else torch.nn.GRU)(f.shape[2], H).double()
        core.weight_ih_l0.copy_(_t(w["rnn_w_ih"])); core.weight_hh_l0.copy_(_t(w["rnn_w_hh"]))
        core.bias_ih_l0.copy_(_t(w["rnn_b_ih"])); core.bias_hh_l0.copy_(_t(w["rnn_b_hh"]))
        s0 = _t(h0)
        if lstm:
            hs, (_, cT) = core(f, (s0[None, :, :H].contiguous(), s0[None, :, H:].contiguous()))
        else:
            hs, _ = core(f, s0[None])
            cT = None
        logits = F.linear(hs, _t(w["pi_w"]), _t(w["pi_b"]))
        value = F.linear(hs, _t(w["v_w"])[None], _t(w["v_b"]))[..., 0]
    return hs.numpy(), None if cT is None else cT[0].numpy(), logits.numpy(), value.numpy()


@pytest.mark.parametrize("net", [SMALL_STD, SMALL_LSTM, SMALL_FULL, SMALL_FULL_LSTM], ids=lambda n: n["name"])
def test_unroll_matches_torch_sequence_modules(ref, net):
    net = dict(net, rnn_type=net.get("rnn_type", "gru"))
    T, N = 6, 3
    w = wl.weights(net)
    obs, h0, done, meas = wl.trajectory_inputs(net, T, N)
    done[:] = 0
    out = ref.policy_unroll(net, w, obs, h0, done, meas=meas)
    hs, cT, logits, value = torch_unroll(net, w, obs, meas, h0)
    H = net["rnn"]
    # (the oracle carries the state as fp32 from step to step, the module in fp64)
    tol = dict(rtol=2e-6, atol=1e-6)
    np.testing.assert_allclose(out["h_seq"][:, :, :H], hs, **tol)
    if cT is not None:
        np.testing.assert_allclose(out["h_seq"][-1, :, H:], cT, **tol)
    np.testing.assert_allclose(out["logits"], logits, **tol)
    np.testing.assert_allclose(out["value"], value, **tol)
    # the sequence matters: the state at the last step differs from a one-step answer
    one = ref.policy_step(net, w, obs[-1], h0, done[-1], 0, 0, meas=None if meas is None else meas[-1])
    assert np.abs(one["h_out"] - out["h_seq"][-1]).max() > 1e-3


@pytest.mark.parametrize("net", [SMALL_STD, SMALL_FULL_LSTM], ids=lambda n: n["name"])
def test_done_restarts_a_trajectory_and_the_past_ignores_the_future(ref, net):
    net = dict(net, rnn_type=net.get("rnn_type", "gru"))
    T, N, t0 = 7, 3, 4
    w = wl.weights(net)
    obs, h0, done, meas = wl.trajectory_inputs(net, T, N)
    done[:] = 0
    done[t0, 1] = 1
    full = ref.policy_unroll(net, w, obs, h0, done, meas=meas)
    # trajectory 1 from t0 on = a fresh unroll of its remaining steps from a zero state
    zero = np.zeros_like(h0)
    d2 = np.zeros((T - t0, N), np.uint8)
    tail = ref.policy_unroll(net, w, obs[t0:], zero, d2, meas=None if meas is None else meas[t0:])
    for k in ("logits", "value", "h_seq"):
        assert np.array_equal(full[k][t0:, 1], tail[k][:, 1]), k
        # the other trajectories carried their state across t0
        assert not np.array_equal(full[k][t0:, 0], tail[k][:, 0]), k
    # causality: changing the frames from t0 on leaves every output before t0 as it was
    obs2 = obs.copy()
    obs2[t0:] = 255 - obs2[t0:]
    other = ref.policy_unroll(net, w, obs2, h0, done, meas=meas)
    for k in ("logits", "value", "h_seq"):
        assert np.array_equal(full[k][:t0], other[k][:t0]), k
        assert not np.array_equal(full[k][t0:], other[k][t0:]), k


def test_one_step_unroll_is_the_step_and_trajectories_are_independent(ref):
    net = dict(SMALL_STD, rnn_type="gru")
    w = wl.weights(net)
    obs, h0, done, _ = wl.trajectory_inputs(net, 3, 4)
    one = ref.policy_unroll(net, w, obs[:1], h0, done[:1])
    step = ref.policy_step(net, w, obs[0], h0, done[0], 5, 9)
    assert np.array_equal(one["logits"][0], step["logits"])
    assert np.array_equal(one["value"][0], step["value"])
    assert np.array_equal(one["h_seq"][0], step["h_out"])
    perm = np.array([2, 0, 3, 1])
    a = ref.policy_unroll(net, w, obs, h0, done)
    b = ref.policy_unroll(net, w, obs[:, perm], h0[perm], done[:, perm])
    for k in ("logits", "value", "h_seq"):
        assert np.array_equal(a[k][:, perm], b[k]), k
    with pytest.raises(ValueError):
        ref.policy_unroll(net, w, obs[:0], h0, done[:0])
