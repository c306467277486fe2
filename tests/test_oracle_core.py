"""Pins for the oracle's LSTM core and for the measurement-vector input of the "full"
architecture (paper, App. "Model architectures" and App. "VizDoom experiments"):
PyTorch's fp64 LSTMCell as the independent library routine, closed-form gate cases, the
whole step against a PyTorch composition, the reset of both state halves, and the
reduction of the measurement path to the plain network when its output is forced to zero.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2006_11751_amd import workloads as wl

SMALL_LSTM = dict(name="lstm_small", B=4, obs=(3, 36, 64), encoder="conv", convs=[(4, 8, 4, 0), (6, 4, 2, 0)],
                  fc=24, rnn=20, rnn_type="lstm", heads=[5, 3], dtype="fp32", p_done=0.4, steps=1,
                  obs_sub=0.0, obs_mul=wl.OBS_MUL, index=5, meas_dim=0, meas_hidden=[])
SMALL_FULL = dict(name="full_small", B=4, obs=(3, 36, 64), encoder="conv", convs=[(4, 8, 4, 0), (6, 4, 2, 0)],
                  fc=24, rnn=20, rnn_type="gru", meas_dim=7, meas_hidden=[10, 6], heads=[3, 3, 2, 2, 2, 8, 21],
                  dtype="fp32", p_done=0.4, steps=1, obs_sub=0.0, obs_mul=wl.OBS_MUL, index=6)
SMALL_FULL_LSTM = dict(SMALL_FULL, name="full_lstm_small", rnn_type="lstm", meas_hidden=[9])


def _t(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).double()


@pytest.mark.parametrize("n_in,H", [(1, 1), (7, 5), (24, 20)])
def test_lstm_cell_matches_torch_lstmcell(ref, n_in, H):
    rng = np.random.default_rng(n_in * 100 + H)
    w_ih, w_hh = rng.standard_normal((4 * H, n_in)).astype(np.float32), rng.standard_normal((4 * H, H)).astype(np.float32)
    b_ih, b_hh = rng.standard_normal(4 * H).astype(np.float32), rng.standard_normal(4 * H).astype(np.float32)
    x, h, c = rng.standard_normal(n_in), rng.standard_normal(H), rng.standard_normal(H)
    hn, cn = ref.lstm_cell(x, h, c, w_ih, w_hh, b_ih, b_hh)
    cell = torch.nn.LSTMCell(n_in, H).double()
    with torch.no_grad():
        cell.weight_ih.copy_(_t(w_ih)); cell.weight_hh.copy_(_t(w_hh))
        cell.bias_ih.copy_(_t(b_ih)); cell.bias_hh.copy_(_t(b_hh))
        th, tc = cell(torch.from_numpy(x)[None], (torch.from_numpy(h)[None], torch.from_numpy(c)[None]))
    np.testing.assert_allclose(hn, th[0].numpy(), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(cn, tc[0].numpy(), rtol=1e-13, atol=1e-14)


def test_lstm_cell_closed_forms(ref):
    H, n_in = 3, 2
    z = lambda *s: np.zeros(s, np.float32)
    x, h, c = np.array([0.3, -1.0]), np.array([0.5, -0.2, 0.9]), np.array([1.0, -2.0, 0.25])
    # no weights, no biases: every sigmoid is 1/2 and the candidate is 0
    hn, cn = ref.lstm_cell(x, h, c, z(4 * H, n_in), z(4 * H, H), z(4 * H), z(4 * H))
    np.testing.assert_allclose(cn, 0.5 * c, rtol=0, atol=1e-16)
    np.testing.assert_allclose(hn, 0.5 * np.tanh(0.5 * c), rtol=1e-15)
    # forget gate open, input gate shut: the cell state passes through unchanged
    b = z(4 * H)
    b[0:H], b[H:2 * H], b[3 * H:] = -60.0, 60.0, 60.0
    hn, cn = ref.lstm_cell(x, h, c, z(4 * H, n_in), z(4 * H, H), b, z(4 * H))
    np.testing.assert_allclose(cn, c, rtol=1e-15)
    np.testing.assert_allclose(hn, np.tanh(c), rtol=1e-15)
    # forget gate shut, input gate open, candidate bias split over both bias vectors
    b1, b2 = z(4 * H), z(4 * H)
    b1[0:H], b1[H:2 * H] = 60.0, -60.0
    b1[2 * H:3 * H], b2[2 * H:3 * H] = 0.25, 0.5          # g = tanh(0.75)
    b2[3 * H:] = math.log(3.0)                            # o = 3/4 up to the fp32 rounding of log 3
    o = 1.0 / (1.0 + math.exp(-float(np.float32(math.log(3.0)))))
    assert abs(o - 0.75) < 1e-8
    hn, cn = ref.lstm_cell(x, h, c, z(4 * H, n_in), z(4 * H, H), b1, b2)
    np.testing.assert_allclose(cn, np.full(H, math.tanh(0.75)), rtol=1e-14)
    np.testing.assert_allclose(hn, o * np.tanh(math.tanh(0.75)), rtol=1e-14)
    # gate rows are ordered i, f, g, o and x, h enter through their own matrices
    w_ih, w_hh = z(4 * H, n_in), z(4 * H, H)
    w_ih[2 * H + 1, 0] = 2.0      # candidate of unit 1 <- x[0]
    w_hh[3 * H + 2, 0] = -1.0     # output gate of unit 2 <- h[0]
    hn, cn = ref.lstm_cell(x, h, c, w_ih, w_hh, z(4 * H), z(4 * H))
    exp_c = 0.5 * c + 0.5 * np.array([0.0, math.tanh(0.6), 0.0])
    exp_o = np.array([0.5, 0.5, 1.0 / (1.0 + math.exp(0.5))])
    np.testing.assert_allclose(cn, exp_c, rtol=1e-15)
    np.testing.assert_allclose(hn, exp_o * np.tanh(exp_c), rtol=1e-15)


def torch_full_step(net, w, obs, meas, state, done):
    """Encoder + optional measurement encoder + GRU/LSTM core + heads in PyTorch fp64."""
    x = (torch.from_numpy(obs).double() - float(np.float32(net["obs_sub"]))) * float(np.float32(net["obs_mul"]))
    for (co, k, s, p), cw, cb in zip(net["convs"], w["conv_w"], w["conv_b"]):
        x = F.relu(F.conv2d(x, _t(cw), _t(cb), stride=s, padding=p))
    f = F.relu(F.linear(x.flatten(1), _t(w["fc_w"]), _t(w["fc_b"])))
    if net["meas_dim"]:
        m = _t(meas)
        for mw, mb in zip(w["meas_w"], w["meas_b"]):
            m = F.relu(F.linear(m, _t(mw), _t(mb)))
        f = torch.cat([f, m], dim=1)
    keep = (1.0 - torch.from_numpy(done.astype(np.float64)))[:, None]
    st = _t(state) * keep
    H = net["rnn"]
    with torch.no_grad():
        if net["rnn_type"] == "lstm":
            cell = torch.nn.LSTMCell(f.shape[1], H).double()
        else:
            cell = torch.nn.GRUCell(f.shape[1], H).double()
        cell.weight_ih.copy_(_t(w["rnn_w_ih"])); cell.weight_hh.copy_(_t(w["rnn_w_hh"]))
        cell.bias_ih.copy_(_t(w["rnn_b_ih"])); cell.bias_hh.copy_(_t(w["rnn_b_hh"]))
        if net["rnn_type"] == "lstm":
            hn, cn = cell(f, (st[:, :H], st[:, H:]))
            new_state = torch.cat([hn, cn], dim=1)
        else:
            hn = cell(f, st)
            new_state = hn
        logits = F.linear(hn, _t(w["pi_w"]), _t(w["pi_b"]))
        value = F.linear(hn, _t(w["v_w"])[None], _t(w["v_b"]))[:, 0]
    return new_state.numpy(), logits.numpy(), value.numpy()


@pytest.mark.parametrize("net", [SMALL_LSTM, SMALL_FULL, SMALL_FULL_LSTM], ids=lambda n: n["name"])
def test_step_matches_torch_composition(ref, net):
    B = net["B"]
    w = wl.weights(net)
    obs, state, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    done[0], done[1] = 1, 0
    meas = wl.measurements(net, 0, B)
    assert state.shape == (B, wl.state_dim(net))
    out = ref.policy_step(net, w, obs, state, done, 1, 0, meas=meas)
    ns, logits, value = torch_full_step(net, w, obs, meas, state, done)
    np.testing.assert_allclose(out["h_out"], ns, rtol=2e-7, atol=1e-7)
    np.testing.assert_allclose(out["logits"], logits, rtol=2e-7, atol=1e-7)
    np.testing.assert_allclose(out["value"], value, rtol=2e-7, atol=1e-7)
    # the indexed variant moves the same state rows through a table
    n_env = 2 * B + 1
    ids = np.array([5, 0, 8, 3], np.int32)
    table = np.zeros((n_env, wl.state_dim(net)), np.float32)
    table[ids] = state
    oi = ref.policy_step_indexed(net, w, obs, table, ids, done, 1, 0, meas=meas)
    np.testing.assert_array_equal(table[ids], out["h_out"])
    np.testing.assert_array_equal(oi["logits"], out["logits"])


def test_done_resets_both_halves_of_an_lstm_state(ref):
    net = SMALL_LSTM
    w = wl.weights(net)
    B = 4
    obs, state = wl.observations(net, 0, B), wl.initial_state(net, B)
    done = np.array([1, 0, 1, 0], np.uint8)
    a = ref.policy_step(net, w, obs, state, done, 1, 0)
    other = state.copy()
    other[0] = 5.0                      # h and c of a reset row: no effect at all
    other[2, net["rnn"]:] = -3.0        # c alone of a reset row: no effect either
    b = ref.policy_step(net, w, obs, other, done, 1, 0)
    for k in ("h_out", "logits", "value", "actions", "logp"):
        assert np.array_equal(a[k], b[k]), k
    zero = state.copy()
    zero[[0, 2]] = 0.0
    c = ref.policy_step(net, w, obs, zero, np.zeros(B, np.uint8), 1, 0)
    assert np.array_equal(a["h_out"], c["h_out"])
    # the cell half matters for rows that are not reset
    other2 = state.copy()
    other2[1, net["rnn"]:] += 0.5
    d = ref.policy_step(net, w, obs, other2, done, 1, 0)
    assert not np.array_equal(a["h_out"][1], d["h_out"][1])
    assert np.array_equal(a["h_out"][[0, 2, 3]], d["h_out"][[0, 2, 3]])


def test_silenced_measurement_path_reduces_to_the_plain_network(ref):
    """Last measurement layer forced to output zero: the step equals the network without
    the measurement input whose core sees only the first fc_dim input columns."""
    net = SMALL_FULL
    w = wl.weights(net)
    B = net["B"]
    obs, state, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    meas = wl.measurements(net, 0, B)
    w0 = dict(w)
    w0["meas_w"] = [w["meas_w"][0], np.zeros_like(w["meas_w"][1])]
    w0["meas_b"] = [w["meas_b"][0], -np.abs(w["meas_b"][1])]          # ReLU(negative) = 0
    a = ref.policy_step(net, w0, obs, state, done, 2, 3, meas=meas)
    plain = dict(net, meas_dim=0, meas_hidden=[])
    wp = dict(w, rnn_w_ih=np.ascontiguousarray(w["rnn_w_ih"][:, :net["fc"]]), meas_w=[], meas_b=[])
    b = ref.policy_step(plain, wp, obs, state, done, 2, 3)
    for k in ("h_out", "logits", "value", "actions", "logp"):
        assert np.array_equal(a[k], b[k]), k
    # and the measurement vector does matter otherwise
    c = ref.policy_step(net, w, obs, state, done, 2, 3, meas=meas)
    d = ref.policy_step(net, w, obs, state, done, 2, 3, meas=meas + 1.0)
    assert not np.array_equal(c["logits"], d["logits"])


def test_full_configuration_has_the_papers_action_space():
    net = wl.network(6)
    assert net["heads"] == [3, 3, 2, 2, 2, 8, 21]
    assert int(np.prod(net["heads"])) == 12096      # total in the paper's action-space table
    assert wl.core_input_dim(net) == 512 + 128 and wl.state_dim(wl.network(5)) == 1024
    w = wl.weights(wl.network(5))
    assert w["rnn_w_ih"].shape == (2048, 512) and w["rnn_w_hh"].shape == (2048, 512)
