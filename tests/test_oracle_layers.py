"""Pins for the oracle's layer routines: hand cases, closed forms and PyTorch's
CPU fp64 routines as an independent opinion (the oracle itself calls no library).
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- convolution

def test_conv_one_pixel_hand_case(ref):
    # 1 channel, 1x1 image, 1x1 kernel: out = relu(w*x + b); numbers chosen exact in fp32.
    x = np.array([[[0.5]]])
    out = ref.conv2d(x, np.array([[[[-2.0]]]]), np.array([0.25]), 1, 0, True)
    assert out.shape == (1, 1, 1) and out[0, 0, 0] == 0.0          # relu(-0.75)
    out = ref.conv2d(x, np.array([[[[-2.0]]]]), np.array([0.25]), 1, 0, False)
    assert out[0, 0, 0] == -0.75
    out = ref.conv2d(x, np.array([[[[3.0]]]]), np.array([0.25]), 1, 0, True)
    assert out[0, 0, 0] == 1.75


def test_conv_two_by_two_hand_case(ref):
    # 2 input channels, 2x3 image, 2x2 kernel, stride 1: two outputs computed by hand.
    x = np.array([[[1, 2, 3], [4, 5, 6]], [[-1, 0, 1], [2, -2, 0.5]]], dtype=np.float64)
    w = np.array([[[[1, 0], [0, -1]], [[2, 1], [0.5, 0]]]], dtype=np.float32)
    b = np.array([0.5], dtype=np.float32)
    # out[0,0,0] = .5 + (1*1 - 1*5) + (2*-1 + 1*0 + .5*2) = .5 - 4 - 1 = -4.5
    # out[0,0,1] = .5 + (1*2 - 1*6) + (2*0 + 1*1 + .5*-2) = .5 - 4 + 0 = -3.5
    out = ref.conv2d(x, w, b, 1, 0, False)
    assert out.shape == (1, 1, 2)
    assert out[0, 0, 0] == -4.5 and out[0, 0, 1] == -3.5


def test_conv_delta_kernel_is_strided_crop(ref):
    rng = _rng(1)
    C, H, W, k, s = 3, 11, 14, 4, 2
    x = rng.standard_normal((C, H, W))
    for c0, p0, q0 in [(0, 0, 0), (2, 3, 1), (1, 1, 3)]:
        w = np.zeros((1, C, k, k), np.float32)
        w[0, c0, p0, q0] = 1.0
        out = ref.conv2d(x, w, np.zeros(1, np.float32), s, 0, False)
        Ho, Wo = (H - k) // s + 1, (W - k) // s + 1
        want = x[c0, p0:p0 + s * Ho:s, q0:q0 + s * Wo:s]
        assert np.array_equal(out[0], want)


def test_conv_floor_ignores_trailing_row_and_column(ref):
    # 17x31 input, 4x4 stride 2 -> 7x14: input row 16 and column 30 are never read.
    rng = _rng(2)
    x = rng.standard_normal((2, 17, 31))
    w = rng.standard_normal((3, 2, 4, 4)).astype(np.float32)
    b = rng.standard_normal(3).astype(np.float32)
    a = ref.conv2d(x, w, b, 2, 0, True)
    assert a.shape == (3, 7, 14)
    y = x.copy()
    y[:, 16, :] = 1e6
    y[:, :, 30] = -1e6
    assert np.array_equal(a, ref.conv2d(y, w, b, 2, 0, True))
    y = x.copy()
    y[:, 15, 29] += 1.0           # the last row/column that IS read
    assert not np.array_equal(a, ref.conv2d(y, w, b, 2, 0, True))


@pytest.mark.parametrize("C,H,W,O,k,s,p,relu", [
    (3, 36, 64, 16, 8, 4, 0, True), (16, 8, 15, 32, 4, 2, 0, True), (5, 9, 7, 4, 3, 1, 1, False),
    (2, 10, 13, 3, 3, 2, 1, True), (4, 7, 14, 6, 3, 2, 0, True), (1, 5, 6, 2, 5, 1, 2, False),
])
def test_conv_matches_torch_fp64(ref, C, H, W, O, k, s, p, relu):
    rng = _rng(10 + C + k)
    x = rng.standard_normal((C, H, W))
    w = rng.standard_normal((O, C, k, k)).astype(np.float32)
    b = rng.standard_normal(O).astype(np.float32)
    got = ref.conv2d(x, w, b, s, p, relu)
    want = F.conv2d(torch.from_numpy(x)[None], torch.from_numpy(w).double(),
                    torch.from_numpy(b).double(), stride=s, padding=p)[0]
    if relu:
        want = want.clamp_min(0)
    assert got.shape == tuple(want.shape)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-12)


def test_conv_rejects_empty_output(ref):
    with pytest.raises(ValueError):
        ref.conv2d(np.zeros((1, 3, 3)), np.zeros((1, 1, 4, 4), np.float32), np.zeros(1, np.float32),
                   1, 0, False)


# -------------------------------------------------------------------- pooling

def test_maxpool_hand_case_negative_border(ref):
    # All-negative 4x4 image.  Zero padding would give 0 everywhere; windows
    # aligned at 2i..2i+2 would give -3 instead of -2 at output (0, 1).
    x = np.array([[[-1, -2, -3, -4],
                   [-5, -6, -7, -8],
                   [-9, -10, -11, -12],
                   [-13, -14, -15, -16]]], dtype=np.float64)
    out = ref.maxpool3x3s2p1(x)
    # output (i,j) covers rows 2i-1..2i+1, cols 2j-1..2j+1 clipped:
    # (0,0): rows 0-1, cols 0-1 -> -1 ; (0,1): rows 0-1, cols 1-3 -> -2
    # (1,0): rows 1-3, cols 0-1 -> -5 ; (1,1): rows 1-3, cols 1-3 -> -6
    assert np.array_equal(out, np.array([[[-1, -2], [-5, -6]]], dtype=np.float64))


@pytest.mark.parametrize("C,H,W", [(2, 72, 128), (3, 9, 16), (1, 5, 7), (2, 1, 1), (1, 2, 3)])
def test_maxpool_matches_torch(ref, C, H, W):
    x = _rng(C * H + W).standard_normal((C, H, W))
    want = F.max_pool2d(torch.from_numpy(x)[None], kernel_size=3, stride=2, padding=1)[0].numpy()
    got = ref.maxpool3x3s2p1(x)
    assert got.shape == want.shape and np.array_equal(got, want)


# --------------------------------------------------------------------- linear

def test_linear_identity_and_hand(ref):
    x = np.array([1.5, -2.0, 0.25])
    assert np.array_equal(ref.linear(x, np.eye(3, dtype=np.float32), np.zeros(3, np.float32), False), x)
    assert np.array_equal(ref.linear(x, np.eye(3, dtype=np.float32), np.zeros(3, np.float32), True),
                          np.array([1.5, 0.0, 0.25]))
    # rows are outputs, columns inputs: a non-symmetric matrix catches a transposed operand
    w = np.array([[1, 2, 3], [0, -1, 4]], np.float32)
    got = ref.linear(x, w, np.array([10, 20], np.float32), False)
    assert np.array_equal(got, np.array([10 + 1.5 - 4 + 0.75, 20 + 2.0 + 1.0]))


def test_linear_matches_torch(ref):
    rng = _rng(5)
    x = rng.standard_normal(37)
    w = rng.standard_normal((11, 37)).astype(np.float32)
    b = rng.standard_normal(11).astype(np.float32)
    want = F.linear(torch.from_numpy(x), torch.from_numpy(w).double(), torch.from_numpy(b).double())
    np.testing.assert_allclose(ref.linear(x, w, b, False), want.numpy(), rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------------ GRU

def _zeros_gru(n_in, H):
    return (np.zeros((3 * H, n_in), np.float32), np.zeros((3 * H, H), np.float32),
            np.zeros(3 * H, np.float32), np.zeros(3 * H, np.float32))


def test_gru_zero_weights_halves_state(ref):
    # r = z = 1/2, n = tanh(0) = 0  =>  h' = h/2
    rng = _rng(6)
    x, h = rng.standard_normal(5), rng.standard_normal(4)
    w_ih, w_hh, b_ih, b_hh = _zeros_gru(5, 4)
    np.testing.assert_allclose(ref.gru_cell(x, h, w_ih, w_hh, b_ih, b_hh), 0.5 * h, rtol=1e-15)


def test_gru_update_gate_limits(ref):
    rng = _rng(7)
    n_in, H = 6, 5
    x, h = rng.standard_normal(n_in), rng.standard_normal(H)
    w_ih = rng.standard_normal((3 * H, n_in)).astype(np.float32)
    w_hh = rng.standard_normal((3 * H, H)).astype(np.float32)
    b_ih = rng.standard_normal(3 * H).astype(np.float32)
    b_hh = rng.standard_normal(3 * H).astype(np.float32)
    big = b_ih.copy()
    big[H:2 * H] = 80.0                     # z -> 1: the state is kept
    np.testing.assert_allclose(ref.gru_cell(x, h, w_ih, w_hh, big, b_hh), h, rtol=1e-12)
    small = b_ih.copy()
    small[H:2 * H] = -80.0                  # z -> 0: the state becomes the candidate n
    wi, wh = w_ih.astype(np.float64), w_hh.astype(np.float64)
    r = 1 / (1 + np.exp(-(wi[:H] @ x + b_ih[:H] + wh[:H] @ h + b_hh[:H])))
    n = np.tanh(wi[2 * H:] @ x + b_ih[2 * H:] + r * (wh[2 * H:] @ h + b_hh[2 * H:]))
    np.testing.assert_allclose(ref.gru_cell(x, h, w_ih, w_hh, small, b_hh), n, rtol=1e-12, atol=1e-15)


def test_gru_one_unit_hand_case(ref):
    # 1 input, 1 unit; every pre-activation chosen so the result can be checked by hand:
    # x = 1, h = 0.5; W_ir = W_hr = 0, b = 0 -> r = 1/2
    # W_iz = 0, W_hz = 0 -> z = 1/2
    # W_in = 0, b_in = 0, W_hn = 2, b_hn = 1 -> n = tanh(r * (2*0.5 + 1)) = tanh(1)
    # h' = 0.5 * tanh(1) + 0.5 * 0.5
    w_ih = np.zeros((3, 1), np.float32)
    w_hh = np.array([[0], [0], [2]], np.float32)
    b_ih = np.zeros(3, np.float32)
    b_hh = np.array([0, 0, 1], np.float32)
    got = ref.gru_cell(np.array([1.0]), np.array([0.5]), w_ih, w_hh, b_ih, b_hh)
    assert abs(got[0] - (0.5 * np.tanh(1.0) + 0.25)) < 1e-15
    # the reset gate multiplies only the recurrent part: moving the 1 from b_hn to b_in changes n
    got2 = ref.gru_cell(np.array([1.0]), np.array([0.5]), w_ih, w_hh, np.array([0, 0, 1], np.float32),
                        np.zeros(3, np.float32))
    assert abs(got2[0] - (0.5 * np.tanh(1.0 + 0.5 * 1.0) + 0.25)) < 1e-15


def test_gru_bounded(ref):
    rng = _rng(8)
    for _ in range(20):
        n_in, H = 7, 9
        x, h = 3 * rng.standard_normal(n_in), 2 * rng.standard_normal(H)
        args = (rng.standard_normal((3 * H, n_in)), rng.standard_normal((3 * H, H)),
                rng.standard_normal(3 * H), rng.standard_normal(3 * H))
        out = ref.gru_cell(x, h, *args)
        assert np.all(np.abs(out) <= np.maximum(np.abs(h), 1.0) + 1e-12)


def test_gru_matches_torch_grucell(ref):
    rng = _rng(9)
    n_in, H = 13, 10
    cell = torch.nn.GRUCell(n_in, H).double()
    w_ih = rng.standard_normal((3 * H, n_in)).astype(np.float32)
    w_hh = rng.standard_normal((3 * H, H)).astype(np.float32)
    b_ih = rng.standard_normal(3 * H).astype(np.float32)
    b_hh = rng.standard_normal(3 * H).astype(np.float32)
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(w_ih).double())
        cell.weight_hh.copy_(torch.from_numpy(w_hh).double())
        cell.bias_ih.copy_(torch.from_numpy(b_ih).double())
        cell.bias_hh.copy_(torch.from_numpy(b_hh).double())
        x, h = rng.standard_normal(n_in), rng.standard_normal(H)
        want = cell(torch.from_numpy(x)[None], torch.from_numpy(h)[None])[0].numpy()
    np.testing.assert_allclose(ref.gru_cell(x, h, w_ih, w_hh, b_ih, b_hh), want, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------ residual encoder

def _tiny_resnet():
    return dict(obs=(2, 9, 12), encoder="resnet", stages=[3, 4], blocks_per_stage=2, fc=8, rnn=8,
                heads=[3], dtype="fp32", obs_sub=0.0, obs_mul=1.0, index=0, p_done=0.0, B=1)


def test_resnet_zero_block_weights_is_identity(ref):
    # With the block convolutions zeroed each block adds nothing, so the encoder is
    # relu(pool(conv(...pool(conv(x))))) -- checked against torch's conv/pool.
    from paper_2006_11751_amd import workloads as wl
    net = _tiny_resnet()
    w = wl.weights(net, seed=3)
    per_stage = 1 + 2 * net["blocks_per_stage"]
    for i in range(len(w["conv_w"])):
        if i % per_stage != 0:
            w["conv_w"][i][:] = 0
            w["conv_b"][i][:] = 0
    x = _rng(4).standard_normal(net["obs"])
    t = torch.from_numpy(x)[None]
    for s in range(len(net["stages"])):
        i = s * per_stage
        t = F.conv2d(t, torch.from_numpy(w["conv_w"][i]).double(), torch.from_numpy(w["conv_b"][i]).double(),
                     padding=1)
        t = F.max_pool2d(t, 3, 2, 1)
    want = t.clamp_min(0)[0].numpy()
    got = ref.resnet_encoder(net, w, x)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_resnet_matches_torch_composition(ref):
    from paper_2006_11751_amd import workloads as wl
    net = _tiny_resnet()
    w = wl.weights(net, seed=5)
    x = _rng(6).standard_normal(net["obs"])
    t = torch.from_numpy(x)[None]
    i = 0

    def conv(t, i):
        return F.conv2d(t, torch.from_numpy(w["conv_w"][i]).double(),
                        torch.from_numpy(w["conv_b"][i]).double(), padding=1)

    for _ in net["stages"]:
        t = F.max_pool2d(conv(t, i), 3, 2, 1)
        i += 1
        for _ in range(net["blocks_per_stage"]):
            u = conv(F.relu(conv(F.relu(t), i)), i + 1)
            t = t + u
            i += 2
    want = F.relu(t)[0].numpy()
    got = ref.resnet_encoder(net, w, x)
    assert got.shape == want.shape == (4, 3, 3)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)
