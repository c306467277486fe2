"""Seeded synthetic workloads: network shapes and input generators.

Serves both the HIP library's callers and the CPU oracle's tests.  Holds none of
the method's arithmetic: only shapes, random draws and the bf16 rounding of the
weight *inputs*.  numpy only.

The observations stand in for the paper's VizDoom frames (128x72 RGB bytes,
paper Sec. 4.1): the step's cost does not depend on pixel content, and the paper
itself benchmarks one domain with random actions for the same reason (paper,
App. "Benchmarking details").
"""
import numpy as np

OBS_MUL = float(np.float32(1.0) / np.float32(255.0))  # the fp32 value nearest 1/255

_STD_CONVS = [(32, 8, 4, 0), (64, 4, 2, 0), (128, 3, 2, 0)]  # (cout, k, stride, pad)

# One entry per benchmark configuration: 0 tiny, 1 standard (the headline one),
# 2 bf16 standard at B=4096, 3 multi-discrete over 16 chained steps, 4 ResNet bf16.
CONFIGS = [
    dict(name="tiny", B=8, obs=(3, 36, 64), encoder="conv", convs=[(16, 8, 4, 0), (32, 4, 2, 0)],
         fc=128, rnn=128, heads=[6], dtype="fp32", p_done=0.1, steps=4),
    dict(name="standard", B=1024, obs=(3, 72, 128), encoder="conv", convs=_STD_CONVS,
         fc=512, rnn=512, heads=[7], dtype="fp32", p_done=0.05, steps=1),
    dict(name="standard_bf16", B=4096, obs=(3, 72, 128), encoder="conv", convs=_STD_CONVS,
         fc=512, rnn=512, heads=[7], dtype="bf16", p_done=0.05, steps=1),
    dict(name="multi_discrete", B=2048, obs=(3, 72, 128), encoder="conv", convs=_STD_CONVS,
         fc=512, rnn=512, heads=[3, 3, 2, 2, 2, 11], dtype="fp32", p_done=0.1, steps=16),
    dict(name="resnet_bf16", B=8192, obs=(3, 72, 128), encoder="resnet", stages=[16, 32, 32],
         blocks_per_stage=2, fc=256, rnn=256, heads=[15], dtype="bf16", p_done=0.05, steps=1),
    # the benchmark model as the paper describes it: the standard network with an LSTM core
    dict(name="standard_lstm", B=1024, obs=(3, 72, 128), encoder="conv", convs=_STD_CONVS,
         fc=512, rnn=512, rnn_type="lstm", heads=[7], dtype="fp32", p_done=0.05, steps=4),
    # the "full" architecture: measurement vector through two FC layers, appended to the
    # encoder's features; GRU core; the seven action heads of the paper's action-space table
    dict(name="full", B=1024, obs=(3, 72, 128), encoder="conv", convs=_STD_CONVS,
         fc=512, rnn=512, meas_dim=23, meas_hidden=[128, 128], heads=[3, 3, 2, 2, 2, 8, 21],
         dtype="fp32", p_done=0.05, steps=4),
]


def network(index, **overrides):
    """A copy of configuration `index` with normalisation defaults filled in."""
    cfg = dict(CONFIGS[index])
    cfg["index"] = index
    cfg.setdefault("obs_sub", 0.0)
    cfg.setdefault("obs_mul", OBS_MUL)
    cfg.setdefault("rnn_type", "gru")
    cfg.setdefault("meas_dim", 0)
    cfg.setdefault("meas_hidden", [])
    cfg.update(overrides)
    return cfg


def state_dim(net):
    """Floats per recurrent-state row: H for a GRU, 2H ([h | c]) for an LSTM."""
    return net["rnn"] * (2 if net.get("rnn_type", "gru") == "lstm" else 1)


def core_input_dim(net):
    hidden = net.get("meas_hidden", []) if net.get("meas_dim", 0) else []
    return net["fc"] + (hidden[-1] if hidden else 0)


def conv_out_hw(h, w, k, s, p):
    return (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1


def conv_tensor_shapes(net):
    """[(cout, cin, k)] for every convolution, in parameter order."""
    c = net["obs"][0]
    shapes = []
    if net["encoder"] == "conv":
        for co, k, _, _ in net["convs"]:
            shapes.append((co, c, k))
            c = co
    else:
        for ch in net["stages"]:
            shapes.append((ch, c, 3))
            c = ch
            for _ in range(net["blocks_per_stage"]):
                shapes.append((ch, ch, 3))
                shapes.append((ch, ch, 3))
    return shapes


def flat_size(net):
    c, h, w = net["obs"]
    if net["encoder"] == "conv":
        for co, k, s, p in net["convs"]:
            h, w = conv_out_hw(h, w, k, s, p)
            c = co
    else:
        for ch in net["stages"]:
            h, w = (h - 1) // 2 + 1, (w - 1) // 2 + 1
            c = ch
    return c * h * w


def round_to_bf16(a):
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(a.shape)


def weights(net, seed=None, dist="normal", rounded=True):
    """Parameters with variance 1/fan_in, biases too (non-zero on purpose): N(0, 1/fan_in)
    (the benchmark recipe), or for robustness tests "laplace", "student3" (heavy tails: Student t
    with 3 degrees of freedom) or "uniform", each scaled to that variance.
    For bf16 configurations every tensor is rounded to bf16 once, so that both
    the oracle and the library start from identical values; rounded=False leaves them
    as drawn (the caller then rounds the oracle's copy itself)."""
    seed = 1000 + net.get("index", 0) if seed is None else seed
    rng = np.random.default_rng(seed)

    def unit(shape):
        if dist == "normal":
            return rng.standard_normal(shape)
        if dist == "laplace":
            return rng.laplace(size=shape) / np.sqrt(2.0)
        if dist == "student3":
            return rng.standard_t(3, size=shape) / np.sqrt(3.0)
        if dist == "uniform":
            return rng.uniform(-1.0, 1.0, size=shape) * np.sqrt(3.0)
        raise ValueError(dist)

    def draw(shape, fan_in):
        a = (unit(shape) / np.sqrt(fan_in)).astype(np.float32)
        return round_to_bf16(a) if net["dtype"] == "bf16" and rounded else a

    w = {"conv_w": [], "conv_b": []}
    for co, ci, k in conv_tensor_shapes(net):
        fan = ci * k * k
        w["conv_w"].append(draw((co, ci, k, k), fan))
        w["conv_b"].append(draw((co,), fan))
    flat, fc, H, sumA = flat_size(net), net["fc"], net["rnn"], sum(net["heads"])
    w["fc_w"], w["fc_b"] = draw((fc, flat), flat), draw((fc,), flat)
    G = 4 if net.get("rnn_type", "gru") == "lstm" else 3      # gate blocks of the recurrent core
    cin = core_input_dim(net)
    w["rnn_w_ih"], w["rnn_b_ih"] = draw((G * H, cin), cin), draw((G * H,), cin)
    w["rnn_w_hh"], w["rnn_b_hh"] = draw((G * H, H), H), draw((G * H,), H)
    w["pi_w"], w["pi_b"] = draw((sumA, H), H), draw((sumA,), H)
    w["v_w"], w["v_b"] = draw((H,), H), draw((1,), H)
    # drawn last, so that networks without a measurement input keep their values
    w["meas_w"], w["meas_b"] = [], []
    n_prev = net.get("meas_dim", 0)
    for m in (net.get("meas_hidden", []) if n_prev else []):
        w["meas_w"].append(draw((m, n_prev), n_prev))
        w["meas_b"].append(draw((m,), n_prev))
        n_prev = m
    return w


def round_weights_to_bf16(w):
    """A copy of a parameter dict with every tensor rounded to bf16 (what a bf16 configuration
    defines its parameters to be)."""
    out = {}
    for k, v in w.items():
        out[k] = [round_to_bf16(a) for a in v] if isinstance(v, list) else round_to_bf16(v)
    return out


# Filter banks for the first convolution whose taps span a wide dynamic range within a channel,
# and the frames that expose them: the cases a per-channel fixed-point image of the bank handles
# worst.  (tap index = (channel, filter row, filter column) of conv_w[0][n])
CONV1_FAMILIES = ("dominant", "log_uniform", "zero_channel", "tiny_equal", "half_half_40",
                  "half_half_1000")


def conv1_family(net, w, kind, seed=77):
    """A copy of parameters w whose first filter bank is of the given kind."""
    rng = np.random.default_rng(seed)
    w = dict(w)
    a = np.array(w["conv_w"][0], dtype=np.float32, copy=True)
    co, ci, k, _ = a.shape
    std = 1.0 / np.sqrt(ci * k * k)
    if kind == "dominant":        # one tap 1000 times the typical one, the same tap in every filter
        a[:, ci - 1, 2, 3] = 1000.0 * std * rng.choice([-1.0, 1.0], size=co)
    elif kind == "log_uniform":   # magnitudes over four decades
        a = (10.0 ** rng.uniform(-4.0, 0.0, a.shape) * rng.choice([-1.0, 1.0], a.shape) * 4.0 * std)
    elif kind == "zero_channel":  # two filters that are zero everywhere
        a[3] = 0.0
        a[co - 1] = 0.0
    elif kind == "tiny_equal":    # every tap the same tiny value
        a[:] = 1e-6
    elif kind in ("half_half_40", "half_half_1000"):  # even filter columns 40x (1000x) the odd ones
        ratio = 40.0 if kind == "half_half_40" else 1000.0
        a = rng.choice([-1.0, 1.0], a.shape) * std
        a[..., 0::2] *= ratio
    else:
        raise ValueError(kind)
    w["conv_w"] = [a.astype(np.float32)] + list(w["conv_w"][1:])
    return w


def conv1_family_frames(net, kind, obs):
    """Frames that put the large taps of the family on dark pixels, i.e. on the byte whose
    normalised value is nearest zero (stride-4 8x8 filter, no padding: filter column q meets
    image columns = q mod 4, filter row p image rows = p mod 4)."""
    obs = obs.copy()
    dark = int(min(255, max(0, round(net["obs_sub"]))))
    if kind == "dominant":
        obs[:, -1, 2::4, 3::4] = dark
    elif kind in ("half_half_40", "half_half_1000"):
        obs[:, :, :, 0::2] = dark
    return obs


def observations(net, t=0, B=None, seed=None):
    B = net["B"] if B is None else B
    seed = 2000 + 100 * net.get("index", 0) + t if seed is None else seed
    rng = np.random.default_rng(seed)
    return rng.integers(0, 256, size=(B,) + tuple(net["obs"]), dtype=np.uint8)


def initial_state(net, B=None, seed=None):
    B = net["B"] if B is None else B
    seed = 3000 + net.get("index", 0) if seed is None else seed
    rng = np.random.default_rng(seed)
    return (0.1 * rng.standard_normal((B, state_dim(net)))).astype(np.float32)


def done_mask(net, t=0, B=None, seed=None):
    B = net["B"] if B is None else B
    seed = 4000 + 100 * net.get("index", 0) + t if seed is None else seed
    rng = np.random.default_rng(seed)
    return (rng.random(B) < net["p_done"]).astype(np.uint8)


def measurements(net, t=0, B=None, seed=None):
    """The "full" architecture's low-dimensional game information (health, ammunition, ...):
    here N(0, 1) fp32 [B, meas_dim], or None for networks without that input."""
    if not net.get("meas_dim", 0):
        return None
    B = net["B"] if B is None else B
    seed = 5000 + 100 * net.get("index", 0) + t if seed is None else seed
    rng = np.random.default_rng(seed)
    return rng.standard_normal((B, net["meas_dim"])).astype(np.float32)


def trajectory_inputs(net, T, N):
    """Inputs of the learner's forward pass over N trajectories of T steps, time-major: the
    per-step draws above stacked.  Returns obs [T,N,C,H,W] u8, h0 [N,state_dim] fp32, done [T,N]
    u8, meas [T,N,meas_dim] fp32 or None."""
    obs = np.stack([observations(net, t, N) for t in range(T)])
    done = np.stack([done_mask(net, t, N) for t in range(T)])
    meas = np.stack([measurements(net, t, N) for t in range(T)]) if net.get("meas_dim", 0) else None
    return obs, initial_state(net, N), done, meas


PHILOX_SEED = 1


# ---- learner-side loss (paper, hyperparameter table of App. "VizDoom experiments") ----

LOSS_HP = dict(gamma=0.99, rho_bar=1.0, c_bar=1.0, clip=1.1, critic_coef=0.5, entropy_coef=0.003)


def loss_config(heads=(7,), T=32, N=64, **overrides):
    """Rollout length 32 and 2048 samples per batch = 64 trajectories, as in the paper."""
    hp = dict(LOSS_HP, heads=list(heads), T=T, N=N)
    hp.update(overrides)
    return hp


def trajectories(hp, seed=6000):
    """Seeded stand-in for a batch of trajectories, time-major.  The behaviour log-probability
    is that of a uniform policy plus noise and the logits are small, so the importance ratios
    scatter around 1 on both sides of the clipping range."""
    rng = np.random.default_rng(seed)
    T, N, heads = hp["T"], hp["N"], hp["heads"]
    logits = (0.3 * rng.standard_normal((T, N, sum(heads)))).astype(np.float32)
    actions = np.stack([rng.integers(0, a, size=(T, N)) for a in heads], axis=-1).astype(np.int32)
    logp_mu = (-float(np.sum(np.log(heads))) + 0.15 * rng.standard_normal((T, N))).astype(np.float32)
    values = rng.standard_normal((T + 1, N)).astype(np.float32)
    rewards = (rng.standard_normal((T, N)) * (rng.random((T, N)) < 0.2)).astype(np.float32)
    dones = (rng.random((T, N)) < 0.03).astype(np.uint8)
    return dict(logits=logits, actions=actions, logp_mu=logp_mu, values=values, rewards=rewards, dones=dones)
