"""ctypes access to the CPU oracle (oracle/sf_oracle.c).

Test infrastructure only: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product package.  Holds no arithmetic
of its own: every function here marshals numpy arrays into the C routines.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# SF_ORACLE_SANITIZE=1: a second build with AddressSanitizer and UndefinedBehaviorSanitizer (no
# OpenMP), for running the CPU tests under the sanitizers:
#   LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
#       SF_ORACLE_SANITIZE=1 python -m pytest tests -m "not gpu"
_SANITIZE = os.environ.get("SF_ORACLE_SANITIZE", "") not in ("", "0")
_SO = os.path.join(_HERE, "libsf_oracle_san.so" if _SANITIZE else "libsf_oracle.so")
_SRC = os.path.join(_HERE, "sf_oracle.c")

MAX_CONV, MAX_STAGE, MAX_HEADS, MAX_CONV_TENSORS = 4, 4, 16, 20
MAX_MEAS_LAYERS = 2


def build(force=True):
    """Compile the oracle with gcc (no fast-math, no contraction)."""
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "sf_oracle.h"))):
        return _SO
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC",
           "-shared", "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
    if _SANITIZE:
        cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
               "-Wall", "-Wextra", "-Wno-unknown-pragmas", "-o", _SO, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _SO


class RefNet(C.Structure):
    _fields_ = [
        ("obs_c", C.c_int32), ("obs_h", C.c_int32), ("obs_w", C.c_int32),
        ("encoder", C.c_int32),
        ("n_conv", C.c_int32),
        ("conv_cout", C.c_int32 * MAX_CONV), ("conv_k", C.c_int32 * MAX_CONV),
        ("conv_stride", C.c_int32 * MAX_CONV), ("conv_pad", C.c_int32 * MAX_CONV),
        ("n_stage", C.c_int32), ("stage_ch", C.c_int32 * MAX_STAGE),
        ("blocks_per_stage", C.c_int32),
        ("fc_dim", C.c_int32), ("rnn_dim", C.c_int32),
        ("n_heads", C.c_int32), ("head_sizes", C.c_int32 * MAX_HEADS),
        ("obs_sub", C.c_float), ("obs_mul", C.c_float),
        ("rnn_type", C.c_int32), ("meas_dim", C.c_int32), ("n_meas_layers", C.c_int32),
        ("meas_hidden", C.c_int32 * MAX_MEAS_LAYERS),
    ]


_FP = C.POINTER(C.c_float)


class RefParams(C.Structure):
    _fields_ = [
        ("conv_w", _FP * MAX_CONV_TENSORS), ("conv_b", _FP * MAX_CONV_TENSORS),
        ("fc_w", _FP), ("fc_b", _FP),
        ("rnn_w_ih", _FP), ("rnn_w_hh", _FP), ("rnn_b_ih", _FP), ("rnn_b_hh", _FP),
        ("pi_w", _FP), ("pi_b", _FP), ("v_w", _FP), ("v_b", _FP),
        ("meas_w", _FP * MAX_MEAS_LAYERS), ("meas_b", _FP * MAX_MEAS_LAYERS),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        L = C.CDLL(_SO)
        L.ref_conv2d.restype = C.c_int
        L.ref_flat_size.restype = C.c_int64
        L.ref_policy_step.restype = C.c_int
        L.ref_policy_step_indexed.restype = C.c_int
        L.ref_num_threads.restype = C.c_int
        L.ref_bits_to_uniform.restype = C.c_float
        L.ref_bits_to_uniform.argtypes = [C.c_uint32]
        L.ref_gumbel.restype = C.c_float
        L.ref_gumbel.argtypes = [C.c_float]
        _lib = L
    return _lib


def _p(a, t=C.c_void_p):
    return a.ctypes.data_as(t)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def make_net(net):
    """net: dict as produced by workloads.network()."""
    r = RefNet()
    r.obs_c, r.obs_h, r.obs_w = net["obs"]
    r.encoder = 1 if net["encoder"] == "resnet" else 0
    if r.encoder == 0:
        r.n_conv = len(net["convs"])
        for i, (co, k, s, p) in enumerate(net["convs"]):
            r.conv_cout[i], r.conv_k[i], r.conv_stride[i], r.conv_pad[i] = co, k, s, p
    else:
        r.n_stage = len(net["stages"])
        for i, ch in enumerate(net["stages"]):
            r.stage_ch[i] = ch
        r.blocks_per_stage = net["blocks_per_stage"]
    r.fc_dim, r.rnn_dim = net["fc"], net["rnn"]
    r.n_heads = len(net["heads"])
    for i, a in enumerate(net["heads"]):
        r.head_sizes[i] = a
    r.obs_sub, r.obs_mul = net["obs_sub"], net["obs_mul"]
    r.rnn_type = 1 if net.get("rnn_type", "gru") == "lstm" else 0
    r.meas_dim = net.get("meas_dim", 0)
    hidden = net.get("meas_hidden", []) if r.meas_dim else []
    r.n_meas_layers = len(hidden)
    for i, m in enumerate(hidden):
        r.meas_hidden[i] = m
    return r


def state_dim(net):
    return net["rnn"] * (2 if net.get("rnn_type", "gru") == "lstm" else 1)


def make_params(w):
    """w: dict of fp32 numpy arrays as produced by workloads.weights().
    Returns (RefParams, keepalive list)."""
    p = RefParams()
    keep = []

    def fp(a):
        a = _f32(a)
        keep.append(a)
        return _p(a, _FP)

    for i, (cw, cb) in enumerate(zip(w["conv_w"], w["conv_b"])):
        p.conv_w[i] = fp(cw)
        p.conv_b[i] = fp(cb)
    for name in ("fc_w", "fc_b", "rnn_w_ih", "rnn_w_hh", "rnn_b_ih", "rnn_b_hh", "pi_w", "pi_b",
                 "v_w", "v_b"):
        setattr(p, name, fp(w[name]))
    for i, (mw, mb) in enumerate(zip(w.get("meas_w", []), w.get("meas_b", []))):
        p.meas_w[i] = fp(mw)
        p.meas_b[i] = fp(mb)
    return p, keep


def flat_size(net):
    return int(lib().ref_flat_size(C.byref(make_net(net))))


def num_threads():
    return int(lib().ref_num_threads())


def _meas_arg(net, meas, B):
    if not net.get("meas_dim", 0):
        return None, None
    meas = _f32(meas)
    assert meas.shape == (B, net["meas_dim"])
    return meas, _p(meas)


def policy_step(net, w, obs, h_in, done, seed, step, want_logits=True, want_margin=True, meas=None):
    """Run one step on host arrays; returns a dict of numpy outputs.  h_in / h_out rows hold
    state_dim(net) floats ([h | c] for an LSTM)."""
    L = lib()
    rn = make_net(net)
    rp, keep = make_params(w)
    B = int(obs.shape[0])
    obs = np.ascontiguousarray(obs, dtype=np.uint8)
    h_in = _f32(h_in)
    done = np.ascontiguousarray(done, dtype=np.uint8)
    nh, sumA, H = len(net["heads"]), int(sum(net["heads"])), state_dim(net)
    meas, meas_p = _meas_arg(net, meas, B)
    out = {
        "actions": np.zeros((B, nh), np.int32), "logp": np.zeros(B, np.float32),
        "value": np.zeros(B, np.float32), "h_out": np.zeros((B, H), np.float32),
        "logits": np.zeros((B, sumA), np.float32) if want_logits else None,
        "margin": np.zeros((B, nh), np.float32) if want_margin else None,
    }
    rc = L.ref_policy_step(
        C.byref(rn), C.byref(rp), C.c_int32(B), _p(obs), meas_p, _p(h_in), _p(done),
        C.c_uint64(seed), C.c_uint64(step), _p(out["actions"]), _p(out["logp"]),
        _p(out["value"]), _p(out["h_out"]),
        _p(out["logits"]) if want_logits else None, _p(out["margin"]) if want_margin else None)
    if rc != 0:
        raise ValueError("ref_policy_step rejected the network description")
    del keep
    return out


def policy_step_indexed(net, w, obs, h_table, env_ids, done, seed, step, meas=None):
    """One step on rows that name environments of a state table; h_table is updated in place."""
    L = lib()
    rn = make_net(net)
    rp, keep = make_params(w)
    B = int(obs.shape[0])
    obs = np.ascontiguousarray(obs, dtype=np.uint8)
    assert h_table.dtype == np.float32 and h_table.flags["C_CONTIGUOUS"]
    env_ids = np.ascontiguousarray(env_ids, dtype=np.int32)
    done = np.ascontiguousarray(done, dtype=np.uint8)
    nh, sumA = len(net["heads"]), int(sum(net["heads"]))
    meas, meas_p = _meas_arg(net, meas, B)
    assert h_table.shape[1] == state_dim(net)
    out = {
        "actions": np.zeros((B, nh), np.int32), "logp": np.zeros(B, np.float32),
        "value": np.zeros(B, np.float32), "logits": np.zeros((B, sumA), np.float32),
        "margin": np.zeros((B, nh), np.float32),
    }
    rc = L.ref_policy_step_indexed(
        C.byref(rn), C.byref(rp), C.c_int32(B), _p(obs), meas_p, _p(h_table), C.c_int32(h_table.shape[0]),
        _p(env_ids), _p(done), C.c_uint64(seed), C.c_uint64(step), _p(out["actions"]),
        _p(out["logp"]), _p(out["value"]), _p(out["logits"]), _p(out["margin"]))
    if rc == -2:
        raise ValueError("env_ids out of range or not distinct")
    if rc != 0:
        raise ValueError("ref_policy_step_indexed rejected the network description")
    del keep
    return out


def policy_unroll(net, w, obs, h0, done, meas=None):
    """The learner's forward pass: obs [T,N,C,H,W] u8, h0 [N,state_dim], done [T,N] (meas
    [T,N,meas_dim]); returns dict(logits [T,N,sumA], value [T,N], h_seq [T,N,state_dim])."""
    L = lib()
    rn = make_net(net)
    rp, keep = make_params(w)
    T, N = int(obs.shape[0]), int(obs.shape[1])
    obs = np.ascontiguousarray(obs, dtype=np.uint8)
    h0 = _f32(h0)
    done = np.ascontiguousarray(done, dtype=np.uint8)
    assert done.shape == (T, N) and h0.shape == (N, state_dim(net))
    sumA, S = int(sum(net["heads"])), state_dim(net)
    meas_p = None
    if net.get("meas_dim", 0) > 0:
        meas = _f32(meas)
        assert meas.shape == (T, N, net["meas_dim"])
        meas_p = _p(meas)
    out = {"logits": np.zeros((T, N, sumA), np.float32), "value": np.zeros((T, N), np.float32),
           "h_seq": np.zeros((T, N, S), np.float32)}
    rc = L.ref_policy_unroll(C.byref(rn), C.byref(rp), C.c_int32(T), C.c_int32(N), _p(obs), meas_p, _p(h0),
                             _p(done), _p(out["logits"]), _p(out["value"]), _p(out["h_seq"]))
    if rc != 0:
        raise ValueError("ref_policy_unroll rejected the arguments")
    del keep
    return out


class RefLossCfg(C.Structure):
    _fields_ = [("T", C.c_int32), ("N", C.c_int32), ("n_heads", C.c_int32),
                ("head_sizes", C.c_int32 * MAX_HEADS),
                ("gamma", C.c_float), ("rho_bar", C.c_float), ("c_bar", C.c_float), ("clip", C.c_float),
                ("critic_coef", C.c_float), ("entropy_coef", C.c_float)]


def appo_loss(hp, logits, actions, logp_mu, values, rewards, dones):
    """hp: dict(heads, gamma, rho_bar, c_bar, clip, critic_coef, entropy_coef); arrays
    time-major: logits [T,N,sumA], actions [T,N,nh], logp_mu/rewards/dones [T,N], values [T+1,N].
    Returns dict(vs, adv, loss[4], dlogits, dvalues) in fp64."""
    T, N, sumA = logits.shape
    cfg = RefLossCfg()
    cfg.T, cfg.N, cfg.n_heads = T, N, len(hp["heads"])
    for i, a in enumerate(hp["heads"]):
        cfg.head_sizes[i] = a
    for k in ("gamma", "rho_bar", "c_bar", "clip", "critic_coef", "entropy_coef"):
        setattr(cfg, k, hp[k])
    logits, logp_mu, values, rewards = _f32(logits), _f32(logp_mu), _f32(values), _f32(rewards)
    actions = np.ascontiguousarray(actions, dtype=np.int32)
    dones = np.ascontiguousarray(dones, dtype=np.uint8)
    assert sumA == sum(hp["heads"]) and values.shape == (T + 1, N) and actions.shape == (T, N, len(hp["heads"]))
    out = dict(vs=np.zeros((T, N)), adv=np.zeros((T, N)), loss=np.zeros(4), dlogits=np.zeros((T, N, sumA)),
               dvalues=np.zeros((T, N)))
    L = lib()
    L.ref_appo_loss.restype = C.c_int
    rc = L.ref_appo_loss(C.byref(cfg), _p(logits), _p(actions), _p(logp_mu), _p(values), _p(rewards), _p(dones),
                         _p(out["vs"]), _p(out["adv"]), _p(out["loss"]), _p(out["dlogits"]), _p(out["dvalues"]))
    if rc != 0:
        raise ValueError("ref_appo_loss rejected its arguments")
    return out


# ---- building blocks ---------------------------------------------------------

def conv2d(x, w, b, stride, pad, relu):
    x = _f64(x)
    w = _f32(w)
    b = _f32(b)
    Cc, H, W = x.shape
    O, _, k, _ = w.shape
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    out = np.zeros((O, max(Ho, 0), max(Wo, 0)), np.float64)
    rc = lib().ref_conv2d(_p(x), Cc, H, W, _p(w), _p(b), O, k, stride, pad, int(relu), _p(out))
    if rc != 0:
        raise ValueError("empty convolution output")
    return out


def maxpool3x3s2p1(x):
    x = _f64(x)
    Cc, H, W = x.shape
    out = np.zeros((Cc, (H - 1) // 2 + 1, (W - 1) // 2 + 1), np.float64)
    lib().ref_maxpool3x3s2p1(_p(x), Cc, H, W, _p(out))
    return out


def linear(x, w, b, relu):
    x = _f64(x)
    w = _f32(w)
    b = _f32(b)
    out = np.zeros(w.shape[0], np.float64)
    lib().ref_linear(_p(x), x.shape[0], _p(w), _p(b), w.shape[0], int(relu), _p(out))
    return out


def lstm_cell(x, h, c, w_ih, w_hh, b_ih, b_hh):
    x, h, c = _f64(x), _f64(h), _f64(c)
    w_ih, w_hh, b_ih, b_hh = _f32(w_ih), _f32(w_hh), _f32(b_ih), _f32(b_hh)
    hn, cn = np.zeros(h.shape[0], np.float64), np.zeros(h.shape[0], np.float64)
    lib().ref_lstm_cell(_p(x), x.shape[0], _p(h), _p(c), h.shape[0], _p(w_ih), _p(w_hh), _p(b_ih),
                        _p(b_hh), _p(hn), _p(cn))
    return hn, cn


def gru_cell(x, h, w_ih, w_hh, b_ih, b_hh):
    x = _f64(x)
    h = _f64(h)
    out = np.zeros_like(h)
    lib().ref_gru_cell(_p(x), x.shape[0], _p(h), h.shape[0], _p(_f32(w_ih)), _p(_f32(w_hh)),
                       _p(_f32(b_ih)), _p(_f32(b_hh)), _p(out))
    return out


def resnet_encoder(net, w, x):
    rn = make_net(net)
    rp, keep = make_params(w)
    x = _f64(x)
    out = np.zeros(flat_size(net), np.float64)
    hf, wf = C.c_int(), C.c_int()
    lib().ref_resnet_encoder(C.byref(rn), C.byref(rp), _p(x), _p(out), C.byref(hf), C.byref(wf))
    del keep
    return out.reshape(net["stages"][-1], hf.value, wf.value)


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, np.uint32)
    key = np.ascontiguousarray(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().ref_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def sampler_words(seed, env, step, head, block):
    out = np.zeros(4, np.uint32)
    lib().ref_sampler_words(C.c_uint64(seed), C.c_uint32(env), C.c_uint64(step), C.c_uint32(head),
                            C.c_uint32(block), _p(out))
    return out


def bits_to_uniform(w):
    return float(lib().ref_bits_to_uniform(int(w)))


def bits_to_uniform_many(words):
    words = np.ascontiguousarray(words, np.uint32)
    out = np.zeros(words.shape, np.float32)
    lib().ref_bits_to_uniform_many(_p(words), C.c_int64(words.size), _p(out))
    return out


def gumbel(u):
    return float(lib().ref_gumbel(C.c_float(u)))


def head_sample(logits, seed, env, step, head, g_override=None):
    logits = _f32(logits)
    a, lp, mg = C.c_int32(), C.c_double(), C.c_float()
    g = _f32(g_override) if g_override is not None else None
    lib().ref_head_sample(_p(logits), logits.shape[0], C.c_uint64(seed), C.c_uint32(env),
                          C.c_uint64(step), C.c_uint32(head), _p(g) if g is not None else None,
                          C.byref(a), C.byref(lp), C.byref(mg))
    return a.value, lp.value, mg.value


def head_histogram(logits, seed, head, n, n_env, step0=0):
    logits = _f32(logits)
    counts = np.zeros(logits.shape[0], np.int64)
    lib().ref_head_histogram(_p(logits), logits.shape[0], C.c_uint64(seed), C.c_uint32(head),
                             C.c_int64(n), C.c_uint32(n_env), C.c_uint64(step0), _p(counts))
    return counts


def log_softmax(logits):
    logits = _f32(logits)
    out = np.zeros(logits.shape[0], np.float64)
    lib().ref_log_softmax(_p(logits), logits.shape[0], _p(out))
    return out
