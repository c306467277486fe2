"""Thin ctypes binding of libsf_policy.so (C ABI in include/sf_policy.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  There is no fallback: if the library has not been built, loading it
raises.  PyTorch appears only as the owner of device memory and streams.
"""
import ctypes as C
import glob
import os
import subprocess

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
_CSRC = os.path.join(_PKG, "csrc")
# SF_POLICY_HOST_SANITIZE=1 selects a second build whose HOST code carries AddressSanitizer and
# UndefinedBehaviorSanitizer (device code unchanged), for running the CPU tests of the host logic:
#   python -c "from paper_2006_11751_amd import binding; binding.build_library(host_sanitize=True)"
#   LD_PRELOAD=$(/opt/rocm/lib/llvm/bin/clang -print-file-name=libclang_rt.asan-x86_64.so) \
#       ASAN_OPTIONS=detect_leaks=0 SF_POLICY_HOST_SANITIZE=1 \
#       python -m pytest tests/test_abi.py tests/test_host_conv1_admission.py
# (the host code is compiled by clang and needs clang's sanitizer runtime; the oracle's own
# sanitizer build uses gcc's, so the two runs are separate)
_HOST_SANITIZE = os.environ.get("SF_POLICY_HOST_SANITIZE", "") not in ("", "0")
_SO = os.path.join(_PKG, "libsf_policy_hostsan.so" if _HOST_SANITIZE else "libsf_policy.so")

SF_ABI_VERSION = 2
SF_MAX_CONV, SF_MAX_STAGE, SF_MAX_HEADS, SF_MAX_CONV_TENSORS = 4, 4, 16, 20
SF_MAX_MEAS_LAYERS = 2
SF_RNN_GRU, SF_RNN_LSTM = 0, 1
SF_OK, SF_ERR_ARG, SF_ERR_SHAPE, SF_ERR_BATCH, SF_ERR_ALIAS = 0, -1, -2, -3, -4
SF_ERR_DEVICE, SF_ERR_OOM, SF_ERR_ARCH = -5, -6, -7

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-fast-math",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall"]


def library_path():
    return _SO


HOST_SANITIZE_FLAGS = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                       "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def build_library(verbose=False, host_sanitize=False):
    """Compile every .hip source for gfx950 and link libsf_policy.so in-tree
    (host_sanitize: libsf_policy_hostsan.so, sanitizers on the host code only)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = sorted(glob.glob(os.path.join(_CSRC, "*.hip")))
    objdir = os.path.join(_PKG, "_build_hostsan" if host_sanitize else "_build")
    os.makedirs(objdir, exist_ok=True)
    inc = ["-I", os.path.join(_ROOT, "include"), "-I", _CSRC]
    flags = HIPCC_FLAGS + (HOST_SANITIZE_FLAGS if host_sanitize else [])
    so = os.path.join(_PKG, "libsf_policy_hostsan.so" if host_sanitize else "libsf_policy.so")
    procs = []
    for s in srcs:
        o = os.path.join(objdir, os.path.basename(s) + ".o")
        cmd = [hipcc] + flags + inc + ["-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd))
        procs.append((s, o, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    objs = []
    for s, o, pr in procs:
        out, _ = pr.communicate()
        text = "\n".join(l for l in out.decode().splitlines()
                         if "packed-fp32-ops" not in l)  # the host pass does not know the feature
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (s, text))
        if verbose and text.strip():
            print(text)
        objs.append(o)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", so] + objs
    if host_sanitize:
        cmd += ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-shared-libsan"]
    subprocess.run(cmd, check=True)
    return so


class SfConv(C.Structure):
    _fields_ = [("cout", C.c_int32), ("k", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32)]


class SfPolicyConfig(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("abi_version", C.c_uint32),
        ("max_batch", C.c_int32), ("obs_c", C.c_int32), ("obs_h", C.c_int32), ("obs_w", C.c_int32),
        ("encoder", C.c_int32), ("n_conv", C.c_int32), ("conv", SfConv * SF_MAX_CONV),
        ("n_stage", C.c_int32), ("stage_ch", C.c_int32 * SF_MAX_STAGE),
        ("blocks_per_stage", C.c_int32),
        ("fc_dim", C.c_int32), ("rnn_dim", C.c_int32), ("n_heads", C.c_int32),
        ("head_sizes", C.c_int32 * SF_MAX_HEADS), ("dtype", C.c_int32),
        ("obs_sub", C.c_float), ("obs_mul", C.c_float),
        ("rnn_type", C.c_int32), ("meas_dim", C.c_int32), ("n_meas_layers", C.c_int32),
        ("meas_hidden", C.c_int32 * SF_MAX_MEAS_LAYERS),
    ]


_FP = C.POINTER(C.c_float)


class SfLossConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("T", C.c_int32), ("N", C.c_int32), ("n_heads", C.c_int32),
                ("head_sizes", C.c_int32 * SF_MAX_HEADS),
                ("gamma", C.c_float), ("rho_bar", C.c_float), ("c_bar", C.c_float), ("clip", C.c_float),
                ("critic_coef", C.c_float), ("entropy_coef", C.c_float)]


class SfPolicyWeights(C.Structure):
    _fields_ = [
        ("conv_w", _FP * SF_MAX_CONV_TENSORS), ("conv_b", _FP * SF_MAX_CONV_TENSORS),
        ("fc_w", _FP), ("fc_b", _FP),
        ("rnn_w_ih", _FP), ("rnn_w_hh", _FP), ("rnn_b_ih", _FP), ("rnn_b_hh", _FP),
        ("pi_w", _FP), ("pi_b", _FP), ("v_w", _FP), ("v_b", _FP),
        ("meas_w", _FP * SF_MAX_MEAS_LAYERS), ("meas_b", _FP * SF_MAX_MEAS_LAYERS),
    ]


EXPORTS = ("sf_policy_create", "sf_policy_step", "sf_policy_destroy", "sf_last_error",
           "sf_policy_flops_per_row", "sf_policy_op_count", "sf_policy_op_name",
           "sf_policy_op_flops_per_row", "sf_policy_set_op_timing", "sf_policy_last_op_times",
           "sf_copy_bytes", "sf_policy_step_indexed", "sf_pipeline_create", "sf_pipeline_submit",
           "sf_pipeline_wait", "sf_pipeline_destroy", "sf_policy_state_dim",
           "sf_policy_update_weights", "sf_appo_loss", "sf_appo_loss_workspace_bytes",
           "sf_policy_op_pipe", "sf_policy_conv1_fixed_point_ratio", "sf_conv1_fixed_point_test",
           "sf_appo_loss_static", "sf_appo_loss_static_max_trajectories", "sf_policy_op_kernel", "sf_policy_unroll")

_lib = None


class SfError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("sf_policy error %d: %s" % (code, text))
        self.code = code


def load_library():
    """Load libsf_policy.so; raises if it has not been built (no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise FileNotFoundError(
                "%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "(hipcc, gfx950) first" % _SO)
        # PyTorch ships its own copy of the HIP runtime.  Import it first so that this
        # library binds to that same copy: two HIP runtimes in one process do not
        # both see the GPU, and the device pointers handed in come from torch's.
        import torch  # noqa: F401
        L = C.CDLL(_SO)
        L.sf_policy_create.restype = C.c_int
        L.sf_policy_create.argtypes = [C.POINTER(SfPolicyConfig), C.POINTER(SfPolicyWeights),
                                       C.c_int, C.POINTER(C.c_void_p)]
        L.sf_policy_step.restype = C.c_int
        L.sf_policy_step.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sf_policy_update_weights.restype = C.c_int
        L.sf_policy_update_weights.argtypes = [C.c_void_p, C.POINTER(SfPolicyWeights), C.c_void_p]
        L.sf_appo_loss_workspace_bytes.restype = C.c_int64
        L.sf_appo_loss_workspace_bytes.argtypes = [C.POINTER(SfLossConfig)]
        L.sf_appo_loss.restype = C.c_int
        L.sf_appo_loss.argtypes = [C.POINTER(SfLossConfig)] + [C.c_void_p] * 13
        L.sf_appo_loss_static.restype = C.c_int
        L.sf_appo_loss_static.argtypes = [C.POINTER(SfLossConfig)] + [C.c_void_p] * 12
        L.sf_appo_loss_static_max_trajectories.restype = C.c_int32
        L.sf_appo_loss_static_max_trajectories.argtypes = []
        L.sf_policy_state_dim.restype = C.c_int32
        L.sf_policy_state_dim.argtypes = [C.c_void_p]
        L.sf_policy_destroy.restype = C.c_int
        L.sf_policy_destroy.argtypes = [C.c_void_p]
        L.sf_last_error.restype = C.c_char_p
        L.sf_policy_flops_per_row.restype = C.c_int64
        L.sf_policy_flops_per_row.argtypes = [C.c_void_p]
        L.sf_policy_op_count.restype = C.c_int
        L.sf_policy_op_count.argtypes = [C.c_void_p]
        L.sf_policy_op_name.restype = C.c_char_p
        L.sf_policy_op_name.argtypes = [C.c_void_p, C.c_int]
        L.sf_policy_op_flops_per_row.restype = C.c_int64
        L.sf_policy_op_flops_per_row.argtypes = [C.c_void_p, C.c_int]
        L.sf_policy_op_pipe.restype = C.c_char_p
        L.sf_policy_op_pipe.argtypes = [C.c_void_p, C.c_int]
        L.sf_policy_op_kernel.restype = C.c_char_p
        L.sf_policy_op_kernel.argtypes = [C.c_void_p, C.c_int]
        L.sf_policy_conv1_fixed_point_ratio.restype = C.c_double
        L.sf_policy_conv1_fixed_point_ratio.argtypes = [C.c_void_p, C.c_int]
        L.sf_conv1_fixed_point_test.restype = C.c_int
        L.sf_conv1_fixed_point_test.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_int32,
                                                C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.sf_policy_set_op_timing.restype = C.c_int
        L.sf_policy_set_op_timing.argtypes = [C.c_void_p, C.c_int]
        L.sf_policy_last_op_times.restype = C.c_int
        L.sf_policy_last_op_times.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_int]
        L.sf_copy_bytes.restype = C.c_int
        L.sf_copy_bytes.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.sf_policy_step_indexed.restype = C.c_int
        L.sf_policy_step_indexed.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_int32, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p]
        L.sf_policy_unroll.restype = C.c_int
        L.sf_policy_unroll.argtypes = [C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 8
        L.sf_pipeline_create.restype = C.c_int
        L.sf_pipeline_create.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
        L.sf_pipeline_submit.restype = C.c_int
        L.sf_pipeline_submit.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_uint64,
                                         C.c_uint64,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
        L.sf_pipeline_wait.restype = C.c_int
        L.sf_pipeline_wait.argtypes = [C.c_void_p, C.c_int32]
        L.sf_pipeline_destroy.restype = C.c_int
        L.sf_pipeline_destroy.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def sf_last_error():
    return load_library().sf_last_error().decode()


def make_config(net, max_batch):
    """net: dict as produced by workloads.network()."""
    c = SfPolicyConfig()
    c.struct_size, c.abi_version = C.sizeof(SfPolicyConfig), SF_ABI_VERSION
    c.max_batch = max_batch
    c.obs_c, c.obs_h, c.obs_w = net["obs"]
    if net["encoder"] == "resnet":
        c.encoder = 1
        c.n_stage = len(net["stages"])
        for i, ch in enumerate(net["stages"]):
            c.stage_ch[i] = ch
        c.blocks_per_stage = net["blocks_per_stage"]
    else:
        c.encoder = 0
        c.n_conv = len(net["convs"])
        for i, (co, k, s, p) in enumerate(net["convs"]):
            c.conv[i] = SfConv(co, k, s, p)
    c.fc_dim, c.rnn_dim, c.n_heads = net["fc"], net["rnn"], len(net["heads"])
    for i, a in enumerate(net["heads"]):
        c.head_sizes[i] = a
    c.dtype = 1 if net["dtype"] == "bf16" else 0
    c.obs_sub, c.obs_mul = net["obs_sub"], net["obs_mul"]
    c.rnn_type = SF_RNN_LSTM if net.get("rnn_type", "gru") == "lstm" else SF_RNN_GRU
    c.meas_dim = net.get("meas_dim", 0)
    hidden = net.get("meas_hidden", []) if c.meas_dim else []
    c.n_meas_layers = len(hidden)
    for i, m in enumerate(hidden):
        c.meas_hidden[i] = m
    return c


def make_weights(w):
    """w: dict of fp32 numpy arrays (workloads.weights()).  Returns (struct, keepalive)."""
    s = SfPolicyWeights()
    keep = []

    def fp(a):
        a = np.ascontiguousarray(a, dtype=np.float32)
        keep.append(a)
        return a.ctypes.data_as(_FP)

    for i, (cw, cb) in enumerate(zip(w["conv_w"], w["conv_b"])):
        s.conv_w[i], s.conv_b[i] = fp(cw), fp(cb)
    for name in ("fc_w", "fc_b", "rnn_w_ih", "rnn_w_hh", "rnn_b_ih", "rnn_b_hh", "pi_w", "pi_b",
                 "v_w", "v_b"):
        setattr(s, name, fp(w[name]))
    for i, (mw, mb) in enumerate(zip(w.get("meas_w", []), w.get("meas_b", []))):
        s.meas_w[i], s.meas_b[i] = fp(mw), fp(mb)
    return s, keep


def sf_conv1_fixed_point_test(conv_w, obs_mul, dtype="fp32"):
    """conv_w: fp32 numpy [32, cin, 8, 8] (host).  Returns (ratio with 2 planes, with 3 planes)."""
    a = np.ascontiguousarray(conv_w, dtype=np.float32)
    assert a.shape[0] == 32 and a.shape[2:] == (8, 8)
    r2, r3 = C.c_double(), C.c_double()
    rc = load_library().sf_conv1_fixed_point_test(a.ctypes.data, a.shape[1], obs_mul,
                                                  1 if dtype == "bf16" else 0, C.byref(r2), C.byref(r3))
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())
    return r2.value, r3.value


def sf_policy_create(cfg, weights, hip_device=0):
    """cfg: SfPolicyConfig, weights: SfPolicyWeights -> opaque handle (int)."""
    h = C.c_void_p()
    rc = load_library().sf_policy_create(C.byref(cfg), C.byref(weights), hip_device, C.byref(h))
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())
    return h.value


def sf_policy_step(handle, B, obs, meas, h_in, done, seed, step, actions, logp, value, h_out,
                   logits_opt=None, hip_stream=None):
    """All buffers are device addresses (ints), e.g. torch.Tensor.data_ptr(); meas is None for
    policies without a measurement input."""
    rc = load_library().sf_policy_step(handle, B, obs, meas, h_in, done, seed, step, actions, logp,
                                       value, h_out, logits_opt, hip_stream)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def sf_policy_step_indexed(handle, B, obs, meas, h_table, n_env, env_ids, done, seed, step, actions,
                           logp, value, logits_opt=None, hip_stream=None):
    """Device addresses (ints); h_table [n_env, state_dim] is read and written at rows env_ids."""
    rc = load_library().sf_policy_step_indexed(handle, B, obs, meas, h_table, n_env, env_ids, done,
                                               seed, step, actions, logp, value, logits_opt, hip_stream)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def sf_policy_unroll(handle, T, N, obs, meas, h0, done, logits, value, h_seq, hip_stream=None):
    """Device addresses (ints) of time-major arrays; see include/sf_policy.h."""
    rc = load_library().sf_policy_unroll(handle, T, N, obs, meas, h0, done, logits, value, h_seq, hip_stream)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def sf_pipeline_create(policy_handle, slot_batch, n_slots):
    h = C.c_void_p()
    rc = load_library().sf_pipeline_create(policy_handle, slot_batch, n_slots, C.byref(h))
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())
    return h


def sf_pipeline_submit(handle, slot, B, host_obs, host_meas, host_done, host_env_ids, h_table, n_env,
                       seed, step, host_actions, host_logp, host_value):
    """host_*: host addresses (page-locked for overlap); h_table: device address."""
    rc = load_library().sf_pipeline_submit(handle, slot, B, host_obs, host_meas, host_done,
                                           host_env_ids, h_table, n_env, seed, step, host_actions,
                                           host_logp, host_value)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def sf_pipeline_wait(handle, slot):
    rc = load_library().sf_pipeline_wait(handle, slot)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def sf_pipeline_destroy(handle):
    rc = load_library().sf_pipeline_destroy(handle)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def sf_policy_update_weights(handle, weights, hip_stream=None):
    """weights: SfPolicyWeights (host pointers); copies are enqueued on hip_stream."""
    rc = load_library().sf_policy_update_weights(handle, C.byref(weights), hip_stream)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def make_loss_config(hp):
    """hp: dict(T, N, heads, gamma, rho_bar, c_bar, clip, critic_coef, entropy_coef)."""
    c = SfLossConfig()
    c.struct_size = C.sizeof(SfLossConfig)
    c.T, c.N, c.n_heads = hp["T"], hp["N"], len(hp["heads"])
    for i, a in enumerate(hp["heads"]):
        c.head_sizes[i] = a
    for k in ("gamma", "rho_bar", "c_bar", "clip", "critic_coef", "entropy_coef"):
        setattr(c, k, hp[k])
    return c


def sf_appo_loss_workspace_bytes(cfg):
    n = load_library().sf_appo_loss_workspace_bytes(C.byref(cfg))
    if n < 0:
        raise SfError(SF_ERR_SHAPE, sf_last_error())
    return int(n)


def sf_appo_loss(cfg, logits, actions, logp_mu, values, rewards, dones, vs, adv, loss, dlogits_opt,
                 dvalues_opt, workspace, hip_stream=None):
    """All buffers are device addresses (ints)."""
    rc = load_library().sf_appo_loss(C.byref(cfg), logits, actions, logp_mu, values, rewards, dones, vs,
                                     adv, loss, dlogits_opt, dvalues_opt, workspace, hip_stream)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def sf_appo_loss_static(cfg, logits, actions, logp_mu, values, rewards, dones, vs, adv, loss, dlogits_opt,
                        dvalues_opt, hip_stream=None):
    """sf_appo_loss without a workspace argument (the library's built-in scratch); device addresses."""
    rc = load_library().sf_appo_loss_static(C.byref(cfg), logits, actions, logp_mu, values, rewards, dones,
                                            vs, adv, loss, dlogits_opt, dvalues_opt, hip_stream)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def appo_loss(hp, tr, want_grads=True, stream=None, out=None):
    """tr: dict of contiguous CUDA tensors (logits, actions, logp_mu, values, rewards, dones),
    time-major.  Returns dict(vs, adv, loss[4], dlogits, dvalues) of CUDA tensors."""
    import torch
    cfg = make_loss_config(hp)
    T, N, sumA = tr["logits"].shape
    d = tr["logits"].device
    for k, dt in (("logits", torch.float32), ("actions", torch.int32), ("logp_mu", torch.float32),
                  ("values", torch.float32), ("rewards", torch.float32), ("dones", torch.uint8)):
        assert tr[k].dtype == dt and tr[k].is_contiguous() and tr[k].is_cuda, k
    assert (T, N) == (hp["T"], hp["N"]) and sumA == sum(hp["heads"]) and tuple(tr["values"].shape) == (T + 1, N)
    if out is None:
        out = dict(vs=torch.empty((T, N), device=d), adv=torch.empty((T, N), device=d),
                   loss=torch.empty(4, device=d),
                   dlogits=torch.empty((T, N, sumA), device=d) if want_grads else None,
                   dvalues=torch.empty((T, N), device=d) if want_grads else None,
                   workspace=torch.empty(sf_appo_loss_workspace_bytes(cfg), dtype=torch.uint8, device=d))
    s = stream if stream is not None else torch.cuda.current_stream(d)
    p = lambda x: None if x is None else x.data_ptr()
    sf_appo_loss(cfg, p(tr["logits"]), p(tr["actions"]), p(tr["logp_mu"]), p(tr["values"]), p(tr["rewards"]),
                 p(tr["dones"]), p(out["vs"]), p(out["adv"]), p(out["loss"]), p(out["dlogits"]),
                 p(out["dvalues"]), p(out["workspace"]), s.cuda_stream)
    return out


def sf_copy_bytes(src, dst, nbytes, hip_stream=None):
    rc = load_library().sf_copy_bytes(src, dst, nbytes, hip_stream)
    if rc != SF_OK:
        raise SfError(rc, sf_last_error())


def sf_policy_destroy(handle):
    load_library().sf_policy_destroy(handle)


class Policy:
    """Convenience owner of one handle; torch tensors in, torch tensors out."""

    def __init__(self, net, weights, max_batch=None, device=0):
        import torch
        self._torch = torch
        self.net = net
        self.device = torch.device("cuda", device)
        self.max_batch = max_batch or net["B"]
        cfg = make_config(net, self.max_batch)
        ws, keep = make_weights(weights)
        self.handle = sf_policy_create(cfg, ws, device)
        del keep
        self.n_heads, self.sumA = len(net["heads"]), sum(net["heads"])
        self.H = int(load_library().sf_policy_state_dim(self.handle))  # floats per state row
        self.meas_dim = net.get("meas_dim", 0)

    def update_weights(self, weights, stream=None):
        """weights: dict as for the constructor; enqueued on `stream` (default: current)."""
        ws, keep = make_weights(weights)
        s = stream if stream is not None else self._torch.cuda.current_stream(self.device)
        sf_policy_update_weights(self.handle, ws, s.cuda_stream)
        del keep

    def flops_per_row(self):
        return int(load_library().sf_policy_flops_per_row(self.handle))

    def ops(self):
        """[(name, flops_per_row)] for each kernel launch of the step."""
        L = load_library()
        return [(L.sf_policy_op_name(self.handle, i).decode(),
                 int(L.sf_policy_op_flops_per_row(self.handle, i)))
                for i in range(L.sf_policy_op_count(self.handle))]

    def op_pipes(self):
        """The arithmetic of each launch: "i8x3", "i8x2", "f32", "bf16", "f16" or "valu"."""
        L = load_library()
        return [L.sf_policy_op_pipe(self.handle, i).decode()
                for i in range(L.sf_policy_op_count(self.handle))]

    def op_kernels(self):
        """The kernel family of each launch ("stem_pool", "res_stage", "gemm_mfma", ...)."""
        L = load_library()
        return [L.sf_policy_op_kernel(self.handle, i).decode()
                for i in range(L.sf_policy_op_count(self.handle))]

    def conv1_fixed_point_ratio(self, planes=3):
        """Worst channel's error-bound ratio of the first convolution's digit planes (<= 1: admitted)."""
        return float(load_library().sf_policy_conv1_fixed_point_ratio(self.handle, planes))

    def set_op_timing(self, enable):
        rc = load_library().sf_policy_set_op_timing(self.handle, int(bool(enable)))
        if rc != SF_OK:
            raise SfError(rc, sf_last_error())

    def last_op_times_ms(self):
        L = load_library()
        n = L.sf_policy_op_count(self.handle)
        buf = (C.c_float * n)()
        rc = L.sf_policy_last_op_times(self.handle, buf, n)
        if rc != SF_OK:
            raise SfError(rc, sf_last_error())
        return list(buf)

    def alloc_outputs(self, B, logits=True):
        t = self._torch
        d = self.device
        return dict(actions=t.empty((B, self.n_heads), dtype=t.int32, device=d),
                    logp=t.empty(B, dtype=t.float32, device=d),
                    value=t.empty(B, dtype=t.float32, device=d),
                    h_out=t.empty((B, self.H), dtype=t.float32, device=d),
                    logits=t.empty((B, self.sumA), dtype=t.float32, device=d) if logits else None)

    def _meas_ptr(self, meas, B):
        if not self.meas_dim:
            return None
        t = self._torch
        assert meas is not None and meas.dtype == t.float32 and meas.is_contiguous()
        assert tuple(meas.shape) == (B, self.meas_dim)
        return meas.data_ptr()

    def step(self, obs, h_in, done, seed, step, out=None, stream=None, meas=None):
        """obs u8 [B,C,H,W], h_in f32 [B,state_dim], done u8 [B], meas f32 [B,meas_dim] (full
        architecture only): contiguous tensors (CUDA, or page-locked for meas in a Pipeline)."""
        t = self._torch
        B = obs.shape[0]
        assert obs.dtype == t.uint8 and h_in.dtype == t.float32 and done.dtype == t.uint8
        assert obs.is_contiguous() and h_in.is_contiguous() and done.is_contiguous()
        assert tuple(obs.shape[1:]) == tuple(self.net["obs"]) and tuple(h_in.shape) == (B, self.H)
        assert done.shape == (B,)
        if out is None:
            out = self.alloc_outputs(B)
        s = stream if stream is not None else t.cuda.current_stream(self.device)
        sf_policy_step(self.handle, B, obs.data_ptr(), self._meas_ptr(meas, B), h_in.data_ptr(),
                       done.data_ptr(), seed, step,
                       out["actions"].data_ptr(), out["logp"].data_ptr(), out["value"].data_ptr(),
                       out["h_out"].data_ptr(),
                       out["logits"].data_ptr() if out.get("logits") is not None else None,
                       s.cuda_stream)
        return out

    def step_indexed(self, obs, h_table, env_ids, done, seed, step, out=None, stream=None, meas=None):
        """obs u8 [B,C,H,W], h_table f32 [n_env,H] (updated in place at rows env_ids),
        env_ids i32 [B], done u8 [B]: contiguous CUDA tensors."""
        t = self._torch
        B = obs.shape[0]
        assert obs.dtype == t.uint8 and h_table.dtype == t.float32 and done.dtype == t.uint8
        assert env_ids.dtype == t.int32 and env_ids.shape == (B,) and done.shape == (B,)
        assert obs.is_contiguous() and h_table.is_contiguous() and done.is_contiguous()
        assert env_ids.is_contiguous() and h_table.shape[1] == self.H
        assert tuple(obs.shape[1:]) == tuple(self.net["obs"])
        if out is None:
            out = self.alloc_outputs(B)
            del out["h_out"]
        s = stream if stream is not None else t.cuda.current_stream(self.device)
        sf_policy_step_indexed(self.handle, B, obs.data_ptr(), self._meas_ptr(meas, B),
                               h_table.data_ptr(), h_table.shape[0],
                               env_ids.data_ptr(), done.data_ptr(), seed, step,
                               out["actions"].data_ptr(), out["logp"].data_ptr(),
                               out["value"].data_ptr(),
                               out["logits"].data_ptr() if out.get("logits") is not None else None,
                               s.cuda_stream)
        return out

    def unroll(self, obs, h0, done, out=None, stream=None, meas=None):
        """The learner's forward pass: obs u8 [T,N,C,H,W], h0 f32 [N,state_dim], done u8 [T,N],
        meas f32 [T,N,meas_dim]: contiguous CUDA tensors.  Returns logits [T,N,sumA], value [T,N],
        h_seq [T,N,state_dim]."""
        t = self._torch
        T, N = obs.shape[0], obs.shape[1]
        assert obs.dtype == t.uint8 and h0.dtype == t.float32 and done.dtype == t.uint8
        assert obs.is_contiguous() and h0.is_contiguous() and done.is_contiguous()
        assert tuple(obs.shape[2:]) == tuple(self.net["obs"]) and tuple(done.shape) == (T, N)
        assert tuple(h0.shape) == (N, self.H)
        if out is None:
            f32 = dict(dtype=t.float32, device=self.device)
            out = {"logits": t.empty((T, N, sum(self.net["heads"])), **f32), "value": t.empty((T, N), **f32),
                   "h_seq": t.empty((T, N, self.H), **f32)}
        meas_ptr = None
        if self.meas_dim:
            assert meas is not None and meas.dtype == t.float32 and meas.is_contiguous()
            assert tuple(meas.shape) == (T, N, self.meas_dim)
            meas_ptr = meas.data_ptr()
        s = stream if stream is not None else t.cuda.current_stream(self.device)
        sf_policy_unroll(self.handle, T, N, obs.data_ptr(), meas_ptr, h0.data_ptr(), done.data_ptr(),
                         out["logits"].data_ptr(), out["value"].data_ptr(), out["h_seq"].data_ptr(), s.cuda_stream)
        return out

    def close(self):
        if self.handle:
            sf_policy_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Pipeline:
    """Double-buffered stepping around a Policy: page-locked host tensors in and out,
    the state table stays on the device.  Marshalling only; see include/sf_policy.h."""

    def __init__(self, policy, slot_batch, n_slots=2):
        import torch
        self._torch = torch
        self.policy = policy
        self.slot_batch = slot_batch
        self.n_slots = n_slots
        self.handle = sf_pipeline_create(policy.handle, slot_batch, n_slots)
        self._keep = [None] * n_slots

    def host_buffers(self, B=None):
        """Page-locked tensors of the right shapes for one slot."""
        t = self._torch
        B = self.slot_batch if B is None else B
        pin = dict(pin_memory=True)
        md = self.policy.meas_dim
        return dict(obs=t.empty((B,) + tuple(self.policy.net["obs"]), dtype=t.uint8, **pin),
                    meas=t.empty((B, md), dtype=t.float32, **pin) if md else None,
                    done=t.empty(B, dtype=t.uint8, **pin), env_ids=t.empty(B, dtype=t.int32, **pin),
                    actions=t.empty((B, self.policy.n_heads), dtype=t.int32, **pin),
                    logp=t.empty(B, dtype=t.float32, **pin), value=t.empty(B, dtype=t.float32, **pin))

    def submit(self, slot, hb, h_table, seed, step, B=None):
        B = hb["obs"].shape[0] if B is None else B
        for k in ("obs", "done", "env_ids", "actions", "logp", "value"):
            assert hb[k].is_contiguous() and not hb[k].is_cuda
        sf_pipeline_submit(self.handle, slot, B, hb["obs"].data_ptr(),
                           self.policy._meas_ptr(hb.get("meas"), hb["obs"].shape[0]),
                           hb["done"].data_ptr(),
                           hb["env_ids"].data_ptr(), h_table.data_ptr(), h_table.shape[0], seed, step,
                           hb["actions"].data_ptr(), hb["logp"].data_ptr(), hb["value"].data_ptr())
        self._keep[slot] = (hb, h_table)  # the buffers stay alive while the slot is in flight

    def wait(self, slot):
        sf_pipeline_wait(self.handle, slot)
        if 0 <= slot < self.n_slots:
            self._keep[slot] = None

    def close(self):
        if self.handle:
            sf_pipeline_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
