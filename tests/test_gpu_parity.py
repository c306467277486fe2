"""GPU parity: sf_policy_step (through the C ABI) against the CPU oracle on the
same seeded inputs, element by element; plus edge cases and the purity /
prefix properties (paper, Sec. 3.1 "Parallelism": stateless policy workers).
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu


def _to_np(out):
    return {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}


def _gpu_step(torch, pol, obs, h_in, done, seed, step):
    d = pol.device
    out = pol.step(torch.from_numpy(obs).to(d), torch.from_numpy(h_in).to(d),
                   torch.from_numpy(done).to(d), seed, step)
    torch.cuda.synchronize()
    return _to_np(out)


def _make(torch, net, max_batch=None):
    from paper_2006_11751_amd import binding
    w = wl.weights(net)
    return binding.Policy(net, w, max_batch=max_batch or net["B"]), w


SMALL_RESNET = dict(name="resnet_small", B=5, obs=(3, 18, 24), encoder="resnet", stages=[4, 6, 6],
                    blocks_per_stage=2, fc=16, rnn=12, heads=[5], dtype="fp32", p_done=0.3, steps=1,
                    obs_sub=0.0, obs_mul=wl.OBS_MUL, index=4)
ODD_NET = dict(name="odd", B=37, obs=(2, 23, 29), encoder="conv", convs=[(5, 5, 2, 1), (7, 3, 1, 0)],
               fc=19, rnn=33, heads=[1, 2, 70, 5], dtype="fp32", p_done=0.5, steps=1,
               obs_sub=127.5, obs_mul=1.0 / 64, index=0)


def test_tiny_four_steps_free_running(torch_cuda, ref):
    """Configuration 0: every element, 4 steps, each side carrying its own state."""
    torch = torch_cuda
    net = wl.network(0)
    pol, w = _make(torch, net)
    h_gpu = wl.initial_state(net)
    h_ref = h_gpu.copy()
    for t in range(net["steps"]):
        obs, done = wl.observations(net, t), wl.done_mask(net, t)
        g = _gpu_step(torch, pol, obs, h_gpu, done, wl.PHILOX_SEED, t)
        o = ref.policy_step(net, w, obs, h_ref, done, wl.PHILOX_SEED, t)
        parity.check_against_oracle(net, g, o, ref, wl.PHILOX_SEED, t)
        h_gpu, h_ref = g["h_out"], o["h_out"]
    pol.close()


RESNET_BF16_SMALL = dict(name="resnet_bf16_small", B=7, obs=(3, 20, 28), encoder="resnet", stages=[16, 32, 32],
                         blocks_per_stage=2, fc=64, rnn=32, heads=[15], dtype="bf16", p_done=0.3, steps=1,
                         obs_sub=0.0, obs_mul=wl.OBS_MUL, index=4)
# several tiles of the fused residual-encoder kernels in both directions, ragged at the edges
RESNET_BF16_MID = dict(RESNET_BF16_SMALL, name="resnet_bf16_mid", B=3, obs=(3, 50, 76))
# width not a multiple of 4 (byte planes not dword-aligned), channel counts 32 -> 16 -> 32
RESNET_BF16_MIX = dict(RESNET_BF16_SMALL, name="resnet_bf16_mix", B=4, obs=(3, 30, 42), stages=[32, 16, 32])
# stage frames of 24 x 64 (16 channels) and 12 x 32 (32 channels): the kernel that runs all blocks
# of a stage with the frame resident in LDS; more frames than its workgroups (256), so some walk
# two frames.  (The last stage, 6 x 16, has fewer tiles than that kernel has waves: four frames
# share an LDS image.)
RESNET_BF16_POW2 = dict(RESNET_BF16_SMALL, name="resnet_bf16_pow2", B=300, obs=(3, 48, 128))
# 136 x 128 frames: the first two stages are too large for that kernel, the last (17 x 16 pixels:
# two image rows per MFMA tile, the ninth tile half empty) runs on it
RESNET_BF16_TALL = dict(RESNET_BF16_SMALL, name="resnet_bf16_tall", B=5, obs=(3, 136, 128))
STD_BF16_SMALL = wl.network(2, B=37, name="standard_bf16_small")
# 76x132 frames: conv2 has 8x15 = 120 output pixels (the eight-tile instantiation of the
# frame-resident kernel), conv3 3x7 = 21 (more than that kernel takes: tiled kernel)
STD_BF16_WIDE = dict(STD_BF16_SMALL, name="standard_bf16_wide", B=9, obs=(3, 76, 132))


@pytest.mark.parametrize("net", [SMALL_RESNET, ODD_NET, RESNET_BF16_SMALL, RESNET_BF16_MID, RESNET_BF16_MIX,
                                 RESNET_BF16_POW2, RESNET_BF16_TALL, STD_BF16_SMALL, STD_BF16_WIDE],
                         ids=lambda n: n["name"])
def test_small_networks_all_elements(torch_cuda, ref, net):
    torch = torch_cuda
    pol, w = _make(torch, net)
    B = net["B"]
    obs, h_in, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    g = _gpu_step(torch, pol, obs, h_in, done, 7, 11)
    o = ref.policy_step(net, w, obs, h_in, done, 7, 11)
    print(net["name"], [n for n, _ in pol.ops()], parity.check_against_oracle(net, g, o, ref, 7, 11))
    pol.close()


def test_standard_full_batch(torch_cuda, ref):
    """Configuration 1 at its full size (B=1024): every row against the oracle."""
    torch = torch_cuda
    net = wl.network(1)
    pol, w = _make(torch, net)
    obs, h_in, done = wl.observations(net), wl.initial_state(net), wl.done_mask(net)
    g = _gpu_step(torch, pol, obs, h_in, done, wl.PHILOX_SEED, 0)
    o = ref.policy_step(net, w, obs, h_in, done, wl.PHILOX_SEED, 0)
    stats = parity.check_against_oracle(net, g, o, ref, wl.PHILOX_SEED, 0)
    print("standard parity:", stats)
    # ragged batch on the same handle: B = 1000 + tail, and the prefix property
    g2 = _gpu_step(torch, pol, obs[:999], h_in[:999], done[:999], wl.PHILOX_SEED, 0)
    for k in ("h_out", "logits", "value", "logp", "actions"):
        assert np.array_equal(g2[k], g[k][:999]), k
    pol.close()


def _tile_edge_rows(B, tile):
    """First and last batch row of every `tile`-row block of a B-row batch."""
    first = np.arange(0, B, tile)
    return np.concatenate([first, np.minimum(first + tile - 1, B - 1)])


def _sampled_rows_check(torch, ref, net, n_rows, n_steps=1, full_steps=1, extra_rows=()):
    """Full-size batch on the GPU; the oracle computes a sample of rows one by one."""
    pol, w = _make(torch, net)
    B = net["B"]
    rng = np.random.default_rng(99)
    rows = np.unique(np.concatenate([[0, 1, B - 1, B - 2, B // 2], rng.integers(0, B, n_rows),
                                     np.asarray(extra_rows, dtype=np.int64)]))
    h_gpu = wl.initial_state(net)
    for t in range(n_steps):
        obs, done = wl.observations(net, t), wl.done_mask(net, t)
        g = _gpu_step(torch, pol, obs, h_gpu, done, wl.PHILOX_SEED, t)
        if t < full_steps or t == n_steps - 1:
            # teacher-forced on the GPU's incoming state for the sampled rows
            o = ref.policy_step(net, w, obs[rows], h_gpu[rows], done[rows], wl.PHILOX_SEED, t)
            # the oracle numbered these rows 0..n-1: redo its sampling with the true row index
            off = 0
            for k, A in enumerate(net["heads"]):
                for i, r in enumerate(rows):
                    a, lp_k, mg = ref.head_sample(o["logits"][i, off:off + A], wl.PHILOX_SEED, int(r), t, k)
                    o["actions"][i, k], o["margin"][i, k] = a, mg
                off += A
            o["logp"] = np.array([
                sum(ref.log_softmax(o["logits"][i, s:s + A])[o["actions"][i, k]]
                    for k, (s, A) in enumerate(zip(np.cumsum([0] + net["heads"][:-1]), net["heads"])))
                for i in range(len(rows))], np.float32)
            gs = {k: v[rows] for k, v in g.items()}
            stats = parity.check_against_oracle(net, gs, o, ref, wl.PHILOX_SEED, t, rows=rows)
            print(net["name"], "step", t, stats)
        # properties that hold at any size
        assert np.all(np.isfinite(g["h_out"])) and np.all(np.abs(g["h_out"]) <= 1.0 + 1e-6)
        assert np.all(g["logp"] <= 1e-6)
        h_gpu = g["h_out"]
    pol.close()


def test_standard_bf16_several_frames_per_workgroup(torch_cuda, ref):
    """Configuration 2's network at B=2101, every row: the frame-resident kernels (conv1 from
    2048 rows on, conv2, conv3) walk several frames or rounds per workgroup here, the last round
    ragged; the 300-row prefix runs conv1 on the gather kernel and must give the same bits."""
    torch = torch_cuda
    net = wl.network(2, B=2101, name="standard_bf16_2101")
    pol, w = _make(torch, net)
    obs, h_in, done = wl.observations(net), wl.initial_state(net), wl.done_mask(net)
    g = _gpu_step(torch, pol, obs, h_in, done, wl.PHILOX_SEED, 2)
    o = ref.policy_step(net, w, obs, h_in, done, wl.PHILOX_SEED, 2)
    parity.check_against_oracle(net, g, o, ref, wl.PHILOX_SEED, 2)
    # prefix property on the same handle (one frame per workgroup below 512 rows)
    g2 = _gpu_step(torch, pol, obs[:300], h_in[:300], done[:300], wl.PHILOX_SEED, 2)
    for k in g:
        assert np.array_equal(g[k][:300], g2[k]), k
    pol.close()


def test_first_convolution_variants_give_the_same_bits(torch_cuda, ref):
    """fp32 standard network at B=2050: the first convolution runs frame-resident from 2048 rows
    on and as a gather kernel below; a 700-row prefix must equal the full call bitwise, and
    sampled rows of the full call must match the oracle."""
    torch = torch_cuda
    net = wl.network(1, B=2050, name="standard_2050")
    pol, w = _make(torch, net)
    obs, h_in, done = wl.observations(net), wl.initial_state(net), wl.done_mask(net)
    g = _gpu_step(torch, pol, obs, h_in, done, wl.PHILOX_SEED, 1)
    g2 = _gpu_step(torch, pol, obs[:700], h_in[:700], done[:700], wl.PHILOX_SEED, 1)
    for k in g:
        assert np.array_equal(g[k][:700], g2[k]), k
    rows = np.array([0, 1, 511, 512, 1023, 1024, 1536, 2047, 2048, 2049])
    o = ref.policy_step(net, w, obs[rows], h_in[rows], done[rows], wl.PHILOX_SEED, 1)
    np.testing.assert_allclose(g["h_out"][rows], o["h_out"], rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(g["value"][rows], o["value"], rtol=1e-4, atol=1e-5)
    pol.close()


def test_standard_bf16_full_size_sampled_rows(torch_cuda, ref):
    """Configuration 2 (B=4096, bf16 weights/activations)."""
    _sampled_rows_check(torch_cuda, ref, wl.network(2), 200)


def test_multi_discrete_16_steps(torch_cuda, ref):
    """Configuration 3 (B=2048, six heads, 16 chained steps), sampled rows: 400 random ones and
    the first and last row of every 64-row block (the row tiles of the GEMM and GRU launches)."""
    _sampled_rows_check(torch_cuda, ref, wl.network(3), 400, n_steps=16, full_steps=2,
                        extra_rows=_tile_edge_rows(2048, 64))


def test_multi_discrete_small_free_running(torch_cuda, ref):
    """Configuration 3's network at B=70, all rows, 16 free-running steps."""
    torch = torch_cuda
    net = wl.network(3, B=70)
    pol, w = _make(torch, net)
    h_gpu = wl.initial_state(net)
    h_ref = h_gpu.copy()
    for t in range(16):
        obs, done = wl.observations(net, t), wl.done_mask(net, t)
        g = _gpu_step(torch, pol, obs, h_gpu, done, wl.PHILOX_SEED, t)
        o = ref.policy_step(net, w, obs, h_ref, done, wl.PHILOX_SEED, t)
        parity.check_against_oracle(net, g, o, ref, wl.PHILOX_SEED, t)
        h_gpu, h_ref = g["h_out"], o["h_out"]
    pol.close()


def test_resnet_bf16_full_size_sampled_rows(torch_cuda, ref):
    """Configuration 4 (B=8192, residual encoder, bf16).  The encoder launches take one
    workgroup per (frame, tile), so every frame runs the same code; the FC and GRU launches tile
    the batch in blocks of 128 and 32/64 rows.  Compared: the first and last row of every
    128-row block, of every eighth 32-row block, and 400 random rows (about 600 in all)."""
    extra = np.concatenate([_tile_edge_rows(8192, 128), _tile_edge_rows(8192, 32)[::8]])
    _sampled_rows_check(torch_cuda, ref, wl.network(4), 400, extra_rows=extra)


def test_purity_done_reset_and_edges(torch_cuda, ref):
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    net = wl.network(0)
    pol, w = _make(torch, net, max_batch=16)
    obs, h_in = wl.observations(net), wl.initial_state(net)
    done = np.array([1, 0, 1, 0, 255, 0, 0, 1], np.uint8)
    a = _gpu_step(torch, pol, obs, h_in, done, 3, 5)
    b = _gpu_step(torch, pol, obs, h_in, done, 3, 5)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    # reset rows ignore h_in and equal the zero-state result bit for bit
    h2 = h_in.copy()
    h2[done != 0] = 55.0
    c = _gpu_step(torch, pol, obs, h2, done, 3, 5)
    h0 = h_in.copy()
    h0[done != 0] = 0.0
    d = _gpu_step(torch, pol, obs, h0, np.zeros(8, np.uint8), 3, 5)
    for k in a:
        assert np.array_equal(a[k], c[k]) and np.array_equal(a[k], d[k]), k
    # single row and prefix
    one = _gpu_step(torch, pol, obs[:1], h_in[:1], done[:1], 3, 5)
    for k in a:
        assert np.array_equal(one[k], a[k][:1]), k
    # seed / step reach the sampler only
    e = _gpu_step(torch, pol, obs, h_in, done, 3, 6)
    assert np.array_equal(e["logits"], a["logits"]) and np.array_equal(e["h_out"], a["h_out"])
    # logits are optional
    dev = pol.device
    out = pol.alloc_outputs(8, logits=False)
    pol.step(torch.from_numpy(obs).to(dev), torch.from_numpy(h_in).to(dev), torch.from_numpy(done).to(dev),
             3, 5, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out["actions"].cpu().numpy(), a["actions"])
    assert np.array_equal(out["logp"].cpu().numpy(), a["logp"])

    # argument errors: nothing is enqueued, a status and a message come back
    t_obs, t_h, t_d = (torch.from_numpy(x).to(dev) for x in (obs, h_in, done))
    o8 = pol.alloc_outputs(8)

    def call(B=8, obs_p=None, h_p=None, hout_p=None, act_p=None):
        binding.sf_policy_step(pol.handle, B, t_obs.data_ptr() if obs_p is None else obs_p, None,
                               t_h.data_ptr() if h_p is None else h_p, t_d.data_ptr(), 1, 0,
                               o8["actions"].data_ptr() if act_p is None else act_p,
                               o8["logp"].data_ptr(), o8["value"].data_ptr(),
                               o8["h_out"].data_ptr() if hout_p is None else hout_p,
                               o8["logits"].data_ptr(), None)

    call(B=0)  # accepted, does nothing
    for kwargs, code in [(dict(B=17), binding.SF_ERR_BATCH), (dict(B=-1), binding.SF_ERR_BATCH),
                         (dict(hout_p=t_h.data_ptr()), binding.SF_ERR_ALIAS),
                         (dict(hout_p=t_h.data_ptr() + 64), binding.SF_ERR_ALIAS),
                         (dict(act_p=o8["actions"].data_ptr() + 2), binding.SF_ERR_ARG)]:
        with pytest.raises(binding.SfError) as ei:
            call(**kwargs)
        assert ei.value.code == code and binding.sf_last_error()
    with pytest.raises(binding.SfError) as ei:
        binding.sf_policy_step(pol.handle, 8, None, None, t_h.data_ptr(), t_d.data_ptr(), 1, 0,
                               o8["actions"].data_ptr(), o8["logp"].data_ptr(), o8["value"].data_ptr(),
                               o8["h_out"].data_ptr(), None, None)
    assert ei.value.code == binding.SF_ERR_ARG
    torch.cuda.synchronize()
    pol.close()


def test_create_rejects_bad_descriptions(torch_cuda):
    from paper_2006_11751_amd import binding
    net = wl.network(0)
    w = wl.weights(net)
    ws, keep = binding.make_weights(w)
    bad = binding.make_config(dict(net, convs=[(16, 8, 4, 0), (32, 40, 2, 0)]), 8)   # empty output
    with pytest.raises(binding.SfError) as ei:
        binding.sf_policy_create(bad, ws, 0)
    assert ei.value.code == binding.SF_ERR_SHAPE
    cfg = binding.make_config(net, 8)
    cfg.abi_version = 99
    with pytest.raises(binding.SfError) as ei:
        binding.sf_policy_create(cfg, ws, 0)
    assert ei.value.code == binding.SF_ERR_ARG
    cfg = binding.make_config(net, 8)
    ws.fc_w = None
    with pytest.raises(binding.SfError) as ei:
        binding.sf_policy_create(cfg, ws, 0)
    assert ei.value.code == binding.SF_ERR_ARG
    with pytest.raises(binding.SfError) as ei:
        binding.sf_policy_create(binding.make_config(net, 8), binding.make_weights(w)[0], 99)
    assert ei.value.code == binding.SF_ERR_DEVICE


def test_sampler_distribution_on_gpu(torch_cuda, ref):
    """Frequencies of GPU-sampled actions follow softmax(logits): a tiny net whose
    logits do not depend on the row (zero head weights, fixed bias)."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    net = dict(name="bias_only", B=4096, obs=(1, 4, 4), encoder="conv", convs=[(2, 2, 2, 0)], fc=4, rnn=4,
               heads=[7, 3], dtype="fp32", p_done=0.0, obs_sub=0.0, obs_mul=wl.OBS_MUL, index=0)
    w = wl.weights(net)
    w["pi_w"][:] = 0
    w["pi_b"][:] = np.array([2.0, 0.5, -1.0, 0.0, 1.5, -3.0, 0.25, 0.0, 1.0, -1.0], np.float32)
    pol = binding.Policy(net, w)
    obs, h_in, done = wl.observations(net), wl.initial_state(net), wl.done_mask(net)
    counts = [np.zeros(7), np.zeros(3)]
    n_steps = 64
    for t in range(n_steps):
        g = _gpu_step(torch, pol, obs, h_in, done, 5, t)
        for k in range(2):
            counts[k] += np.bincount(g["actions"][:, k], minlength=len(counts[k]))
        if t == 0:  # bit-identical to the oracle's draws for these logits
            for bb in range(0, 4096, 97):
                assert ref.head_sample(w["pi_b"][:7], 5, bb, 0, 0)[0] == g["actions"][bb, 0]
                assert ref.head_sample(w["pi_b"][7:], 5, bb, 0, 1)[0] == g["actions"][bb, 1]
    n = 4096 * n_steps
    for k, sl in enumerate([slice(0, 7), slice(7, 10)]):
        p = np.exp(ref.log_softmax(w["pi_b"][sl]))
        chi2 = float(((counts[k] - n * p) ** 2 / (n * p)).sum())
        dof = len(p) - 1
        assert chi2 < dof + 5 * np.sqrt(2 * dof) + 5
    pol.close()


def _random_net(rng, dtype):
    """A random small plain-stack network; channel counts are drawn so that both the
    MFMA kernels (multiples of 32 / 8) and the shape-agnostic ones are exercised."""
    chans = [int(rng.choice([8, 16, 24, 32, 64])) for _ in range(int(rng.integers(1, 4)))]
    convs, h, w = [], int(rng.integers(20, 41)), int(rng.integers(6, 13)) * 4
    H, W = h, w
    first = True
    for co in chans:
        if first and rng.random() < 0.6:
            k, s, p, co = 8, 4, 0, 32          # the byte-input MFMA kernel's shape
        else:
            k = int(rng.choice([1, 2, 3, 4])); s = int(rng.choice([1, 2])); p = int(rng.choice([0, 0, 1]))
        if (h + 2 * p - k) // s + 1 < 1 or (w + 2 * p - k) // s + 1 < 1 or h + 2 * p < k or w + 2 * p < k:
            break
        convs.append((co, k, s, p))
        h, w = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
        first = False
    if not convs:
        convs = [(32, 8, 4, 0)]
    return dict(name="rand", B=int(rng.integers(1, 90)), obs=(int(rng.choice([1, 3, 4])), H, W), encoder="conv",
                convs=convs, fc=int(rng.choice([32, 48, 64, 128])), rnn=int(rng.choice([32, 40, 64, 96])),
                heads=[int(a) for a in rng.integers(1, 12, size=int(rng.integers(1, 5)))], dtype=dtype,
                p_done=0.3, steps=1, obs_sub=float(rng.choice([0.0, 127.5])), obs_mul=wl.OBS_MUL, index=0)


@pytest.mark.parametrize("seed", range(18))
def test_random_network_shapes(torch_cuda, ref, seed):
    """Randomly drawn network descriptions, every element against the oracle.  Seeds from 12 on
    draw the parameters from non-Gaussian laws (Laplace, Student t with 3 degrees of freedom,
    uniform) of the same variance."""
    torch = torch_cuda
    rng = np.random.default_rng(500 + seed)
    net = _random_net(rng, "bf16" if seed % 3 == 2 else "fp32")
    dist = "normal" if seed < 12 else ("laplace", "student3", "uniform")[(seed - 12) // 2]
    w = wl.weights(net, seed=600 + seed, dist=dist)
    from paper_2006_11751_amd import binding
    pol = binding.Policy(net, w)
    B = net["B"]
    obs = wl.observations(net, 0, B, seed=700 + seed)
    h_in = wl.initial_state(net, B, seed=800 + seed)
    done = wl.done_mask(net, 0, B, seed=900 + seed)
    g = _gpu_step(torch, pol, obs, h_in, done, 11, seed)
    o = ref.policy_step(net, w, obs, h_in, done, 11, seed)
    stats = parity.check_against_oracle(net, g, o, ref, 11, seed)
    print(net["obs"], net["convs"], net["fc"], net["rnn"], net["heads"], net["dtype"], B, stats)
    pol.close()


def test_maximum_batch_size(torch_cuda, ref):
    """max_batch = 65535 (the largest the boundary accepts) on the standard network: offsets
    beyond 2^32 bytes, grids of 200,000 workgroups.  Sampled rows against the oracle, and the
    first 1024 rows bit for bit against a B = 1024 call on the same handle."""
    torch = torch_cuda
    net = wl.network(1, B=65535, name="standard_max_batch")
    pol, w = _make(torch, net)
    B, d = net["B"], pol.device
    rng = np.random.default_rng(12345)
    obs = rng.integers(0, 256, size=(B,) + tuple(net["obs"]), dtype=np.uint8)
    h_in = (0.1 * rng.standard_normal((B, net["rnn"]))).astype(np.float32)
    done = (rng.random(B) < 0.05).astype(np.uint8)
    t_obs, t_h, t_d = torch.from_numpy(obs).to(d), torch.from_numpy(h_in).to(d), torch.from_numpy(done).to(d)
    big = pol.step(t_obs, t_h, t_d, 1, 3)
    torch.cuda.synchronize()
    small = pol.step(t_obs[:1024].contiguous(), t_h[:1024].contiguous(), t_d[:1024].contiguous(), 1, 3)
    torch.cuda.synchronize()
    for k in ("actions", "logp", "value", "h_out", "logits"):
        assert torch.equal(big[k][:1024], small[k]), k
    g = _to_np(big)
    rows = np.unique(np.concatenate([[0, B - 1, B - 2, 40000, 65000], rng.integers(0, B, 40)]))
    o = ref.policy_step(net, w, obs[rows], h_in[rows], done[rows], 1, 3)
    off = 0
    for k, A in enumerate(net["heads"]):
        for i, r in enumerate(rows):
            a, _, mg = ref.head_sample(o["logits"][i, off:off + A], 1, int(r), 3, k)
            o["actions"][i, k], o["margin"][i, k] = a, mg
        off += A
    o["logp"] = np.array([ref.log_softmax(o["logits"][i])[o["actions"][i, 0]] for i in range(len(rows))], np.float32)
    parity.check_against_oracle(net, {k: v[rows] for k, v in g.items()}, o, ref, 1, 3, rows=rows)
    assert np.all(np.isfinite(g["h_out"])) and np.all(np.abs(g["h_out"]) <= 1.0 + 1e-6)
    pol.close()


def test_fused_first_two_layers_equal_the_separate_kernels(torch_cuda, ref, monkeypatch):
    """bf16 standard network: the launch that runs the first two convolutions with the first
    layer's image in LDS gives the bits of the two separate kernels, at a batch that makes its
    workgroups walk several frames with a ragged last round, on a misaligned observation buffer
    (which takes the separate kernels), and on a second frame shape (76 x 120: 18 x 29 and
    8 x 13 pixels after the two layers)."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    for net in (wl.network(2, B=1100, name="standard_bf16_1100"),
                wl.network(2, B=23, name="standard_bf16_76x120", obs=(3, 76, 120))):
        w = wl.weights(net)
        B = net["B"]
        obs, h_in, done = wl.observations(net), wl.initial_state(net), wl.done_mask(net)
        fused = binding.Policy(net, w)
        assert fused.op_pipes()[0] == "i8x2+bf16" and [n for n, _ in fused.ops()][0] == "conv1+conv2"
        g = _gpu_step(torch, fused, obs, h_in, done, 1, 0)
        monkeypatch.setenv("SF_NO_CONV12_FUSE", "1")
        plain = binding.Policy(net, w)
        monkeypatch.delenv("SF_NO_CONV12_FUSE")
        assert plain.op_pipes()[:2] == ["i8x2", "bf16"]
        g2 = _gpu_step(torch, plain, obs, h_in, done, 1, 0)
        for k in g:
            assert np.array_equal(g[k], g2[k]), (net["name"], k)
        # observations at an address that is 4-byte but not 16-byte aligned
        d = fused.device
        raw = torch.empty(obs.size + 16, dtype=torch.uint8, device=d)
        t_obs = raw[4:4 + obs.size].view(obs.shape)
        t_obs.copy_(torch.from_numpy(obs))
        assert t_obs.data_ptr() % 16 == 4
        out = fused.step(t_obs, torch.from_numpy(h_in).to(d), torch.from_numpy(done).to(d), 1, 0)
        torch.cuda.synchronize()
        for k in g:
            assert np.array_equal(g[k], out[k].cpu().numpy()), (net["name"], "misaligned", k)
        rows = np.arange(0, B, max(1, B // 40))
        o = ref.policy_step(net, w, obs[rows], h_in[rows], done[rows], 1, 0)
        parity.assert_close("h_out", g["h_out"][rows], o["h_out"], 2e-2)
        parity.assert_close("value", g["value"][rows], o["value"], 2e-2)
        fused.close()
        plain.close()


# frame shapes for the kernel that pools the first convolution in registers: odd height and a
# last column group with four live lanes; two frames with fewer pooled rows than waves;
# the benchmark's frame with more frames than workgroups (512), so some walk two
STEM_POOL_NETS = [dict(RESNET_BF16_SMALL, name="resnet_bf16_37x40", B=6, obs=(3, 37, 40)),
                  dict(RESNET_BF16_SMALL, name="resnet_bf16_9x12", B=3, obs=(3, 9, 12)),
                  dict(RESNET_BF16_SMALL, name="resnet_bf16_10x16", B=2, obs=(3, 10, 16)),
                  dict(RESNET_BF16_SMALL, name="resnet_bf16_72x128", B=600, obs=(3, 72, 128))]


@pytest.mark.parametrize("net", STEM_POOL_NETS, ids=lambda n: n["name"])
def test_first_convolution_pooled_in_registers(torch_cuda, ref, monkeypatch, net):
    """Residual encoder, fp16 activations: the first convolution and its max-pool as one launch
    that never stores the full-resolution output against the oracle, and against the kernel that
    pools out of LDS (same values up to the summation order inside the matrix cores)."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    w = wl.weights(net)
    B = net["B"]
    obs, h_in, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    pol = binding.Policy(net, w)
    assert pol.op_kernels()[0] == "stem_pool", pol.op_kernels()
    g = _gpu_step(torch, pol, obs, h_in, done, 7, 11)
    rows = np.arange(B) if B <= 16 else np.unique(np.concatenate([np.arange(0, B, 23), [B - 1, 511, 512]]))
    o = ref.policy_step(net, w, obs[rows], h_in[rows], done[rows], 7, 11)
    parity.assert_close("h_out", g["h_out"][rows], o["h_out"], 2e-2)
    parity.assert_close("value", g["value"][rows], o["value"], 2e-2)
    monkeypatch.setenv("SF_NO_STEM_POOL", "1")
    old = binding.Policy(net, w)
    monkeypatch.delenv("SF_NO_STEM_POOL")
    assert old.op_kernels()[0] == "conv3x3_pool", old.op_kernels()
    g2 = _gpu_step(torch, old, obs, h_in, done, 7, 11)
    parity.assert_close("h_out vs LDS-pooled kernel", g["h_out"], g2["h_out"], 4e-3)
    parity.assert_close("value vs LDS-pooled kernel", g["value"], g2["value"], 4e-3)
    pol.close()
    old.close()


# stage inputs for the kernel that pools a stage convolution in registers: 24 x 64 x 16 and
# 12 x 32 x 32 (one and two frames per workgroup round, more rounds than workgroups);
# 25 x 38 x 16 (odd height, 19 pooled columns); 19 x 20 and 10 x 10 (two frames per round, five
# and ten live lanes per frame); 5 x 8 and 3 x 4 (fewer pooled rows than waves); odd batch sizes
# leave the second frame of the last round empty
CONV_POOL_REGS_NETS = [(dict(RESNET_BF16_POW2, name="resnet_bf16_pow2_601", B=601), 2),
                       (dict(RESNET_BF16_MID, B=5), 1),
                       (dict(RESNET_BF16_SMALL, name="resnet_bf16_37x40", B=7, obs=(3, 37, 40)), 2),
                       (dict(RESNET_BF16_SMALL, name="resnet_bf16_10x16", B=3, obs=(3, 10, 16)), 2)]


@pytest.mark.parametrize("net,n_regs", CONV_POOL_REGS_NETS, ids=lambda v: v["name"] if isinstance(v, dict) else str(v))
def test_stage_convolution_pooled_in_registers(torch_cuda, ref, monkeypatch, net, n_regs):
    """Residual encoder, fp16 activations: the second and third stage convolutions with their
    max-pools as launches that never store the full-resolution output, against the oracle and
    against the kernels that pool out of LDS (same values up to the summation order inside the
    matrix cores)."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    w = wl.weights(net)
    B = net["B"]
    obs, h_in, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    pol = binding.Policy(net, w)
    assert pol.op_kernels().count("conv_pool_regs") == n_regs, pol.op_kernels()
    g = _gpu_step(torch, pol, obs, h_in, done, 7, 11)
    rows = np.arange(B) if B <= 16 else np.unique(np.concatenate([np.arange(0, B, 29), [B - 1, B - 2, 255, 256, 511, 512]]))
    o = ref.policy_step(net, w, obs[rows], h_in[rows], done[rows], 7, 11)
    parity.assert_close("h_out", g["h_out"][rows], o["h_out"], 2e-2)
    parity.assert_close("value", g["value"][rows], o["value"], 2e-2)
    monkeypatch.setenv("SF_NO_CONV_POOL_REGS", "1")
    old = binding.Policy(net, w)
    monkeypatch.delenv("SF_NO_CONV_POOL_REGS")
    assert "conv_pool_regs" not in old.op_kernels(), old.op_kernels()
    g2 = _gpu_step(torch, old, obs, h_in, done, 7, 11)
    parity.assert_close("h_out vs LDS-pooled kernels", g["h_out"], g2["h_out"], 4e-3)
    parity.assert_close("value vs LDS-pooled kernels", g["value"], g2["value"], 4e-3)
    pol.close()
    old.close()


# last-stage frames (32 channels) with fewer 32-pixel tiles than the stage kernel has waves: the
# kernel stacks them in its LDS image.  9 x 16 (three to a stack; 7 frames: the last stack holds
# one), 6 x 16 (four to a stack; 302 frames: more stacks than workgroups would be at 256, the last
# holds two), 13 x 16 (two to a stack, the last holds one); 5 x 32 and 3 x 16 (second and third
# stage both stacked by four, the last stack with three).
STACKED_STAGE_NETS = [(dict(RESNET_BF16_SMALL, name="resnet_bf16_72x128", B=7, obs=(3, 72, 128)), 3),
                      (dict(RESNET_BF16_SMALL, name="resnet_bf16_48x128", B=302, obs=(3, 48, 128)), 3),
                      (dict(RESNET_BF16_SMALL, name="resnet_bf16_100x128", B=5, obs=(3, 100, 128)), 2),
                      (dict(RESNET_BF16_SMALL, name="resnet_bf16_20x128", B=11, obs=(3, 20, 128)), 3)]


@pytest.mark.parametrize("net,n_stage", STACKED_STAGE_NETS, ids=lambda v: v["name"] if isinstance(v, dict) else str(v))
def test_small_stage_frames_stacked_in_lds(torch_cuda, ref, monkeypatch, net, n_stage):
    """Residual blocks of a stage whose frames are smaller than the stage kernel's eight tiles:
    several frames share one LDS image, a row of zeros between them.  Against the oracle, and
    against the per-block kernels (same arithmetic per output up to the summation order inside
    the matrix cores)."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    w = wl.weights(net)
    B = net["B"]
    obs, h_in, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    pol = binding.Policy(net, w)
    assert pol.op_kernels().count("res_stage") == n_stage, pol.op_kernels()
    g = _gpu_step(torch, pol, obs, h_in, done, 7, 11)
    rows = np.arange(B) if B <= 16 else np.unique(np.concatenate([np.arange(0, B, 23), np.arange(B - 6, B), [255, 256, 257]]))
    o = ref.policy_step(net, w, obs[rows], h_in[rows], done[rows], 7, 11)
    parity.assert_close("h_out", g["h_out"][rows], o["h_out"], 1e-2)
    parity.assert_close("value", g["value"][rows], o["value"], 1e-2)
    monkeypatch.setenv("SF_NO_RES_STAGE", "1")
    old = binding.Policy(net, w)
    monkeypatch.delenv("SF_NO_RES_STAGE")
    assert "res_stage" not in old.op_kernels(), old.op_kernels()
    g2 = _gpu_step(torch, old, obs, h_in, done, 7, 11)
    # (both keep the residual stream in fp16 and round it at different points: each measured about
    # 1e-3 from the oracle, so twice that from one another)
    parity.assert_close("h_out vs per-block kernels", g["h_out"], g2["h_out"], 1e-2)
    parity.assert_close("value vs per-block kernels", g["value"], g2["value"], 1e-2)
    pol.close()
    old.close()
