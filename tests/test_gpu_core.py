"""GPU parity of the LSTM core and of the "full" architecture's measurement input
(paper, App. "Model architectures", App. "VizDoom experiments") against the oracle,
through the C ABI: small networks on every element (generic and MFMA kernels), the two
benchmark-shaped configurations at full size, chained steps with the state carried, and
the indexed / pipelined variants with [h | c] state rows and a measurement vector.
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests import parity
from tests.test_gpu_parity import _make, _to_np

pytestmark = pytest.mark.gpu

_BASE = dict(B=37, obs=(3, 36, 64), encoder="conv", convs=[(16, 8, 4, 0), (32, 4, 2, 0)], dtype="fp32",
             p_done=0.3, steps=1, obs_sub=0.0, obs_mul=wl.OBS_MUL, meas_dim=0, meas_hidden=[], rnn_type="gru")
NETS = [
    dict(_BASE, name="lstm_odd", fc=24, rnn=20, rnn_type="lstm", heads=[5, 3], index=5),          # generic kernels
    dict(_BASE, name="lstm_mfma", fc=64, rnn=64, rnn_type="lstm", heads=[6], index=5),            # MFMA, BM=32
    dict(_BASE, name="lstm_bf16", fc=64, rnn=96, rnn_type="lstm", heads=[4, 4], index=5, dtype="bf16"),
    dict(_BASE, name="full_odd", fc=24, rnn=20, meas_dim=7, meas_hidden=[10, 6], heads=[3, 3, 2, 2, 2, 8, 21], index=6),
    dict(_BASE, name="full_mfma", fc=64, rnn=64, meas_dim=23, meas_hidden=[40, 32], heads=[3, 3, 2, 2, 2, 8, 21], index=6),
    dict(_BASE, name="full_lstm_mfma", fc=96, rnn=32, rnn_type="lstm", meas_dim=5, meas_hidden=[64], heads=[7], index=6),
    dict(_BASE, name="full_mixed", fc=64, rnn=64, meas_dim=9, meas_hidden=[17], heads=[2, 3], index=6),  # x2 not a K chunk
    # bf16 configurations whose core runs on the 16-bit MFMA (64-wide K chunks), ragged batch of 137
    dict(_BASE, name="lstm_bf16_mfma", B=137, fc=64, rnn=128, rnn_type="lstm", heads=[4, 4], index=5, dtype="bf16"),
    dict(_BASE, name="gru_bf16_mfma", B=137, fc=128, rnn=64, heads=[9], index=5, dtype="bf16"),
    dict(_BASE, name="full_bf16_mfma", B=137, fc=64, rnn=64, meas_dim=11, meas_hidden=[20, 64], heads=[3, 2], index=6,
         dtype="bf16"),
    # GRU of a bf16 configuration with 128 and 256 hidden units (several unit tiles per row block;
    # ragged batches of 137 and 65 rows; bf16 features from the FC kernel, and fp32 ones with a
    # measurement input)
    dict(_BASE, name="gru_bf16_wide", B=137, fc=64, rnn=128, heads=[5], index=5, dtype="bf16"),
    dict(_BASE, name="full_bf16_wide", B=65, fc=128, rnn=256, meas_dim=7, meas_hidden=[64], heads=[4, 2], index=6,
         dtype="bf16"),
]


def _gpu_step(torch, pol, net, obs, state, done, seed, step, meas):
    d = pol.device
    out = pol.step(torch.from_numpy(obs).to(d), torch.from_numpy(state).to(d), torch.from_numpy(done).to(d),
                   seed, step, meas=None if meas is None else torch.from_numpy(meas).to(d))
    torch.cuda.synchronize()
    return _to_np(out)


@pytest.mark.parametrize("net", NETS, ids=lambda n: n["name"])
def test_small_networks_all_elements(torch_cuda, ref, net):
    torch = torch_cuda
    pol, w = _make(torch, net)
    B = net["B"]
    obs, state, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    meas = wl.measurements(net, 0, B)
    assert state.shape[1] == wl.state_dim(net) == pol.H
    g = _gpu_step(torch, pol, net, obs, state, done, 7, 11, meas)
    o = ref.policy_step(net, w, obs, state, done, 7, 11, meas=meas)
    parity.check_against_oracle(net, g, o, ref, 7, 11)
    pol.close()


@pytest.mark.parametrize("index", [5, 6])
def test_benchmark_shaped_configurations_full_batch_chained(torch_cuda, ref, index):
    """standard_lstm and full (B=1024): every row, 2 free-running steps, each side carrying
    its own state."""
    torch = torch_cuda
    net = wl.network(index)
    pol, w = _make(torch, net)
    s_gpu = wl.initial_state(net)
    s_ref = s_gpu.copy()
    for t in range(2):
        obs, done, meas = wl.observations(net, t), wl.done_mask(net, t), wl.measurements(net, t)
        g = _gpu_step(torch, pol, net, obs, s_gpu, done, wl.PHILOX_SEED, t, meas)
        o = ref.policy_step(net, w, obs, s_ref, done, wl.PHILOX_SEED, t, meas=meas)
        stats = parity.check_against_oracle(net, g, o, ref, wl.PHILOX_SEED, t)
        print(net["name"], "step", t, stats)
        s_gpu, s_ref = g["h_out"], o["h_out"]
    pol.close()


def test_lstm_done_resets_both_halves(torch_cuda):
    torch = torch_cuda
    net = NETS[1]
    pol, _ = _make(torch, net)
    B = net["B"]
    obs, state = wl.observations(net, 0, B), wl.initial_state(net, B)
    done = (np.arange(B) % 3 == 0).astype(np.uint8)
    a = _gpu_step(torch, pol, net, obs, state, done, 1, 0, None)
    other = state.copy()
    other[done == 1] = 9.0
    b = _gpu_step(torch, pol, net, obs, other, done, 1, 0, None)
    zero = state.copy()
    zero[done == 1] = 0.0
    c = _gpu_step(torch, pol, net, obs, zero, np.zeros(B, np.uint8), 1, 0, None)
    for k in ("h_out", "logits", "value", "actions", "logp"):
        assert np.array_equal(a[k], b[k]) and np.array_equal(a[k], c[k]), k
    pol.close()


@pytest.mark.parametrize("net", [NETS[1], NETS[5], NETS[3], NETS[7], NETS[9]], ids=lambda n: n["name"])
def test_indexed_step_and_pipeline_with_wide_state_rows_and_measurements(torch_cuda, ref, net):
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    pol, w = _make(torch, net)
    d = pol.device
    B, n_env, S = net["B"], 2 * net["B"] + 3, wl.state_dim(net)
    obs, done, meas = wl.observations(net, 0, B), wl.done_mask(net, 0, B), wl.measurements(net, 0, B)
    ids = np.random.default_rng(3).permutation(n_env)[:B].astype(np.int32)
    table = (0.1 * np.random.default_rng(4).standard_normal((n_env, S))).astype(np.float32)
    before = table.copy()
    tdev = torch.from_numpy(table).to(d)
    out = pol.step_indexed(torch.from_numpy(obs).to(d), tdev, torch.from_numpy(ids).to(d),
                           torch.from_numpy(done).to(d), 7, 2,
                           meas=None if meas is None else torch.from_numpy(meas).to(d))
    torch.cuda.synchronize()
    g = _to_np(out)
    o = ref.policy_step_indexed(net, w, obs, table, ids, done, 7, 2, meas=meas)
    after = tdev.cpu().numpy()
    g["h_out"], o["h_out"] = after[ids], table[ids]
    parity.check_against_oracle(net, g, o, ref, 7, 2, rows=ids)
    rest = np.setdiff1d(np.arange(n_env), ids)
    assert np.array_equal(after[rest], before[rest])
    # the pipeline gives the same bits as the direct call
    t2 = torch.from_numpy(before).to(d)
    pipe = binding.Pipeline(pol, B, 1)
    hb = pipe.host_buffers()
    hb["obs"].copy_(torch.from_numpy(obs))
    hb["done"].copy_(torch.from_numpy(done))
    hb["env_ids"].copy_(torch.from_numpy(ids))
    if meas is not None:
        hb["meas"].copy_(torch.from_numpy(meas))
    pipe.submit(0, hb, t2, 7, 2)
    pipe.wait(0)
    assert np.array_equal(hb["actions"].numpy(), g["actions"])
    assert np.array_equal(hb["logp"].numpy(), g["logp"])
    assert np.array_equal(t2.cpu().numpy(), after)
    pipe.close()
    pol.close()


def test_create_rejects_bad_core_descriptions(torch_cuda):
    from paper_2006_11751_amd import binding
    net = NETS[4]
    w = wl.weights(net)
    ws, keep = binding.make_weights(w)
    for patch, code in [(dict(rnn_type=2), binding.SF_ERR_SHAPE), (dict(meas_dim=-1), binding.SF_ERR_SHAPE),
                        (dict(n_meas_layers=3), binding.SF_ERR_SHAPE), (dict(n_meas_layers=0), binding.SF_ERR_SHAPE)]:
        cfg = binding.make_config(net, 8)
        for k, v in patch.items():
            setattr(cfg, k, v)
        with pytest.raises(binding.SfError) as e:
            binding.sf_policy_create(cfg, ws, 0)
        assert e.value.code == code
    cfg = binding.make_config(net, 8)
    ws2, keep2 = binding.make_weights(dict(w, meas_w=[w["meas_w"][0]], meas_b=[w["meas_b"][0]]))
    with pytest.raises(binding.SfError) as e:                 # second measurement layer missing
        binding.sf_policy_create(cfg, ws2, 0)
    assert e.value.code == binding.SF_ERR_ARG
    # a policy with a measurement input refuses a step without it
    pol = binding.Policy(net, w, max_batch=8)
    import torch
    d = pol.device
    out = pol.alloc_outputs(8)
    with pytest.raises(binding.SfError) as e:
        binding.sf_policy_step(pol.handle, 8, torch.zeros((8,) + net["obs"], dtype=torch.uint8, device=d).data_ptr(),
                               None, torch.zeros((8, pol.H), device=d).data_ptr(),
                               torch.zeros(8, dtype=torch.uint8, device=d).data_ptr(), 1, 0,
                               out["actions"].data_ptr(), out["logp"].data_ptr(), out["value"].data_ptr(),
                               out["h_out"].data_ptr(), None, None)
    assert e.value.code == binding.SF_ERR_ARG
    pol.close()
