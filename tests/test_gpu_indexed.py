"""GPU parity of the indexed step and the double-buffered pipeline (through the C ABI)
against the oracle's indexed step (paper, Sec. 3.2 double-buffered sampling, Sec. 3.3
index-based exchange): element by element on seeded inputs, untouched table rows bit for
bit, identity ids equal to the plain step, two slots in alternation over several steps,
ids outside the table, and the error paths.
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests import parity
from tests.test_gpu_parity import RESNET_BF16_SMALL, _make, _to_np

pytestmark = pytest.mark.gpu


def _table(net, n_env, seed=77):
    rng = np.random.default_rng(seed)
    return (0.1 * rng.standard_normal((n_env, net["rnn"]))).astype(np.float32)


def _ids(B, n_env, seed=5):
    return np.random.default_rng(seed).permutation(n_env)[:B].astype(np.int32)


def _gpu_indexed(torch, pol, obs, table_dev, ids, done, seed, step):
    d = pol.device
    out = pol.step_indexed(torch.from_numpy(obs).to(d), table_dev, torch.from_numpy(ids).to(d),
                           torch.from_numpy(done).to(d), seed, step)
    torch.cuda.synchronize()
    return _to_np(out)


STD_SMALL = wl.network(1, B=70, name="standard_small")
STD_BF16_SMALL = wl.network(2, B=37, name="standard_bf16_small")


@pytest.mark.parametrize("net", [wl.network(0), STD_SMALL, STD_BF16_SMALL, RESNET_BF16_SMALL],
                         ids=lambda n: n["name"])
def test_indexed_step_all_elements(torch_cuda, ref, net):
    torch = torch_cuda
    pol, w = _make(torch, net)
    B, n_env = net["B"], 3 * net["B"] + 5
    obs, done = wl.observations(net, 0, B), wl.done_mask(net, 0, B)
    ids = _ids(B, n_env)
    table = _table(net, n_env)
    before = table.copy()
    tdev = torch.from_numpy(table).to(pol.device)
    g = _gpu_indexed(torch, pol, obs, tdev, ids, done, 7, 11)
    o = ref.policy_step_indexed(net, w, obs, table, ids, done, 7, 11)   # updates `table`
    after = tdev.cpu().numpy()
    g["h_out"], o["h_out"] = after[ids], table[ids]
    parity.check_against_oracle(net, g, o, ref, 7, 11, rows=ids)
    rest = np.setdiff1d(np.arange(n_env), ids)
    assert np.array_equal(after[rest], before[rest])
    pol.close()


def test_identity_ids_equal_the_plain_step_bitwise(torch_cuda):
    torch = torch_cuda
    net = wl.network(1, B=200)
    pol, _ = _make(torch, net)
    B, d = net["B"], pol.device
    obs, h_in, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    plain = pol.step(torch.from_numpy(obs).to(d), torch.from_numpy(h_in).to(d),
                     torch.from_numpy(done).to(d), 3, 4)
    tdev = torch.from_numpy(h_in).to(d)
    idx = _gpu_indexed(torch, pol, obs, tdev, np.arange(B, dtype=np.int32), done, 3, 4)
    plain = _to_np(plain)
    assert np.array_equal(tdev.cpu().numpy(), plain["h_out"])
    for k in ("actions", "logp", "value", "logits"):
        assert np.array_equal(idx[k], plain[k]), k
    pol.close()


def test_ids_outside_the_table_read_zero_state_and_write_nothing(torch_cuda):
    torch = torch_cuda
    net = wl.network(0)
    pol, _ = _make(torch, net)
    B, n_env, d = net["B"], 20, pol.device
    obs, done = wl.observations(net, 0, B), np.zeros(B, np.uint8)
    ids = _ids(B, n_env)
    table = _table(net, n_env)
    good = torch.from_numpy(table).to(d)
    g = _gpu_indexed(torch, pol, obs, good, ids, done, 1, 0)
    bad_ids = ids.copy()
    bad_ids[2], bad_ids[5] = n_env, -3
    bad = torch.from_numpy(table).to(d)
    b = _gpu_indexed(torch, pol, obs, bad, bad_ids, done, 1, 0)
    keep = np.ones(B, bool)
    keep[[2, 5]] = False
    for k in ("logits", "value"):
        assert np.array_equal(b[k][keep], g[k][keep]), k
    ga, ba = good.cpu().numpy(), bad.cpu().numpy()
    assert np.array_equal(ba[ids[keep]], ga[ids[keep]])
    assert np.array_equal(ba[ids[~keep]], table[ids[~keep]])      # never written
    # the two rows were computed from a zero state: same logits as with done = 1
    done1 = done.copy()
    done1[[2, 5]] = 1
    z = _gpu_indexed(torch, pol, obs, torch.from_numpy(table).to(d), ids, done1, 1, 0)
    assert np.array_equal(b["logits"][~keep], z["logits"][~keep])
    pol.close()


def test_pipeline_two_slots_alternating(torch_cuda, ref):
    """Two halves of the environments take turns for several steps; every result equals
    the oracle's alternation, and the direct indexed calls bit for bit."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    net = wl.network(0)
    n_env, half, steps = 16, 8, 3
    pol, w = _make(torch, net, max_batch=half)
    pol2, _ = _make(torch, net, max_batch=half)
    d = pol.device
    table0 = _table(net, n_env)
    t_pipe = torch.from_numpy(table0).to(d)
    t_direct = torch.from_numpy(table0).to(d)
    t_ref = table0.copy()
    pipe = binding.Pipeline(pol, half, 2)
    hb = [pipe.host_buffers(), pipe.host_buffers()]
    groups = [np.arange(0, half, dtype=np.int32), np.arange(half, n_env, dtype=np.int32)]
    for t in range(steps):
        obs, done = wl.observations(net, t, n_env), wl.done_mask(net, t, n_env)
        for s in (0, 1):
            ids = groups[s]
            hb[s]["obs"].copy_(torch.from_numpy(obs[ids]))
            hb[s]["done"].copy_(torch.from_numpy(done[ids]))
            hb[s]["env_ids"].copy_(torch.from_numpy(ids))
            pipe.submit(s, hb[s], t_pipe, wl.PHILOX_SEED, t)
        for s in (0, 1):
            pipe.wait(s)
            ids = groups[s]
            o = ref.policy_step_indexed(net, w, obs[ids], t_ref, ids, done[ids], wl.PHILOX_SEED, t)
            g = _gpu_indexed(torch, pol2, obs[ids], t_direct, ids, done[ids], wl.PHILOX_SEED, t)
            assert np.array_equal(hb[s]["actions"].numpy(), g["actions"])
            assert np.array_equal(hb[s]["logp"].numpy(), g["logp"])
            assert np.array_equal(hb[s]["value"].numpy(), g["value"])
            g["h_out"], o["h_out"] = t_direct.cpu().numpy()[ids], t_ref[ids]
            parity.check_against_oracle(net, g, o, ref, wl.PHILOX_SEED, t, rows=ids)
        assert np.array_equal(t_pipe.cpu().numpy(), t_direct.cpu().numpy())
    pipe.close()
    pol.close()
    pol2.close()


def test_pipeline_standard_size_one_and_two_slots_agree(torch_cuda):
    """Configuration 1's shapes, B = 1024 as two slots of 512, against one slot of 1024."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    net = wl.network(1)
    B = net["B"]
    pol, _ = _make(torch, net)
    d = pol.device
    obs, done = wl.observations(net), wl.done_mask(net)
    table0 = wl.initial_state(net)
    ids = np.arange(B, dtype=np.int32)
    res = {}
    for n_slots in (1, 2):
        tab = torch.from_numpy(table0).to(d)
        per = B // n_slots
        pipe = binding.Pipeline(pol, per, n_slots)
        hbs = [pipe.host_buffers() for _ in range(n_slots)]
        for s in range(n_slots):
            sl = slice(s * per, (s + 1) * per)
            hbs[s]["obs"].copy_(torch.from_numpy(obs[sl]))
            hbs[s]["done"].copy_(torch.from_numpy(done[sl]))
            hbs[s]["env_ids"].copy_(torch.from_numpy(ids[sl]))
            pipe.submit(s, hbs[s], tab, 1, 0)
        for s in range(n_slots):
            pipe.wait(s)
        res[n_slots] = (np.concatenate([h["actions"].numpy() for h in hbs]),
                        np.concatenate([h["logp"].numpy() for h in hbs]), tab.cpu().numpy())
        pipe.close()
    for a, b in zip(res[1], res[2]):
        assert np.array_equal(a, b)
    pol.close()


def test_indexed_and_pipeline_error_paths(torch_cuda):
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    net = wl.network(0)
    pol, _ = _make(torch, net)
    d = pol.device
    B = net["B"]
    obs = torch.from_numpy(wl.observations(net, 0, B)).to(d)
    done = torch.zeros(B, dtype=torch.uint8, device=d)
    ids = torch.arange(B, dtype=torch.int32, device=d)
    tab = torch.zeros((B, net["rnn"]), dtype=torch.float32, device=d)
    out = pol.alloc_outputs(B)

    def call(**kw):
        a = dict(B=B, obs=obs.data_ptr(), tab=tab.data_ptr(), n_env=B, ids=ids.data_ptr())
        a.update(kw)
        binding.sf_policy_step_indexed(pol.handle, a["B"], a["obs"], None, a["tab"], a["n_env"], a["ids"],
                                       done.data_ptr(), 1, 0, out["actions"].data_ptr(),
                                       out["logp"].data_ptr(), out["value"].data_ptr(), None, None)

    for kw, code in [(dict(B=B + 1), binding.SF_ERR_BATCH), (dict(obs=None), binding.SF_ERR_ARG),
                     (dict(ids=None), binding.SF_ERR_ARG), (dict(n_env=0), binding.SF_ERR_ARG),
                     (dict(tab=tab.data_ptr() + 4), binding.SF_ERR_ARG)]:
        with pytest.raises(binding.SfError) as e:
            call(**kw)
        assert e.value.code == code
    call(B=0)

    with pytest.raises(binding.SfError) as e:
        binding.sf_pipeline_create(pol.handle, B + 1, 2)
    assert e.value.code == binding.SF_ERR_BATCH
    with pytest.raises(binding.SfError) as e:
        binding.sf_pipeline_create(pol.handle, B, 3)
    assert e.value.code == binding.SF_ERR_ARG
    pipe = binding.Pipeline(pol, B, 2)
    hb = pipe.host_buffers()
    hb["obs"].copy_(obs.cpu())
    hb["done"].zero_()
    hb["env_ids"].copy_(ids.cpu())
    pipe.submit(0, hb, tab, 1, 0)
    with pytest.raises(binding.SfError) as e:      # slot 0 is in flight
        pipe.submit(0, hb, tab, 1, 1)
    assert e.value.code == binding.SF_ERR_ARG
    with pytest.raises(binding.SfError) as e:
        pipe.submit(2, hb, tab, 1, 1)
    assert e.value.code == binding.SF_ERR_ARG
    pipe.wait(0)
    pipe.wait(1)                                    # idle slot: returns at once
    pipe.close()
    pol.close()
