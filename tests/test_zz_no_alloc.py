"""The entry point that allocates nothing: sf_appo_loss_static keeps the per-trajectory partial
sums in an array inside the library's device image instead of a caller workspace.  Through the
C ABI, twice in a row on one GPU, the second call on a smaller batch (so that stale contents of
the shared array beyond its N would show): every output must equal sf_appo_loss's bit for bit
(same kernels), and match the oracle to the fp32 tolerance; a batch beyond the built-in limit is
refused with a clear error.
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu


def _both(torch, binding, hp, seed):
    d = torch.device("cuda", 0)
    tr_np = wl.trajectories(hp, seed)
    tr = {k: torch.from_numpy(v).to(d) for k, v in tr_np.items()}
    T, N, sumA = tr["logits"].shape
    want = binding.appo_loss(hp, tr)            # the existing entry point, caller workspace
    got = dict(vs=torch.full((T, N), 7.0, device=d), adv=torch.full((T, N), 7.0, device=d),
               loss=torch.full((4,), 7.0, device=d), dlogits=torch.full((T, N, sumA), 7.0, device=d),
               dvalues=torch.full((T, N), 7.0, device=d))
    p = lambda x: x.data_ptr()
    binding.sf_appo_loss_static(binding.make_loss_config(hp), p(tr["logits"]), p(tr["actions"]), p(tr["logp_mu"]),
                                p(tr["values"]), p(tr["rewards"]), p(tr["dones"]), p(got["vs"]), p(got["adv"]),
                                p(got["loss"]), p(got["dlogits"]), p(got["dvalues"]),
                                torch.cuda.current_stream(d).cuda_stream)
    torch.cuda.synchronize()
    return tr_np, {k: got[k].cpu().numpy() for k in got}, {k: want[k].cpu().numpy() for k in got}


def test_static_scratch_entry_point_twice_second_call_smaller(torch_cuda, ref):
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    assert binding.load_library().sf_appo_loss_static_max_trajectories() == 16384
    for hp, seed in ((wl.loss_config((3, 3, 2, 2, 2, 8, 21), 32, 300), 6101),
                     (wl.loss_config((7,), 70, 37, rho_bar=0.9, c_bar=0.8), 6102)):
        tr, got, want = _both(torch, binding, hp, seed)
        for k in got:
            assert np.array_equal(got[k], want[k]), k
        o = ref.appo_loss(hp, **tr)
        for k in ("vs", "adv", "dvalues"):
            parity.assert_close(k, got[k], o[k], 1e-4)
        scale = np.abs(o["loss"][:3]).max()
        assert np.all(np.abs(got["loss"] - o["loss"]) <= 1e-4 * (np.abs(o["loss"]) + scale))


def test_static_scratch_entry_point_rejects_sizes_beyond_its_limit(torch_cuda):
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    hp = wl.loss_config((2,), 1, 16385)
    x = torch.zeros(8, device="cuda")
    with pytest.raises(binding.SfError) as e:
        binding.sf_appo_loss_static(binding.make_loss_config(hp), *([x.data_ptr()] * 11), None)
    assert e.value.code == binding.SF_ERR_SHAPE and "16384" in str(e.value)
    with pytest.raises(binding.SfError) as e:   # argument checks still come first
        binding.sf_appo_loss_static(binding.make_loss_config(wl.loss_config((2,), 4, 4)), None,
                                    *([x.data_ptr()] * 10), None)
    assert e.value.code == binding.SF_ERR_ARG
