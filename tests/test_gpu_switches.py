"""Every kernel-selection switch still gives the oracle's result: the fallback kernels
(shape-agnostic kernels, fp32 kernels on bf16 weights, per-layer residual-encoder kernels,
fp32-MFMA core in bf16 configurations, fp32 first convolution) are exercised on small
networks through the C ABI.  The switches are read when a policy is created, once: a weight
update on such a policy, made after the variable has been removed, still packs for the kernels
chosen at create.
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests import parity
from tests.test_gpu_parity import RESNET_BF16_MID, RESNET_BF16_POW2, RESNET_BF16_SMALL, _make, _to_np
from tests.test_gpu_core import NETS

pytestmark = pytest.mark.gpu

STD_SMALL = wl.network(1, B=70, name="standard_small")
STD_BF16_SMALL = wl.network(2, B=37, name="standard_bf16_small")
BY_NAME = {n["name"]: n for n in NETS}

CASES = [
    ("SF_FORCE_GENERIC", "1", STD_SMALL),
    ("SF_FORCE_GENERIC", "1", BY_NAME["lstm_mfma"]),
    ("SF_FORCE_GENERIC", "1", BY_NAME["full_mfma"]),
    ("SF_FORCE_GENERIC", "1", RESNET_BF16_SMALL),
    ("SF_CONV1", "fp32", STD_SMALL),
    ("SF_CONV1", "i8", STD_SMALL),
    ("SF_GEMM_TILE", "4", STD_SMALL),
    ("SF_GRU_BM", "64", STD_SMALL),
    ("SF_NO_RNN_PAIRS", "1", STD_SMALL),
    ("SF_NO_BF16_PATH", "1", STD_BF16_SMALL),
    ("SF_NO_RNN_BF16", "1", STD_BF16_SMALL),
    ("SF_CONV_BF16_TC", "2", STD_BF16_SMALL),
    ("SF_FC_OUT_F32", "1", STD_BF16_SMALL),
    ("SF_NO_CONV_IMAGE", "1", STD_BF16_SMALL),
    ("SF_NO_CONV12_FUSE", "1", STD_BF16_SMALL),
    ("SF_NO_RNN_BF16", "1", BY_NAME["lstm_bf16_mfma"]),
    ("SF_NO_FUSED_RESNET", "1", RESNET_BF16_MID),
    ("SF_NO_RES_STAGE", "1", dict(RESNET_BF16_POW2, B=9)),
    ("SF_NO_STEM_POOL", "1", RESNET_BF16_MID),
    ("SF_NO_CONV_POOL_REGS", "1", RESNET_BF16_MID),
    ("SF_NO_PATCH_CONV", "1", RESNET_BF16_SMALL),
    ("SF_STREAM_F32", "1", RESNET_BF16_SMALL),
]


@pytest.mark.parametrize("var,val,net", CASES, ids=["%s=%s-%s" % (v, x, n["name"]) for v, x, n in CASES])
def test_switch(torch_cuda, ref, monkeypatch, var, val, net):
    torch = torch_cuda
    monkeypatch.setenv(var, val)
    pol, w = _make(torch, net)
    monkeypatch.delenv(var)
    d = pol.device
    B = net["B"]
    obs, state, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    meas = wl.measurements(net, 0, B)
    out = pol.step(torch.from_numpy(obs).to(d), torch.from_numpy(state).to(d), torch.from_numpy(done).to(d),
                   5, 3, meas=None if meas is None else torch.from_numpy(meas).to(d))
    torch.cuda.synchronize()
    o = ref.policy_step(net, w, obs, state, done, 5, 3, meas=meas)
    parity.check_against_oracle(net, _to_np(out), o, ref, 5, 3)
    # The switches were read at create and are kept in the policy: a weight update made after
    # the variable is gone must pack for the kernels chosen then, not for the default ones.
    w2 = wl.weights(net, seed=9090)
    pol.update_weights(w2)
    out = pol.step(torch.from_numpy(obs).to(d), torch.from_numpy(state).to(d), torch.from_numpy(done).to(d),
                   5, 3, meas=None if meas is None else torch.from_numpy(meas).to(d))
    torch.cuda.synchronize()
    o = ref.policy_step(net, w2, obs, state, done, 5, 3, meas=meas)
    parity.check_against_oracle(net, _to_np(out), o, ref, 5, 3)
    pol.close()
