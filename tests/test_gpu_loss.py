"""GPU parity of the learner-side loss kernels (paper, Sec. 3.4 and the hyperparameter
table of App. "VizDoom experiments") against the oracle, through the C ABI: targets,
advantages, the four loss values and both gradients on seeded trajectory batches, including
trajectories longer than one wavefront, truncation levels below 1, episode ends, bitwise
reproducibility, and the error paths.
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu

RTOL = 1e-4

CASES = [
    ("paper_batch", wl.loss_config((7,), 32, 64), 6001),
    ("full_action_space", wl.loss_config((3, 3, 2, 2, 2, 8, 21), 16, 9), 6002),
    ("three_chunks", wl.loss_config((5, 4), 150, 3, rho_bar=0.9, c_bar=0.8, gamma=0.97), 6003),
    ("one_sample", wl.loss_config((2,), 1, 1), 6004),
    ("exact_chunk", wl.loss_config((6,), 64, 5), 6005),
    ("large", wl.loss_config((7,), 32, 2048), 6006),
    # 133 logits per sample: the tiles do not fit LDS, the kernel that reads memory directly runs
    ("wide_head_direct_kernel", wl.loss_config((130, 3), 20, 5), 6007),
    # an even number of logits (padded LDS rows, element-wise tile copies), three chunks of 64
    # steps, and a last workgroup with 3 of its 4 trajectories
    ("even_width_staged", wl.loss_config((60, 4), 150, 7), 6008),
    # 32 lanes per trajectory, eight per workgroup, the last workgroup with 3; 16-byte tile copies
    ("short_trajectories", wl.loss_config((5, 4), 32, 19), 6010),
    ("short_trajectories_scalar_copies", wl.loss_config((5, 4), 17, 19), 6011),
    ("full_action_space_large", wl.loss_config((3, 3, 2, 2, 2, 8, 21), 32, 515), 6009),
]


def _run(torch, hp, tr, grads=True):
    from paper_2006_11751_amd import binding
    d = torch.device("cuda", 0)
    dev = {k: torch.from_numpy(v).to(d) for k, v in tr.items()}
    out = binding.appo_loss(hp, dev, want_grads=grads)
    torch.cuda.synchronize()
    return {k: (v.cpu().numpy() if v is not None and k != "workspace" else None) for k, v in out.items()}


def _ratios(hp, tr):
    """fp64 importance ratios, only to find samples that sit on a clipping boundary."""
    lp, off = 0.0, 0
    for k, A in enumerate(hp["heads"]):
        l = tr["logits"][..., off:off + A].astype(np.float64)
        ls = l - l.max(-1, keepdims=True)
        ls = ls - np.log(np.exp(ls).sum(-1, keepdims=True))
        lp = lp + np.take_along_axis(ls, tr["actions"][..., k:k + 1].astype(np.int64), -1)[..., 0]
        off += A
    return np.exp(lp - tr["logp_mu"].astype(np.float64))


@pytest.mark.parametrize("name,hp,seed", CASES, ids=[c[0] for c in CASES])
def test_loss_matches_the_oracle(torch_cuda, ref, name, hp, seed):
    tr = wl.trajectories(hp, seed)
    g = _run(torch_cuda, hp, tr)
    o = ref.appo_loss(hp, **tr)
    stats = {k: parity.assert_close(k, g[k], o[k], RTOL) for k in ("vs", "adv", "dvalues")}
    # the loss values: each against its own magnitude plus the scale of the terms it sums
    scale = np.abs(o["loss"][:3]).max()
    assert np.all(np.abs(g["loss"] - o["loss"]) <= RTOL * (np.abs(o["loss"]) + scale)), (g["loss"], o["loss"])
    # the clipped / unclipped choice is a decision on ratio: samples within 1e-4 of a boundary
    # of the clipping range may legitimately fall on either side in fp32
    r = _ratios(hp, tr)
    clip = float(np.float32(hp["clip"]))
    sure = np.minimum(np.abs(r - clip), np.abs(r - 1.0 / clip)) > 1e-4
    assert sure.mean() > 0.99 or r.size < 200
    stats["dlogits"] = parity.assert_close("dlogits", g["dlogits"][sure], o["dlogits"][sure], RTOL)
    print(name, stats, "undecided samples:", int((~sure).sum()))


def test_forward_only_and_bitwise_reproducible(torch_cuda):
    hp = wl.loss_config((7,), 32, 64)
    tr = wl.trajectories(hp, 6001)
    a = _run(torch_cuda, hp, tr)
    b = _run(torch_cuda, hp, tr)
    c = _run(torch_cuda, hp, tr, grads=False)
    for k in ("vs", "adv", "loss", "dlogits", "dvalues"):
        assert np.array_equal(a[k], b[k]), k
    for k in ("vs", "adv", "loss"):
        assert np.array_equal(a[k], c[k]), k
    assert c["dlogits"] is None


def test_episode_ends_cut_the_recursion(torch_cuda):
    """Changing anything after a done does not change the targets before it."""
    hp = wl.loss_config((4,), 40, 2)
    tr = wl.trajectories(hp, 6010)
    tr["dones"][:] = 0
    tr["dones"][17, 0] = 1
    a = _run(torch_cuda, hp, tr)
    tr2 = {k: v.copy() for k, v in tr.items()}
    tr2["rewards"][18:, 0] += 3.0
    tr2["values"][18:, 0] -= 2.0
    b = _run(torch_cuda, hp, tr2)
    assert np.array_equal(a["vs"][:18, 0], b["vs"][:18, 0]) and np.array_equal(a["adv"][:18, 0], b["adv"][:18, 0])
    assert not np.array_equal(a["vs"][18:, 0], b["vs"][18:, 0])
    assert np.array_equal(a["vs"][:, 1], b["vs"][:, 1])


def test_loss_error_paths(torch_cuda):
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    hp = wl.loss_config((3,), 4, 2)
    for bad, code in [(dict(T=0), binding.SF_ERR_SHAPE), (dict(clip=0.5), binding.SF_ERR_SHAPE),
                      (dict(heads=[0]), binding.SF_ERR_SHAPE)]:
        cfg = binding.make_loss_config(dict(hp, **bad))
        assert binding.load_library().sf_appo_loss_workspace_bytes(cfg) == -1
        rc = binding.load_library().sf_appo_loss(cfg, *([None] * 13))
        assert rc == code
    cfg = binding.make_loss_config(hp)
    assert binding.sf_appo_loss_workspace_bytes(cfg) == 2 * 4 * 4 + 16   # partial sums + alignment room
    assert binding.load_library().sf_appo_loss(cfg, *([None] * 13)) == binding.SF_ERR_ARG
    cfg.struct_size = 8
    assert binding.load_library().sf_appo_loss(cfg, *([None] * 13)) == binding.SF_ERR_ARG


def test_loss_is_independent_of_the_workspace_contents(torch_cuda, ref):
    """Whatever the workspace held before (zeros, ones, random bytes, the previous call's partial
    sums), repeated calls on it give the same bits, and the loss terms equal the oracle's
    (515 trajectories: 129 workgroups, the last with three trajectories)."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    hp = wl.loss_config((3, 3, 2, 2, 2, 8, 21), 32, 515)
    tr = wl.trajectories(hp, 6020)
    d = torch.device("cuda", 0)
    dev = {k: torch.from_numpy(v).to(d) for k, v in tr.items()}
    out = binding.appo_loss(hp, dev)
    torch.cuda.synchronize()
    want = out["loss"].cpu().numpy().copy()
    o = ref.appo_loss(hp, **tr)
    scale = np.abs(o["loss"][:3]).max()
    assert np.all(np.abs(want - o["loss"]) <= RTOL * (np.abs(o["loss"]) + scale)), (want, o["loss"])
    cfg = binding.make_loss_config(hp)
    ws = out["workspace"]
    st = torch.cuda.current_stream().cuda_stream
    ptrs = [dev[k].data_ptr() for k in ("logits", "actions", "logp_mu", "values", "rewards", "dones")] + \
           [out[k].data_ptr() for k in ("vs", "adv", "loss", "dlogits", "dvalues", "workspace")]
    gen = torch.Generator(device="cpu").manual_seed(5)
    for fill in ("zeros", "ones", "random", "keep", "keep"):
        if fill == "zeros":
            ws.zero_()
        elif fill == "ones":
            ws.fill_(255)
        elif fill == "random":
            ws.copy_(torch.randint(0, 256, (ws.numel(),), dtype=torch.uint8, generator=gen))
        out["loss"].fill_(float("nan"))
        binding.sf_appo_loss(cfg, *ptrs, st)
        torch.cuda.synchronize()
        assert np.array_equal(out["loss"].cpu().numpy(), want), fill


def test_loss_replayed_from_a_graph(torch_cuda, ref):
    """The entry point that allocates nothing, recorded into a HIP graph once and replayed with the
    program's own eager calls and synchronisations in between: every replay gives the eager call's
    bits (two kernel nodes, no memset node: nothing has to start at zero)."""
    torch = torch_cuda
    from paper_2006_11751_amd import binding
    hp = wl.loss_config((3, 3, 2, 2, 2, 8, 21), 32, 259)
    tr = wl.trajectories(hp, 6021)
    d = torch.device("cuda", 0)
    dev = {k: torch.from_numpy(v).to(d) for k, v in tr.items()}
    eager = binding.appo_loss(hp, dev)
    torch.cuda.synchronize()
    want = {k: eager[k].cpu().numpy().copy() for k in ("vs", "adv", "loss", "dlogits", "dvalues")}
    cfg = binding.make_loss_config(hp)
    out = {k: torch.empty_like(eager[k]) for k in want}
    ptrs = [dev[k].data_ptr() for k in ("logits", "actions", "logp_mu", "values", "rewards", "dones")] + \
           [out[k].data_ptr() for k in ("vs", "adv", "loss", "dlogits", "dvalues")]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        binding.sf_appo_loss_static(cfg, *ptrs, side.cuda_stream)   # first use on this device, outside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        binding.sf_appo_loss_static(cfg, *ptrs, torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        for v in out.values():
            v.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in want:
            assert np.array_equal(out[k].cpu().numpy(), want[k]), (rep, k)
        # eager work of the same kind between the replays
        again = binding.appo_loss(hp, dev)
        torch.cuda.synchronize()
        assert np.array_equal(again["loss"].cpu().numpy(), want["loss"])
