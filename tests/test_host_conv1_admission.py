"""Host logic of the library, no GPU: the admission test that decides whether the first
convolution may run on int8 digit planes (a per-channel fixed-point image of its filter bank)
instead of fp32.  The library's figures are compared with an independent numpy computation of
the same definition, and the decision is checked on the filter families that a fixed-point
image handles well and badly.  Alongside, an fp64 emulation of the digit-plane arithmetic shows
what the decision protects: admitted banks stay far inside the fp32 tolerance even on the
frames that are worst for them, rejected ones do not."""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl

NET = dict(name="one_conv", B=6, obs=(3, 36, 64), encoder="conv", convs=[(32, 8, 4, 0)], fc=64, rnn=32,
           heads=[5], dtype="fp32", p_done=0.3, steps=1, obs_sub=0.0, obs_mul=wl.OBS_MUL, index=0)


def _digits(wp, planes):
    """Fixed-point image of one channel's folded taps wp (fp64): scale max/127 held in fp32,
    signed digits of radix 254."""
    mx = np.abs(wp).max()
    s = float(np.float32(mx / 127.0)) if mx > 0 else 1.0
    q = wp / s
    d1 = np.clip(np.rint(q), -127, 127)
    r = (q - d1) * 254.0
    d2 = np.clip(np.rint(r), -127, 127)
    d3 = np.clip(np.rint((r - d2) * 254.0), -127, 127)
    return s * (d1 + d2 / 254.0 + (d3 / 64516.0 if planes == 3 else 0.0))


def _ratios(conv_w, obs_mul, bf16):
    a = wl.round_to_bf16(conv_w) if bf16 else np.asarray(conv_w, np.float32)
    worst = [0.0, 0.0]
    for n in range(a.shape[0]):
        wp = np.float64(np.float32(obs_mul)) * a[n].astype(np.float64).ravel()
        K = wp.size
        mag = np.sort(np.abs(wp[wp != 0]))
        if mag.size == 0:
            continue
        m = mag[(mag.size - 1) // 2]
        l1 = np.minimum(np.abs(wp), m).sum()
        refs = (2.0 ** -9 * 255.0 * l1, np.sqrt(K) * 2.0 ** -24 * 255.0 * l1)
        for i, planes in enumerate((2, 3)):
            e_fix = 128.0 * np.abs(wp - _digits(wp, planes)).sum()
            worst[i] = max(worst[i], e_fix / refs[i])
    return tuple(worst)


def _bank(kind):
    w = wl.weights(NET, seed=31)
    if kind != "gaussian":
        w = wl.conv1_family(NET, w, kind)
    return w["conv_w"][0]


@pytest.mark.parametrize("kind", ("gaussian",) + wl.CONV1_FAMILIES)
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_library_ratio_equals_the_definition(kind, dtype):
    from paper_2006_11751_amd import binding
    bank = _bank(kind)
    got = binding.sf_conv1_fixed_point_test(bank, wl.OBS_MUL, dtype)
    want = _ratios(bank, wl.OBS_MUL, dtype == "bf16")
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-300)


def test_decisions_on_the_families():
    from paper_2006_11751_amd import binding
    r3 = {k: binding.sf_conv1_fixed_point_test(_bank(k), wl.OBS_MUL, "fp32")[1]
          for k in ("gaussian",) + wl.CONV1_FAMILIES}
    # admitted: the benchmark recipe (with a wide margin, whatever the seed), all-zero filters,
    # equal tiny taps (exact: one digit), a 1:40 split
    assert r3["gaussian"] < 0.25 and r3["zero_channel"] < 0.25
    assert r3["tiny_equal"] < 0.05 and r3["half_half_40"] < 1.0
    # rejected: one dominant tap, four decades of magnitudes, a 1:1000 split
    assert r3["dominant"] > 10 and r3["log_uniform"] > 1.0 and r3["half_half_1000"] > 10
    for seed in range(20):   # the benchmark recipe never comes near the limit
        w = wl.weights(wl.network(1), seed=seed)["conv_w"][0]
        assert binding.sf_conv1_fixed_point_test(w, wl.OBS_MUL, "fp32")[1] < 0.25
    # bf16 parameters: two planes are admitted for the recipe, not for a dominant tap
    assert binding.sf_conv1_fixed_point_test(_bank("gaussian"), wl.OBS_MUL, "bf16")[0] < 0.1
    assert binding.sf_conv1_fixed_point_test(_bank("dominant"), wl.OBS_MUL, "bf16")[0] > 1.0


def test_bad_arguments():
    from paper_2006_11751_amd import binding
    lib = binding.load_library()
    import ctypes as C
    r = C.c_double()
    a = np.zeros((32, 2, 8, 8), np.float32)
    assert lib.sf_conv1_fixed_point_test(a.ctypes.data, 2, 1.0, 0, C.byref(r), C.byref(r)) == binding.SF_ERR_ARG
    assert lib.sf_conv1_fixed_point_test(None, 3, 1.0, 0, C.byref(r), C.byref(r)) == binding.SF_ERR_ARG


@pytest.mark.parametrize("kind", ("gaussian",) + wl.CONV1_FAMILIES)
def test_what_the_decision_protects(kind):
    """fp64 emulation of the three-plane arithmetic on the family's worst frames: relative to
    the rms of the layer's pre-activations, an admitted bank errs by less than a tenth of the fp32
    tolerance (1e-4); the rejected dominant-tap and 1:1000 banks exceed a quarter of it, which
    is why they must not run in fixed point."""
    from paper_2006_11751_amd import binding
    bank = _bank(kind)
    ratio = binding.sf_conv1_fixed_point_test(bank, wl.OBS_MUL, "fp32")[1]
    obs = wl.conv1_family_frames(NET, kind, wl.observations(NET, 0, 4, seed=5))
    # all 8x8 windows at stride 4 as rows [pixels][K]
    C_, H, W = NET["obs"]
    cols = []
    for b in range(obs.shape[0]):
        for i in range((H - 8) // 4 + 1):
            for j in range((W - 8) // 4 + 1):
                cols.append(obs[b, :, 4 * i:4 * i + 8, 4 * j:4 * j + 8].ravel())
    X = np.asarray(cols, np.float64)
    worst = 0.0
    for n in range(32):
        wp = np.float64(np.float32(wl.OBS_MUL)) * bank[n].astype(np.float64).ravel()
        exact = X @ wp
        fixed = (X - 128.0) @ _digits(wp, 3) + 128.0 * wp.sum()
        rms = np.sqrt(np.mean(exact ** 2))
        if rms > 0:
            worst = max(worst, np.abs(fixed - exact).max() / rms)
    if ratio <= 1.0:
        assert worst < 1e-5, (kind, ratio, worst)
    elif kind in ("dominant", "half_half_1000"):
        assert worst > 2.5e-5, (kind, ratio, worst)
