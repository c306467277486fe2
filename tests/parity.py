"""Comparison rules shared by the GPU parity tests.

Floating point: |gpu - ref| <= rtol * |ref| + atol with atol = rtol * rms(ref
tensor); rtol = 1e-4 for fp32 configurations, 2e-2 for bf16 ones.
Actions: bit-identical, except in heads whose top-2 perturbed-logit margin in the
oracle is below 1e-3 (fp32).  For bf16 configurations a mismatch is accepted only
if that margin is below twice the largest logit error of the row; the sampler
itself is checked exactly by running the oracle's sampler on the GPU's logits.
"""
import numpy as np

RTOL = {"fp32": 1e-4, "bf16": 2e-2}
MARGIN = 1e-3


def violation(gpu, ref, rtol):
    """max over elements of |gpu - ref| / (rtol*|ref| + atol); <= 1 passes."""
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    atol = rtol * float(np.sqrt(np.mean(ref * ref)))
    bound = rtol * np.abs(ref) + max(atol, 1e-30)
    return float(np.max(np.abs(gpu - ref) / bound))


def assert_close(name, gpu, ref, rtol):
    assert np.all(np.isfinite(np.asarray(gpu))), name + " has non-finite values"
    v = violation(gpu, ref, rtol)
    assert v <= 1.0, "%s: violation ratio %.3f (rtol %.0e)" % (name, v, rtol)
    return v


def check_against_oracle(net, gpu, ora, ref_mod, seed, step, rows=None):
    """gpu, ora: dicts of numpy arrays with keys actions, logp, value, h_out,
    logits (ora also margin).  rows: the batch row index of each compared row
    (the sampler's env word); default 0..n-1."""
    rtol = RTOL[net["dtype"]]
    n = ora["h_out"].shape[0]
    rows = np.arange(n) if rows is None else np.asarray(rows)
    stats = {}
    stats["h_out"] = assert_close("h_out", gpu["h_out"], ora["h_out"], rtol)
    stats["logits"] = assert_close("logits", gpu["logits"], ora["logits"], rtol)
    stats["value"] = assert_close("value", gpu["value"], ora["value"], rtol)

    # sampler exactness: the oracle's sampler on the GPU's own logits
    heads = net["heads"]
    excused_exact = 0
    for i in range(n):
        off = 0
        for k, A in enumerate(heads):
            a, _, mg = ref_mod.head_sample(gpu["logits"][i, off:off + A], seed, int(rows[i]), step, k)
            if a != gpu["actions"][i, k]:
                assert mg < MARGIN, "row %d head %d: sampler mismatch on identical logits (margin %g)" % (
                    rows[i], k, mg)
                excused_exact += 1
            off += A
    # end to end against the oracle's actions
    mism = gpu["actions"] != ora["actions"]
    if net["dtype"] == "fp32":
        bad = mism & ~(ora["margin"] < MARGIN)
    else:
        dl = np.max(np.abs(gpu["logits"].astype(np.float64) - ora["logits"]), axis=1, keepdims=True)
        bad = mism & ~(ora["margin"] < np.maximum(2 * dl, MARGIN))
    assert not bad.any(), "actions differ outside the margin rule in rows %s" % (rows[np.where(bad)[0]][:10],)
    same = ~mism.any(axis=1)
    if same.any():
        stats["logp"] = assert_close("logp", gpu["logp"][same], ora["logp"][same], rtol)
    assert np.all(gpu["actions"] >= 0) and np.all(gpu["actions"] < np.array(heads)[None, :])
    stats["action_mismatch_rate"] = float(mism.mean())
    stats["excused_exact"] = excused_exact
    return stats
