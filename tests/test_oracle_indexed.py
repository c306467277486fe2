"""Pins for the oracle's indexed step (rows name environments of a state table; paper,
Sec. 3.2 double-buffered sampling and Sec. 3.3 index-based exchange): the independent
PyTorch fp64 composition on gathered rows, reduction to the plain step, the sampler's
counter word, untouched rows, order independence, two half-batches in alternation, and
the rejection of bad ids.
"""
import numpy as np
import pytest

from paper_2006_11751_amd import workloads as wl
from tests.test_oracle_step import SMALL_STD, torch_step


def _table(net, n_env, seed=77):
    rng = np.random.default_rng(seed)
    return (0.1 * rng.standard_normal((n_env, net["rnn"]))).astype(np.float32)


def test_indexed_step_matches_torch_composition_on_gathered_rows(ref):
    net = SMALL_STD
    w = wl.weights(net)
    B, n_env = 3, 9
    obs, _, done = wl.observations(net, 0, B), None, np.array([0, 1, 0], np.uint8)
    table = _table(net, n_env)
    before = table.copy()
    ids = np.array([7, 2, 4], np.int32)
    out = ref.policy_step_indexed(net, w, obs, table, ids, done, 3, 5)
    hn, logits, value = torch_step(net, w, obs, before[ids], done)
    np.testing.assert_allclose(table[ids], hn, rtol=2e-7, atol=1e-7)
    np.testing.assert_allclose(out["logits"], logits, rtol=2e-7, atol=1e-7)
    np.testing.assert_allclose(out["value"], value, rtol=2e-7, atol=1e-7)
    # rows nobody named keep their state, bit for bit
    rest = np.setdiff1d(np.arange(n_env), ids)
    assert np.array_equal(table[rest], before[rest])
    # the sampler's counter word is the environment id, not the batch row
    off = 0
    for k, A in enumerate(net["heads"]):
        for b in range(B):
            a, _, _ = ref.head_sample(out["logits"][b, off:off + A], 3, int(ids[b]), 5, k)
            assert a == out["actions"][b, k]
        off += A


def test_identity_ids_reduce_to_the_plain_step(ref):
    net = wl.network(0)
    w = wl.weights(net)
    B = net["B"]
    obs, h_in, done = wl.observations(net, 0, B), wl.initial_state(net, B), wl.done_mask(net, 0, B)
    plain = ref.policy_step(net, w, obs, h_in, done, 1, 2)
    table = h_in.copy()
    out = ref.policy_step_indexed(net, w, obs, table, np.arange(B, dtype=np.int32), done, 1, 2)
    assert np.array_equal(table, plain["h_out"])
    for k in ("actions", "logp", "value", "logits"):
        assert np.array_equal(out[k], plain[k]), k


def test_result_does_not_depend_on_where_an_environment_sits(ref):
    net = wl.network(0)
    w = wl.weights(net)
    B, n_env = 6, 10
    obs, done = wl.observations(net, 0, B), np.array([0, 1, 0, 0, 1, 0], np.uint8)
    ids = np.array([9, 0, 3, 5, 2, 7], np.int32)
    t1 = _table(net, n_env)
    t2 = t1.copy()
    o1 = ref.policy_step_indexed(net, w, obs, t1, ids, done, 4, 0)
    perm = np.array([4, 2, 0, 5, 1, 3])
    o2 = ref.policy_step_indexed(net, w, obs[perm], t2, ids[perm], done[perm], 4, 0)
    assert np.array_equal(t1, t2)
    for k in ("actions", "logp", "value", "logits"):
        assert np.array_equal(o1[k][perm], o2[k]), k


def test_two_half_batches_in_alternation_equal_one_full_batch_per_step(ref):
    """Double-buffered sampling: the two halves of the environments are served by separate
    calls; every environment still sees the same sequence as when all are served at once."""
    net = wl.network(0)
    w = wl.weights(net)
    n_env = 8
    full = _table(net, n_env)
    split = full.copy()
    ids = np.arange(n_env, dtype=np.int32)
    for t in range(3):
        obs, done = wl.observations(net, t, n_env), wl.done_mask(net, t, n_env)
        a = ref.policy_step_indexed(net, w, obs, full, ids, done, 1, t)
        lo, hi = ids[: n_env // 2], ids[n_env // 2:]
        b1 = ref.policy_step_indexed(net, w, obs[lo], split, lo, done[lo], 1, t)
        b2 = ref.policy_step_indexed(net, w, obs[hi], split, hi, done[hi], 1, t)
        assert np.array_equal(full, split)
        assert np.array_equal(a["actions"], np.concatenate([b1["actions"], b2["actions"]]))
        assert np.array_equal(a["logp"], np.concatenate([b1["logp"], b2["logp"]]))


@pytest.mark.parametrize("ids", [[0, 0], [0, 5], [-1, 1]])
def test_bad_ids_are_rejected_and_nothing_is_written(ref, ids):
    net = wl.network(0)
    w = wl.weights(net)
    obs, done = wl.observations(net, 0, 2), np.zeros(2, np.uint8)
    table = _table(net, 5)
    before = table.copy()
    with pytest.raises(ValueError):
        ref.policy_step_indexed(net, w, obs, table, np.array(ids, np.int32), done, 1, 0)
    assert np.array_equal(table, before)
