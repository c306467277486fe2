"""Pins for the oracle's sampler: Philox structure, bits->uniform exactness,
Gumbel moments, softmax invariants, distributional correctness, tie rule.

Philox4x32-10 is pinned three ways: its published known answers (tests/golden), an
independent big-integer implementation written from the algorithm's description, and
the statistical behaviour of the draws.
"""
import math
import os

import numpy as np
import pytest


# ---- Philox: independent big-integer implementation ---------------------------

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def philox_py(ctr, key, rounds=10):
    c = [int(v) for v in ctr]
    k = [int(v) for v in key]
    for _ in range(rounds):
        prod0, prod1 = M0 * c[0], M1 * c[2]
        c = [((prod1 >> 32) ^ c[1] ^ k[0]) & MASK, prod1 & MASK,
             ((prod0 >> 32) ^ c[3] ^ k[1]) & MASK, prod0 & MASK]
        k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
    return c


def philox_inverse_py(out, key, rounds=10):
    """Run the rounds backwards: the round function is a bijection because the
    multipliers are odd (invertible mod 2^32)."""
    inv0, inv1 = pow(M0, -1, 1 << 32), pow(M1, -1, 1 << 32)
    c = [int(v) for v in out]
    keys = [((int(key[0]) + r * W0) & MASK, (int(key[1]) + r * W1) & MASK) for r in range(rounds)]
    for r in reversed(range(rounds)):
        k0, k1 = keys[r]
        c2 = (c[1] * inv1) & MASK          # lo(M1*c2) = c[1]
        c0 = (c[3] * inv0) & MASK          # lo(M0*c0) = c[3]
        c1 = c[0] ^ ((M1 * c2) >> 32) ^ k0
        c3 = c[2] ^ ((M0 * c0) >> 32) ^ k1
        c = [c0, c1 & MASK, c2, c3 & MASK]
    return c


def test_philox_matches_bigint_implementation(ref):
    rng = np.random.default_rng(11)
    for _ in range(10000):
        ctr = rng.integers(0, 1 << 32, 4, dtype=np.uint64).astype(np.uint32)
        key = rng.integers(0, 1 << 32, 2, dtype=np.uint64).astype(np.uint32)
        assert list(ref.philox4x32_10(ctr, key)) == philox_py(ctr, key)
    for ctr, key in [((0, 0, 0, 0), (0, 0)), ((MASK,) * 4, (MASK, MASK))]:
        assert list(ref.philox4x32_10(ctr, key)) == philox_py(ctr, key)


def test_philox_known_answers(ref):
    """The published known answers of Philox4x32-10: a wrong round constant, multiplier, round
    count or word order in the oracle and in the big-integer copy above alike would pass the
    comparison of the two, but not this."""
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_known_answers.txt")
    cases = [[int(w, 16) for w in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    assert len(cases) == 3
    for words in cases:
        ctr, key, want = words[:4], words[4:6], words[6:]
        assert [int(v) for v in ref.philox4x32_10(np.array(ctr, np.uint32), np.array(key, np.uint32))] == want
        assert philox_py(ctr, key) == want


def test_philox_is_invertible(ref):
    rng = np.random.default_rng(12)
    for _ in range(500):
        ctr = rng.integers(0, 1 << 32, 4, dtype=np.uint64).astype(np.uint32)
        key = rng.integers(0, 1 << 32, 2, dtype=np.uint64).astype(np.uint32)
        out = ref.philox4x32_10(ctr, key)
        assert philox_inverse_py(out, key) == [int(v) for v in ctr]


def test_philox_distinct_counters_distinct_outputs_and_avalanche(ref):
    key = np.array([1, 0], np.uint32)
    seen = set()
    flips = []
    base = ref.philox4x32_10(np.array([0, 0, 0, 0], np.uint32), key)
    for i in range(4096):
        out = ref.philox4x32_10(np.array([i, 0, 0, 0], np.uint32), key)
        seen.add(tuple(int(v) for v in out))
        if i:
            flips.append(sum(bin(int(a) ^ int(b)).count("1") for a, b in zip(out, base)))
    assert len(seen) == 4096
    # neighbouring counters give unrelated 128-bit blocks: about 64 differing bits
    assert 60 < np.mean(flips) < 68


def test_philox_bits_are_uniform(ref):
    # bit balance over 4096 blocks x 128 bits: each bit position near 1/2
    key = np.array([7, 9], np.uint32)
    acc = np.zeros(128)
    n = 4096
    for i in range(n):
        out = ref.philox4x32_10(np.array([i, 3, 0, 5], np.uint32), key)
        bits = np.unpackbits(out.view(np.uint8), bitorder="little")
        acc += bits
    assert np.all(np.abs(acc / n - 0.5) < 5 * 0.5 / math.sqrt(n))


def test_sampler_words_keying(ref):
    # key = (seed lo, seed hi); counter = (env, step lo, step hi, head<<16 | block)
    seed, env, step, head, block = 0x1234567890ABCDEF, 77, 0xA1B2C3D4E5F60718, 5, 2
    got = ref.sampler_words(seed, env, step, head, block)
    want = philox_py([env, step & MASK, step >> 32, (head << 16) | block], [seed & MASK, seed >> 32])
    assert list(got) == want
    # every argument matters
    base = tuple(ref.sampler_words(1, 0, 0, 0, 0))
    for args in [(2, 0, 0, 0, 0), (1, 1, 0, 0, 0), (1, 0, 1, 0, 0), (1, 0, 1 << 32, 0, 0),
                 (1, 0, 0, 1, 0), (1, 0, 0, 0, 1), (1 + (1 << 32), 0, 0, 0, 0)]:
        assert tuple(ref.sampler_words(*args)) != base


# ---- bits -> uniform -> Gumbel -------------------------------------------------

def test_uniform_exhaustive(ref):
    # all 2^23 values: exactly (k + 1/2) / 2^23, strictly inside (0, 1), low 9 bits ignored
    k = np.arange(1 << 23, dtype=np.uint32)
    u = ref.bits_to_uniform_many(k << np.uint32(9))
    exact = (k.astype(np.float64) + 0.5) / float(1 << 23)
    assert np.array_equal(u.astype(np.float64), exact)
    assert u.min() == 2.0 ** -24 and u.max() == 1.0 - 2.0 ** -24
    u2 = ref.bits_to_uniform_many((k[::4097] << np.uint32(9)) | np.uint32(0x1FF))
    assert np.array_equal(u2, u[::4097])
    assert ref.bits_to_uniform(0) == 2.0 ** -24
    assert ref.bits_to_uniform(0xFFFFFFFF) == 1.0 - 2.0 ** -24


def test_gumbel_values_and_moments(ref):
    # selected points against the fp64 value, at fp32 accuracy
    for u in [2.0 ** -24, 0.1, 0.25, 0.5, 0.75, 0.999, 1.0 - 2.0 ** -24]:
        uf = float(np.float32(u))
        want = -math.log(-math.log(uf))
        assert abs(ref.gumbel(uf) - want) <= 4e-7 * max(1.0, abs(want))
    # the extremes stay finite
    assert math.isfinite(ref.gumbel(2.0 ** -24)) and math.isfinite(ref.gumbel(1.0 - 2.0 ** -24))
    assert ref.gumbel(float(np.float32(0.2))) < ref.gumbel(float(np.float32(0.8)))
    # moments over 10^6 draws from the generator itself: mean -> Euler-Mascheroni, var -> pi^2/6
    n = 250000
    words = np.concatenate([ref.sampler_words(3, e, 0, 0, 0) for e in range(n)])
    u = ref.bits_to_uniform_many(words)
    g = np.array([ref.gumbel(float(v)) for v in u[:200000]])
    assert abs(g.mean() - 0.5772156649) < 4 * math.sqrt(math.pi ** 2 / 6 / len(g))
    assert abs(g.var() - math.pi ** 2 / 6) < 0.03
    # uniform moments over the full million
    assert abs(u.mean() - 0.5) < 4 / math.sqrt(12 * len(u))
    assert abs(u.var() - 1 / 12) < 1e-3


# ---- softmax / log-probability -------------------------------------------------

def test_log_softmax_invariants(ref):
    rng = np.random.default_rng(21)
    for A in [1, 2, 3, 7, 11, 21]:
        l = (3 * rng.standard_normal(A)).astype(np.float32)
        ls = ref.log_softmax(l)
        assert abs(np.exp(ls).sum() - 1.0) < 1e-12
        # exact shift (power of two keeps fp32 logits exactly shifted)
        shifted = ref.log_softmax((l.astype(np.float64) + 64.0).astype(np.float32))
        np.testing.assert_allclose(shifted, ls, atol=2e-5)
        assert np.argmax(ls) == np.argmax(l)
    # large logits do not overflow
    ls = ref.log_softmax(np.array([1000.0, 999.0], np.float32))
    assert abs(ls[0] + math.log1p(math.exp(-1.0))) < 1e-12
    # two actions: log sigmoid(+-(l0 - l1))
    l = np.array([0.75, -1.5], np.float32)
    d = float(l[0]) - float(l[1])
    ls = ref.log_softmax(l)
    assert abs(ls[0] + math.log1p(math.exp(-d))) < 1e-14
    assert abs(ls[1] + math.log1p(math.exp(d))) < 1e-14
    # uniform logits
    np.testing.assert_allclose(ref.log_softmax(np.full(8, 2.5, np.float32)), -math.log(8), rtol=1e-14)


def test_head_sample_logp_is_log_softmax_at_action(ref):
    rng = np.random.default_rng(22)
    for trial in range(200):
        A = int(rng.integers(1, 22))
        l = (2 * rng.standard_normal(A)).astype(np.float32)
        a, lp, mg = ref.head_sample(l, 1, trial, 5, 0)
        assert 0 <= a < A
        assert lp == ref.log_softmax(l)[a]
        assert mg >= 0


def test_head_sample_is_argmax_of_perturbed_logits(ref):
    # rebuild the perturbed logits from the exported pieces and take the argmax
    rng = np.random.default_rng(23)
    for trial in range(300):
        A = int(rng.integers(2, 22))
        l = rng.standard_normal(A).astype(np.float32)
        seed, env, step, head = 9, trial, 1000 + trial, trial % 6
        pert = np.zeros(A, np.float32)
        for i in range(A):
            w = ref.sampler_words(seed, env, step, head, i // 4)[i % 4]
            pert[i] = np.float32(l[i]) + np.float32(ref.gumbel(ref.bits_to_uniform(int(w))))
        a, _, mg = ref.head_sample(l, seed, env, step, head)
        assert a == int(np.argmax(pert))
        top2 = np.sort(pert)[-2:]
        assert mg == np.float32(top2[1] - top2[0])


def test_tie_rule_lowest_index(ref):
    l = np.array([0.5, 0.5, 0.5, 0.25], np.float32)
    a, _, mg = ref.head_sample(l, 1, 0, 0, 0, g_override=np.zeros(4, np.float32))
    assert a == 0 and mg == 0.0
    a, _, _ = ref.head_sample(np.array([0.0, 1.0, 1.0], np.float32), 1, 0, 0, 0,
                              g_override=np.zeros(3, np.float32))
    assert a == 1
    # noise can overturn the logits
    a, _, _ = ref.head_sample(np.array([0.0, 1.0, 1.0], np.float32), 1, 0, 0, 0,
                              g_override=np.array([2.0, 0.0, 0.5], np.float32))
    assert a == 0


def test_single_action_head(ref):
    a, lp, mg = ref.head_sample(np.array([3.0], np.float32), 1, 0, 0, 0)
    assert a == 0 and lp == 0.0 and math.isinf(mg)


@pytest.mark.parametrize("logits", [
    [0.0, 0.0, 0.0], [1.0, -1.0], [2.0, 0.5, -1.0, 0.0, 1.5, -3.0, 0.25],
    [0.1 * i for i in range(11)], [3.0, -2.0, 0.0, 0.0, 1.0, 1.0, -1.0, 2.0, 0.5, 0.5, 0.5, -4.0, 0.0, 1.0, 2.5],
])
def test_sampler_frequencies_match_softmax(ref, logits):
    # Gumbel-max is an exact categorical sampler: chi-square of 10^6 draws against softmax
    l = np.array(logits, np.float32)
    n = 1_000_000
    counts = ref.head_histogram(l, seed=1, head=2, n=n, n_env=1024)
    assert counts.sum() == n
    p = np.exp(ref.log_softmax(l))
    chi2 = float(((counts - n * p) ** 2 / (n * p)).sum())
    dof = len(l) - 1
    # mean dof, sd sqrt(2 dof): 5 sigma
    assert chi2 < dof + 5 * math.sqrt(2 * dof) + 5
    assert np.all(np.abs(counts - n * p) < 5 * np.sqrt(n * p * (1 - p)) + 1)


def test_sampler_streams_differ_and_repeat(ref):
    l = np.zeros(16, np.float32)
    draws = lambda **kw: [ref.head_sample(l, kw.get("seed", 1), e, kw.get("step", 0), kw.get("head", 0))[0]
                          for e in range(256)]
    base = draws()
    assert base == draws()
    assert base != draws(seed=2) and base != draws(step=1) and base != draws(head=1)
    # uses several Philox blocks: with 16 equal logits all 16 actions occur
    assert set(base) == set(range(16))
