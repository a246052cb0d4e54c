"""Pins for the oracle's counter-based sampler (Sec. 4.1: the seed that travels with each observation)."""
import math
import os

import numpy as np

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers(oracle):
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        assert oracle.philox4x32_10(w[:4], w[4:6]) == w[6:]
        n += 1
    assert n >= 2


def test_philox_is_sensitive_to_every_input_word(oracle):
    base = oracle.philox4x32_10([1, 2, 3, 4], [5, 6])
    outs = {tuple(base)}
    for i in range(4):
        c = [1, 2, 3, 4]; c[i] ^= 1
        outs.add(tuple(oracle.philox4x32_10(c, [5, 6])))
    for i in range(2):
        k = [5, 6]; k[i] ^= 1
        outs.add(tuple(oracle.philox4x32_10([1, 2, 3, 4], k)))
    assert len(outs) == 7
    # swapping counter words or key words is not a symmetry
    assert oracle.philox4x32_10([2, 1, 3, 4], [5, 6]) != base
    assert oracle.philox4x32_10([1, 2, 3, 4], [6, 5]) != base


def test_uniform_range_and_moments(oracle):
    u = np.array([oracle.uniform(99, e, s) for e in range(200) for s in range(100)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2 ** 24 == np.round(u * 2 ** 24))      # 24-bit grid
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1 / 12) < 0.005
    # word 0's top 24 bits, key = seed lo/hi, counter = (env, step, 0, 0)
    seed = 0x0123456789ABCDEF
    w = oracle.philox4x32_10([7, 11, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
    assert oracle.uniform(seed, 7, 11) == (w[0] >> 8) / 2.0 ** 24


def test_expf_accuracy_and_edges(oracle):
    assert oracle.expf(0.0) == np.float32(1.0)
    assert oracle.expf(-87.5) == np.float32(0.0)
    xs = np.concatenate([-np.linspace(0, 87, 3001), -np.logspace(-8, 1.9, 500)]).astype(np.float32)
    for x in xs:
        got, want = float(oracle.expf(float(x))), math.exp(float(x))
        assert abs(got - want) <= 4e-7 * want, (x, got, want)


def test_one_hot_and_single_action(oracle):
    l = np.full((64, 6), -40.0, np.float32); l[:, 4] = 40.0
    a, lp, _ = oracle.sample(l, seed=3, step=0)
    assert np.all(a == 4) and np.allclose(lp, 0.0, atol=1e-6)
    a, lp, _ = oracle.sample(np.zeros((10, 1), np.float32), seed=3, step=0)
    assert np.all(a == 0) and np.all(lp == 0.0)


def test_inverse_cdf_rule_against_float64(oracle):
    """Every sampled action must be the inverse-CDF action of the float64 softmax, except within rounding of a boundary."""
    rng = np.random.default_rng(0)
    N, A = 20000, 18
    l = rng.normal(0, 2, size=(N, A)).astype(np.float32)
    a, lp, u = oracle.sample(l, seed=1234, step=5)
    p = np.exp(l.astype(np.float64) - l.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    cdf = np.cumsum(p, 1)
    want = np.minimum((cdf <= u.astype(np.float64)[:, None]).sum(1), A - 1)
    bad = np.nonzero(want != a)[0]
    for i in bad:  # only allowed when u sits within 1e-6 of a boundary
        assert np.min(np.abs(cdf[i] - u[i])) < 1e-6
    assert bad.size < 20
    np.testing.assert_allclose(lp, np.log(p[np.arange(N), a]), atol=2e-6)


def test_empirical_frequencies_over_seeds(oracle):
    """Fixed logits, many (seed, env, step) counters: chi-square of action counts against the float64 softmax."""
    A = 6
    logits = np.array([0.3, -1.2, 2.0, 0.0, 1.1, -0.5], np.float32)
    p = np.exp(logits.astype(np.float64) - logits.max()); p /= p.sum()
    counts = np.zeros(A)
    n_env = 5000
    tile = np.tile(logits, (n_env, 1))
    for seed in range(40):
        a, _, _ = oracle.sample(tile, seed=1000 + seed, step=seed % 7, env_offset=seed * 13)
        counts += np.bincount(a, minlength=A)
    n = counts.sum()
    chi2 = float(((counts - n * p) ** 2 / (n * p)).sum())
    assert chi2 < 25.0, (chi2, counts / n, p)     # 5 dof: P(chi2 > 25) ~ 1.4e-4; seeds are fixed so not flaky


def test_action_depends_only_on_seed_env_step(oracle):
    """Batch-partition invariance: splitting the batch (with env_offset) cannot change any action."""
    rng = np.random.default_rng(2)
    l = rng.normal(size=(37, 18)).astype(np.float32)
    a, lp, _ = oracle.sample(l, seed=77, step=9, env_offset=100)
    a1, lp1, _ = oracle.sample(l[:10], seed=77, step=9, env_offset=100)
    a2, lp2, _ = oracle.sample(l[10:], seed=77, step=9, env_offset=110)
    assert np.array_equal(a, np.concatenate([a1, a2])) and np.array_equal(lp, np.concatenate([lp1, lp2]))
    b, _, _ = oracle.sample(l, seed=77, step=10, env_offset=100)
    assert not np.array_equal(a, b)
