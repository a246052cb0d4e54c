"""Pins for the oracle's returns / GAE recurrence (Sec. 3, n-step truncated return; GAE generalisation)."""
import numpy as np
import pytest


def _run(orc, r, V, d, gamma, lam):
    r = np.asarray(r, dtype=np.float64).reshape(-1, 1)
    V = np.asarray(V, dtype=np.float64).reshape(-1, 1)
    d = np.asarray(d, dtype=np.uint8).reshape(-1, 1)
    a, R = orc.gae(r, V, d, gamma, lam)
    return a[:, 0], R[:, 0]


def test_hand_trajectory_lambda1(oracle):
    # T=3, r=1, V=0, gamma=.5: A2 = 1, A1 = 1 + .5, A0 = 1 + .5*1.5 (all exact in binary)
    a, R = _run(oracle, [1, 1, 1], [0, 0, 0, 0], [0, 0, 0], 0.5, 1.0)
    assert a.tolist() == [1.75, 1.5, 1.0]
    assert R.tolist() == [1.75, 1.5, 1.0]


def test_hand_trajectory_lambda_half(oracle):
    # gamma*lambda = .25: A2 = 1, A1 = 1.25, A0 = 1 + .25*1.25
    a, _ = _run(oracle, [1, 1, 1], [0, 0, 0, 0], [0, 0, 0], 0.5, 0.5)
    assert a.tolist() == [1.3125, 1.25, 1.0]


def test_done_resets(oracle):
    # done after step 1: chain cut between t=1 and t=2
    a, _ = _run(oracle, [1, 1, 1], [0, 0, 0, 0], [0, 1, 0], 0.5, 0.5)
    assert a.tolist() == [1.25, 1.0, 1.0]
    a, _ = _run(oracle, [1, 1, 1], [0, 0, 0, 0], [1, 0, 0], 0.5, 0.5)
    assert a.tolist() == [1.0, 1.25, 1.0]
    # a done also masks the bootstrap value of the next state
    a, R = _run(oracle, [0, 0], [1, 2, 100], [0, 1], 1.0, 1.0)
    assert a.tolist() == [-1.0, -2.0] and R.tolist() == [0.0, 0.0]


def test_zero_reward_bootstrap(oracle):
    a, R = _run(oracle, [0, 0, 0], [1, 2, 3, 4], [0, 0, 0], 1.0, 1.0)
    assert a.tolist() == [3.0, 2.0, 1.0]
    assert R.tolist() == [4.0, 4.0, 4.0]


def test_geometric_closed_form(oracle):
    T, gamma, lam, r = 40, 0.97, 0.9, 0.3
    a, _ = _run(oracle, [r] * T, [0] * (T + 1), [0] * T, gamma, lam)
    gl = gamma * lam
    want = np.array([r * (1 - gl ** (T - t)) / (1 - gl) for t in range(T)])
    np.testing.assert_allclose(a, want, rtol=1e-13)


def test_lambda0_is_td_error(oracle):
    rng = np.random.default_rng(3)
    T = 17
    r, V = rng.normal(size=T), rng.normal(size=T + 1)
    d = (rng.random(T) < 0.2).astype(np.uint8)
    a, _ = _run(oracle, r, V, d, 0.9, 0.0)
    want = r + 0.9 * (1 - d) * V[1:] - V[:-1]
    np.testing.assert_allclose(a, want, rtol=1e-14, atol=1e-15)


def test_lambda1_equals_nstep_return_double_sum(oracle):
    """R_t = sum_{i<n} gamma^i r_{t+i} + gamma^n V(s_{t+n}) with n = T - t (Sec. 3), by the direct double sum."""
    rng = np.random.default_rng(5)
    T, N, gamma = 12, 7, 0.99
    r, V = rng.normal(size=(T, N)), rng.normal(size=(T + 1, N))
    _, R = oracle.gae(r, V, np.zeros((T, N), np.uint8), gamma, 1.0)
    want = np.zeros((T, N))
    for t in range(T):
        n = T - t
        for i in range(n):
            want[t] += gamma ** i * r[t + i]
        want[t] += gamma ** n * V[T]
    np.testing.assert_allclose(R, want, rtol=1e-12, atol=1e-13)


def test_done_splits_into_independent_problems(oracle):
    rng = np.random.default_rng(7)
    T, gamma, lam, cut = 11, 0.95, 0.8, 6          # done at t = cut-1
    r, V = rng.normal(size=T), rng.normal(size=T + 1)
    d = np.zeros(T, np.uint8); d[cut - 1] = 1
    a, R = _run(oracle, r, V, d, gamma, lam)
    # first segment: terminal, i.e. bootstrap value 0; second: its own problem
    V1 = np.concatenate([V[:cut], [0.0]])
    a1, R1 = _run(oracle, r[:cut], V1, np.zeros(cut, np.uint8), gamma, lam)
    a2, R2 = _run(oracle, r[cut:], V[cut:], np.zeros(T - cut, np.uint8), gamma, lam)
    np.testing.assert_allclose(a, np.concatenate([a1, a2]), rtol=1e-14)
    np.testing.assert_allclose(R, np.concatenate([R1, R2]), rtol=1e-14)


def test_columns_independent_and_layout(oracle):
    """[T,N] time-major layout: column n of the batched call equals the single-column call."""
    rng = np.random.default_rng(11)
    T, N = 9, 5
    r, V = rng.normal(size=(T, N)), rng.normal(size=(T + 1, N))
    d = (rng.random((T, N)) < 0.15).astype(np.uint8)
    a, R = oracle.gae(r, V, d, 0.99, 0.95)
    for n in range(N):
        an, Rn = _run(oracle, r[:, n], V[:, n], d[:, n], 0.99, 0.95)
        assert np.array_equal(a[:, n], an) and np.array_equal(R[:, n], Rn)


def test_normalize_adv(oracle):
    rng = np.random.default_rng(1)
    a = rng.normal(2.0, 3.0, size=1000)
    z = oracle.normalize_adv(a)
    want = (a - a.mean()) / (a.std(ddof=1) + 1e-5)
    np.testing.assert_allclose(z, want, rtol=1e-12, atol=1e-13)
    assert abs(z.mean()) < 1e-12 and abs(z.std(ddof=1) - 1.0) < 1e-4
