"""Pins for the oracle's gradient-norm clip and Adam step."""
import numpy as np


def test_adam_first_step_closed_form(oracle):
    rng = np.random.default_rng(0)
    g = rng.normal(size=100); g[:5] = 0.0
    th = rng.normal(size=100)
    hp = oracle.make_hparams(lr=1e-3, adam_eps=1e-5)
    t1, m, v = oracle.adam(th, g, np.zeros(100), np.zeros(100), 1, hp)
    # bias corrections cancel at t=1: step = lr * g / (|g| + eps)
    np.testing.assert_allclose(t1 - th, -1e-3 * g / (np.abs(g) + 1e-5), rtol=1e-12, atol=1e-18)
    assert np.all(t1[:5] == th[:5])
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-14)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)


def test_adam_three_step_scalar_by_hand(oracle):
    hp = oracle.make_hparams(lr=0.1, beta1=0.5, beta2=0.5, adam_eps=0.0)
    th, m, v = np.array([1.0]), np.zeros(1), np.zeros(1)
    gs = [2.0, -1.0, 4.0]
    # by hand: m1=1, v1=2 -> mhat=2, vhat=4 -> th=1-.1*2/2=.9
    #          m2=0, v2=1.5 -> mhat=0 -> th=.9
    #          m3=2, v3=8.75 -> mhat=2/.875, vhat=10 -> th=.9-.1*(2/.875)/sqrt(10)
    want = [0.9, 0.9, 0.9 - 0.1 * (2 / 0.875) / np.sqrt(10.0)]
    for t, g in enumerate(gs, start=1):
        th, m, v = oracle.adam(th, np.array([g]), m, v, t, hp)
        np.testing.assert_allclose(th[0], want[t - 1], rtol=1e-14)


def test_clip(oracle):
    rng = np.random.default_rng(1)
    g = rng.normal(size=1000)
    n = np.linalg.norm(g)
    s = oracle.clip_coef(g, 0.5)
    np.testing.assert_allclose(np.linalg.norm(s * g), 0.5 * n / (n + 1e-6), rtol=1e-12)
    assert oracle.clip_coef(g * 1e-3, 0.5) == 1.0
    assert oracle.clip_coef(g, 0.0) == 1.0 and oracle.clip_coef(g, -1.0) == 1.0


def test_learner_step_composes(oracle):
    """learner_step == loss_grads -> clip -> adam, and gscale enters Adam as a plain factor on g."""
    import hts_synth as syn
    kw = dict(convs=((3, 8, 4), (4, 3, 1), (4, 2, 1)), hidden=8)
    net = oracle.make_net(2, 20, 20, 3, **kw)
    rng = np.random.default_rng(2)
    p = syn.init_params(1, 2, 20, 20, 3, bias_scale=0.1, **kw).astype(np.float64)
    B = 10
    obs = rng.integers(0, 256, size=(B, 2, 20, 20), dtype=np.uint8)
    act = rng.integers(0, 3, size=B).astype(np.int32)
    adv, ret, olp = rng.normal(size=B) * 30, rng.normal(size=B), -np.ones(B)
    hp = oracle.make_hparams(algo=0, max_grad_norm=0.5, lr=1e-2)
    m0, v0 = np.zeros(p.size), np.zeros(p.size)
    p1, m1, v1, g, st = oracle.learner_step(net, p, m0, v0, 1, obs, act, olp, adv, ret, hp)
    g2, st2 = oracle.loss_grads(net, p, obs, act, olp, adv, ret, hp)
    assert np.array_equal(g, g2)
    s = oracle.clip_coef(g2, 0.5)
    assert s < 1.0
    p2, m2, v2 = oracle.adam(p, g2 * s, m0, v0, 1, hp)
    np.testing.assert_allclose(p1, p2, rtol=1e-14, atol=1e-16)
    np.testing.assert_allclose(m1, m2, rtol=1e-14, atol=1e-300)


def test_delayed_gradient_step(oracle):
    """Sec. 4.1 "Delayed gradient": theta_{j+1} = theta_j + step(grad J(theta_{j-1}; D)).
    Pins: (i) with theta_{j-1} == theta_j it is the ordinary update; (ii) the gradient and the loss statistics depend on
    the behaviour parameters only; (iii) from zero moments the displacement theta_{j+1} - theta_j is the same whichever
    target it is applied to (Adam's first step is a function of g alone), and equals -lr*g/(|g|+eps)."""
    import hts_synth as syn
    kw = dict(convs=((3, 8, 4), (4, 3, 1), (4, 2, 1)), hidden=8)
    net = oracle.make_net(2, 20, 20, 3, **kw)
    rng = np.random.default_rng(5)
    pb = syn.init_params(1, 2, 20, 20, 3, bias_scale=0.1, **kw).astype(np.float64)
    pt1 = syn.init_params(2, 2, 20, 20, 3, bias_scale=0.1, **kw).astype(np.float64)
    pt2 = syn.init_params(3, 2, 20, 20, 3, bias_scale=0.1, **kw).astype(np.float64)
    B = 12
    obs = rng.integers(0, 256, size=(B, 2, 20, 20), dtype=np.uint8)
    act = rng.integers(0, 3, size=B).astype(np.int32)
    adv, ret, olp = rng.normal(size=B), rng.normal(size=B), -np.ones(B)
    hp = oracle.make_hparams(algo=0, lr=1e-2)
    z = np.zeros(pb.size)
    same = oracle.learner_step_delayed(net, pb, pb, z, z, 1, obs, act, olp, adv, ret, hp)
    plain = oracle.learner_step(net, pb, z, z, 1, obs, act, olp, adv, ret, hp)
    np.testing.assert_allclose(same[0], plain[0], rtol=1e-14, atol=1e-16)
    a = oracle.learner_step_delayed(net, pb, pt1, z, z, 1, obs, act, olp, adv, ret, hp)
    b = oracle.learner_step_delayed(net, pb, pt2, z, z, 1, obs, act, olp, adv, ret, hp)
    assert np.array_equal(a[3], b[3]) and np.array_equal(a[3], plain[3]) and a[4] == b[4]
    np.testing.assert_allclose(a[0] - pt1, b[0] - pt2, rtol=0, atol=1e-15)
    g = a[3]
    np.testing.assert_allclose(a[0] - pt1, -1e-2 * g / (np.abs(g) + 1e-5), rtol=1e-9, atol=1e-15)
    # a gradient taken at the target instead would differ
    g_t, _ = oracle.loss_grads(net, pt1, obs, act, olp, adv, ret, hp)
    assert np.linalg.norm(g_t - g) > 1e-3 * np.linalg.norm(g)


def test_rmsprop(oracle):
    """RMSProp without momentum: first step from v = 0 is -lr g / (sqrt(1-alpha)|g| + eps); g = 0 leaves theta alone;
    a three-step scalar sequence worked by hand."""
    rng = np.random.default_rng(3)
    g = rng.normal(size=50)
    th0 = rng.normal(size=50)
    th, v = oracle.rmsprop(th0, g, np.zeros(50), 7e-4, 0.99, 1e-5)
    np.testing.assert_allclose(th - th0, -7e-4 * g / (np.sqrt(0.01) * np.abs(g) + 1e-5), rtol=1e-12)
    np.testing.assert_allclose(v, 0.01 * g * g, rtol=1e-14)
    th2, v2 = oracle.rmsprop(th0, np.zeros(50), v, 7e-4, 0.99, 1e-5)
    assert np.array_equal(th2, th0)
    np.testing.assert_allclose(v2, 0.99 * v, rtol=1e-15)
    # alpha = 0.5, lr = 0.1, eps = 0, g = 2, 0, 4:  v = 2, 1, 8.5
    t, vv = np.array([1.0]), np.zeros(1)
    want = [1.0 - 0.1 * 2 / np.sqrt(2.0), 1.0 - 0.1 * 2 / np.sqrt(2.0),
            1.0 - 0.1 * 2 / np.sqrt(2.0) - 0.1 * 4 / np.sqrt(8.5)]
    for k, gk in enumerate([2.0, 0.0, 4.0]):
        t, vv = oracle.rmsprop(t, np.array([gk]), vv, 0.1, 0.5, 0.0 if gk else 1e-30)
        np.testing.assert_allclose(t[0], want[k], rtol=1e-14)
    # gscale is a plain factor on g
    a = oracle.rmsprop(th0, g, np.zeros(50), 1e-3, 0.9, 1e-5, gscale=0.25)
    b = oracle.rmsprop(th0, 0.25 * g, np.zeros(50), 1e-3, 0.9, 1e-5)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-15)
