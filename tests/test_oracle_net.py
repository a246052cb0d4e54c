"""Pins for the oracle's network forward, loss and hand-derived backward.

The architecture is the one in the paper's appendix "Implementation Details"; the loss is eq. (4) of Sec. 3 plus the
squared value loss, and PPO's clipped surrogate.  The library cross-check uses torch's CPU conv2d/linear/autograd in
float64 on random inputs: an independent formulation, not a copy of the oracle's loops.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import hts_synth as syn

TINY = dict(C=2, H=20, W=20, A=3, convs=((3, 8, 4), (4, 3, 1), (4, 2, 1)), hidden=8)


def _tiny(oracle):
    net = oracle.make_net(TINY["C"], TINY["H"], TINY["W"], TINY["A"], TINY["convs"], TINY["hidden"])
    return net


def _torch_forward(p, obs, convs):
    x = torch.from_numpy(obs.astype(np.float64)) / 255.0
    for i, (co, k, s) in enumerate(convs):
        x = F.relu(F.conv2d(x, p[f"conv{i + 1}.w"], p[f"conv{i + 1}.b"], stride=s))
    h = F.relu(F.linear(x.flatten(1), p["fc.w"], p["fc.b"]))
    return F.linear(h, p["pi.w"], p["pi.b"]), F.linear(h, p["v.w"], p["v.b"])[:, 0]


def _torch_loss(p, obs, convs, actions, old_logp, adv, ret, algo, eps, cv, ce, rho_bar=1.0, old_values=None,
                value_clip=0.0):
    logits, v = _torch_forward(p, obs, convs)
    lsm = F.log_softmax(logits, dim=1)
    logp = lsm.gather(1, torch.from_numpy(actions.astype(np.int64))[:, None])[:, 0]
    ent = -(lsm.exp() * lsm).sum(1)
    adv_t, ret_t = torch.from_numpy(adv), torch.from_numpy(ret)
    if algo == 0:
        lpi = -(logp * adv_t).mean()
    elif algo == 2:
        w = (logp - torch.from_numpy(old_logp)).exp().clamp(max=rho_bar).detach()
        lpi = -(w * logp * adv_t).mean()
    else:
        rho = (logp - torch.from_numpy(old_logp)).exp()
        lpi = -torch.minimum(rho * adv_t, rho.clamp(1 - eps, 1 + eps) * adv_t).mean()
    lv = (ret_t - v) ** 2
    if value_clip > 0:
        ov = torch.from_numpy(old_values)
        lv = torch.maximum(lv, (ov + (v - ov).clamp(-value_clip, value_clip) - ret_t) ** 2)
    lv = lv.mean()
    return lpi + cv * lv - ce * ent.mean(), lpi, lv, ent.mean()


def _torch_params(flat, shape_kw, A):
    parts = syn.split_params(flat.astype(np.float64), shape_kw["C"], shape_kw["H"], shape_kw["W"], A,
                             convs=shape_kw["convs"], hidden=shape_kw["hidden"])
    return {k: torch.from_numpy(np.ascontiguousarray(v)).requires_grad_(True) for k, v in parts.items()}


def test_param_count_closed_forms(oracle):
    atari = lambda A: 32 * 4 * 64 + 32 + 64 * 32 * 16 + 64 + 64 * 64 * 9 + 64 + 512 * 3136 + 512 + A * 512 + A + 512 + 1
    assert oracle.param_count(oracle.make_net(4, 84, 84, 6)) == atari(6) == 1687719
    assert oracle.param_count(oracle.make_net(4, 84, 84, 18)) == atari(18) == 1693875
    assert oracle.param_count(oracle.make_net(16, 72, 96, 19)) == 1424052
    for (C, H, W, A) in [(4, 84, 84, 6), (16, 72, 96, 19)]:
        assert oracle.param_count(oracle.make_net(C, H, W, A)) == syn.param_count(C, H, W, A)


def test_zero_weights_give_head_biases(oracle):
    net = oracle.make_net(4, 84, 84, 6)
    P = oracle.param_count(net)
    p = np.zeros(P)
    p[-1] = 0.7                                  # v.b
    p[-1 - 512 - 6:-1 - 512] = np.arange(6) - 2  # pi.b
    obs = syn.obs_uniform(3, 2)
    logits, v = oracle.forward(net, p, obs)
    assert np.array_equal(logits, np.tile(np.arange(6) - 2.0, (2, 1))) and np.array_equal(v, [0.7, 0.7])


def test_kernel_equal_to_input_is_dot_product(oracle):
    """A single conv layer whose kernel covers the whole input is one dot product per filter."""
    net = oracle.make_net(3, 5, 5, 2, convs=((4, 5, 1),), hidden=4)
    rng = np.random.default_rng(0)
    P = oracle.param_count(net)
    p = rng.normal(size=P)
    obs = rng.integers(0, 256, size=(1, 3, 5, 5), dtype=np.uint8)
    w1, b1 = p[:300].reshape(4, 75), p[300:304]
    y1 = np.maximum(w1 @ (obs.reshape(75) / 255.0) + b1, 0)
    off = 304
    fw, fb = p[off:off + 16].reshape(4, 4), p[off + 16:off + 20]; off += 20
    h = np.maximum(fw @ y1 + fb, 0)
    pw, pb = p[off:off + 8].reshape(2, 4), p[off + 8:off + 10]; off += 10
    vw, vb = p[off:off + 4], p[off + 4]
    logits, v = oracle.forward(net, p, obs)
    np.testing.assert_allclose(logits[0], pw @ h + pb, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(v[0], vw @ h + vb, rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("shape", [(4, 84, 84, 6), (16, 72, 96, 19)])
def test_forward_matches_torch_cpu(oracle, shape):
    C, H, W, A = shape
    net = oracle.make_net(C, H, W, A)
    flat = syn.init_params(5, C, H, W, A, bias_scale=0.1)
    obs = syn.obs_uniform(9, 3, C, H, W)
    logits, v = oracle.forward(net, flat, obs)
    kw = dict(C=C, H=H, W=W, convs=((32, 8, 4), (64, 4, 2), (64, 3, 1)), hidden=512)
    with torch.no_grad():
        tl, tv = _torch_forward(_torch_params(flat, kw, A), obs, kw["convs"])
    np.testing.assert_allclose(logits, tl.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(v, tv.numpy(), rtol=1e-10, atol=1e-12)
    # gather by index
    l2, v2 = oracle.forward(net, flat, obs, index=np.array([2, 0], np.int32))
    assert np.array_equal(l2, logits[[2, 0]]) and np.array_equal(v2, v[[2, 0]])


def _problem(oracle, seed, B, algo, kw=TINY):
    rng = np.random.default_rng(seed)
    net = oracle.make_net(kw["C"], kw["H"], kw["W"], kw["A"], kw["convs"], kw["hidden"])
    flat = syn.init_params(seed, kw["C"], kw["H"], kw["W"], kw["A"], bias_scale=0.2, convs=kw["convs"],
                           hidden=kw["hidden"]).astype(np.float64)
    obs = rng.integers(0, 256, size=(B, kw["C"], kw["H"], kw["W"]), dtype=np.uint8)
    actions = rng.integers(0, kw["A"], size=B).astype(np.int32)
    adv, ret = rng.normal(size=B), rng.normal(size=B)
    logits, _ = oracle.forward(net, flat, obs)
    lsm = logits - logits.max(1, keepdims=True); lsm -= np.log(np.exp(lsm).sum(1, keepdims=True))
    old_logp = lsm[np.arange(B), actions] + rng.normal(0, 0.15, size=B) * (algo != 0)
    return net, flat, obs, actions, old_logp, adv, ret


@pytest.mark.parametrize("algo,eps", [(0, 0.1), (1, 0.1), (1, 0.3)])
def test_loss_and_grads_match_torch_autograd(oracle, algo, eps):
    net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 21 + algo, 16, algo)
    hp = oracle.make_hparams(algo=algo, clip_eps=eps, vf_coef=0.5, ent_coef=0.01)
    g, st = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, hp)
    p = _torch_params(flat, TINY, TINY["A"])
    loss, lpi, lv, ent = _torch_loss(p, obs, TINY["convs"], actions, old_logp, adv, ret, algo, eps, 0.5, 0.01)
    loss.backward()
    tg = np.concatenate([p[name].grad.numpy().ravel() for name, _ in
                         syn.param_shapes(TINY["C"], TINY["H"], TINY["W"], TINY["A"], convs=TINY["convs"],
                                          hidden=TINY["hidden"])])
    np.testing.assert_allclose(st["total_loss"], loss.item(), rtol=1e-12)
    np.testing.assert_allclose(st["policy_loss"], lpi.item(), rtol=1e-12)
    np.testing.assert_allclose(st["value_loss"], lv.item(), rtol=1e-12)
    np.testing.assert_allclose(st["entropy"], ent.item(), rtol=1e-12)
    np.testing.assert_allclose(g, tg, rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(st["grad_norm"], np.linalg.norm(tg), rtol=1e-10)
    if algo == 1:
        assert 0.0 < st["clip_frac"] < 1.0      # the case exercises both clipped and unclipped rows


def test_full_size_gradient_matches_torch_autograd(oracle):
    """Full Atari-shaped net, 4 rows, PPO: every parameter tensor's gradient against autograd."""
    kw = dict(C=4, H=84, W=84, A=6, convs=((32, 8, 4), (64, 4, 2), (64, 3, 1)), hidden=512)
    net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 4, 4, 1, kw)
    hp = oracle.make_hparams(algo=1, clip_eps=0.1)
    idx = np.array([3, 1, 0], np.int32)
    g, st = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, hp, index=idx)
    p = _torch_params(flat, kw, 6)
    sel = idx.astype(np.int64)
    loss, *_ = _torch_loss(p, obs[sel], kw["convs"], actions[sel], old_logp[sel], adv[sel], ret[sel], 1, 0.1, 0.5, 0.01)
    loss.backward()
    tg = np.concatenate([p[name].grad.numpy().ravel() for name, _ in syn.param_shapes(4, 84, 84, 6)])
    np.testing.assert_allclose(g, tg, rtol=1e-8, atol=1e-13)


def test_finite_differences(oracle):
    """Central differences in float64 on the tiny net, at a point away from ReLU / clip kinks."""
    for algo in (0, 1):
        net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 31 + algo, 6, algo)
        hp = oracle.make_hparams(algo=algo, clip_eps=0.2, vf_coef=0.5, ent_coef=0.01)
        g, _ = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, hp)
        rng = np.random.default_rng(0)
        picks = rng.choice(flat.size, size=60, replace=False)
        picks = np.concatenate([picks, np.arange(flat.size - 40, flat.size)])   # fc tail, heads, biases
        h = 1e-6
        for i in picks:
            pp, pm = flat.copy(), flat.copy()
            pp[i] += h; pm[i] -= h
            lp_ = oracle.loss_grads(net, pp, obs, actions, old_logp, adv, ret, hp, want_grads=False)[1]["total_loss"]
            lm_ = oracle.loss_grads(net, pm, obs, actions, old_logp, adv, ret, hp, want_grads=False)[1]["total_loss"]
            fd = (lp_ - lm_) / (2 * h)
            assert abs(fd - g[i]) <= 1e-6 * max(1.0, abs(g[i])) + 2e-8, (algo, i, fd, g[i])


def test_ppo_ratio_one_is_a2c(oracle):
    """rho == 1 (old_logp = current logp): PPO's gradient equals A2C's whatever eps is (Sec. 3 eq. (4))."""
    net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 41, 12, 0)     # algo 0 -> old_logp is exact
    ga, sa = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, oracle.make_hparams(algo=0))
    for eps in (0.0, 0.1, 1e9):
        gp, sp = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, oracle.make_hparams(algo=1, clip_eps=eps))
        np.testing.assert_allclose(gp, ga, rtol=1e-12, atol=1e-15)
        assert sp["clip_frac"] == 0.0 and abs(sp["approx_kl"]) < 1e-15
    # without clipping and arbitrary old_logp: PPO gradient = A2C gradient with adv scaled by rho
    rng = np.random.default_rng(1)
    olp = old_logp + rng.normal(0, 0.3, size=old_logp.size)
    gp, _ = oracle.loss_grads(net, flat, obs, actions, olp, adv, ret, oracle.make_hparams(algo=1, clip_eps=1e9))
    rho = np.exp(old_logp - olp)
    ga2, _ = oracle.loss_grads(net, flat, obs, actions, old_logp, adv * rho, ret, oracle.make_hparams(algo=0))
    np.testing.assert_allclose(gp, ga2, rtol=1e-12, atol=1e-15)


def _flat_grad(p, kw):
    return np.concatenate([p[name].grad.numpy().ravel() for name, _ in
                           syn.param_shapes(kw["C"], kw["H"], kw["W"], kw["A"], convs=kw["convs"], hidden=kw["hidden"])])


@pytest.mark.parametrize("rho_bar", [1.0, 1.1, 1e9])
def test_truncated_importance_weights(oracle, rho_bar):
    """The alternative to the delayed gradient in the appendix's ablation ("Delayed Gradient"): importance weights
    w = min(rho, rho_bar), constants in the derivative.  Pinned three ways: torch autograd with the weight detached,
    A2C on advantages pre-multiplied by weights computed here from the forward pass, and the on-policy case."""
    net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 61, 16, 2)
    hp = oracle.make_hparams(algo="a2c_tis", rho_bar=rho_bar)
    g, st = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, hp)
    p = _torch_params(flat, TINY, TINY["A"])
    loss, lpi, lv, ent = _torch_loss(p, obs, TINY["convs"], actions, old_logp, adv, ret, 2, 0.0, 0.5, 0.01, rho_bar=rho_bar)
    loss.backward()
    np.testing.assert_allclose(st["total_loss"], loss.item(), rtol=1e-12)
    np.testing.assert_allclose(st["policy_loss"], lpi.item(), rtol=1e-12)
    np.testing.assert_allclose(g, _flat_grad(p, TINY), rtol=1e-9, atol=1e-13)
    # the same gradient from the A2C branch with w folded into the advantages
    logits, _ = oracle.forward(net, flat, obs)
    lsm = logits - logits.max(1, keepdims=True); lsm -= np.log(np.exp(lsm).sum(1, keepdims=True))
    rho = np.exp(lsm[np.arange(16), actions] - old_logp)
    w = np.minimum(rho, rho_bar)
    ga, _ = oracle.loss_grads(net, flat, obs, actions, old_logp, adv * w, ret, oracle.make_hparams(algo=0))
    np.testing.assert_allclose(g, ga, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(st["clip_frac"], np.mean(rho > rho_bar), rtol=0, atol=1e-15)
    if rho_bar == 1.1:
        assert 0.0 < st["clip_frac"] < 1.0          # both truncated and untruncated rows occur
    # on-policy data (rho == 1): the plain actor-critic gradient whenever rho_bar >= 1
    net, flat, obs, actions, exact_logp, adv, ret = _problem(oracle, 62, 8, 0)
    g1, _ = oracle.loss_grads(net, flat, obs, actions, exact_logp, adv, ret, hp)
    g0, _ = oracle.loss_grads(net, flat, obs, actions, exact_logp, adv, ret, oracle.make_hparams(algo=0))
    np.testing.assert_allclose(g1, g0, rtol=1e-12, atol=1e-15)


def test_clipped_value_loss(oracle):
    """max((v-R)^2, (old_v + clip(v - old_v, +-c) - R)^2) per row: torch autograd; a radius that never binds gives the
    plain squared loss; rows whose clipped term wins while v is outside the radius send no gradient to the value head."""
    net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 71, 16, 1)
    _, v = oracle.forward(net, flat, obs)
    rng = np.random.default_rng(5)
    old_values = v + rng.normal(0, 0.2, size=16)
    c = 0.1
    hp = oracle.make_hparams(algo=1, clip_eps=0.1, value_clip=c)
    g, st = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, hp, old_values=old_values)
    p = _torch_params(flat, TINY, TINY["A"])
    loss, lpi, lv, ent = _torch_loss(p, obs, TINY["convs"], actions, old_logp, adv, ret, 1, 0.1, 0.5, 0.01,
                                     old_values=old_values, value_clip=c)
    loss.backward()
    np.testing.assert_allclose(st["value_loss"], lv.item(), rtol=1e-12)
    np.testing.assert_allclose(st["total_loss"], loss.item(), rtol=1e-12)
    np.testing.assert_allclose(g, _flat_grad(p, TINY), rtol=1e-9, atol=1e-13)
    vc = old_values + np.clip(v - old_values, -c, c)
    wins = (vc - ret) ** 2 > (v - ret) ** 2
    outside = np.abs(v - old_values) > c
    assert (wins & outside).any() and (~wins).any()       # the case has rows of both kinds
    # never binding: identical to the unclipped loss
    g_big, s_big = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret,
                                     oracle.make_hparams(algo=1, clip_eps=0.1, value_clip=1e9), old_values=old_values)
    g_off, s_off = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, oracle.make_hparams(algo=1, clip_eps=0.1))
    np.testing.assert_array_equal(g_big, g_off)
    assert s_big["value_loss"] == s_off["value_loss"]
    # every row clipped away from v with the clipped term winning: the value head gets no gradient at all
    far, target = v + 10.0, v - 5.0             # clipped value v + 10 - c is further from the target than v is
    g_far, s_far = oracle.loss_grads(net, flat, obs, actions, old_logp, np.zeros(16), target,
                                     oracle.make_hparams(algo=0, ent_coef=0.0, value_clip=c), old_values=far)
    assert not g_far.any(), "with adv = 0, no entropy term and a dead value term nothing has a gradient"
    np.testing.assert_allclose(s_far["value_loss"], (15.0 - c) ** 2, rtol=1e-12)


def test_uniform_policy_entropy_and_zero_sum(oracle):
    """Zero policy-head weights: p = 1/A, H = log A, and the policy-bias gradient sums to zero."""
    net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 51, 8, 0)
    A, Hd = TINY["A"], TINY["hidden"]
    P = flat.size
    piw = P - 1 - Hd - A - A * Hd
    flat[piw:piw + A * Hd + A] = 0.0
    g, st = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, oracle.make_hparams(algo=0, ent_coef=0.5))
    np.testing.assert_allclose(st["entropy"], np.log(A), rtol=1e-14)
    gb = g[piw + A * Hd:piw + A * Hd + A]
    assert abs(gb.sum()) < 1e-15
    # at the uniform policy the entropy term has zero gradient: bias grad = -mean(adv * (onehot - 1/A))
    want = -np.array([(adv * ((actions == j) - 1.0 / A)).mean() for j in range(A)])
    np.testing.assert_allclose(gb, want, rtol=1e-12, atol=1e-15)


# ---- the reduced-precision operand model (operand_bf16 = 1) -------------------------------------------------------
def test_round_bf16_against_torch_and_ties(oracle):
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.normal(size=2000) * 10.0 ** rng.integers(-6, 6, size=2000), [0.0, -0.0, 1.0, 255.0]])
    xs = xs.astype(np.float32)
    want = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.round_bf16(float(x)) for x in xs], np.float32)
    assert np.array_equal(got, want)
    # ties go to the even 8-bit significand
    assert oracle.round_bf16(1.0 + 2.0 ** -8) == 1.0
    assert oracle.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert oracle.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert oracle.round_bf16(255.0) == 255.0 and oracle.round_bf16(257.0) == 256.0


class _RoundGrad(torch.autograd.Function):
    """Identity whose derivative rounds the incoming gradient to bfloat16 (placed on a pre-activation, it rounds the
    gradient with respect to that pre-activation before any product of the backward pass uses it)."""

    @staticmethod
    def forward(ctx, x):
        return x.view_as(x)

    @staticmethod
    def backward(ctx, g):
        return g.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def _rb(t):
    q = t.detach().to(torch.float32).to(torch.bfloat16).to(torch.float64)
    return t + (q - t).detach()


def _rounded_model_torch(kw, p, obs, gate_masks=None, round_grads=True):
    """Forward pass with every operand of a conv/FC product rounded to bfloat16 (straight-through); with round_grads
    the gradients of the pre-activations are rounded too.  gate_masks: ReLU gates to use in the derivative instead of
    the pass's own.  -> (logits, values, list of pre-activations)."""
    def relu(pre, li):
        if gate_masks is None:
            return F.relu(pre)
        y = pre * gate_masks[li]
        return F.relu(pre).detach() + (y - y.detach())

    rg = _RoundGrad.apply if round_grads else (lambda t: t)
    pres = []
    x = torch.from_numpy(obs.astype(np.float64)) / 255.0
    for i, (co, k, s) in enumerate(kw["convs"]):
        pre = rg(F.conv2d(x, _rb(p[f"conv{i + 1}.w"]), p[f"conv{i + 1}.b"], stride=s))
        pres.append(pre)
        x = _rb(relu(pre, i))
    pre = rg(F.linear(x.flatten(1), _rb(p["fc.w"]), p["fc.b"]))
    pres.append(pre)
    h = relu(pre, len(kw["convs"]))
    return F.linear(h, p["pi.w"], p["pi.b"]), F.linear(h, p["v.w"], p["v.b"])[:, 0], pres


def _ppo_loss_torch(logits, v, actions, old_logp, adv, ret):
    lsm = F.log_softmax(logits, dim=1)
    logp = lsm.gather(1, torch.from_numpy(actions.astype(np.int64))[:, None])[:, 0]
    rho = (logp - torch.from_numpy(old_logp)).exp()
    ad = torch.from_numpy(adv)
    return (-torch.minimum(rho * ad, rho.clamp(0.9, 1.1) * ad).mean() + 0.5 * ((torch.from_numpy(ret) - v) ** 2).mean()
            - 0.01 * (-(lsm.exp() * lsm).sum(1)).mean())


_QKW = dict(C=3, H=44, W=52, A=5, convs=((32, 8, 4), (64, 4, 2), (64, 3, 1)), hidden=512)


def _qflat_grad(p):
    return np.concatenate([p[name].grad.numpy().ravel() for name, _ in syn.param_shapes(3, 44, 52, 5)])


def test_operand_model_matches_torch_with_rounded_operands(oracle):
    """Forward and gradients in the operand-rounding model vs autograd through the same roundings: weights and layer
    outputs rounded straight-through in the forward pass, pre-activation gradients rounded in the backward pass."""
    kw = _QKW
    net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 61, 4, 1, kw)
    flat = flat.astype(np.float32).astype(np.float64)
    qnet = oracle.make_net(3, 44, 52, 5, operand_bf16=True)
    p = _torch_params(flat, kw, 5)
    logits, v, _ = _rounded_model_torch(kw, p, obs)
    ql, qv = oracle.forward(qnet, flat, obs)
    np.testing.assert_allclose(ql, logits.detach().numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(qv, v.detach().numpy(), rtol=1e-9, atol=1e-12)
    el, _ = oracle.forward(net, flat, obs)
    assert 1e-5 < np.abs(ql - el).max() < 0.1 * np.abs(el).max()       # the rounding is really applied
    loss = _ppo_loss_torch(logits, v, actions, old_logp, adv, ret)
    loss.backward()
    tg = _qflat_grad(p)
    g, st = oracle.loss_grads(qnet, flat, obs, actions, old_logp, adv, ret, oracle.make_hparams(algo=1, clip_eps=0.1))
    np.testing.assert_allclose(st["total_loss"], loss.item(), rtol=1e-11)
    np.testing.assert_allclose(g, tg, rtol=1e-8, atol=1e-13)
    # the backward roundings are really applied: with the forward roundings alone the gradient differs, a little
    p2 = _torch_params(flat, kw, 5)
    l2, v2, _ = _rounded_model_torch(kw, p2, obs, round_grads=False)
    _ppo_loss_torch(l2, v2, actions, old_logp, adv, ret).backward()
    fg = _qflat_grad(p2)
    rel = np.linalg.norm(g - fg) / np.linalg.norm(fg)
    assert 1e-5 < rel < 2e-2


def test_exact_gate_diagnostic_matches_torch(oracle):
    """gates_exact: rounded operands, but every discontinuous decision of the derivative (ReLU gates, the clipped
    surrogate's band decision) comes from the unrounded forward pass."""
    kw = _QKW
    net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 62, 8, 1, kw)
    flat = flat.astype(np.float32).astype(np.float64)
    pe = _torch_params(flat, kw, 5)                                   # unrounded forward pass: its gates
    x = torch.from_numpy(obs.astype(np.float64)) / 255.0
    masks = []
    with torch.no_grad():
        for i, (co, k, s) in enumerate(kw["convs"]):
            pre = F.conv2d(x, pe[f"conv{i + 1}.w"], pe[f"conv{i + 1}.b"], stride=s)
            masks.append((pre > 0).to(torch.float64))
            x = F.relu(pre)
        pre = F.linear(x.flatten(1), pe["fc.w"], pe["fc.b"])
        masks.append((pre > 0).to(torch.float64))
        h = F.relu(pre)
        lsm_e = F.log_softmax(F.linear(h, pe["pi.w"], pe["pi.b"]), dim=1)
        logp_e = lsm_e.gather(1, torch.from_numpy(actions.astype(np.int64))[:, None])[:, 0].numpy()
    # put the unrounded ratio of every row a hair inside or outside the band's edge that its advantage makes active, so
    # that the rounded pass lands on the other side for some of them
    eps = 0.1
    edge = np.where(adv > 0, 1.0 + eps, 1.0 - eps)
    old_logp = logp_e - np.log(edge * (1.0 + 1e-6 * np.where(np.arange(8) % 2 == 0, 1.0, -1.0)))
    rho_e = np.exp(logp_e - old_logp)
    cut_e = ((adv > 0) & (rho_e > 1 + eps)) | ((adv < 0) & (rho_e < 1 - eps))
    assert cut_e.any() and not cut_e.all()
    p = _torch_params(flat, kw, 5)
    logits, v, pres = _rounded_model_torch(kw, p, obs, gate_masks=masks)
    flips = sum(int(((pr.detach() > 0).to(torch.float64) != mk).sum()) for pr, mk in zip(pres, masks))
    assert flips > 0                                                   # otherwise the case tests nothing
    lsm = F.log_softmax(logits, dim=1)
    logp = lsm.gather(1, torch.from_numpy(actions.astype(np.int64))[:, None])[:, 0]
    rho = (logp - torch.from_numpy(old_logp)).exp()
    rho_q = rho.detach().numpy()
    cut_q = ((adv > 0) & (rho_q > 1 + eps)) | ((adv < 0) & (rho_q < 1 - eps))
    assert (cut_q != cut_e).any()                                      # the rounded pass decides differently somewhere
    ad = torch.from_numpy(adv)
    keep = torch.from_numpy((~cut_e).astype(np.float64))
    surrogate = -(rho * ad * keep).mean()                              # derivative: -adv rho / B where not cut (unrounded decision)
    loss = surrogate + 0.5 * ((torch.from_numpy(ret) - v) ** 2).mean() - 0.01 * (-(lsm.exp() * lsm).sum(1)).mean()
    loss.backward()
    tg = _qflat_grad(p)
    hp = oracle.make_hparams(algo=1, clip_eps=eps)
    gnet = oracle.make_net(3, 44, 52, 5, operand_bf16=True, gates_exact=True)
    g, st = oracle.loss_grads(gnet, flat, obs, actions, old_logp, adv, ret, hp)
    np.testing.assert_allclose(g, tg, rtol=1e-8, atol=1e-13)
    gq, stq = oracle.loss_grads(oracle.make_net(3, 44, 52, 5, operand_bf16=True), flat, obs, actions, old_logp, adv,
                                ret, hp)
    assert st["total_loss"] == stq["total_loss"]                       # the losses are those of the rounded pass
    assert np.abs(g - gq).max() > 0                                    # and the flipped decisions do change the gradient


def test_threaded_variants_equal_the_plain_calls(oracle):
    """The threaded gradient is the slot-ordered combination of plain calls: equal to the plain call up to the
    reassociation of its float64 sums, and independent of the number of threads; the threaded forward is identical."""
    net, flat, obs, actions, old_logp, adv, ret = _problem(oracle, 63, 37, 1, _QKW)
    hp = oracle.make_hparams(algo=1, clip_eps=0.1)
    idx = np.array([5, 3, 36, 0, 7, 7, 12, 30, 2, 1, 35], np.int32)
    for index in (None, idx):
        g1, s1 = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, hp, index=index)
        g2, s2 = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, hp, index=index, threads=2)
        g3, s3 = oracle.loss_grads(net, flat, obs, actions, old_logp, adv, ret, hp, index=index, threads=5)
        assert np.array_equal(g2, g3) and s2 == s3
        np.testing.assert_allclose(g2, g1, rtol=1e-11, atol=1e-15)
        for k in s1:
            np.testing.assert_allclose(s2[k], s1[k], rtol=1e-12, atol=1e-15)
        l1, v1 = oracle.forward(net, flat, obs, index=index)
        l2, v2 = oracle.forward(net, flat, obs, index=index, threads=3)
        assert np.array_equal(l1, l2) and np.array_equal(v1, v2)
    z = np.zeros(flat.size)
    th1 = oracle.learner_step(net, flat, z, z, 1, obs, actions, old_logp, adv, ret, hp)
    th2 = oracle.learner_step(net, flat, z, z, 1, obs, actions, old_logp, adv, ret, hp, threads=4)
    big = np.abs(th1[3]) > 1e-4 * np.abs(th1[3]).max()    # Adam's first step is ~lr*sign(g): compare where g is not ~0
    np.testing.assert_allclose(th2[0][big], th1[0][big], rtol=0, atol=1e-10)
