"""GPU parity: every call of the C ABI against the CPU oracle on the same seeded inputs.

Tolerances (relative, per output tensor; both ||x-y||2/||y||2 and max|x-y|/max|y| must hold):
  fp32: logits/values/losses/gradients 1e-4, GAE and returns 1e-6, parameters after an update 1e-5;
  bf16 operands: 2e-2 on forward outputs and losses (gradients: see test_bf16_* below);
  actions: bit-exact for the same logits and the same Philox counters.
"""
import numpy as np
import pytest
import torch

import hts_synth as syn

pytestmark = pytest.mark.gpu

ATARI = (4, 84, 84)
FOOT = (16, 72, 96)


@pytest.fixture(scope="module")
def hts():
    import paper_2012_09849_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return m


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def oracle_hp(oracle, hp):
    """The oracle's hyper-parameters with exactly the binary32 values the GPU call receives."""
    return oracle.make_hparams(algo=hp.algo, clip_eps=float(hp.clip_eps), vf_coef=float(hp.vf_coef),
                               ent_coef=float(hp.ent_coef), max_grad_norm=float(hp.max_grad_norm), lr=float(hp.lr),
                               beta1=float(hp.beta1), beta2=float(hp.beta2), adam_eps=float(hp.adam_eps),
                               rho_bar=float(hp.rho_bar), value_clip=float(hp.value_clip))


def rel_err(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    l2 = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    mx = np.abs(got - want).max() / max(np.abs(want).max(), 1e-300)
    return max(l2, mx)


def assert_close(got, want, tol, name=""):
    e = rel_err(got, want)
    assert e <= tol, f"{name}: relative error {e:.3e} > {tol:.1e}"


# ------------------------------------------------------------------------------------------------------------
# tile core
# ------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("prec,tol", [(0, 1e-5), (1, 1e-2)])
@pytest.mark.parametrize("shape", [(64, 64, 32), (1, 1, 8), (70, 33, 40), (257, 130, 328), (16, 512, 3136)])
def test_tile_core_matches_matmul(hts, prec, tol, shape):
    M, N, K = shape
    ctx = hts.Context(4, 84, 84, 6, max_act_batch=1)
    rng = np.random.default_rng(M * 1000 + N)
    A, B = rng.normal(size=(M, K)).astype(np.float32), rng.normal(size=(N, K)).astype(np.float32)
    out = torch.full((M, N), float("nan"), device="cuda")
    ctx.hts_test_gemm(prec, dev(A), dev(B), out)
    torch.cuda.synchronize()
    want = A.astype(np.float64) @ B.astype(np.float64).T
    assert_close(out.cpu().numpy(), want, tol, f"gemm {shape}")
    ctx.close()


# ------------------------------------------------------------------------------------------------------------
# sampler
# ------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("A", [1, 6, 18, 64])
def test_sampler_bit_exact(hts, oracle, A):
    ctx = hts.Context(4, 84, 84, A, max_act_batch=1)
    rng = np.random.default_rng(A)
    N = 20001
    logits = (rng.normal(0, 2.5, size=(N, A))).astype(np.float32)
    logits[:50] = 0.0                        # exact ties
    logits[50:60, 0] = 100.0                 # underflow of the other terms
    actions = torch.full((N,), -1, dtype=torch.int32, device="cuda")
    logp = torch.zeros(N, device="cuda")
    ctx.hts_sample_from_logits(dev(logits), 0xDEADBEEF12345678, 77, 1000, actions, logp)
    torch.cuda.synchronize()
    a_ref, lp_ref, _ = oracle.sample(logits, 0xDEADBEEF12345678, 77, 1000)
    assert np.array_equal(actions.cpu().numpy(), a_ref)
    np.testing.assert_allclose(logp.cpu().numpy(), lp_ref, atol=1e-6, rtol=0)
    ctx.close()


# ------------------------------------------------------------------------------------------------------------
# returns / GAE
# ------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("T,N,gamma,lam", [(5, 4, 0.99, 1.0), (5, 16, 0.99, 1.0), (128, 32, 0.99, 0.95),
                                           (512, 16, 0.993, 0.95), (1, 1, 0.9, 0.9), (7, 65, 0.99, 0.95),
                                           (33, 1000, 0.99, 0.95), (128, 4096, 0.99, 0.95),
                                           (40, 70001, 0.99, 0.95), (17, 20000, 0.99, 0.95),    # plain / chunked
                                           (11, 262144, 0.99, 0.95), (6, 262147, 0.99, 0.95)])   # very wide
def test_gae_parity(hts, oracle, T, N, gamma, lam):
    ctx = hts.Context(4, 84, 84, 6, max_act_batch=1)
    seed = T * 131 + N
    r = syn.normal_f32(seed, syn.S_REW, (T, N)) if N > 100 else syn.rewards_ternary(seed, T, N)
    v = syn.normal_f32(seed, syn.S_VAL, (T + 1, N))
    d = syn.dones_bernoulli(seed, T, N, 0.05 if T < 100 else 0.01)
    adv, ret = torch.zeros(T, N, device="cuda"), torch.zeros(T, N, device="cuda")
    ctx.hts_returns_gae(dev(r), dev(v), dev(d), gamma, lam, adv, ret)
    torch.cuda.synchronize()
    a_ref, r_ref = oracle.gae(r, v, d, np.float32(gamma), np.float32(lam))
    for got, want, nm in ((adv, a_ref, "adv"), (ret, r_ref, "ret")):
        g = got.cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(g - want) / np.maximum(1.0, np.abs(want)))) <= 1e-6, nm
        assert_close(g, want, 1e-6, nm)
    ctx.close()


def test_normalize_advantages(hts, oracle):
    ctx = hts.Context(4, 84, 84, 6, max_act_batch=1)
    for n in (1, 2, 20, 4096, 8192 + 3):
        a = syn.normal_f32(n, syn.S_MISC, (n,)) * 3 + 1
        t = dev(a)
        ctx.hts_normalize_advantages(t)
        torch.cuda.synchronize()
        want = oracle.normalize_adv(a)
        np.testing.assert_allclose(t.cpu().numpy(), want, rtol=2e-6, atol=2e-6)
    ctx.close()


# ------------------------------------------------------------------------------------------------------------
# hts_act
# ------------------------------------------------------------------------------------------------------------
def _act(ctx, obs, params, seed, step, env_offset, A):
    N = obs.shape[0]
    actions = torch.full((N,), -1, dtype=torch.int32, device="cuda")
    logp, values = torch.zeros(N, device="cuda"), torch.zeros(N, device="cuda")
    logits = torch.zeros(N, A, device="cuda")
    ctx.hts_act(obs, params, seed, step, env_offset, actions, logp, values, logits)
    torch.cuda.synchronize()
    return actions.cpu().numpy(), logp.cpu().numpy(), values.cpu().numpy(), logits.cpu().numpy()


@pytest.mark.parametrize("shape,A,N,prec,tol", [
    (ATARI, 6, 4, 0, 1e-4), (ATARI, 18, 16, 0, 1e-4), (ATARI, 18, 37, 0, 1e-4), (FOOT, 19, 16, 0, 1e-4),
    ((2, 36, 36), 5, 9, 0, 1e-4), ((3, 44, 52), 7, 130, 0, 1e-4),
    (ATARI, 18, 32, 1, 2e-2), (FOOT, 19, 16, 1, 2e-2), ((3, 44, 52), 7, 130, 1, 2e-2),
    # the multi-agent football workload: 16 environments x 3 controlled players = 48 rows per call
    (FOOT, 19, 48, 1, 2e-2), (FOOT, 19, 48, 0, 1e-4),
    # many actions: a second round of policy-head rows (A > 20), one lane per row sum (A > 32), the largest head, and
    # more than 512 rows (four wavefronts per workgroup, more than 64 KiB of LDS with 64 actions)
    ((2, 36, 36), 21, 9, 0, 1e-4), ((2, 36, 36), 33, 40, 0, 1e-4), ((2, 36, 36), 64, 17, 0, 1e-4),
    ((2, 36, 36), 64, 530, 0, 1e-4), ((2, 36, 36), 33, 530, 1, 2e-2)])
def test_act_parity(hts, oracle, shape, A, N, prec, tol):
    Cc, H, W = shape
    ctx = hts.Context(Cc, H, W, A, precision=prec, max_act_batch=N)
    net = oracle.make_net(Cc, H, W, A)
    params = syn.init_params(7, Cc, H, W, A, bias_scale=0.05)
    if shape == ATARI:
        obs = syn.obs_atari(11, 1, N)[0]
    elif shape == FOOT:
        obs = syn.obs_football(11, 1, N)[0]
    else:
        obs = syn.obs_uniform(11, N, Cc, H, W)
    seed, step, off = 20201209, 3, 40
    a, lp, v, lg = _act(ctx, dev(obs), dev(params), seed, step, off, A)
    l_ref, v_ref = oracle.forward(net, params, obs)
    assert_close(lg, l_ref, tol, "logits")
    assert_close(v, v_ref, tol, "values")
    # actions: bit-exact given the logits the GPU produced and the same counters
    a_ref, lp_ref, u = oracle.sample(lg, seed, step, off)
    assert np.array_equal(a, a_ref)
    np.testing.assert_allclose(lp, lp_ref, atol=1e-6, rtol=0)
    # against the oracle's own logits the action may differ only where u sits at a CDF boundary
    a_or, _, _ = oracle.sample(l_ref.astype(np.float32), seed, step, off)
    p = np.exp(l_ref - l_ref.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    cdf = np.cumsum(p, 1)
    for i in np.nonzero(a_or != a)[0]:
        assert np.min(np.abs(cdf[i] - u[i])) < (1e-5 if prec == 0 else 3e-2)
    # batch-partition invariance and run-to-run determinism (bitwise)
    k = max(1, N // 3)
    a1, lp1, v1, lg1 = _act(ctx, dev(obs[:k]), dev(params), seed, step, off, A)
    a2, lp2, v2, lg2 = _act(ctx, dev(obs[k:]), dev(params), seed, step, off + k, A) if N > k else (a[:0], lp[:0], v[:0], lg[:0])
    assert np.array_equal(np.concatenate([a1, a2]), a)
    assert np.array_equal(np.concatenate([lg1, lg2]), lg)
    assert np.array_equal(np.concatenate([lp1, lp2]), lp) and np.array_equal(np.concatenate([v1, v2]), v)
    for _ in range(3):
        b = _act(ctx, dev(obs), dev(params), seed, step, off, A)
        assert all(np.array_equal(x, y) for x, y in zip(b, (a, lp, v, lg)))
    ctx.close()


@pytest.mark.parametrize("shape,A,prec", [(ATARI, 18, 0), (FOOT, 19, 0), ((3, 44, 52), 7, 0), (ATARI, 18, 1), (FOOT, 19, 1)])
def test_act_small_and_large_batch_kernels_agree_bitwise(hts, shape, A, prec, monkeypatch):
    """Small batches run wave-per-segment kernels, large ones the tile kernels; both add the same K segments in the
    same order, so an observation's outputs do not depend on which kernels served it."""
    Cc, H, W = shape
    N = 40
    params = dev(syn.init_params(9, Cc, H, W, A, bias_scale=0.05))
    obs = dev(syn.obs_uniform(13, N, Cc, H, W))
    outs = []
    # all small / all tile kernels / mixed (the 40-batch is "large", splits small) / tile kernels with the FC layer's
    # groups added inside the FC kernel (the form large batches take) instead of by the heads kernel
    # ... and the wave-per-segment kernels with 32x32 tiles only / with 16x16 tiles in every layer
    for knob, fold, t16 in (("128", None, None), ("0", None, None), ("16", None, None), ("0", "1", None),
                            ("128", None, "0"), ("128", None, "100000")):
        monkeypatch.setenv("HTS_SMALL_BATCH", knob)
        if t16 is None:
            monkeypatch.delenv("HTS_TILE16_BELOW", raising=False)
        else:
            monkeypatch.setenv("HTS_TILE16_BELOW", t16)
        if fold is None:
            monkeypatch.delenv("HTS_FC_FOLD_ROWS", raising=False)
        else:
            monkeypatch.setenv("HTS_FC_FOLD_ROWS", fold)
        ctx = hts.Context(Cc, H, W, A, precision=prec, max_act_batch=N)
        full = _act(ctx, obs, params, 5, 1, 0, A)
        a = _act(ctx, obs[:16], params, 5, 1, 0, A)
        b = _act(ctx, obs[16:], params, 5, 1, 16, A)
        assert all(np.array_equal(np.concatenate([x, y]), z) for x, y, z in zip(a, b, full))
        outs.append(full)
        ctx.close()
    for o in outs[1:]:
        assert all(np.array_equal(x, y) for x, y in zip(o, outs[0]))


@pytest.mark.parametrize("shape,A,N", [(FOOT, 19, 256), (FOOT, 19, 301), (FOOT, 19, 700), (ATARI, 18, 300), (ATARI, 18, 2100)])
def test_conv1_slab_kernel_agrees_bitwise(hts, shape, A, N, monkeypatch):
    """Large bf16 batches of 16x72x96 frames take a conv1 kernel of their own (frame slabs of four channels resident in
    LDS, producer and consumer wavefronts); it adds the same 64-long segments in the same order as the tile kernel, so
    an observation's outputs do not depend on which of them served it.  N = 301 and 700 leave workgroups with
    different numbers of observations (256 workgroups walk the batch).  4x84x84 frames take it too (there
    against the LDS-image kernel of that shape)."""
    Cc, H, W = shape
    params = dev(syn.init_params(21, Cc, H, W, A, bias_scale=0.05))
    obs = dev(syn.obs_football(23, 1, N)[0] if shape == FOOT else syn.obs_atari(23, 1, N)[0])
    outs = []
    for rows in ("256", "100000000"):
        monkeypatch.setenv("HTS_CONV1_SLAB_ROWS", rows)
        ctx = hts.Context(Cc, H, W, A, precision=1, max_act_batch=N)
        outs.append(_act(ctx, obs, params, 5, 1, 0, A))
        ctx.close()
    assert all(np.array_equal(x, y) for x, y in zip(*outs))
    # and against the wave-per-segment kernels, 100 observations at a time
    monkeypatch.delenv("HTS_CONV1_SLAB_ROWS", raising=False)
    ctx = hts.Context(Cc, H, W, A, precision=1, max_act_batch=N)
    for lo in range(0, N, 100):
        part = _act(ctx, obs[lo:lo + 100], params, 5, 1, lo, A)
        assert all(np.array_equal(x, y[lo:lo + 100]) for x, y in zip(part, outs[0]))
    ctx.close()


@pytest.mark.parametrize("count,B", [(330, 301), (600, 600)])
def test_conv1_slab_gradient_kernels_agree(hts, oracle, count, B, monkeypatch):
    """The learner's two conv1 kernels for large bf16 batches of 16x72x96 frames (forward and weight gradient, both with
    producer and consumer wavefronts) against the kernels they replace: the forward bits are identical, and the weight
    gradient adds the same products in the same order -- only the bias column is formed differently (column sums
    taken by the threads that copy the gradient rows) -- so every tensor of the gradient but conv1.b is bitwise the same."""
    shape, A = FOOT, 19
    Cc, H, W = shape
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 1200 + count, True)
    index = syn.permutation(9, count)[:B]
    out = []
    for rows in ("256", "100000000"):
        monkeypatch.setenv("HTS_CONV1_SLAB_ROWS", rows)
        ctx = hts.Context(Cc, H, W, A, precision=1, max_learn_batch=B)
        hp = hts.HParams(algo=1, clip_eps=0.1)
        grads = torch.full((ctx.P,), float("nan"), device="cuda")
        stats = ctx.new_stats()
        ctx.hts_loss_and_grads(dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), dev(params), hp, grads,
                               index=dev(index), stats=stats)
        torch.cuda.synchronize()
        out.append((grads.cpu().numpy(), ctx.read_stats(stats)))
        ctx.close()
    (g_new, st_new), (g_old, st_old) = out
    assert np.all(np.isfinite(g_new))
    for k in ("policy_loss", "value_loss", "entropy"):
        assert st_new[k] == st_old[k], (k, st_new[k], st_old[k])
    for name, gn in _split(g_new, shape, A).items():
        go = _split(g_old, shape, A)[name]
        if name == "conv1.b":
            assert rel_err(gn, go) <= 1e-5, (name, rel_err(gn, go))
        else:
            assert np.array_equal(gn, go), (name, rel_err(gn, go))


@pytest.mark.parametrize("prec", [0, 1])
def test_act_with_loaded_parameters(hts, prec):
    """hts_act(params = NULL) reuses the parameters loaded before (bitwise the same outputs); it is refused when
    nothing is loaded, and after a learner update has moved the caller's vector on."""
    Cc, H, W = ATARI
    A, N = 6, 20
    ctx = hts.Context(Cc, H, W, A, precision=prec, max_act_batch=N, max_learn_batch=N)
    params = dev(syn.init_params(21, Cc, H, W, A, bias_scale=0.05))
    other = dev(syn.init_params(22, Cc, H, W, A, bias_scale=0.05))
    obs = dev(syn.obs_uniform(23, N, Cc, H, W))
    with pytest.raises(hts.HtsError):
        _act(ctx, obs, None, 5, 1, 0, A)
    ref = _act(ctx, obs, params, 5, 1, 0, A)
    again = _act(ctx, obs, None, 5, 1, 0, A)
    assert all(np.array_equal(x, y) for x, y in zip(ref, again))
    ctx.hts_sync_params(other)
    o1 = _act(ctx, obs, None, 5, 1, 0, A)
    o2 = _act(ctx, obs, other, 5, 1, 0, A)
    assert all(np.array_equal(x, y) for x, y in zip(o1, o2))
    assert not np.array_equal(o1[3], ref[3])
    # an update through the library invalidates the loaded copy
    P = params.numel()
    opt = hts.OptState(torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda"))
    ctx.hts_adam_apply(params, torch.ones(P, device="cuda"), opt, hts.HParams())
    with pytest.raises(hts.HtsError):
        _act(ctx, obs, None, 5, 1, 0, A)
    ctx.close()


# ------------------------------------------------------------------------------------------------------------
# learner
# ------------------------------------------------------------------------------------------------------------
def _rollout(oracle, shape, A, count, seed, ppo):
    Cc, H, W = shape
    net = oracle.make_net(Cc, H, W, A)
    params = syn.init_params(seed, Cc, H, W, A, bias_scale=0.05)
    if shape == ATARI:
        obs = syn.obs_uniform(seed + 1, count) if count <= 20 else syn.obs_atari(seed + 1, 1, count)[0]
    elif shape == FOOT:
        obs = syn.obs_football(seed + 1, 1, count)[0]
    else:
        obs = syn.obs_uniform(seed + 1, count, Cc, H, W)
    logits, values = oracle.forward(net, params, obs)
    actions, logp, _ = oracle.sample(logits.astype(np.float32), seed, 0, 0)
    old_logp = logp.astype(np.float64) + (syn.normal(seed, syn.S_MISC, count) * 0.08 if ppo else 0.0)
    adv = syn.normal(seed, syn.S_MISC + 1, count)
    ret = values + adv
    return net, params, obs, actions, old_logp.astype(np.float32), adv.astype(np.float32), ret.astype(np.float32)


def _split(flat, shape, A):
    Cc, H, W = shape
    out, off = {}, 0
    for name, shp in syn.param_shapes(Cc, H, W, A):
        n = int(np.prod(shp)); out[name] = flat[off:off + n]; off += n
    return out


LEARN_CASES = [
    # shape, A, count, B(index?), algo, clip, max_norm, prec
    (ATARI, 6, 20, None, 0, 0.1, 0.0, 0),          # tiny A2C config
    (ATARI, 18, 24, 17, 1, 0.1, 0.5, 0),           # PPO, gathered ragged minibatch, clip on
    (FOOT, 19, 6, 5, 1, 0.08, 0.0, 0),
    ((3, 44, 52), 7, 70, 67, 1, 0.1, 0.5, 0),       # several tiles and ragged tails in every contraction
    ((2, 36, 36), 5, 3, None, 0, 0.1, 0.0, 0),
    # many actions: policy-head weight gradient with more than 32 rows, second round of head rows in the heads kernel
    ((2, 36, 36), 21, 30, 23, 1, 0.1, 0.0, 0),
    ((2, 36, 36), 33, 30, None, 0, 0.1, 0.5, 0),
    ((2, 36, 36), 64, 140, 131, 1, 0.1, 0.0, 0),
    ((2, 36, 36), 64, 560, 530, 1, 0.1, 0.0, 0),   # more than 512 rows: four wavefronts per heads workgroup
    (FOOT, 19, 50, 48, 1, 0.08, 0.0, 0),           # the multi-agent workload's rows per call as a minibatch
]


@pytest.mark.parametrize("small_batch", ["128", "0"])      # wave-per-segment kernels / tile kernels
@pytest.mark.parametrize("shape,A,count,B,algo,eps,max_norm,prec", LEARN_CASES)
def test_loss_and_grads_parity(hts, oracle, shape, A, count, B, algo, eps, max_norm, prec, small_batch, monkeypatch):
    monkeypatch.setenv("HTS_SMALL_BATCH", small_batch)
    Cc, H, W = shape
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 100 + count, algo == 1)
    index = None if B is None else syn.permutation(5, count)[:B]
    nb = count if B is None else B
    ctx = hts.Context(Cc, H, W, A, precision=prec, max_learn_batch=nb)
    hp = hts.HParams(algo=algo, clip_eps=eps, vf_coef=0.5, ent_coef=0.01, max_grad_norm=max_norm)
    grads = torch.full((ctx.P,), float("nan"), device="cuda")
    stats = ctx.new_stats()
    args = (dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), dev(params), hp, grads)
    ctx.hts_loss_and_grads(*args, index=None if index is None else dev(index), stats=stats)
    torch.cuda.synchronize()
    ohp = oracle_hp(oracle, hp)
    g_ref, st_ref = oracle.loss_grads(net, params, obs, actions, old_logp, adv, ret, ohp, index=index)
    g = grads.cpu().numpy()
    assert np.all(np.isfinite(g))
    tol = 1e-4
    for name, gg in _split(g, shape, A).items():
        assert_close(gg, _split(g_ref, shape, A)[name], tol, f"grad {name}")
    st = ctx.read_stats(stats)
    for k in ("policy_loss", "value_loss", "entropy", "grad_norm"):
        assert abs(st[k] - st_ref[k]) <= tol * max(1.0, abs(st_ref[k])), (k, st[k], st_ref[k])
    assert abs(st["clip_frac"] - st_ref["clip_frac"]) < 1e-6 and abs(st["approx_kl"] - st_ref["approx_kl"]) < 1e-5
    assert st["nonfinite"] == 0
    # run-to-run bit identity
    g2 = torch.zeros_like(grads)
    ctx.hts_loss_and_grads(*args[:-1], g2, index=None if index is None else dev(index))
    torch.cuda.synchronize()
    assert torch.equal(grads, g2)
    ctx.close()


@pytest.mark.parametrize("max_norm", [0.0, 0.5])
def test_adam_apply_parity(hts, oracle, max_norm):
    ctx = hts.Context(4, 84, 84, 6, max_learn_batch=1)
    P = ctx.P
    th = syn.normal_f32(1, syn.S_MISC, (P,))
    hp = hts.HParams(lr=7e-4, max_grad_norm=max_norm)
    ohp = oracle_hp(oracle, hp)
    th_d, m_d, v_d = dev(th), torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
    opt = hts.OptState(m_d, v_d, 0)
    th_o, m_o, v_o = th.astype(np.float64), np.zeros(P), np.zeros(P)
    for t in range(1, 4):
        g = syn.normal_f32(10 + t, syn.S_MISC, (P,)) * np.float32(0.01 * t)
        g[::7] = 0.0
        ctx.hts_adam_apply(th_d, dev(g), opt, hp)
        torch.cuda.synchronize()
        sc = oracle.clip_coef(g, max_norm)
        th_o, m_o, v_o = oracle.adam(th_o, g, m_o, v_o, t, ohp, gscale=sc)
        assert opt.step == t
        got = th_d.cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(got - th_o) / np.maximum(1.0, np.abs(th_o)))) <= 1e-6
        # the update itself (not just theta) is right
        assert_close(got - th.astype(np.float64), th_o - th.astype(np.float64), 1e-3, "delta theta")   # theta is fp32: its ulp is ~1e-4 of a step
        assert_close(m_d.cpu().numpy(), m_o, 1e-5, "m")
        assert_close(v_d.cpu().numpy(), v_o, 1e-5, "v")
    ctx.close()


@pytest.mark.parametrize("shape,A,count,B,algo,eps,max_norm,prec", LEARN_CASES[:2] + LEARN_CASES[3:4])
def test_learner_step_parity(hts, oracle, shape, A, count, B, algo, eps, max_norm, prec):
    Cc, H, W = shape
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 200 + count, algo == 1)
    index = None if B is None else syn.permutation(6, count)[:B]
    nb = count if B is None else B
    ctx = hts.Context(Cc, H, W, A, precision=prec, max_learn_batch=nb)
    lr = 7e-4
    hp = hts.HParams(algo=algo, clip_eps=eps, max_grad_norm=max_norm, lr=lr)
    ohp = oracle_hp(oracle, hp)
    P = ctx.P
    p_d, m_d, v_d = dev(params), torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
    opt = hts.OptState(m_d, v_d, 0)
    p_o, m_o, v_o = params.astype(np.float64), np.zeros(P), np.zeros(P)
    idx_d = None if index is None else dev(index)
    g_hist = []
    for t in (1, 2):
        ctx.hts_learner_step(dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), p_d, opt, hp, index=idx_d)
        torch.cuda.synchronize()
        p_prev = p_o.copy()
        p_o, m_o, v_o, g_o, _ = oracle.learner_step(net, p_o, m_o, v_o, t, obs, actions, old_logp, adv, ret, ohp, index=index)
        got = p_d.cpu().numpy().astype(np.float64)
        d_got, d_ref = got - p_prev, p_o - p_prev
        g_hist.append(g_o)
        if t == 1:
            # first update from zero moments: step = lr*g/(|g|+eps), insensitive to small gradient errors: 1e-5
            for name, pp in _split(got, shape, A).items():
                assert_close(pp, _split(p_o, shape, A)[name], 1e-5, f"update {t} param {name}")
        else:
            # later updates: step = lr*mhat/(sqrt(vhat)+eps) with mhat a signed mix of g1, g2, so its error is lr
            # times the ENTRYWISE relative error of the gradients -- small where |g| is a fair fraction of the
            # tensor's largest gradient, unbounded where g nearly vanishes.  Hence: entries with sizeable gradients
            # to 5e-2*lr; of all entries at most 0.5% beyond 1e-2*lr (a ReLU gate whose pre-activation lies within
            # binary32 rounding of zero opens on one side only and moves its weights by a full step), none beyond 2*lr.
            err = np.abs(d_got - d_ref)
            assert err.max() <= 2.0 * lr and float(np.mean(err > 1e-2 * lr)) < 5e-3
            off = 0
            for name, shp in syn.param_shapes(Cc, H, W, A):
                n = int(np.prod(shp)); sl = slice(off, off + n); off += n
                sizeable = np.ones(n, bool)
                for gh in g_hist:
                    sizeable &= np.abs(gh[sl]) > 1e-2 * np.abs(gh[sl]).max()
                if sizeable.any():
                    worst = err[sl][sizeable].max() / lr
                    print(f"update {t} {name}: worst step error on sizeable-gradient entries {worst:.2e} lr")
                    assert worst <= 5e-2, name
        # Each update is checked as ONE update from a common state: the second starts, on both sides, from the
        # oracle's state after the first rounded to binary32 (the step counter carries over).
        p32, m32, v32 = (x.astype(np.float32) for x in (p_o, m_o, v_o))
        p_d.copy_(dev(p32)); m_d.copy_(dev(m32)); v_d.copy_(dev(v32))
        p_o, m_o, v_o = (x.astype(np.float64) for x in (p32, m32, v32))
    assert opt.step == 2
    ctx.close()


@pytest.mark.parametrize("algo,max_norm", [(0, 0.0), (1, 0.5)])
def test_delayed_gradient_step_parity(hts, oracle, algo, max_norm):
    """hts_learner_step_delayed: gradient at the behaviour parameters, update applied to the target parameters."""
    shape, A, count = ATARI, 18, 24
    Cc, H, W = shape
    net, p_b, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 500, algo == 1)
    p_t = (p_b + 0.01 * syn.normal_f32(77, syn.S_MISC, p_b.shape)).astype(np.float32)
    ctx = hts.Context(Cc, H, W, A, max_learn_batch=count)
    hp = hts.HParams(algo=algo, max_grad_norm=max_norm, lr=7e-4)
    P = ctx.P
    pb_d, pt_d = dev(p_b), dev(p_t)
    opt = hts.OptState(torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda"), 0)
    args = (dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret))
    ctx.hts_learner_step_delayed(*args, pb_d, pt_d, opt, hp)
    torch.cuda.synchronize()
    p_ref, m_ref, v_ref, _, _ = oracle.learner_step_delayed(net, p_b, p_t, np.zeros(P), np.zeros(P), 1, obs, actions,
                                                            old_logp, adv, ret, oracle_hp(oracle, hp))
    got = pt_d.cpu().numpy().astype(np.float64)
    for name, pp in _split(got, shape, A).items():
        assert_close(pp, _split(p_ref, shape, A)[name], 1e-5, f"param {name}")
    assert_close(opt.m.cpu().numpy(), m_ref, 1e-4, "m")
    assert torch.equal(pb_d, dev(p_b)), "behaviour parameters must not change"
    assert opt.step == 1
    with pytest.raises(hts.HtsError):          # one vector for both roles is the ordinary step, not this call
        ctx.hts_learner_step_delayed(*args, pt_d, pt_d, opt, hp)
    ctx.close()


def test_rmsprop_parity(hts, oracle):
    """The paper's optimiser: three RMSProp steps on random gradients (with and without the norm clip), then one whole
    learner step with it."""
    rng = np.random.default_rng(9)
    ctx = hts.Context(4, 84, 84, 6, max_learn_batch=8)
    P = ctx.P
    th = rng.normal(size=P).astype(np.float32)
    th_d, m_d, v_d = dev(th), torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
    opt = hts.OptState(m_d, v_d, 0)
    th_o, v_o = th.astype(np.float64), np.zeros(P)
    for step, max_norm in enumerate((0.0, 0.5, 0.0)):
        hp = hts.HParams(optimizer=hts.OPT_RMSPROP, rms_alpha=0.99, lr=7e-4, adam_eps=1e-5, max_grad_norm=max_norm)
        g = (rng.normal(size=P) * 10.0 ** rng.uniform(-4, 0, size=P)).astype(np.float32)
        ctx.hts_adam_apply(th_d, dev(g), opt, hp)
        torch.cuda.synchronize()
        sc = oracle.clip_coef(g, max_norm) if max_norm > 0 else 1.0
        th_o, v_o = oracle.rmsprop(th_o, g, v_o, float(hp.lr), float(hp.rms_alpha), float(hp.adam_eps), gscale=sc)
        np.testing.assert_allclose(th_d.cpu().numpy(), th_o, rtol=0, atol=2e-6)
        np.testing.assert_allclose(v_d.cpu().numpy(), v_o, rtol=1e-5, atol=1e-12)
        th_o = th_d.cpu().numpy().astype(np.float64); v_o = v_d.cpu().numpy().astype(np.float64)
    assert opt.step == 3
    ctx.close()
    # whole learner step
    shape, A, count = ATARI, 6, 8
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 600, False)
    ctx = hts.Context(*shape, A, max_learn_batch=count)
    hp = hts.HParams(algo=0, optimizer=hts.OPT_RMSPROP, lr=7e-4)
    p_d = dev(params)
    opt = hts.OptState(torch.zeros(ctx.P, device="cuda"), torch.zeros(ctx.P, device="cuda"), 0)
    ctx.hts_learner_step(dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), p_d, opt, hp)
    torch.cuda.synchronize()
    g_ref, _ = oracle.loss_grads(net, params, obs, actions, old_logp, adv, ret, oracle_hp(oracle, hp))
    p_ref, _ = oracle.rmsprop(params, g_ref, np.zeros(ctx.P), float(hp.lr), float(hp.rms_alpha), float(hp.adam_eps))
    # From v = 0 the step is lr*g/(sqrt(1-alpha)|g| + eps): ten times Adam's first step, and sensitive to the
    # gradient's rounding over a ten times wider band (|g| <~ eps/sqrt(1-alpha)); hence 1e-4 where Adam's test has 1e-5.
    for name, pp in _split(p_d.cpu().numpy().astype(np.float64), shape, A).items():
        assert_close(pp, _split(p_ref, shape, A)[name], 1e-4, f"param {name}")
    with pytest.raises(hts.HtsError):
        ctx.hts_adam_apply(p_d, p_d, opt, hts.HParams(optimizer=7))
    ctx.close()


@pytest.mark.parametrize("small_batch", ["128", "0"])
@pytest.mark.parametrize("shape,A,count,B,algo,rho_bar,value_clip,prec", [
    (ATARI, 18, 24, 17, 2, 1.0, 0.0, 0),            # truncated importance weights, about half the rows truncated
    (ATARI, 18, 24, 17, 2, 1.05, 0.1, 0),           # ... with the clipped value loss as well
    (ATARI, 6, 20, None, 1, 1.0, 0.15, 0),          # PPO with the clipped value loss
    (FOOT, 19, 6, 5, 2, 1.0, 0.01, 0),
    ((3, 44, 52), 7, 70, 67, 2, 1.0, 0.1, 0),
])
def test_loss_variants_parity(hts, oracle, shape, A, count, B, algo, rho_bar, value_clip, prec, small_batch, monkeypatch):
    """Truncated importance weights (the alternative to the delayed gradient in the appendix's ablation) and the clipped
    value loss, against the oracle; then one full optimiser step with them."""
    monkeypatch.setenv("HTS_SMALL_BATCH", small_batch)
    Cc, H, W = shape
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 300 + count, True)
    _, values = oracle.forward(net, params, obs)
    old_values = (values + 0.2 * syn.normal(300 + count, syn.S_MISC + 2, count)).astype(np.float32)
    index = None if B is None else syn.permutation(7, count)[:B]
    nb = count if B is None else B
    ctx = hts.Context(Cc, H, W, A, precision=prec, max_learn_batch=nb)
    hp = hts.HParams(algo=algo, clip_eps=0.1, vf_coef=0.5, ent_coef=0.01, rho_bar=rho_bar, value_clip=value_clip,
                     max_grad_norm=0.5, lr=2.5e-4)
    ohp = oracle_hp(oracle, hp)
    ov = old_values if value_clip > 0 else None
    d_idx = None if index is None else dev(index)
    d_ov = None if ov is None else dev(ov)
    grads = torch.full((ctx.P,), float("nan"), device="cuda")
    stats = ctx.new_stats()
    d_params = dev(params)
    ctx.hts_loss_and_grads(dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), d_params, hp, grads, index=d_idx,
                           stats=stats, old_values=d_ov)
    torch.cuda.synchronize()
    g_ref, st_ref = oracle.loss_grads(net, params, obs, actions, old_logp, adv, ret, ohp, index=index, old_values=ov)
    rows = np.arange(count) if index is None else index
    if algo == 2:
        assert 0.0 < st_ref["clip_frac"] < 1.0, "the case should have truncated and untruncated rows"
    if value_clip > 0:
        d = values[rows] - old_values[rows]
        wins = (old_values[rows] + np.clip(d, -value_clip, value_clip) - ret[rows]) ** 2 > (values[rows] - ret[rows]) ** 2
        assert wins.any() and (~wins).any(), "the case should have rows on both sides of the maximum"
    g = grads.cpu().numpy()
    for name, gg in _split(g, shape, A).items():
        assert_close(gg, _split(g_ref, shape, A)[name], 1e-4, f"grad {name}")
    st = ctx.read_stats(stats)
    for k in ("policy_loss", "value_loss", "entropy", "grad_norm"):
        assert abs(st[k] - st_ref[k]) <= 1e-4 * max(1.0, abs(st_ref[k])), (k, st[k], st_ref[k])
    assert abs(st["clip_frac"] - st_ref["clip_frac"]) < 1e-6 and abs(st["approx_kl"] - st_ref["approx_kl"]) < 1e-5
    # one optimiser step
    P = ctx.P
    opt = hts.OptState(torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda"))
    ctx.hts_learner_step(dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), d_params, opt, hp, index=d_idx,
                         old_values=d_ov)
    torch.cuda.synchronize()
    th, m, v, _, _ = oracle.learner_step(net, params, np.zeros(P), np.zeros(P), 1, obs, actions, old_logp, adv, ret, ohp,
                                         index=index, old_values=ov)
    assert_close(opt.m.cpu().numpy(), m, 1e-4, "m")
    step_ref = th - params.astype(np.float64)
    step = d_params.cpu().numpy().astype(np.float64) - params.astype(np.float64)
    err = np.abs(step - step_ref)          # first Adam step: |step| ~ lr per entry, sensitive where |g| ~ adam_eps
    assert err.max() <= 2.0 * float(hp.lr) and float(np.mean(err > 1e-2 * float(hp.lr))) < 5e-3
    ctx.close()


def test_no_correction_is_plain_actor_critic_on_a_stale_storage(hts, oracle):
    """The ablation's third arm, "no correction": the plain actor-critic gradient at the current parameters on a storage
    collected with the previous ones.  The stored log-probabilities play no part in it."""
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, ATARI, 6, 20, 77, False)
    stale = params + 1e-3 * syn.normal(78, syn.S_MISC, params.size).astype(np.float32)     # "current" parameters
    ctx = hts.Context(4, 84, 84, 6, max_learn_batch=20)
    hp = hts.HParams(algo=0)
    g1, g2 = torch.zeros(ctx.P, device="cuda"), torch.zeros(ctx.P, device="cuda")
    ctx.hts_loss_and_grads(dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), dev(stale), hp, g1)
    ctx.hts_loss_and_grads(dev(obs), dev(actions), None, dev(adv), dev(ret), dev(stale), hp, g2)
    torch.cuda.synchronize()
    assert torch.equal(g1, g2)
    g_ref, _ = oracle.loss_grads(net, stale, obs, actions, None, adv, ret, oracle_hp(oracle, hp))
    for name, gg in _split(g1.cpu().numpy(), ATARI, 6).items():
        assert_close(gg, _split(g_ref, ATARI, 6)[name], 1e-4, f"grad {name}")
    ctx.close()


def test_learner_errors_launch_nothing(hts):
    ctx = hts.Context(4, 84, 84, 6, max_act_batch=4, max_learn_batch=4)
    obs = torch.zeros(8, 4, 84, 84, dtype=torch.uint8, device="cuda")
    p = torch.zeros(ctx.P, device="cuda")
    a, lp, v = torch.zeros(8, dtype=torch.int32, device="cuda"), torch.zeros(8, device="cuda"), torch.zeros(8, device="cuda")
    with pytest.raises(hts.HtsError):
        ctx.hts_act(obs, p, 1, 0, 0, a, lp, v)                 # N = 8 > max_act_batch
    with pytest.raises(hts.HtsError):
        ctx.hts_loss_and_grads(obs, a, None, lp, v, p, hts.HParams(algo=1), torch.zeros(ctx.P, device="cuda"))  # PPO needs old_logp
    with pytest.raises(hts.HtsError):
        ctx.hts_loss_and_grads(obs, a, None, lp, v, p, hts.HParams(algo=2), torch.zeros(ctx.P, device="cuda"), B=4)   # needs old_logp
    with pytest.raises(hts.HtsError):
        ctx.hts_loss_and_grads(obs, a, lp, lp, v, p, hts.HParams(algo=2, rho_bar=0.0), torch.zeros(ctx.P, device="cuda"), B=4)
    with pytest.raises(hts.HtsError):
        ctx.hts_loss_and_grads(obs, a, lp, lp, v, p, hts.HParams(algo=0, value_clip=0.1), torch.zeros(ctx.P, device="cuda"), B=4)  # needs old_values
    with pytest.raises(hts.HtsError):
        ctx.hts_loss_and_grads(obs, a, lp, lp, v, p, hts.HParams(algo=3), torch.zeros(ctx.P, device="cuda"), B=4)
    with pytest.raises(hts.HtsError):
        ctx.hts_loss_and_grads(obs, a, lp, lp, v, p, hts.HParams(algo=0), torch.zeros(ctx.P, device="cuda"))    # B = 8 > max
    torch.cuda.synchronize()
    ctx.close()


@pytest.mark.parametrize("prec", [0, 1])
def test_tracked_parameters_give_the_same_bits(hts, oracle, prec):
    """hts_track_params: the optimiser kernel rewrites the context's copy of the network and later calls skip the load.
    Rollout, three updates, rollout -- with and without -- must agree bit for bit; a write by the caller is announced
    with hts_sync_params."""
    shape, A, count, B = (3, 44, 52), 7, 40, 24
    Cc, H, W = shape
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 91, True)
    hp = hts.HParams(algo=1, clip_eps=0.1, max_grad_norm=0.5, lr=1e-3)
    outs = []
    for track in (False, True):
        ctx = hts.Context(Cc, H, W, A, precision=prec, max_act_batch=count, max_learn_batch=B)
        ctx.hts_track_params(track)
        p_d = dev(params)
        P = ctx.P
        opt = hts.OptState(torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda"), 0)
        data = (dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret))
        res = [_act(ctx, data[0], p_d, 5, 1, 0, A)]
        for k in range(3):
            ctx.hts_learner_step(*data, p_d, opt, hp, index=dev(syn.permutation(60 + k, count)[:B]))
        res.append(_act(ctx, data[0], p_d, 5, 2, 0, A))
        if track:       # the loaded copy followed the updates: params = NULL acts on the updated network
            z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device="cuda")
            a2, lp2, v2, lg2 = z(count, dt=torch.int32), z(count), z(count), z(count, A)
            ctx.hts_act(data[0], None, 5, 2, 0, a2, lp2, v2, lg2)
            torch.cuda.synchronize()
            assert np.array_equal(lg2.cpu().numpy(), res[-1][3]) and np.array_equal(a2.cpu().numpy(), res[-1][0])
        # a write by the caller, announced
        p_d.mul_(0.5)
        ctx.hts_sync_params(p_d)
        ctx.hts_learner_step(*data, p_d, opt, hp, index=dev(syn.permutation(70, count)[:B]))
        res.append(_act(ctx, data[0], p_d, 5, 3, 0, A))
        torch.cuda.synchronize()
        outs.append((res, p_d.cpu().numpy(), opt.m.cpu().numpy(), opt.v.cpu().numpy()))
        ctx.close()
    (r0, p0, m0, v0), (r1, p1, m1, v1) = outs
    assert np.array_equal(p0, p1) and np.array_equal(m0, m1) and np.array_equal(v0, v1)
    for x, y in zip(r0, r1):
        assert all(np.array_equal(u, w) for u, w in zip(x, y))
    assert not np.array_equal(r0[0][3], r0[1][3])            # the updates did change the network


def test_nonfinite_flag_on_injected_infinity(hts, oracle):
    """hts_stats.nonfinite is 0 on a healthy minibatch and 1 when a loss term is not finite (an infinite advantage)."""
    shape, A, count = (2, 36, 36), 5, 12
    Cc, H, W = shape
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 77, True)
    ctx = hts.Context(Cc, H, W, A, max_learn_batch=count)
    hp = hts.HParams(algo=1, clip_eps=0.1)
    grads, stats = torch.zeros(ctx.P, device="cuda"), ctx.new_stats()
    for bad in (False, True):
        a = adv.copy()
        if bad:
            a[5] = np.inf
        ctx.hts_loss_and_grads(dev(obs), dev(actions), dev(old_logp), dev(a), dev(ret), dev(params), hp, grads, stats=stats)
        torch.cuda.synchronize()
        st = ctx.read_stats(stats)
        assert st["nonfinite"] == (1 if bad else 0), st
    # the same through hts_learner_step (the flag is raised; what the caller does with the update is its business)
    P = ctx.P
    opt = hts.OptState(torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda"), 0)
    r = ret.copy(); r[3] = np.nan
    ctx.hts_learner_step(dev(obs), dev(actions), dev(old_logp), dev(adv), dev(r), dev(params), opt, hp, stats=stats)
    torch.cuda.synchronize()
    assert ctx.read_stats(stats)["nonfinite"] == 1
    ctx.close()


# ------------------------------------------------------------------------------------------------------------
# bf16 operands (fp32 accumulate, fp32 heads/loss/optimiser); the oracle is the unrounded computation
# ------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("small_batch", ["128", "0"])
@pytest.mark.parametrize("shape,A,count,B,algo", [(ATARI, 18, 48, 40, 1), (FOOT, 19, 10, 8, 1), ((3, 44, 52), 7, 70, 67, 0)])
def test_bf16_loss_and_grads(hts, oracle, shape, A, count, B, algo, small_batch, monkeypatch):
    monkeypatch.setenv("HTS_SMALL_BATCH", small_batch)
    Cc, H, W = shape
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 300 + count, algo == 1)
    index = syn.permutation(8, count)[:B]
    ctx = hts.Context(Cc, H, W, A, precision=1, max_learn_batch=B)
    hp = hts.HParams(algo=algo, clip_eps=0.1)
    grads = torch.full((ctx.P,), float("nan"), device="cuda")
    stats = ctx.new_stats()
    ctx.hts_loss_and_grads(dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), dev(params), hp, grads,
                           index=dev(index), stats=stats)
    torch.cuda.synchronize()
    ohp = oracle_hp(oracle, hp)
    g_ref, st_ref = oracle.loss_grads(net, params, obs, actions, old_logp, adv, ret, ohp, index=index)
    qnet = oracle.make_net(Cc, H, W, A, operand_bf16=True)
    g_q, st_q = oracle.loss_grads(qnet, params, obs, actions, old_logp, adv, ret, ohp, index=index)
    st = ctx.read_stats(stats)
    g = grads.cpu().numpy()
    # (1) against the unrounded oracle: losses within 2e-2
    for k in ("policy_loss", "value_loss", "entropy"):
        assert abs(st[k] - st_ref[k]) <= 2e-2 * max(1.0, abs(st_ref[k])), (k, st[k], st_ref[k])
    # (2) against the oracle's operand-rounding model (same bf16 operands, exact sums): losses and every gradient
    # tensor within 2e-2.  This is the sharp check: both sides open the same ReLU gates.
    for k in ("policy_loss", "value_loss", "entropy", "grad_norm"):
        assert abs(st[k] - st_q[k]) <= 2e-2 * max(1.0, abs(st_q[k])), (k, st[k], st_q[k])
    errs_q = {name: rel_err(gg, _split(g_q, shape, A)[name]) for name, gg in _split(g, shape, A).items()}
    print("bf16 gradient errors vs operand-rounding oracle:", {k: f"{v:.1e}" for k, v in errs_q.items()})
    for name, e in errs_q.items():
        assert e <= 2e-2, (name, e)
    # (3) against the unrounded oracle the gradient differs by the ReLU gates that bf16 rounding of the forward
    # pass flips (pre-activations within ~2^-8 relative of zero): a discontinuous change no bf16 forward avoids.
    # Held to a direction bound, and reported.
    errs = {name: rel_err(gg, _split(g_ref, shape, A)[name]) for name, gg in _split(g, shape, A).items()}
    cos = float(np.dot(g, g_ref) / (np.linalg.norm(g) * np.linalg.norm(g_ref)))
    print("bf16 gradient errors vs unrounded oracle:", {k: f"{v:.1e}" for k, v in errs.items()}, f"cosine {cos:.5f}")
    assert cos >= 0.98
    ctx.close()


@pytest.mark.parametrize("shape,A,count,B", [(ATARI, 18, 140, 131), (FOOT, 19, 140, 133)])
def test_bf16_ragged_large_batch_agrees_with_small_batch_kernels(hts, oracle, shape, A, count, B, monkeypatch):
    """A minibatch just above the boundary between the kernel families, of a size that leaves the last group of
    every LDS-resident kernel part full and every tile kernel a ragged tail: the large-batch kernels (tile kernels,
    image kernels, split reductions) against the wave-per-segment kernels on the same bf16 problem.  The two differ in
    the order of the backward reductions only (forward bits are identical), so the gradients agree far inside the bf16
    tolerance; the wave-per-segment kernels are the ones held against the oracle above."""
    Cc, H, W = shape
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, count, 900 + count, True)
    index = syn.permutation(8, count)[:B]
    out = {}
    for knob, fold in (("128", "1000000"), ("1000", "1000000"), ("128", "1")):
        monkeypatch.setenv("HTS_SMALL_BATCH", knob)
        monkeypatch.setenv("HTS_FC_FOLD_ROWS", fold)     # "1": the FC kernel adds its K groups itself, as for large batches
        ctx = hts.Context(Cc, H, W, A, precision=1, max_learn_batch=B)
        hp = hts.HParams(algo=1, clip_eps=0.1)
        grads = torch.full((ctx.P,), float("nan"), device="cuda")
        stats = ctx.new_stats()
        ctx.hts_loss_and_grads(dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), dev(params), hp, grads,
                               index=dev(index), stats=stats)
        torch.cuda.synchronize()
        out[knob, fold] = (grads.cpu().numpy(), ctx.read_stats(stats))
        ctx.close()
    (g_large, st_large), (g_small, st_small) = out["128", "1000000"], out["1000", "1000000"]
    assert np.all(np.isfinite(g_large))
    assert np.array_equal(out["128", "1"][0], g_large) and out["128", "1"][1] == st_large     # same bits either way
    for k in ("policy_loss", "value_loss", "entropy"):
        assert st_large[k] == st_small[k], (k, st_large[k], st_small[k])          # forward bits are identical
    for name, gl in _split(g_large, shape, A).items():
        e = rel_err(gl, _split(g_small, shape, A)[name])
        assert e <= 1e-3, (name, e)
