"""Full-size GPU checks: the shapes, batch sizes and call sequences that bench.py times.

Where the CPU oracle finishes in seconds the comparison is complete (the Atari A2C iteration); at the PPO and
sweep sizes the oracle computes sampled outputs (whole calls at sampled steps, one whole minibatch, sampled rows of a
large batch), and properties that hold at any size cover the rest: actions are a bit-exact function of the
logits and counters, an observation's outputs do not depend on the batch it was served in, and a mean loss's
gradient over a minibatch is the mean of its chunks' gradients.
"""
import numpy as np
import pytest
import torch

import hts_synth as syn
from test_gpu_parity import ATARI, FOOT, _split, assert_close, dev, hts, oracle_hp, rel_err  # noqa: F401

pytestmark = pytest.mark.gpu

SEED = 20201209


def _storage(ctx, T, N, A):
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device="cuda")
    return dict(actions=z(T + 1, N, dt=torch.int32), logp=z(T + 1, N), values=z(T + 1, N), logits=z(T + 1, N, A))


def _rollout_gpu(ctx, obs_d, params_d, st, T, base_step=0):
    """T+1 hts_act calls as bench.py issues them: parameters loaded by the first call, reused by the others."""
    for t in range(T + 1):
        ctx.hts_act(obs_d[t], params_d if t == 0 else None, SEED, base_step + t, 0, st["actions"][t], st["logp"][t],
                    st["values"][t], st["logits"][t])
    torch.cuda.synchronize()


def test_atari_a2c_fp32_whole_iteration(hts, oracle):
    """N=16, T=5, 18 actions, fp32: every output of one iteration against the oracle."""
    N, T, A = 16, 5, 18
    Cc, H, W = ATARI
    ctx = hts.Context(Cc, H, W, A, precision=0, max_act_batch=N, max_learn_batch=N * T)
    net = oracle.make_net(Cc, H, W, A)
    params = syn.init_params(31, Cc, H, W, A, bias_scale=0.05)
    obs = syn.obs_atari(32, T + 1, N)
    rew = syn.rewards_ternary(33, T, N)
    dones = syn.dones_bernoulli(34, T, N, 0.05)
    obs_d, params_d = dev(obs), dev(params)
    st = _storage(ctx, T, N, A)
    _rollout_gpu(ctx, obs_d, params_d, st, T)
    logits, values = st["logits"].cpu().numpy(), st["values"].cpu().numpy()
    for t in range(T + 1):
        l_ref, v_ref = oracle.forward(net, params, obs[t])
        assert_close(logits[t], l_ref, 1e-4, f"logits step {t}")
        assert_close(values[t], v_ref, 1e-4, f"values step {t}")
        a_ref, lp_ref, _ = oracle.sample(logits[t], SEED, t, 0)
        assert np.array_equal(st["actions"][t].cpu().numpy(), a_ref)
        np.testing.assert_allclose(st["logp"][t].cpu().numpy(), lp_ref, atol=1e-6, rtol=0)
    # returns (lambda = 1: the n-step return of Sec. 3) from the GPU's own values
    adv_d, ret_d = torch.zeros(T, N, device="cuda"), torch.zeros(T, N, device="cuda")
    ctx.hts_returns_gae(dev(rew), st["values"], dev(dones), 0.99, 1.0, adv_d, ret_d)
    torch.cuda.synchronize()
    adv_ref, ret_ref = oracle.gae(rew, values, dones, 0.99, 1.0)
    np.testing.assert_allclose(adv_d.cpu().numpy(), adv_ref, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(ret_d.cpu().numpy(), ret_ref, rtol=1e-6, atol=1e-6)
    # one A2C update on the 80 rows
    hp = hts.HParams(algo=0, lr=7e-4)
    P = ctx.P
    opt = hts.OptState(torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda"), 0)
    rows = N * T
    flat_obs = obs_d[:T].reshape(rows, Cc, H, W)
    acts, lps = st["actions"][:T].reshape(rows).contiguous(), st["logp"][:T].reshape(rows).contiguous()
    ctx.hts_learner_step(flat_obs, acts, lps, adv_d.reshape(rows), ret_d.reshape(rows), params_d, opt, hp)
    torch.cuda.synchronize()
    p_ref, _, _, g_ref, _ = oracle.learner_step(
        net, params.astype(np.float64), np.zeros(P), np.zeros(P), 1, obs[:T].reshape(rows, Cc, H, W),
        acts.cpu().numpy(), lps.cpu().numpy(), adv_d.reshape(rows).cpu().numpy(), ret_d.reshape(rows).cpu().numpy(),
        oracle_hp(oracle, hp))
    got = params_d.cpu().numpy().astype(np.float64)
    for name, pp in _split(got, ATARI, A).items():
        assert_close(pp, _split(p_ref, ATARI, A)[name], 1e-5, f"param {name}")
    ctx.close()


def _chunk_mean_grads(ctx, hts_mod, args, index_d, B, chunk, hp):
    """Mean over equal chunks of the chunk gradients (each chunk is its own library call)."""
    acc = torch.zeros(ctx.P, dtype=torch.float64, device="cuda")
    g = torch.zeros(ctx.P, device="cuda")
    for c0 in range(0, B, chunk):
        ctx.hts_loss_and_grads(*args, hp, g, index=index_d[c0:c0 + chunk].contiguous())
        acc += g.double()
    torch.cuda.synchronize()
    return (acc / (B // chunk)).cpu().numpy()


def test_atari_ppo_bf16_full_size(hts, oracle):
    """N=32, T=128, minibatch 1024 of 4096 rows, bf16 operands."""
    N, T, A, B = 32, 128, 18, 1024
    Cc, H, W = ATARI
    ctx = hts.Context(Cc, H, W, A, precision=1, max_act_batch=N, max_learn_batch=B)
    net, qnet = oracle.make_net(Cc, H, W, A), oracle.make_net(Cc, H, W, A, operand_bf16=True)
    params = syn.init_params(41, Cc, H, W, A, bias_scale=0.05)
    obs = syn.obs_atari(42, T + 1, N)
    rew = syn.rewards_score_clipped(43, T, N)
    dones = syn.dones_bernoulli(44, T, N, 0.01)
    obs_d, params_d = dev(obs), dev(params)
    st = _storage(ctx, T, N, A)
    _rollout_gpu(ctx, obs_d, params_d, st, T)
    logits, values = st["logits"].cpu().numpy(), st["values"].cpu().numpy()
    actions, logp = st["actions"].cpu().numpy(), st["logp"].cpu().numpy()
    for t in (0, 63, T):                       # whole calls at sampled steps against the unrounded oracle
        l_ref, v_ref = oracle.forward(net, params, obs[t])
        assert_close(logits[t], l_ref, 2e-2, f"logits step {t}")
        assert_close(values[t], v_ref, 2e-2, f"values step {t}")
    for t in range(T + 1):                     # every action: bit-exact given the logits and the counters
        a_ref, lp_ref, _ = oracle.sample(logits[t], SEED, t, 0)
        assert np.array_equal(actions[t], a_ref), t
        np.testing.assert_allclose(logp[t], lp_ref, atol=1e-6, rtol=0)
    adv_d, ret_d = torch.zeros(T, N, device="cuda"), torch.zeros(T, N, device="cuda")
    ctx.hts_returns_gae(dev(rew), st["values"], dev(dones), 0.99, 0.95, adv_d, ret_d)
    ctx.hts_normalize_advantages(adv_d)
    torch.cuda.synchronize()
    adv_ref, ret_ref = oracle.gae(rew, values, dones, 0.99, 0.95)
    np.testing.assert_allclose(ret_d.cpu().numpy(), ret_ref, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(adv_d.cpu().numpy(), oracle.normalize_adv(adv_ref), rtol=1e-5, atol=1e-5)
    # one minibatch of 1024 gathered rows: losses against the unrounded oracle, gradients against the oracle's
    # operand-rounding model (the same bf16 operands, exact sums)
    rows = N * T
    index = syn.permutation(45, rows)[:B]
    hp = hts.HParams(algo=1, clip_eps=0.1, max_grad_norm=0.5, lr=2.5e-4)
    flat = (obs_d[:T].reshape(rows, Cc, H, W), st["actions"][:T].reshape(rows).contiguous(),
            (st["logp"][:T].reshape(rows) + 0.05 * torch.sin(torch.arange(rows, device="cuda"))).contiguous(),
            adv_d.reshape(rows), ret_d.reshape(rows), params_d)
    grads, stats = torch.zeros(ctx.P, device="cuda"), ctx.new_stats()
    ctx.hts_loss_and_grads(*flat, hp, grads, index=dev(index), stats=stats)
    torch.cuda.synchronize()
    host = [x.cpu().numpy() for x in flat[1:5]]
    ohp = oracle_hp(oracle, hp)
    flat_obs = obs[:T].reshape(rows, Cc, H, W)
    _, st_ref = oracle.loss_grads(net, params, flat_obs, *host, ohp, index=index)
    g_q, st_q = oracle.loss_grads(qnet, params, flat_obs, *host, ohp, index=index)
    s = ctx.read_stats(stats)
    for k in ("policy_loss", "value_loss", "entropy"):
        assert abs(s[k] - st_ref[k]) <= 2e-2 * max(1.0, abs(st_ref[k])), (k, s[k], st_ref[k])
    g = grads.cpu().numpy()
    for name, gg in _split(g, ATARI, A).items():
        assert rel_err(gg, _split(g_q, ATARI, A)[name]) <= 2e-2, name
    assert abs(s["grad_norm"] - st_q["grad_norm"]) <= 2e-2 * st_q["grad_norm"]
    # the same minibatch as 8 chunks of 128 rows (wave-per-segment kernels): the PPO loss is a mean over rows
    g_chunks = _chunk_mean_grads(ctx, hts, flat, dev(index), B, 128, hp)
    for name, gg in _split(g, ATARI, A).items():
        assert rel_err(gg, _split(g_chunks, ATARI, A)[name]) <= 5e-3, name
    ctx.close()


def test_football_ppo_bf16_full_size(hts, oracle):
    """16x72x96 observations, 19 actions, minibatch 2048, bf16: one 128-row chunk against the oracle, the full
    minibatch through the chunk-mean property; actor calls at N=16 against the oracle."""
    N, A, B, count = 16, 19, 2048, 2304
    Cc, H, W = FOOT
    ctx = hts.Context(Cc, H, W, A, precision=1, max_act_batch=N, max_learn_batch=B)
    net, qnet = oracle.make_net(Cc, H, W, A), oracle.make_net(Cc, H, W, A, operand_bf16=True)
    params = syn.init_params(51, Cc, H, W, A, bias_scale=0.05)
    obs = syn.obs_football(52, 1, count)[0]
    obs_d, params_d = dev(obs), dev(params)
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device="cuda")
    actions, logp, values, logits = z(count, dt=torch.int32), z(count), z(count), z(count, A)
    for i, c0 in enumerate(range(0, count, N)):            # the actor's launch shape: 16 observations per call
        ctx.hts_act(obs_d[c0:c0 + N], params_d if i == 0 else None, SEED, i, 0, actions[c0:c0 + N], logp[c0:c0 + N],
                    values[c0:c0 + N], logits[c0:c0 + N])
    torch.cuda.synchronize()
    lg = logits.cpu().numpy()
    for c0 in (0, 1152, count - N):
        l_ref, v_ref = oracle.forward(net, params, obs[c0:c0 + N])
        assert_close(lg[c0:c0 + N], l_ref, 2e-2, f"logits rows {c0}")
        assert_close(values[c0:c0 + N].cpu().numpy(), v_ref, 2e-2, f"values rows {c0}")
    for i, c0 in enumerate(range(0, count, N)):
        a_ref, _, _ = oracle.sample(lg[c0:c0 + N], SEED, i, 0)
        assert np.array_equal(actions[c0:c0 + N].cpu().numpy(), a_ref)
    adv = dev(syn.normal(53, syn.S_MISC, count).astype(np.float32))
    ret = (values + adv).contiguous()
    old_logp = (logp + 0.05 * torch.cos(torch.arange(count, device="cuda"))).contiguous()
    hp = hts.HParams(algo=1, clip_eps=0.08, ent_coef=0.003, lr=3.4e-4)
    index = syn.permutation(54, count)[:B]
    flat = (obs_d, actions, old_logp, adv, ret, params_d)
    grads = torch.zeros(ctx.P, device="cuda")
    ctx.hts_loss_and_grads(*flat, hp, grads, index=dev(index))
    torch.cuda.synchronize()
    g = grads.cpu().numpy()
    g_chunks = _chunk_mean_grads(ctx, hts, flat, dev(index), B, 128, hp)
    for name, gg in _split(g, FOOT, A).items():
        assert rel_err(gg, _split(g_chunks, FOOT, A)[name]) <= 5e-3, name
    # first chunk against the oracle's operand-rounding model
    g1 = torch.zeros(ctx.P, device="cuda")
    ctx.hts_loss_and_grads(*flat, hp, g1, index=dev(index[:128]))
    torch.cuda.synchronize()
    host = [x.cpu().numpy() for x in flat[1:5]]
    g_q, _ = oracle.loss_grads(qnet, params, obs, *host, oracle_hp(oracle, hp), index=index[:128])
    for name, gg in _split(g1.cpu().numpy(), FOOT, A).items():
        assert rel_err(gg, _split(g_q, FOOT, A)[name]) <= 2e-2, name
    ctx.close()


@pytest.mark.parametrize("N", [256, 1024, 4096])
def test_large_batch_act_bf16(hts, oracle, N):
    """Inference sweep: sampled rows against the oracle; the same rows served in a batch of 32 give the same bits;
    all actions follow from the logits."""
    A = 18
    Cc, H, W = ATARI
    ctx = hts.Context(Cc, H, W, A, precision=1, max_act_batch=N)
    net = oracle.make_net(Cc, H, W, A)
    params = syn.init_params(61, Cc, H, W, A, bias_scale=0.05)
    obs = syn.obs_atari(62, 1, N)[0]
    obs_d, params_d = dev(obs), dev(params)
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device="cuda")
    actions, logp, values, logits = z(N, dt=torch.int32), z(N), z(N), z(N, A)
    ctx.hts_act(obs_d, params_d, SEED, 9, 0, actions, logp, values, logits)
    torch.cuda.synchronize()
    lg = logits.cpu().numpy()
    a_ref, lp_ref, _ = oracle.sample(lg, SEED, 9, 0)
    assert np.array_equal(actions.cpu().numpy(), a_ref)
    np.testing.assert_allclose(logp.cpu().numpy(), lp_ref, atol=1e-6, rtol=0)
    rows = np.unique(np.concatenate([[0, 1, N - 1], syn.permutation(63, N)[:13]]))
    l_ref, v_ref = oracle.forward(net, params, obs[rows])
    assert_close(lg[rows], l_ref, 2e-2, "sampled logits")
    assert_close(values.cpu().numpy()[rows], v_ref, 2e-2, "sampled values")
    for c0 in (0, N // 2 + 32, N - 32):         # batch-partition invariance across the two kernel families
        a2, lp2, v2, lg2 = z(32, dt=torch.int32), z(32), z(32), z(32, A)
        ctx.hts_act(obs_d[c0:c0 + 32], None, SEED, 9, c0, a2, lp2, v2, lg2)
        torch.cuda.synchronize()
        assert torch.equal(lg2, logits[c0:c0 + 32]) and torch.equal(a2, actions[c0:c0 + 32])
        assert torch.equal(v2, values[c0:c0 + 32]) and torch.equal(lp2, logp[c0:c0 + 32])
    ctx.close()


def test_gae_sweep_size(hts, oracle):
    T, N = 128, 4096
    r, v = syn.normal_f32(71, syn.S_REW, (T, N)), syn.normal_f32(72, syn.S_VAL, (T + 1, N))
    d = syn.dones_bernoulli(73, T, N, 0.01)
    ctx = hts.Context(4, 84, 84, 18, max_act_batch=1)
    adv, ret = torch.zeros(T, N, device="cuda"), torch.zeros(T, N, device="cuda")
    ctx.hts_returns_gae(dev(r), dev(v), dev(d), 0.99, 0.95, adv, ret)
    torch.cuda.synchronize()
    a_ref, r_ref = oracle.gae(r, v, d, 0.99, 0.95)
    np.testing.assert_allclose(adv.cpu().numpy(), a_ref, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(ret.cpu().numpy(), r_ref, rtol=1e-6, atol=1e-6)
    ctx.close()


MAX_BATCH = 65536          # the largest batch a context accepts


@pytest.mark.parametrize("shape,A,prec", [(ATARI, 18, 1), (FOOT, 19, 1), (ATARI, 18, 0)])
def test_maximum_batch_act(hts, oracle, shape, A, prec):
    """hts_act at the largest batch a context accepts (offsets beyond 2^31 bytes in every activation).  The batch is
    64 distinct frames repeated 1024 times: batch-partition invariance makes every copy's logits and value equal,
    bit for bit, to those of the 64 frames served alone, which the oracle checks; actions and log-probabilities of all
    65536 rows (every row has its own Philox counter) follow from the logits."""
    Cc, H, W = shape
    N, R = MAX_BATCH, 64
    net = oracle.make_net(Cc, H, W, A)
    params = syn.init_params(81, Cc, H, W, A, bias_scale=0.05)
    frames = syn.obs_atari(82, 1, R)[0] if shape == ATARI else syn.obs_football(82, 1, R)[0]
    ctx = hts.Context(Cc, H, W, A, precision=prec, max_act_batch=N)
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device="cuda")
    params_d, frames_d = dev(params), dev(frames)
    a64, lp64, v64, lg64 = z(R, dt=torch.int32), z(R), z(R), z(R, A)
    ctx.hts_act(frames_d, params_d, SEED, 3, 0, a64, lp64, v64, lg64)
    obs_d = frames_d.repeat(N // R, 1, 1, 1)                  # row k*64 + i is frame i
    actions, logp, values, logits = z(N, dt=torch.int32), z(N), z(N), z(N, A)
    ctx.hts_act(obs_d, None, SEED, 3, 0, actions, logp, values, logits)
    torch.cuda.synchronize()
    assert torch.equal(logits.view(N // R, R, A), lg64.expand(N // R, R, A))
    assert torch.equal(values.view(N // R, R), v64.expand(N // R, R))
    l_ref, v_ref = oracle.forward(net, params, frames)
    tol = 2e-2 if prec == 1 else 1e-4
    assert_close(lg64.cpu().numpy(), l_ref, tol, "logits")
    assert_close(v64.cpu().numpy(), v_ref, tol, "values")
    a_ref, lp_ref, _ = oracle.sample(logits.cpu().numpy(), SEED, 3, 0)
    assert np.array_equal(actions.cpu().numpy(), a_ref)
    np.testing.assert_allclose(logp.cpu().numpy(), lp_ref, atol=1e-6, rtol=0)
    ctx.close()


@pytest.mark.parametrize("shape,A,prec,algo", [(ATARI, 18, 0, 0), (ATARI, 18, 1, 1), (FOOT, 19, 1, 1)])
def test_maximum_minibatch_gradient(hts, oracle, shape, A, prec, algo):
    """Forward, loss and backward on the largest minibatch a context accepts: 65536 rows gathered (through `index`)
    from a 64-row storage, every row 1024 times.  The mean loss over the repeated rows is the mean over the 64, so the
    oracle's gradient on the 64 rows is the expected value."""
    Cc, H, W = shape
    B, R = MAX_BATCH, 64
    from test_gpu_parity import _rollout
    net, params, obs, actions, old_logp, adv, ret = _rollout(oracle, shape, A, R, 500, algo == 1)
    index = np.tile(np.arange(R, dtype=np.int32), B // R)
    ctx = hts.Context(Cc, H, W, A, precision=prec, max_learn_batch=B)
    hp = hts.HParams(algo=algo, clip_eps=0.1, vf_coef=0.5, ent_coef=0.01)
    grads = torch.full((ctx.P,), float("nan"), device="cuda")
    stats = ctx.new_stats()
    args = (dev(obs), dev(actions), dev(old_logp), dev(adv), dev(ret), dev(params), hp)
    ctx.hts_loss_and_grads(*args, grads, index=dev(index), stats=stats)
    torch.cuda.synchronize()
    if prec == 1:       # the oracle's operand-rounding model (same bf16 operands, exact sums): both sides open the same ReLU gates
        net = oracle.make_net(Cc, H, W, A, operand_bf16=True)
    g_ref, st_ref = oracle.loss_grads(net, params, obs, actions, old_logp, adv, ret, oracle_hp(oracle, hp))
    g = grads.cpu().numpy()
    assert np.all(np.isfinite(g))
    # binary32 tolerance at this size: the FC and heads weight gradients are single accumulation chains over the 65536
    # rows; with unit roundoff u = 6e-8 a chain of n additions errs by sqrt(n) u = 1.5e-5 for independent addends and by
    # up to n u = 3.9e-3 in the worst case, and repeated rows (equal addends, partial sums growing linearly) lie in
    # between (1.4e-4 observed on fc.w).  5e-4 is allowed here; the 1e-4 of the other tests stands for n <= 4096.
    tol = 2e-2 if prec == 1 else 5e-4
    for name, gg in _split(g, shape, A).items():
        assert_close(gg, _split(g_ref, shape, A)[name], tol, f"grad {name}")
    st = ctx.read_stats(stats)
    for k in ("policy_loss", "value_loss", "entropy"):
        assert abs(st[k] - st_ref[k]) <= tol * max(1.0, abs(st_ref[k])), (k, st[k], st_ref[k])
    g2 = torch.zeros_like(grads)                                # run-to-run bit identity at this size
    ctx.hts_loss_and_grads(*args, g2, index=dev(index))
    torch.cuda.synchronize()
    assert torch.equal(grads, g2)
    ctx.close()
