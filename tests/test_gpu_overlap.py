"""The concurrent schedule of bench.py (rollout on one stream, one-step-delayed learner update on another) must give
the same bits as the same calls issued one after the other on a single stream: concurrency changes when things run,
never what they compute (the paper's determinism claim, Sec. 4.1)."""

import pytest
import torch

import hts_synth as syn

pytestmark = pytest.mark.gpu


def test_overlapped_schedule_equals_serial_schedule():
    import bench
    import paper_2012_09849_amd as hts
    cfg = dict(bench.CONFIGS["atari_a2c_n16_t5_fp32"])
    base = bench.Loop(cfg, hts, torch, syn)
    ov = bench.OverlapLoop(base)
    iters = 5
    for _ in range(iters):
        ov.step()
    torch.cuda.synchronize()
    got = [t.clone() for t in ov.theta]
    got_actions = [s["actions"].clone() for s in ov.store]

    # serial replay of the same schedule: one context, one stream
    N, T = cfg["N"], cfg["T"]
    ctx = hts.Context(cfg["C"], cfg["H"], cfg["W"], cfg["A"], precision=cfg["precision"], max_act_batch=N,
                      max_learn_batch=N * T)
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device="cuda")
    store = [dict(actions=z(T + 1, N, dt=torch.int32), logp=z(T + 1, N), values=z(T + 1, N), adv=z(T, N), ret=z(T, N))
             for _ in range(2)]
    theta = [base.params.clone() for _ in range(3)]
    P = base.params.numel()
    opt = hts.OptState(z(P), z(P), 0)
    obs_flat = base.obs[:T].reshape(T * N, cfg["C"], cfg["H"], cfg["W"])
    for j in range(iters):
        prev, cur, nxt = theta
        st = store[j % 2]
        for t in range(T + 1):
            ctx.hts_act(base.obs[t], cur, 20201209, j * (T + 1) + t, 0, st["actions"][t], st["logp"][t], st["values"][t])
        ctx.hts_returns_gae(base.rew, st["values"], base.dones, cfg["gamma"], cfg["lam"], st["adv"], st["ret"])
        nxt.copy_(cur)
        if j > 0:
            old = store[(j - 1) % 2]
            ctx.hts_learner_step_delayed(obs_flat, old["actions"][:T].reshape(-1), old["logp"][:T].reshape(-1),
                                         old["adv"].reshape(-1), old["ret"].reshape(-1), prev, nxt, opt, base.hp)
        theta = [cur, nxt, prev]
    torch.cuda.synchronize()
    for a, b in zip(got, theta):
        assert torch.equal(a, b)
    for a, b in zip(got_actions, store):
        assert torch.equal(a, b["actions"])
    assert opt.step == iters - 1 and ov.opt.step == iters - 1
    # and the parameters did move
    assert not torch.equal(theta[1], base.params)
    ctx.close()
