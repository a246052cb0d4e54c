"""The concurrent schedule of the package (schedule.OverlapLoop: rollout on one stream, one-step-delayed learner update on another) must give
the same bits as the same calls issued one after the other on a single stream: concurrency changes when things run,
never what they compute (the paper's determinism claim, Sec. 4.1)."""

import pytest
import torch

import hts_synth as syn

pytestmark = pytest.mark.gpu


def test_overlapped_schedule_equals_serial_schedule():
    import paper_2012_09849_amd as hts
    from paper_2012_09849_amd import schedule
    cfg = dict(schedule.CONFIGS["atari_a2c_n16_t5_fp32"])
    base = schedule.Loop(cfg, hts, torch, syn)
    ov = schedule.OverlapLoop(base)
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


def test_overlapped_ppo_schedule_equals_serial_schedule():
    """Several minibatch steps per storage: the learner's epochs on storage j-1 run beside the rollout of storage j;
    the serial replay of the same calls gives the same parameters and actions."""
    import paper_2012_09849_amd as hts
    from paper_2012_09849_amd import schedule
    cfg = dict(schedule.CONFIGS["atari_ppo_n32_t128_bf16"], N=8, T=12, epochs=2, minibatches=2)
    base = schedule.Loop(cfg, hts, torch, syn)
    ov = schedule.OverlapLoop(base)
    iters = 4
    for _ in range(iters):
        ov.step()
    torch.cuda.synchronize()
    N, T, B = cfg["N"], cfg["T"], base.B
    ctx = hts.Context(cfg["C"], cfg["H"], cfg["W"], cfg["A"], precision=cfg["precision"], max_act_batch=N,
                      max_learn_batch=B)
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
        ctx.hts_normalize_advantages(st["adv"])
        nxt.copy_(cur)
        if j > 0:
            old = store[(j - 1) % 2]
            for e in range(cfg["epochs"]):
                for k in range(cfg["minibatches"]):
                    ctx.hts_learner_step(obs_flat, old["actions"][:T].reshape(-1), old["logp"][:T].reshape(-1),
                                         old["adv"].reshape(-1), old["ret"].reshape(-1), nxt, opt, base.hp,
                                         index=base.perms[e][k * B:(k + 1) * B], B=B)
        theta = [cur, nxt, prev]
    torch.cuda.synchronize()
    for a, b in zip(ov.theta, theta):
        assert torch.equal(a, b)
    for a, b in zip(ov.store, store):
        assert torch.equal(a["actions"], b["actions"])
    assert opt.step == (iters - 1) * 4 and ov.opt.step == opt.step
    assert not torch.equal(theta[1], base.params)
    ctx.close()


def test_compute_unit_ranges_do_not_change_results():
    """The concurrent schedule with the actors' and the learner's streams confined to disjoint ranges of compute units
    (hts_stream_create_cu_range) gives the same bits as with ordinary streams: where a kernel runs never enters what it
    computes.  Football-shaped frames, a few steps of a short unroll."""
    import paper_2012_09849_amd as hts
    from paper_2012_09849_amd import schedule
    cfg = dict(schedule.CONFIGS["football_ppo_n16_t512_bf16"], N=16, T=6, epochs=1, minibatches=2)
    outs = []
    for cus in (None, 192, 64):
        base = schedule.Loop(cfg, hts, torch, syn)
        ov = schedule.OverlapLoop(base, actor_cus=cus)
        for _ in range(3):
            ov.step()
        torch.cuda.synchronize()
        outs.append(([t.clone() for t in ov.theta], [s["actions"].clone() for s in ov.store]))
        ov.close()
        base.ctx.close()
    for theta, actions in outs[1:]:
        assert all(torch.equal(a, b) for a, b in zip(theta, outs[0][0]))
        assert all(torch.equal(a, b) for a, b in zip(actions, outs[0][1]))
    assert not torch.equal(outs[0][0][1], outs[0][0][0])


def test_compute_unit_range_stream_errors():
    import ctypes as C
    import paper_2012_09849_amd as hts
    lib = hts.load_library()
    h = C.c_void_p()
    total = torch.cuda.get_device_properties(0).multi_processor_count
    assert lib.hts_stream_create_cu_range(0, 0, C.byref(h)) == -1            # HTS_EINVAL: empty range
    assert lib.hts_stream_create_cu_range(-1, 4, C.byref(h)) == -1
    assert lib.hts_stream_create_cu_range(total - 3, 4, C.byref(h)) == -1    # leaves the device
    assert lib.hts_stream_create_cu_range(0, 4, None) == -1
    assert lib.hts_stream_destroy(None) == -1
    s = hts.CuRangeStream(total - 8, 8)                                      # the last eight compute units (one per die): fine
    x = torch.zeros(1024, device="cuda")
    with torch.cuda.stream(s.stream):
        x += 1.0
    s.close()
    assert float(x.sum()) == 1024.0
