"""Call schedules of one training iteration on top of the binding (no arithmetic of the method lives here).

`Loop` issues the sequential schedule: the T actor calls of one unroll plus the bootstrap call, the returns over the
filled storage and the learner's minibatch steps, back to back on one stream.  `OverlapLoop` issues the paper's
concurrent schedule (Sec. 4.1 "Concurrent rollout and learning"): the actors fill storage j on one stream while the
learner consumes storage j-1 on another; the streams meet once per iteration.  `CONFIGS` holds the workloads the
benchmark and the full-size tests run.  The synthetic input generator is passed in by the caller (`syn`), so that this
package does not depend on where the test inputs come from.
"""
from __future__ import annotations

CONFIGS = {
    # Atari-shaped A2C: 16 environments, unroll 5 (the paper's A2C setting), fp32, one Adam update on the 80 rows
    "atari_a2c_n16_t5_fp32": dict(C=4, H=84, W=84, A=18, N=16, T=5, precision=0, algo=0, gamma=0.99, lam=1.0,
                                  lr=7e-4, epochs=1, minibatches=1, clip=0.1, max_norm=0.0, ent=0.01, obs="atari"),
    # Atari-shaped PPO: 32 environments, unroll 128, bf16 operands, 4 epochs x 4 minibatches of 1024, norm clip 0.5
    "atari_ppo_n32_t128_bf16": dict(C=4, H=84, W=84, A=18, N=32, T=128, precision=1, algo=1, gamma=0.99, lam=0.95,
                                    lr=2.5e-4, epochs=4, minibatches=4, clip=0.1, max_norm=0.5, ent=0.01, obs="atari"),
    # Football-shaped PPO: 16x72x96 extracted-map stacks, 16 environments, unroll 512, 2 epochs x 4 minibatches of 2048
    "football_ppo_n16_t512_bf16": dict(C=16, H=72, W=96, A=19, N=16, T=512, precision=1, algo=1, gamma=0.993,
                                       lam=0.95, lr=3.4e-4, epochs=2, minibatches=4, clip=0.08, max_norm=0.0,
                                       ent=0.003, obs="football", overlap_actor_cus=192),
    # the paper's multi-agent football experiment controls three players per environment: every controlled player is
    # one row of every call (16 environments x 3 players = 48 rows per step), unroll 128 as in the paper's runs
    "football_multiagent_ppo_n16x3_t128_bf16": dict(C=16, H=72, W=96, A=19, N=48, T=128, precision=1, algo=1,
                                                    gamma=0.993, lam=0.95, lr=3.4e-4, epochs=2, minibatches=4,
                                                    clip=0.08, max_norm=0.0, ent=0.003, obs="football"),
}

ACT_SEED = 20201209


def make_inputs(cfg, syn):
    """Host arrays of one storage: observations [T+1,N,C,H,W], rewards, dones [T,N], initial parameters."""
    N, T = cfg["N"], cfg["T"]
    if cfg["obs"] == "atari":
        obs = syn.obs_atari(syn.MASTER_SEED, T + 1, N)
        rew = syn.rewards_ternary(syn.MASTER_SEED, T, N) if cfg["algo"] == 0 else syn.rewards_score_clipped(syn.MASTER_SEED, T, N)
        dones = syn.dones_bernoulli(syn.MASTER_SEED, T, N, 0.05 if cfg["algo"] == 0 else 0.01)
    else:
        obs = syn.obs_football(syn.MASTER_SEED, T + 1, N)
        rew = syn.rewards_ternary(syn.MASTER_SEED, T, N, p_nonzero=0.002)
        dones = ((rew != 0) | (syn.dones_bernoulli(syn.MASTER_SEED, T, N, 0.001) != 0)).astype("uint8")
    params = syn.init_params(syn.MASTER_SEED, cfg["C"], cfg["H"], cfg["W"], cfg["A"])
    return obs, rew, dones, params


class Loop:
    """Device buffers of one storage plus the calls of one iteration, all on the context's stream."""

    def __init__(self, cfg, hts, torch, syn):
        self.cfg, self.hts, self.torch = cfg, hts, torch
        N, T, A = cfg["N"], cfg["T"], cfg["A"]
        obs, rew, dones, params = make_inputs(cfg, syn)
        self.host = dict(obs=obs, rew=rew, dones=dones, params=params)
        dev = "cuda"
        self.obs = torch.from_numpy(obs).to(dev)                      # [T+1, N, C, H, W]
        self.rew = torch.from_numpy(rew).to(dev)
        self.dones = torch.from_numpy(dones).to(dev)
        self.params = torch.from_numpy(params).to(dev)
        B = N * T // cfg["minibatches"]
        self.B = B
        self.ctx = hts.Context(cfg["C"], cfg["H"], cfg["W"], A, precision=cfg["precision"], max_act_batch=N,
                               max_learn_batch=B)
        # this loop writes self.params through this context's learner calls only, so the context may keep its copy of
        # the network in step with it instead of re-loading the vector before every update and every rollout
        self.ctx.hts_track_params(True)
        P = self.ctx.P
        self.opt = hts.OptState(torch.zeros(P, device=dev), torch.zeros(P, device=dev), 0)
        self.actions = torch.zeros(T + 1, N, dtype=torch.int32, device=dev)
        self.logp = torch.zeros(T + 1, N, device=dev)
        self.values = torch.zeros(T + 1, N, device=dev)
        self.adv = torch.zeros(T, N, device=dev)
        self.ret = torch.zeros(T, N, device=dev)
        self.hp = hts.HParams(algo=cfg["algo"], clip_eps=cfg["clip"], vf_coef=0.5, ent_coef=cfg["ent"],
                              max_grad_norm=cfg["max_norm"], lr=cfg["lr"])
        self.perms = [torch.from_numpy(syn.permutation(syn.MASTER_SEED, N * T, e)).to(dev) for e in range(cfg["epochs"])]
        self.iteration = 0
        # device addresses of every step's rows, taken once: a rollout is T+1 calls of a few microseconds each, and
        # slicing tensors for every call would cost more host time than the GPU needs for the call
        self._act_rows = self.ctx.act_rows(self.obs, self.actions, self.logp, self.values)

    def rollout(self):
        c, cfg = self.ctx, self.cfg
        base = self.iteration * (cfg["T"] + 1)
        # the actors keep one parameter version for a whole storage: it is loaded by the first call only
        c.hts_act_rows(self._act_rows, self.params, ACT_SEED, base, 0)

    def returns(self):
        cfg = self.cfg
        self.ctx.hts_returns_gae(self.rew, self.values, self.dones, cfg["gamma"], cfg["lam"], self.adv, self.ret)
        if cfg["algo"] == 1:
            self.ctx.hts_normalize_advantages(self.adv)

    def learn(self):
        cfg, T, N = self.cfg, self.cfg["T"], self.cfg["N"]
        obs = self.obs[:T].reshape(T * N, cfg["C"], cfg["H"], cfg["W"])
        actions, logp = self.actions[:T].reshape(-1), self.logp[:T].reshape(-1)
        adv, ret = self.adv.reshape(-1), self.ret.reshape(-1)
        for e in range(cfg["epochs"]):
            for k in range(cfg["minibatches"]):
                idx = None if cfg["minibatches"] == 1 and cfg["epochs"] == 1 else self.perms[e][k * self.B:(k + 1) * self.B]
                self.ctx.hts_learner_step(obs, actions, logp, adv, ret, self.params, self.opt, self.hp, index=idx,
                                          B=self.B)

    def step(self):
        self.rollout()
        self.returns()
        self.learn()
        self.iteration += 1


class OverlapLoop:
    """The paper's schedule (Sec. 4.1 "Concurrent rollout and learning"): while the actors fill storage j with theta_j
    on one stream, the learner works on storage j-1 on another; the streams meet once per iteration.  Two contexts
    (calls on one context must not overlap), two storages, three parameter vectors in rotation.

    One update per storage (A2C): the paper's one-step-delayed rule -- gradient at theta_{j-1} on storage j-1, applied to
    theta_j (hts_learner_step_delayed).  Several minibatch steps per storage (PPO): the paper states its rule for a
    single gradient step only; here the learner runs its ordinary epochs on storage j-1 starting from theta_j, the
    stored behaviour log-probabilities (of theta_{j-1}) entering through PPO's own probability ratio."""

    def __init__(self, base, learner_after=8, actor_cus=None):
        torch, hts, cfg = base.torch, base.hts, base.cfg
        self.base, self.cfg, self.torch = base, cfg, torch
        self.learner_after = learner_after          # actor calls issued before the learner's calls (see step)
        N, T = cfg["N"], cfg["T"]
        # actor_cus: the actors' stream is confined to the first `actor_cus` compute units and the learner's to the
        # rest.  It pays where the two sides' workgroups each want a whole compute unit's LDS (16x72x96 frames: the actor's
        # conv1 and the learner's conv1 kernels), so that on shared compute units every actor call waits for a learner
        # workgroup to leave; it costs where they interleave well anyway (4x84x84 frames).  Results do not depend on it.
        self._masked = []
        if actor_cus:
            total = torch.cuda.get_device_properties(torch.cuda.current_device()).multi_processor_count
            self._masked = [hts.CuRangeStream(0, actor_cus), hts.CuRangeStream(actor_cus, total - actor_cus)]
            self.s_roll, self.s_learn = self._masked[0].stream, self._masked[1].stream
        else:
            self.s_roll, self.s_learn = torch.cuda.Stream(), torch.cuda.Stream()
        mk = lambda **kw: hts.Context(cfg["C"], cfg["H"], cfg["W"], cfg["A"], precision=cfg["precision"], **kw)
        self.ctx_act = mk(max_act_batch=N, stream=self.s_roll)
        self.ctx_learn = mk(max_learn_batch=base.B, stream=self.s_learn)
        z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device="cuda")
        self.store = [dict(actions=z(T + 1, N, dt=torch.int32), logp=z(T + 1, N), values=z(T + 1, N), adv=z(T, N),
                           ret=z(T, N)) for _ in range(2)]
        self.rows = [self.ctx_act.act_rows(base.obs, st["actions"], st["logp"], st["values"]) for st in self.store]
        self.theta = [base.params.clone() for _ in range(3)]        # prev, cur, next
        P = base.params.numel()
        self.opt = hts.OptState(z(P), z(P), 0)
        self.ev_roll, self.ev_learn = torch.cuda.Event(), torch.cuda.Event()
        self.j = 0
        torch.cuda.synchronize()

    def step(self):
        torch, cfg, b = self.torch, self.cfg, self.base
        T, N = cfg["T"], cfg["N"]
        prev, cur, nxt = self.theta
        st = self.store[self.j % 2]
        single = cfg["epochs"] * cfg["minibatches"] == 1
        # When the learner's calls are issued matters on this hardware (it changes nothing in what either stream
        # computes): the rollout is hundreds of short calls whose issue alone takes the host milliseconds, so a learner
        # issued after it starts when the actors are nearly done; a learner issued before it fills the machine with
        # large kernels first, and the actors' short dependent kernels then wait behind them.  So the first
        # `learner_after` actor calls go out first, then the learner's calls, then the rest of the rollout.
        k = min(self.learner_after, T + 1)
        self.ctx_act.hts_act_rows(self.rows[self.j % 2], cur, ACT_SEED, self.j * (T + 1), 0, 0, k)
        with torch.cuda.stream(self.s_learn):
            nxt.copy_(cur)
            if self.j > 0:
                old = self.store[(self.j - 1) % 2]
                obs = b.obs[:T].reshape(T * N, cfg["C"], cfg["H"], cfg["W"])
                data = (obs, old["actions"][:T].reshape(-1), old["logp"][:T].reshape(-1), old["adv"].reshape(-1),
                        old["ret"].reshape(-1))
                if single:
                    self.ctx_learn.hts_learner_step_delayed(*data, prev, nxt, self.opt, b.hp)
                else:
                    for e in range(cfg["epochs"]):
                        for m in range(cfg["minibatches"]):
                            self.ctx_learn.hts_learner_step(*data, nxt, self.opt, b.hp,
                                                            index=b.perms[e][m * b.B:(m + 1) * b.B], B=b.B)
        self.ctx_act.hts_act_rows(self.rows[self.j % 2], cur, ACT_SEED, self.j * (T + 1), 0, k, T + 1)
        self.ctx_act.hts_returns_gae(b.rew, st["values"], b.dones, cfg["gamma"], cfg["lam"], st["adv"], st["ret"])
        if cfg["algo"] == 1:
            self.ctx_act.hts_normalize_advantages(st["adv"])
        self.ev_roll.record(self.s_roll)
        self.ev_learn.record(self.s_learn)
        self.s_roll.wait_event(self.ev_learn)
        self.s_learn.wait_event(self.ev_roll)
        self.theta = [cur, nxt, prev]
        self.j += 1

    def close(self):
        """Ends the two contexts and gives back the hardware queues of compute-unit-confined streams."""
        self.torch.cuda.synchronize()
        self.ctx_act.close()
        self.ctx_learn.close()
        for m in self._masked:
            m.close()
        self._masked = []
