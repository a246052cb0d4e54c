#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One step = one training iteration of a workload: T batched hts_act calls with seeded sampling plus the bootstrap call,
hts_returns_gae (and the advantage normalisation of the PPO workloads), and every learner minibatch step of the
iteration -- all enqueued back to back on one stream, no host synchronisation inside the timed region, inputs resident
in HBM.  The default workload is the largest single-GPU configuration, the Football-shaped PPO iteration (16x72x96
observations, 16 environments, unroll 512, 2 epochs x 4 minibatches of 2048, bf16 operands).

Prints ONE JSON line: env-frames/s (N*T per step over wall time) and learner samples/s of that workload, a roofline
entry for its dominant kernel (timed live with HIP events inside the library, a sample of its launches inside the
timed region), the other workloads (Atari-shaped PPO and A2C, the large-batch actor / returns sweep) in
`other_workloads`, and the CPU oracle timed on the host beside it (one core, and all cores).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2012_09849_amd.schedule import CONFIGS, Loop, OverlapLoop  # noqa: E402  (no GPU needed to import)

DEFAULT_WORKLOAD = "football_ppo_n16_t512_bf16"
METRIC = "env-frames/sec (act+GAE+PPO update) and learner samples/sec, 1×MI355X"
PEAK = {"mfma_f32": 157.3e12, "mfma_bf16": 2.5e15, "hbm": 8.0e12}


def layer_flops(cfg):
    """2*MACs per observation of the four contractions (unpadded)."""
    C, H, W = cfg["C"], cfg["H"], cfg["W"]
    H1, W1 = (H - 8) // 4 + 1, (W - 8) // 4 + 1
    H2, W2 = (H1 - 4) // 2 + 1, (W1 - 4) // 2 + 1
    P1, P2, P3 = H1 * W1, H2 * W2, (H2 - 2) * (W2 - 2)
    return {"conv1": 2.0 * P1 * 32 * 64 * C, "conv2": 2.0 * P2 * 64 * 512, "conv3": 2.0 * P3 * 64 * 576,
            "fc": 2.0 * 512 * 64 * P3}


def site_work(cfg, P):
    """Algorithmic work PER LAUNCH of every launch site: name -> (kind, amount, rows per launch).

    FLOPs are 2*MACs of the unpadded contraction times the rows one launch processes (N for an actor call, the
    minibatch size for a learner call); bytes are the arrays a streaming kernel must read and write once."""
    N, T = cfg["N"], cfg["T"]
    B = N * T // cfg["minibatches"]
    f = layer_flops(cfg)
    w = {}
    for layer in ("conv1", "conv2", "conv3", "fc"):
        w[f"{layer}_fwd"] = ("flop", N * f[layer], N)
        w[f"{layer}_fwd_learn"] = ("flop", B * f[layer], B)
    for layer in ("conv3", "conv2"):
        w[f"{layer}_wgrad"] = ("flop", B * f[layer], B)
        w[f"{layer}_dgrad"] = ("flop", B * f[layer], B)
    w["conv1_wgrad"] = ("flop", B * f["conv1"], B)
    w["fc_wgrad"] = ("flop", B * f["fc"], B)
    w["fc_dgrad"] = ("flop", B * f["fc"], B)
    w["adam"] = ("byte", 28.0 * P, B)
    w["grad_norm"] = ("byte", 4.0 * P, B)
    w["gae"] = ("byte", 17.0 * T * N + 4.0 * N, N)
    return w


def time_sites(loop, steps=2):
    """Every launch site bracketed in turn over a few steps: name -> (bracket ms per step, launches per step)."""
    names = loop.ctx.profile_sites()
    per_step = {}
    for i, nm in enumerate(names):
        loop.ctx.hts_profile_begin(i)
        for _ in range(steps):
            loop.step()
        n, ms = loop.ctx.hts_profile_end()
        if n:
            per_step[nm] = (ms / steps, n / steps)
    return per_step


ACT_SITES = ("prep", "conv1_fwd", "conv2_fwd", "conv3_fwd", "fc_fwd", "heads_act")


def bracket_overhead(loop, torch, per_step):
    """What an event bracket adds to a kernel's time IN SITU, from this workload's own rollout: the actor calls' launches
    run back to back on one stream, so the rollout's wall time is the sum of its kernels' times, and the sum of the raw
    brackets of the same launches exceeds it by (launches x overhead).  (An empty bracket -- two events with nothing
    between them -- reads about 4.5 us on this machine, but a bracket around a kernel costs less than that: the
    kernel's own completion covers part of it.)  -> (overhead ms, rollout ms per step)."""
    for _ in range(2):
        loop.rollout()
    torch.cuda.synchronize()
    reps = 3
    t0 = time.perf_counter()
    for _ in range(reps):
        loop.rollout()
    torch.cuda.synchronize()
    roll_ms = (time.perf_counter() - t0) / reps * 1e3
    raw = sum(per_step[k][0] for k in ACT_SITES if k in per_step)
    n = sum(per_step[k][1] for k in ACT_SITES if k in per_step)
    return max((raw - roll_ms) / max(n, 1), 0.0), roll_ms


def roofline_entry(cfg, name, kind, per_launch, rows, avg_bracket_s, overhead_s, n_timed, launches_per_step, traffic):
    """The dominant kernel against its roofline.  `achieved` uses the event bracket less the bracket's own in-situ cost
    (see bracket_overhead); the raw bracket and that cost are printed beside it."""
    net_s = max(avg_bracket_s - overhead_s, 1e-9)
    if kind == "flop":
        peak = PEAK["mfma_f32"] if cfg["precision"] == 0 else PEAK["mfma_bf16"]
        ach, unit, scale, bound = per_launch / net_s, "TFLOP/s", 1e12, "mfma"
    else:
        peak, ach, unit, scale, bound = PEAK["hbm"], per_launch / net_s, "GB/s", 1e9, "hbm"
    return {"kernel": name, "bound": bound, "achieved": ach / scale, "peak": peak / scale, "unit": unit,
            "frac": ach / peak, "traffic": traffic, "rows_per_launch": rows, "work_per_launch": per_launch,
            "avg_launch_us": net_s * 1e6, "raw_bracket_us": avg_bracket_s * 1e6, "event_overhead_us": overhead_s * 1e6,
            "frac_from_raw_bracket": per_launch / avg_bracket_s / peak,
            "launches_timed": n_timed, "launches_per_step": launches_per_step}


def cpu_baseline(cfg, loop, budget_s=14.0, threads=1):
    """The oracle as it stands on a bounded sample of the same workload (about budget_s of wall time).
    threads > 1: its threaded variants (rows spread over host threads, fixed-order combination)."""
    import numpy as np
    import oracle
    h = loop.host
    N, T = cfg["N"], cfg["T"]
    net = oracle.make_net(cfg["C"], cfg["H"], cfg["W"], cfg["A"])
    p = h["params"].astype(np.float64)
    hp = oracle.make_hparams(algo=cfg["algo"], clip_eps=cfg["clip"], lr=cfg["lr"], max_grad_norm=cfg["max_norm"])
    all_obs = h["obs"][:T].reshape(N * T, cfg["C"], cfg["H"], cfg["W"])
    # actor: whole hts_act steps (N frames each, cycling through the iteration's T+1) for 40% of the budget
    t0 = time.perf_counter()
    n_steps = 0
    while n_steps == 0 or time.perf_counter() - t0 < 0.4 * budget_s:
        logits, _ = oracle.forward(net, p, h["obs"][n_steps % (T + 1)], threads=threads)
        oracle.sample(logits.astype(np.float32), 1, n_steps, 0)
        n_steps += 1
    t_act = (time.perf_counter() - t0) / n_steps
    t0 = time.perf_counter()
    oracle.gae(h["rew"], np.zeros((T + 1, N)), h["dones"], cfg["gamma"], cfg["lam"])
    t_gae = time.perf_counter() - t0
    # learner: one update on a calibration sample, then on as many rows as the rest of the budget allows

    def learn(rows):
        t = time.perf_counter()
        oracle.learner_step(net, p, np.zeros(p.size), np.zeros(p.size), 1, all_obs[:rows], np.zeros(rows, np.int32),
                            np.zeros(rows), np.ones(rows), np.ones(rows), hp, threads=threads)
        return time.perf_counter() - t
    rows0 = min(N * T, 16 * max(1, threads))
    t_cal = learn(rows0)
    mb_rows = N * T // cfg["minibatches"]
    rows = int(min(mb_rows, max(rows0, 0.6 * budget_s * rows0 / t_cal)))
    t_learn, reps = learn(rows), 1
    while t_learn * (reps + 1) / reps < 0.6 * budget_s - t_cal:       # small workloads: repeat the whole update
        t_learn += learn(rows)
        reps += 1
    t_learn /= reps
    learn_rows = N * T * cfg["epochs"]
    total = t_act * (T + 1) + t_gae + t_learn * (learn_rows / rows)
    return {"value": N * T / total, "unit": "env-frames/s", "cores": threads, "kind": "oracle",
            "sample": f"{n_steps} hts_act steps of {N} frames (an iteration has {T + 1}), GAE in full, {reps} learner "
                      f"update(s) on {rows} rows scaled linearly to the iteration's {learn_rows}; "
                      f"{t_act * n_steps + t_gae + t_cal + t_learn * reps:.1f} s of wall time on {threads} thread(s)",
            "learner_samples_per_s": rows / t_learn, "host_cores": os.cpu_count()}


def source_digest():
    """SHA-256 over the kernel sources: hardware-counter figures are only reported for the sources they were taken on.
    (api.hip holds the C entry points and no kernel: it is not part of the digest.)"""
    import glob
    import hashlib
    h = hashlib.sha256()
    root = os.path.join(ROOT, "paper_2012_09849_amd", "csrc")
    for f in sorted(glob.glob(os.path.join(root, "*.hip")) + glob.glob(os.path.join(root, "*.hpp"))):
        if os.path.basename(f) != "api.hip":
            h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


# HBM bytes per launch of the launch sites that can come out as a workload's dominant kernel, from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE (KiB per dispatch, averaged over the site's launches of the run, each scaled by what the
# counter reads for a plain copy of known size): workload -> ({launch site: bytes per launch}, digest of the kernel
# sources the counters were taken on).
TRAFFIC = {
    "football_ppo_n16_t512_bf16": ({"conv1_fwd": 5099060, "conv1_fwd_learn": 279396464, "conv1_wgrad": 314394353,
                                    "conv2_fwd": 2626307, "conv3_fwd": 1214351, "fc_fwd": 3475119}, "394f517a35e13028"),
    "atari_ppo_n32_t128_bf16": ({"conv1_fwd": 2846561, "conv1_fwd_learn": 55546870, "conv1_wgrad": 63732383,
                                 "conv2_wgrad": 45561325}, "394f517a35e13028"),
}


# Average duration (us) of the same launch sites' kernels in the committed rocprofv3 kernel traces
# (profiles/all_kernels_<workload>.txt), for comparison with the live event figure; same digest rule as TRAFFIC.
TRACE_AVG_US = {
    "football_ppo_n16_t512_bf16": ({"conv1_fwd": 6.30, "heads_act": 5.07, "conv2_fwd": 3.87, "conv3_fwd": 3.52,
                                    "fc_fwd": 3.20, "conv1_fwd_learn": 86.50, "conv1_wgrad": 78.18}, "394f517a35e13028"),
    "atari_ppo_n32_t128_bf16": ({"conv1_fwd": 5.03, "heads_act": 5.20, "conv1_fwd_learn": 20.44, "conv1_wgrad": 19.09,
                                 "conv2_wgrad": 22.54}, "394f517a35e13028"),
}


def run_iterations(loop, torch, steps, warmup, sample_site=None, sample_every=1):
    """warmup untimed steps, then `steps` timed ones between two synchronisations.  sample_site: bracket every
    sample_every-th launch of that site with events during the timed steps."""
    for _ in range(warmup):
        loop.step()
    torch.cuda.synchronize()
    if sample_site is not None:
        loop.ctx.hts_profile_begin_sampled(sample_site, sample_every)
    t0 = time.perf_counter()
    for _ in range(steps):
        loop.step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    timed = loop.ctx.hts_profile_end() if sample_site is not None else (0, 0.0)
    return wall, timed


def time_learner(loop, torch, n):
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(n):
        loop.learn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t1) / n


def workload_summary(name, steps, warmup, hts, torch, syn):
    """One of the other workloads, timed the same way (no brackets)."""
    cfg = CONFIGS[name]
    loop = Loop(cfg, hts, torch, syn)
    wall, _ = run_iterations(loop, torch, steps, warmup)
    t_learn = time_learner(loop, torch, max(1, steps // 4))
    frames = cfg["N"] * cfg["T"]
    out = {"value": frames * steps / wall, "unit": "env-frames/s", "ms_per_step": wall / steps * 1e3, "steps": steps,
           "warmup": warmup, "dtype": "f32" if cfg["precision"] == 0 else "bf16",
           "learner_samples_per_s": frames * cfg["epochs"] / t_learn, "learner_ms_per_step": t_learn * 1e3,
           "config": {"envs": cfg["N"], "unroll": cfg["T"], "obs": [cfg["C"], cfg["H"], cfg["W"]],
                      "epochs": cfg["epochs"], "minibatches": cfg["minibatches"]}}
    loop.ctx.close()
    del loop
    torch.cuda.empty_cache()
    return out


def act_sweep(hts, torch, syn):
    """Large-batch actor / returns sweep: hts_act over N in {256, 1024, 4096} Atari-shaped observations (bf16, 18
    actions, seeded sampling), frames/s per call with the parameters already loaded; returns/GAE at 128 x 4096 and,
    for a bandwidth- rather than launch-bound figure, at 128 x 262144."""
    import numpy as np
    out = {}
    params = torch.from_numpy(syn.init_params(syn.MASTER_SEED, 4, 84, 84, 18)).cuda()
    base = syn.obs_atari(syn.MASTER_SEED, 1, 256)[0]                 # 256 distinct environments, tiled to N
    for N in (256, 1024, 4096):
        obs = torch.from_numpy(np.ascontiguousarray(np.tile(base, (N // 256, 1, 1, 1)))).cuda()
        ctx = hts.Context(4, 84, 84, 18, precision=1, max_act_batch=N)
        actions = torch.zeros(N, dtype=torch.int32, device="cuda")
        logp, values = torch.zeros(N, device="cuda"), torch.zeros(N, device="cuda")
        ctx.hts_act(obs, params, 7, 0, 0, actions, logp, values)
        reps = 200 if N <= 1024 else 60
        for s in range(5):
            ctx.hts_act(obs, None, 7, s, 0, actions, logp, values)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(reps):
            ctx.hts_act(obs, None, 7, s, 0, actions, logp, values)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        out[f"act_n{N}"] = {"frames_per_s": N / dt, "us_per_call": dt * 1e6,
                            "frac_of_bf16_mfma_peak": N * sum(layer_flops(dict(C=4, H=84, W=84)).values()) / dt / PEAK["mfma_bf16"]}
        ctx.close()
        del obs
    ctx = hts.Context(4, 84, 84, 18, precision=1, max_act_batch=1)
    overhead_ms = ctx.hts_profile_overhead(256)
    g = torch.Generator(device="cuda").manual_seed(1)
    for T, N, reps in ((128, 4096, 200), (128, 262144, 20)):
        r, v = torch.randn(T, N, device="cuda", generator=g), torch.randn(T + 1, N, device="cuda", generator=g)
        d = (torch.rand(T, N, device="cuda", generator=g) < 0.01).to(torch.uint8)
        adv, ret = torch.empty_like(r), torch.empty_like(r)
        for _ in range(3):
            ctx.hts_returns_gae(r, v, d, 0.99, 0.95, adv, ret)
        ctx.hts_profile_begin(ctx.profile_sites().index("gae"))
        for _ in range(reps):
            ctx.hts_returns_gae(r, v, d, 0.99, 0.95, adv, ret)
        n, ms = ctx.hts_profile_end()
        nbytes = 17.0 * T * N + 4.0 * N
        raw_us = ms / n * 1e3
        us = max(raw_us - overhead_ms * 1e3, 1e-3)
        out[f"gae_{T}x{N}"] = {"GB/s": nbytes / (us * 1e-6) / 1e9, "frac_of_hbm_peak": nbytes / (us * 1e-6) / PEAK["hbm"],
                               "avg_launch_us": us, "raw_bracket_us": raw_us, "event_overhead_us": overhead_ms * 1e3}
        del r, v, d, adv, ret
    ctx.close()
    torch.cuda.empty_cache()
    return out


def progress(msg):
    """A line on stderr at the end of each phase (stdout carries the one JSON line)."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other workloads and the overlapped schedule")
    ap.add_argument("--site", default=None, help="bracket this launch site instead of discovering the dominant one")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="calibration for hardware counters: run a plain device copy of this many MiB and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); multi-GPU sharding is a design note, not code",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import hts_synth as syn
    import paper_2012_09849_amd as hts

    cfg = CONFIGS[args.workload]
    torch.cuda.set_device(0)
    if args.copy_probe > 0:
        n = args.copy_probe * (1 << 20) // 4
        src = torch.arange(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_MiB": args.copy_probe, "bytes_read": 4 * n, "bytes_written": 4 * n}))
        return
    loop = Loop(cfg, hts, torch, syn)
    for _ in range(args.warmup):
        loop.step()
    torch.cuda.synchronize()
    work = site_work(cfg, loop.ctx.P)
    names = loop.ctx.profile_sites()
    empty_bracket_ms = loop.ctx.hts_profile_overhead(256)     # what two events with nothing between them read
    progress(f"{args.workload}: warm-up done")
    if args.site:
        # light form for runs under a profiler's counter collection (every dispatch is slow there): one bracketed
        # step of the named site, the empty bracket's reading as the bracket cost
        dominant = args.site
        loop.ctx.hts_profile_begin(names.index(dominant))
        loop.step()
        n1, ms1 = loop.ctx.hts_profile_end()
        per_step = {dominant: (ms1, float(n1))}
        overhead_ms, rollout_ms = empty_bracket_ms, None
    else:
        per_step = time_sites(loop)
        overhead_ms, rollout_ms = bracket_overhead(loop, torch, per_step)
    progress("launch sites timed")
    if not args.site:
        ranked = sorted(((v[0] - v[1] * overhead_ms, k) for k, v in per_step.items() if k in work), reverse=True)
        dominant = ranked[0][1]
    launches_per_step = per_step[dominant][1]
    # about 16 brackets per step: a bracket costs the stream about as much as a small kernel
    every = max(1, int(launches_per_step // 16))
    torch.cuda.synchronize()

    # timed region: a sample of the dominant kernel's launches is bracketed by HIP events on the library's stream
    wall, (n_timed, ms_timed) = run_iterations(loop, torch, args.steps, 0, names.index(dominant), every)
    progress(f"{args.steps} timed steps done")
    t_learn = time_learner(loop, torch, max(1, args.steps // 4))

    N, T = cfg["N"], cfg["T"]
    frames = N * T
    learn_rows = frames * cfg["epochs"]
    out = {
        "metric": METRIC,
        "value": frames * args.steps / wall,
        "unit": "env-frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if cfg["precision"] == 0 else "bf16",
        "data": "synthetic",
        "config": {"workload": args.workload, "envs": N, "unroll": T, "actions": cfg["A"],
                   "obs": [cfg["C"], cfg["H"], cfg["W"]], "epochs": cfg["epochs"], "minibatches": cfg["minibatches"],
                   "minibatch_rows": loop.B, "learner_rows_per_step": learn_rows},
        "learner_samples_per_s": learn_rows / t_learn,
        "learner_ms_per_step": t_learn * 1e3,
    }
    kind, per_launch, rows = work[dominant]
    traffic = None
    if args.workload in TRAFFIC and dominant in TRAFFIC[args.workload][0] and TRAFFIC[args.workload][1] == source_digest():
        traffic = TRAFFIC[args.workload][0][dominant]
    out["roofline"] = roofline_entry(cfg, dominant, kind, per_launch, rows, ms_timed / max(n_timed, 1) * 1e-3,
                                     overhead_ms * 1e-3, n_timed, launches_per_step, traffic)
    out["roofline"]["empty_bracket_us"] = empty_bracket_ms * 1e3
    if args.workload in TRACE_AVG_US and dominant in TRACE_AVG_US[args.workload][0] and TRACE_AVG_US[args.workload][1] == source_digest():
        tr_us = TRACE_AVG_US[args.workload][0][dominant]
        out["roofline"]["trace_avg_us"] = tr_us        # the kernel's average in profiles/all_kernels_<workload>.txt
        out["roofline"]["frac_from_trace"] = per_launch / (tr_us * 1e-6) / (out["roofline"]["peak"] * (1e12 if kind == "flop" else 1e9))
    out["rollout_ms_per_step"] = rollout_ms
    # the same accounting for the learner's dominant kernel (minibatch-sized launches: a throughput figure, where the
    # actor kernels at N rows per call are latency figures); brackets from the per-site pass
    learn_sites = [(v[0] - v[1] * overhead_ms, k) for k, v in per_step.items()
                   if k in work and work[k][2] == loop.B and work[k][0] == "flop"]
    if learn_sites and not args.site:
        _, lk = max(learn_sites)
        lkind, lper, lrows = work[lk]
        lms, ln = per_step[lk]
        ltraffic = None
        if args.workload in TRAFFIC and lk in TRAFFIC[args.workload][0] and TRAFFIC[args.workload][1] == source_digest():
            ltraffic = TRAFFIC[args.workload][0][lk]
        out["roofline_learner"] = roofline_entry(cfg, lk, lkind, lper, lrows, lms / ln * 1e-3, overhead_ms * 1e-3, int(ln * 2),
                                                 ln, ltraffic)
        if args.workload in TRACE_AVG_US and lk in TRACE_AVG_US[args.workload][0] and TRACE_AVG_US[args.workload][1] == source_digest():
            tr_us = TRACE_AVG_US[args.workload][0][lk]
            out["roofline_learner"]["trace_avg_us"] = tr_us
            out["roofline_learner"]["frac_from_trace"] = lper / (tr_us * 1e-6) / (out["roofline_learner"]["peak"] * 1e12)
    # every launch site of this workload: event-bracket time per launch (raw, and less the empty bracket) and its share
    kernels = {}
    for k, (ms, n) in sorted(per_step.items(), key=lambda kv: -(kv[1][0] - kv[1][1] * overhead_ms)):
        raw_us = ms / n * 1e3
        e = {"launches_per_step": n, "raw_bracket_us": round(raw_us, 3),
             "avg_launch_us": round(max(raw_us - overhead_ms * 1e3, 0.0), 3),
             "ms_per_step": round(max(ms - n * overhead_ms, 0.0), 5)}
        if k in work:
            wk, amount, _ = work[k]
            pk = PEAK["hbm"] if wk == "byte" else (PEAK["mfma_f32"] if cfg["precision"] == 0 else PEAK["mfma_bf16"])
            e["frac_of_peak"] = round(amount / max((raw_us - overhead_ms * 1e3) * 1e-6, 1e-9) / pk, 5)
        kernels[k] = e
    out["kernels"] = kernels
    if not args.site and not args.no_others:
        actor_cus = cfg.get("overlap_actor_cus")
        try:
            ov = OverlapLoop(loop, actor_cus=actor_cus)
        except hts.HtsError as err:                    # e.g. a device with another number of compute units
            progress(f"compute-unit ranges refused ({err}); concurrent schedule on ordinary streams")
            actor_cus = None
            ov = OverlapLoop(loop)
        ov_steps = max(1, args.steps // 2)
        for _ in range(2):
            ov.step()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(ov_steps):
            ov.step()
        torch.cuda.synchronize()
        ov_wall = time.perf_counter() - t2
        out["overlapped"] = {"value": frames * ov_steps / ov_wall, "unit": "env-frames/s",
                             "ms_per_step": ov_wall / ov_steps * 1e3, "steps": ov_steps,
                             "schedule": "rollout with theta_j on one stream while the learner works on the previous "
                                         "storage on a second stream (one update per storage: the one-step-delayed "
                                         "update; several: ordinary epochs from theta_j); same work per step as "
                                         "`value`, which runs the three parts in sequence",
                             "actor_compute_units": actor_cus or "all (shared with the learner)"}
        ov.close()
        del ov
    if not args.no_cpu_baseline:
        import oracle
        progress("timing the CPU oracle")
        out["cpu_baseline"] = cpu_baseline(cfg, loop)
        out["cpu_baseline_all_cores"] = cpu_baseline(cfg, loop, budget_s=8.0, threads=oracle.host_threads())
    loop.ctx.close()
    del loop
    torch.cuda.empty_cache()
    if not args.site and not args.no_others:
        others = {}
        for name, steps, warmup in (("atari_ppo_n32_t128_bf16", 40, 3), ("atari_a2c_n16_t5_fp32", 1000, 50)):
            if name != args.workload:
                progress(f"other workload {name}")
                others[name] = workload_summary(name, steps, warmup, hts, torch, syn)
        others["act_sweep_bf16"] = act_sweep(hts, torch, syn)
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
