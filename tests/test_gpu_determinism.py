"""Run-to-run bit identity at the scale of the benchmark loops: the same iterations from the same state give the same
parameters, optimiser moments and actions (the paper's "full determinism", Sec. 1 and Sec. 4.1)."""
import hashlib

import pytest
import torch

import hts_synth as syn

pytestmark = pytest.mark.gpu


def _digest(loop):
    h = hashlib.sha256()
    for t in (loop.params, loop.opt.m, loop.opt.v, loop.actions, loop.logp, loop.values, loop.adv, loop.ret):
        h.update(t.detach().cpu().numpy().tobytes())
    return h.hexdigest()


@pytest.mark.parametrize("workload,overrides,iters", [
    ("atari_a2c_n16_t5_fp32", {}, 25),
    ("atari_ppo_n32_t128_bf16", {}, 2),                              # 32 minibatch steps of 1024 rows
    ("football_ppo_n16_t512_bf16", {"T": 64, "N": 16}, 2),           # 16x72x96 frames, minibatches of 256
])
def test_bench_loop_is_bit_reproducible(workload, overrides, iters):
    import bench
    import paper_2012_09849_amd as hts
    cfg = dict(bench.CONFIGS[workload], **overrides)
    digests = []
    for _ in range(2):
        loop = bench.Loop(cfg, hts, torch, syn)
        for _ in range(iters):
            loop.step()
        torch.cuda.synchronize()
        digests.append(_digest(loop))
        assert bool(torch.isfinite(loop.params).all())
        loop.ctx.close()
    assert digests[0] == digests[1]
