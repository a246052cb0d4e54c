"""numpy front-end of the CPU oracle (oracle/hts_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never imports or calls it.

All floating-point arrays cross this boundary as float64 (the oracle's
arithmetic type), except the sampler's logits, which are float32 because the
sampling decision is defined in binary32.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hts_oracle.c")
_LIB = os.path.join(_HERE, "libhts_oracle.so")

MAX_CONV = 4
GRAD_SLOTS = 32       # slots of the threaded gradient (fixed, so that its result does not depend on the thread count)


def host_threads() -> int:
    """Worker threads for the threaded variants: the host's cores, at most 16."""
    return max(1, min(16, os.cpu_count() or 1))


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Net(C.Structure):
    _fields_ = [("C", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("nconv", C.c_int32),
                ("cout", C.c_int32 * MAX_CONV), ("ksz", C.c_int32 * MAX_CONV), ("stride", C.c_int32 * MAX_CONV),
                ("hidden", C.c_int32), ("A", C.c_int32), ("operand_bf16", C.c_int32), ("gates_exact", C.c_int32)]


class HParams(C.Structure):
    _fields_ = [("algo", C.c_int32), ("clip_eps", C.c_double), ("vf_coef", C.c_double), ("ent_coef", C.c_double),
                ("max_grad_norm", C.c_double), ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("adam_eps", C.c_double), ("rho_bar", C.c_double), ("value_clip", C.c_double)]


class Stats(C.Structure):
    _fields_ = [("policy_loss", C.c_double), ("value_loss", C.c_double), ("entropy", C.c_double),
                ("grad_norm", C.c_double), ("clip_frac", C.c_double), ("approx_kl", C.c_double),
                ("total_loss", C.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


def make_net(C_in, H, W, A, convs=((32, 8, 4), (64, 4, 2), (64, 3, 1)), hidden=512, operand_bf16=False,
             gates_exact=False) -> Net:
    """operand_bf16: every operand of a conv/FC matrix product (forward and backward) rounded to bfloat16;
    gates_exact (with operand_bf16): the backward pass takes its ReLU gates from an unrounded forward pass."""
    n = Net()
    n.operand_bf16 = 1 if operand_bf16 else 0
    n.gates_exact = 1 if gates_exact else 0
    n.C, n.H, n.W, n.A, n.hidden, n.nconv = C_in, H, W, A, hidden, len(convs)
    for i, (co, k, s) in enumerate(convs):
        n.cout[i], n.ksz[i], n.stride[i] = co, k, s
    return n


def make_hparams(algo=0, clip_eps=0.1, vf_coef=0.5, ent_coef=0.01, max_grad_norm=0.0, lr=7e-4, beta1=0.9,
                 beta2=0.999, adam_eps=1e-5, rho_bar=1.0, value_clip=0.0) -> HParams:
    algo_id = {"a2c": 0, "ppo": 1, "a2c_tis": 2}.get(algo, algo)
    return HParams(algo_id, clip_eps, vf_coef, ent_coef, max_grad_norm, lr, beta1, beta2, adam_eps, rho_bar,
                   value_clip)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_param_count.restype = C.c_int64
        _lib.orc_uniform.restype = C.c_float
        _lib.orc_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        _lib.orc_expf.restype = C.c_float
        _lib.orc_expf.argtypes = [C.c_float]
        _lib.orc_round_bf16.restype = C.c_double
        _lib.orc_round_bf16.argtypes = [C.c_double]
        _lib.orc_clip_coef.restype = C.c_double
        _lib.orc_clip_coef.argtypes = [C.c_void_p, C.c_int64, C.c_double]
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def param_count(net: Net) -> int:
    return int(lib().orc_param_count(C.byref(net)))


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (C.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(v) for v in o]


def uniform(seed: int, env: int, step: int) -> float:
    return float(lib().orc_uniform(C.c_uint64(seed), C.c_uint32(env), C.c_uint32(step)))


def expf(x: float) -> np.float32:
    return np.float32(lib().orc_expf(C.c_float(float(x))))


def round_bf16(x: float) -> float:
    return float(lib().orc_round_bf16(C.c_double(float(x))))


def forward(net: Net, params, obs, index=None, B=None, threads=1):
    """-> logits float64 [B,A], values float64 [B].  threads > 1: rows spread over host threads (same values)."""
    p = _f64(params)
    obs = np.ascontiguousarray(obs, dtype=np.uint8).reshape(-1, net.C, net.H, net.W)
    idx = None if index is None else np.ascontiguousarray(index, dtype=np.int32)
    if B is None:
        B = obs.shape[0] if idx is None else idx.size
    logits = np.empty((B, net.A), dtype=np.float64)
    values = np.empty(B, dtype=np.float64)
    if threads > 1:
        rc = lib().orc_forward_mt(C.byref(net), _ptr(p), _ptr(obs), _ptr(idx), C.c_int32(B), _ptr(logits),
                                  _ptr(values), C.c_int32(threads))
    else:
        rc = lib().orc_forward(C.byref(net), _ptr(p), _ptr(obs), _ptr(idx), C.c_int32(B), _ptr(logits), _ptr(values))
    assert rc == 0
    return logits, values


def sample(logits, seed: int, step: int, env_offset: int = 0):
    """float32 logits [N,A] -> (actions int32 [N], logp float32 [N], u float32 [N])."""
    l = np.ascontiguousarray(logits, dtype=np.float32)
    N, A = l.shape
    actions = np.empty(N, dtype=np.int32)
    logp = np.empty(N, dtype=np.float32)
    u = np.empty(N, dtype=np.float32)
    rc = lib().orc_sample(_ptr(l), C.c_int32(N), C.c_int32(A), C.c_uint64(seed), C.c_uint32(step),
                          C.c_int32(env_offset), _ptr(actions), _ptr(logp), _ptr(u))
    assert rc == 0
    return actions, logp, u


def gae(rewards, values, dones, gamma: float, lam: float):
    """rewards [T,N], values [T+1,N], dones [T,N] -> (adv, ret) float64 [T,N]."""
    r, v = _f64(rewards), _f64(values)
    d = np.ascontiguousarray(dones, dtype=np.uint8)
    T, N = r.shape
    assert v.shape == (T + 1, N) and d.shape == (T, N)
    adv, ret = np.empty((T, N)), np.empty((T, N))
    lib().orc_gae(_ptr(r), _ptr(v), _ptr(d), C.c_double(gamma), C.c_double(lam), C.c_int32(T), C.c_int32(N),
                  _ptr(adv), _ptr(ret))
    return adv, ret


def normalize_adv(adv):
    a = _f64(adv).copy()
    lib().orc_normalize_adv(_ptr(a), C.c_int64(a.size))
    return a


def _buffer_args(net, obs, index, actions, old_logp, adv, ret, old_values=None):
    obs = np.ascontiguousarray(obs, dtype=np.uint8).reshape(-1, net.C, net.H, net.W)
    count = obs.shape[0]
    idx = None if index is None else np.ascontiguousarray(index, dtype=np.int32)
    B = count if idx is None else idx.size
    act = np.ascontiguousarray(actions, dtype=np.int32).reshape(-1)
    olp = _f64(old_logp if old_logp is not None else np.zeros(count)).reshape(-1)
    ad, rt = _f64(adv).reshape(-1), _f64(ret).reshape(-1)
    assert act.size == count and olp.size == count and ad.size == count and rt.size == count
    olv = None if old_values is None else _f64(old_values).reshape(-1)
    assert olv is None or olv.size == count
    return obs, idx, B, act, olp, ad, rt, olv


def loss_grads(net: Net, params, obs, actions, old_logp, adv, ret, hp: HParams, index=None, want_grads=True,
               old_values=None, threads=1):
    """-> (grads float64 [P] or None, stats dict).  old_values is read only when hp.value_clip > 0.
    threads > 1: the rows are cut into GRAD_SLOTS slots, each a plain call, combined in slot order."""
    p = _f64(params)
    obs, idx, B, act, olp, ad, rt, olv = _buffer_args(net, obs, index, actions, old_logp, adv, ret, old_values)
    assert hp.value_clip <= 0 or olv is not None
    g = np.empty(p.size) if want_grads else None
    st = Stats()
    if threads > 1:
        rc = lib().orc_loss_grads_mt(C.byref(net), _ptr(p), _ptr(obs), _ptr(idx), C.c_int32(B), _ptr(act), _ptr(olp),
                                     _ptr(olv), _ptr(ad), _ptr(rt), C.byref(hp), _ptr(g), C.byref(st),
                                     C.c_int32(GRAD_SLOTS), C.c_int32(threads))
    else:
        rc = lib().orc_loss_grads(C.byref(net), _ptr(p), _ptr(obs), _ptr(idx), C.c_int32(B), _ptr(act), _ptr(olp),
                                  _ptr(olv), _ptr(ad), _ptr(rt), C.byref(hp), _ptr(g), C.byref(st))
    assert rc == 0
    return g, st.as_dict()


def clip_coef(g, max_norm: float) -> float:
    g = _f64(g)
    return float(lib().orc_clip_coef(_ptr(g), C.c_int64(g.size), C.c_double(max_norm)))


def adam(theta, g, m, v, t: int, hp: HParams, gscale: float = 1.0):
    """-> new (theta, m, v) float64 copies."""
    th, m2, v2 = _f64(theta).copy(), _f64(m).copy(), _f64(v).copy()
    g = _f64(g)
    lib().orc_adam(_ptr(th), _ptr(g), _ptr(m2), _ptr(v2), C.c_int64(th.size), C.c_int64(t), C.c_double(gscale),
                   C.byref(hp))
    return th, m2, v2


def learner_step(net: Net, params, m, v, t: int, obs, actions, old_logp, adv, ret, hp: HParams, index=None,
                 old_values=None, threads=1):
    """-> (params, m, v, grads, stats), all new float64 arrays.  threads > 1: the threaded gradient, then the same
    clip and optimiser step."""
    if threads > 1:
        g, st = loss_grads(net, params, obs, actions, old_logp, adv, ret, hp, index=index, old_values=old_values,
                           threads=threads)
        scale = clip_coef(g, hp.max_grad_norm) if hp.max_grad_norm > 0 else 1.0
        th, m2, v2 = adam(params, g, m, v, t, hp, gscale=scale)
        return th, m2, v2, g, st
    th, m2, v2 = _f64(params).copy(), _f64(m).copy(), _f64(v).copy()
    obs, idx, B, act, olp, ad, rt, olv = _buffer_args(net, obs, index, actions, old_logp, adv, ret, old_values)
    assert hp.value_clip <= 0 or olv is not None
    g = np.empty(th.size)
    st = Stats()
    rc = lib().orc_learner_step(C.byref(net), _ptr(th), _ptr(m2), _ptr(v2), C.c_int64(t), _ptr(obs), _ptr(idx),
                                C.c_int32(B), _ptr(act), _ptr(olp), _ptr(olv), _ptr(ad), _ptr(rt), C.byref(hp),
                                _ptr(g), C.byref(st))
    assert rc == 0
    return th, m2, v2, g, st.as_dict()


def learner_step_delayed(net: Net, params_behaviour, params_target, m, v, t: int, obs, actions, old_logp, adv, ret,
                         hp: HParams, index=None, old_values=None):
    """The paper's one-step-delayed update (Sec. 4.1 "Delayed gradient"): the gradient of the objective at the behaviour
    parameters theta_{j-1}, on the storage collected with them, goes through clip + optimiser into the target
    parameters theta_j.  -> (theta_{j+1}, m, v, grads, stats), new float64 arrays."""
    g, st = loss_grads(net, params_behaviour, obs, actions, old_logp, adv, ret, hp, index=index, old_values=old_values)
    scale = clip_coef(g, hp.max_grad_norm) if hp.max_grad_norm > 0 else 1.0
    th, m2, v2 = adam(params_target, g, m, v, t, hp, gscale=scale)
    return th, m2, v2, g, st


def rmsprop(theta, g, v, lr: float, alpha: float, eps: float, gscale: float = 1.0):
    """-> new (theta, v) float64 copies."""
    th, v2 = _f64(theta).copy(), _f64(v).copy()
    g = _f64(g)
    lib().orc_rmsprop(_ptr(th), _ptr(g), _ptr(v2), C.c_int64(th.size), C.c_double(gscale), C.c_double(lr),
                      C.c_double(alpha), C.c_double(eps))
    return th, v2
