"""ctypes binding with the same names as the C ABI (include/hts.h).  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhts.so")

PRECISION_FP32, PRECISION_BF16 = 0, 1
ALGO_A2C, ALGO_PPO, ALGO_A2C_TIS = 0, 1, 2
OPT_ADAM, OPT_RMSPROP = 0, 1

EXPORTS = ["hts_param_count", "hts_create", "hts_destroy", "hts_act", "hts_sync_params", "hts_sample_from_logits", "hts_returns_gae",
           "hts_normalize_advantages", "hts_learner_step", "hts_learner_step_delayed", "hts_loss_and_grads", "hts_adam_apply", "hts_test_gemm",
           "hts_last_hip_error", "hts_strerror", "hts_profile_site_count", "hts_profile_site_name", "hts_profile_begin",
           "hts_profile_end", "hts_profile_overhead", "hts_profile_begin_sampled", "hts_adam_apply_static", "hts_track_params",
           "hts_stream_create_cu_range", "hts_stream_destroy"]


class HtsError(RuntimeError):
    pass


class NetDesc(C.Structure):
    _fields_ = [("C", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("A", C.c_int32), ("precision", C.c_int32)]


class Buffer(C.Structure):
    _fields_ = [("obs", C.c_void_p), ("actions", C.c_void_p), ("old_logp", C.c_void_p), ("old_values", C.c_void_p),
                ("advantages", C.c_void_p), ("returns", C.c_void_p), ("count", C.c_int32), ("index", C.c_void_p),
                ("B", C.c_int32)]


class HParams(C.Structure):
    _fields_ = [("algo", C.c_int32), ("clip_eps", C.c_float), ("vf_coef", C.c_float), ("ent_coef", C.c_float),
                ("max_grad_norm", C.c_float), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("adam_eps", C.c_float), ("optimizer", C.c_int32), ("rms_alpha", C.c_float), ("rho_bar", C.c_float),
                ("value_clip", C.c_float)]

    def __init__(self, algo=ALGO_A2C, clip_eps=0.1, vf_coef=0.5, ent_coef=0.01, max_grad_norm=0.0, lr=7e-4,
                 beta1=0.9, beta2=0.999, adam_eps=1e-5, optimizer=OPT_ADAM, rms_alpha=0.99, rho_bar=1.0,
                 value_clip=0.0):
        super().__init__(algo, clip_eps, vf_coef, ent_coef, max_grad_norm, lr, beta1, beta2, adam_eps, optimizer,
                         rms_alpha, rho_bar, value_clip)


class _OptStateC(C.Structure):
    _fields_ = [("m", C.c_void_p), ("v", C.c_void_p), ("step", C.c_int64)]


class OptState:
    """Adam moments (device fp32 [P]) and the host-side count of completed updates."""

    def __init__(self, m: torch.Tensor, v: torch.Tensor, step: int = 0):
        self.m, self.v, self.step = m, v, step


STATS_FIELDS = ("policy_loss", "value_loss", "entropy", "grad_norm", "clip_frac", "approx_kl", "nonfinite")

_lib = None


def load_library():
    """Load libhts.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise HtsError(f"{LIB_PATH} not found: build it with `python -m paper_2012_09849_amd.build`")
        lib = C.CDLL(LIB_PATH)
        lib.hts_param_count.restype = C.c_int64
        lib.hts_param_count.argtypes = [C.POINTER(NetDesc)]
        lib.hts_strerror.restype = C.c_char_p
        lib.hts_strerror.argtypes = [C.c_int32]
        lib.hts_create.argtypes = [C.POINTER(NetDesc), C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_void_p)]
        lib.hts_destroy.argtypes = [C.c_void_p]
        lib.hts_act.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_int32, C.c_int32,
                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.hts_sync_params.argtypes = [C.c_void_p, C.c_void_p]
        lib.hts_track_params.argtypes = [C.c_void_p, C.c_int32]
        lib.hts_sample_from_logits.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_int32, C.c_int32,
                                               C.c_void_p, C.c_void_p]
        lib.hts_returns_gae.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float,
                                        C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        lib.hts_normalize_advantages.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        lib.hts_learner_step.argtypes = [C.c_void_p, C.POINTER(Buffer), C.c_void_p, C.POINTER(_OptStateC),
                                         C.POINTER(HParams), C.c_void_p]
        lib.hts_loss_and_grads.argtypes = [C.c_void_p, C.POINTER(Buffer), C.c_void_p, C.POINTER(HParams), C.c_void_p,
                                           C.c_void_p]
        lib.hts_adam_apply.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_OptStateC), C.POINTER(HParams),
                                       C.c_int64]
        lib.hts_adam_apply_static.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(_OptStateC), C.POINTER(HParams),
                                              C.c_int64, C.c_void_p]
        lib.hts_test_gemm.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_int32]
        lib.hts_profile_site_name.restype = C.c_char_p
        lib.hts_profile_site_name.argtypes = [C.c_int32]
        lib.hts_profile_begin.argtypes = [C.c_void_p, C.c_int32]
        lib.hts_profile_begin_sampled.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        lib.hts_profile_end.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_double)]
        lib.hts_profile_overhead.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double)]
        lib.hts_stream_create_cu_range.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
        lib.hts_stream_destroy.argtypes = [C.c_void_p]
        _lib = lib
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        lib = load_library()
        raise HtsError(f"{what}: {lib.hts_strerror(rc).decode()} (code {rc}, hip {lib.hts_last_hip_error()})")


def param_count(C_in: int, H: int, W: int, A: int, precision: int = PRECISION_FP32) -> int:
    d = NetDesc(C_in, H, W, A, precision)
    n = load_library().hts_param_count(C.byref(d))
    if n < 0:
        _check(int(n), "hts_param_count")
    return int(n)


def _ptr(t, dtype, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise HtsError(f"{name}: expected a contiguous {dtype} device tensor")
    return C.c_void_p(t.data_ptr())


def hts_adam_apply_static(params, grads, opt: OptState, hp: HParams, stream=None):
    """Clip + optimiser step through the library's static scratch array: no context, no allocation."""
    lib = load_library()
    stream = stream if stream is not None else torch.cuda.current_stream()
    oc = _OptStateC(_ptr(opt.m, torch.float32, "m"), _ptr(opt.v, torch.float32, "v"), opt.step)
    _check(lib.hts_adam_apply_static(_ptr(params, torch.float32, "params"), _ptr(grads, torch.float32, "grads"),
                                     C.byref(oc), C.byref(hp), params.numel(), C.c_void_p(stream.cuda_stream)),
           "hts_adam_apply_static")
    opt.step = oc.step


class CuRangeStream:
    """hts_stream_create_cu_range: a stream whose kernels run on compute units [first_cu, first_cu + n_cus) only, wrapped
    as a torch stream (`.stream`).  close() synchronises and destroys it."""

    def __init__(self, first_cu: int, n_cus: int):
        lib = load_library()
        h = C.c_void_p()
        _check(lib.hts_stream_create_cu_range(first_cu, n_cus, C.byref(h)), "hts_stream_create_cu_range")
        self._h = h
        self.stream = torch.cuda.ExternalStream(h.value)

    def close(self):
        if self._h is not None and self._h.value:
            _check(load_library().hts_stream_destroy(self._h), "hts_stream_destroy")
            self._h = None


class Context:
    """Owns an hts_ctx bound to a torch stream (default: the current stream at construction)."""

    def __init__(self, C_in, H, W, A, precision=PRECISION_FP32, max_act_batch=0, max_learn_batch=0, stream=None):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise HtsError("no GPU visible: the library has no CPU path")
        self.desc = NetDesc(C_in, H, W, A, precision)
        self.A = A
        self.P = param_count(C_in, H, W, A, precision)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self._h = C.c_void_p()
        _check(self.lib.hts_create(C.byref(self.desc), max_act_batch, max_learn_batch,
                                   C.c_void_p(self.stream.cuda_stream), C.byref(self._h)), "hts_create")

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            self.stream.synchronize()
            self.lib.hts_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the three calls of the hot path ------------------------------------------------------------------
    def hts_act(self, obs, params, seed, step, env_offset, actions, logp, values, logits=None):
        N = obs.shape[0]
        _check(self.lib.hts_act(self._h, _ptr(obs, torch.uint8, "obs"), _ptr(params, torch.float32, "params"),
                                C.c_uint64(seed), C.c_uint32(step), N, env_offset,
                                _ptr(actions, torch.int32, "actions"), _ptr(logp, torch.float32, "logp"),
                                _ptr(values, torch.float32, "values"), _ptr(logits, torch.float32, "logits")),
               "hts_act")

    def act_rows(self, obs, actions, logp, values, logits=None):
        """Pre-marshalled hts_act arguments, one entry per leading index s of obs [S,N,C,H,W], actions / logp / values
        [S,N] (and logits [S,N,A]): the tensors are checked once and only raw device addresses are kept."""
        S, N = obs.shape[0], obs.shape[1]
        for t, dt, nm in ((obs, torch.uint8, "obs"), (actions, torch.int32, "actions"), (logp, torch.float32, "logp"),
                          (values, torch.float32, "values"), (logits, torch.float32, "logits")):
            if t is not None:
                _ptr(t, dt, nm)
                if t.shape[0] != S or t.shape[1] != N:
                    raise HtsError(f"{nm}: leading dimensions must be [{S},{N}]")
        ob, so = obs.data_ptr(), obs[0].numel()
        ab, lb, vb = actions.data_ptr(), logp.data_ptr(), values.data_ptr()
        gb, sg = (logits.data_ptr(), 4 * logits[0].numel()) if logits is not None else (0, 0)
        rows = [(ob + s * so, ab + 4 * s * N, lb + 4 * s * N, vb + 4 * s * N, (gb + s * sg) if gb else None)
                for s in range(S)]
        return (N, rows, (obs, actions, logp, values, logits))

    def hts_act_rows(self, act_rows, params, seed, step0, env_offset, first=0, last=None):
        """One hts_act call per entry [first, last) of act_rows (see act_rows); entry s is step step0 + s.  The
        parameters are passed to entry 0 only (the actors keep one parameter version for a whole storage)."""
        N, rows, _keep = act_rows
        fn, h = self.lib.hts_act, self._h
        pp = _ptr(params, torch.float32, "params")
        last = len(rows) if last is None else last
        for s in range(first, last):
            o, a, l, v, g = rows[s]
            rc = fn(h, o, pp if s == 0 else None, seed, step0 + s, N, env_offset, a, l, v, g)
            if rc != 0:
                _check(rc, "hts_act")

    def hts_track_params(self, on: bool):
        _check(self.lib.hts_track_params(self._h, 1 if on else 0), "hts_track_params")

    def hts_sync_params(self, params):
        _check(self.lib.hts_sync_params(self._h, _ptr(params, torch.float32, "params")), "hts_sync_params")

    def hts_sample_from_logits(self, logits, seed, step, env_offset, actions, logp):
        N = logits.shape[0]
        _check(self.lib.hts_sample_from_logits(self._h, _ptr(logits, torch.float32, "logits"), C.c_uint64(seed),
                                               C.c_uint32(step), N, env_offset,
                                               _ptr(actions, torch.int32, "actions"),
                                               _ptr(logp, torch.float32, "logp")), "hts_sample_from_logits")

    def hts_returns_gae(self, rewards, values, dones, gamma, lam, advantages, returns):
        T, N = rewards.shape
        if tuple(values.shape) != (T + 1, N) or tuple(dones.shape) != (T, N):
            raise HtsError("hts_returns_gae: values must be [T+1,N] and dones [T,N]")
        _check(self.lib.hts_returns_gae(self._h, _ptr(rewards, torch.float32, "rewards"),
                                        _ptr(values, torch.float32, "values"), _ptr(dones, torch.uint8, "dones"),
                                        gamma, lam, T, N, _ptr(advantages, torch.float32, "advantages"),
                                        _ptr(returns, torch.float32, "returns")), "hts_returns_gae")

    def hts_normalize_advantages(self, adv):
        _check(self.lib.hts_normalize_advantages(self._h, _ptr(adv, torch.float32, "adv"), adv.numel()),
               "hts_normalize_advantages")

    def _buffer(self, obs, actions, old_logp, advantages, returns, index, B, old_values=None):
        count = obs.shape[0]
        if B is None:
            B = count if index is None else index.numel()
        keep = (obs, actions, old_logp, advantages, returns, index, old_values)
        return Buffer(_ptr(obs, torch.uint8, "obs"), _ptr(actions, torch.int32, "actions"),
                      _ptr(old_logp, torch.float32, "old_logp"), _ptr(old_values, torch.float32, "old_values"),
                      _ptr(advantages, torch.float32, "advantages"), _ptr(returns, torch.float32, "returns"), count,
                      _ptr(index, torch.int32, "index"), B), keep

    def hts_learner_step(self, obs, actions, old_logp, advantages, returns, params, opt: OptState, hp: HParams,
                         index=None, B=None, stats=None, old_values=None):
        buf, _keep = self._buffer(obs, actions, old_logp, advantages, returns, index, B, old_values)
        oc = _OptStateC(_ptr(opt.m, torch.float32, "m"), _ptr(opt.v, torch.float32, "v"), opt.step)
        _check(self.lib.hts_learner_step(self._h, C.byref(buf), _ptr(params, torch.float32, "params"), C.byref(oc),
                                         C.byref(hp), _ptr(stats, torch.float32, "stats")), "hts_learner_step")
        opt.step = oc.step

    def hts_learner_step_delayed(self, obs, actions, old_logp, advantages, returns, params_behaviour, params_target,
                                 opt: OptState, hp: HParams, index=None, B=None, stats=None, old_values=None):
        buf, _keep = self._buffer(obs, actions, old_logp, advantages, returns, index, B, old_values)
        oc = _OptStateC(_ptr(opt.m, torch.float32, "m"), _ptr(opt.v, torch.float32, "v"), opt.step)
        _check(self.lib.hts_learner_step_delayed(self._h, C.byref(buf),
                                                 _ptr(params_behaviour, torch.float32, "params_behaviour"),
                                                 _ptr(params_target, torch.float32, "params_target"), C.byref(oc),
                                                 C.byref(hp), _ptr(stats, torch.float32, "stats")),
               "hts_learner_step_delayed")
        opt.step = oc.step

    def hts_loss_and_grads(self, obs, actions, old_logp, advantages, returns, params, hp: HParams, grads, index=None,
                           B=None, stats=None, old_values=None):
        buf, _keep = self._buffer(obs, actions, old_logp, advantages, returns, index, B, old_values)
        _check(self.lib.hts_loss_and_grads(self._h, C.byref(buf), _ptr(params, torch.float32, "params"), C.byref(hp),
                                           _ptr(grads, torch.float32, "grads"), _ptr(stats, torch.float32, "stats")),
               "hts_loss_and_grads")

    def hts_adam_apply(self, params, grads, opt: OptState, hp: HParams):
        oc = _OptStateC(_ptr(opt.m, torch.float32, "m"), _ptr(opt.v, torch.float32, "v"), opt.step)
        _check(self.lib.hts_adam_apply(self._h, _ptr(params, torch.float32, "params"),
                                       _ptr(grads, torch.float32, "grads"), C.byref(oc), C.byref(hp), params.numel()),
               "hts_adam_apply")
        opt.step = oc.step

    def hts_test_gemm(self, precision, A, B, out):
        M, K = A.shape
        N = B.shape[0]
        _check(self.lib.hts_test_gemm(self._h, precision, _ptr(A, torch.float32, "A"), _ptr(B, torch.float32, "B"),
                                      _ptr(out, torch.float32, "out"), M, N, K), "hts_test_gemm")

    def profile_sites(self):
        return [self.lib.hts_profile_site_name(i).decode() for i in range(self.lib.hts_profile_site_count())]

    def hts_profile_begin(self, site: int):
        _check(self.lib.hts_profile_begin(self._h, site), "hts_profile_begin")

    def hts_profile_begin_sampled(self, site: int, every: int):
        _check(self.lib.hts_profile_begin_sampled(self._h, site, every), "hts_profile_begin_sampled")

    def hts_profile_end(self):
        """-> (timed launches, total milliseconds)."""
        n, ms = C.c_int32(), C.c_double()
        _check(self.lib.hts_profile_end(self._h, C.byref(n), C.byref(ms)), "hts_profile_end")
        return n.value, ms.value

    def hts_profile_overhead(self, reps=256):
        """-> mean milliseconds of an empty event bracket."""
        ms = C.c_double()
        _check(self.lib.hts_profile_overhead(self._h, reps, C.byref(ms)), "hts_profile_overhead")
        return ms.value

    @staticmethod
    def new_stats(device="cuda"):
        """Device buffer for hts_stats (6 floats + 1 int32, viewed as 7 float32 words)."""
        return torch.zeros(7, dtype=torch.float32, device=device)

    @staticmethod
    def read_stats(stats) -> dict:
        h = stats.cpu()
        d = {k: float(h[i]) for i, k in enumerate(STATS_FIELDS[:6])}
        d["nonfinite"] = int(h[6:7].view(torch.int32)[0])
        return d
