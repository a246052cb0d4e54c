"""Seeded synthetic inputs for the actor / returns / learner path.

This module only *generates data* (frames, rewards, dones, initial weights,
minibatch permutations).  It contains none of the method's arithmetic and is
the one module that both the CPU oracle's tests and the GPU path's tests and
benchmark may import, so that both sides see byte-identical inputs.

Every array is a pure function of (master seed, stream id, element index):
a SplitMix64-style counter hash, so any slice can be regenerated on its own
and nothing depends on call order.

Stand-ins (the paper's simulators are not available): Atari-shaped frames
(4x84x84 stacked grey frames) and GFootball "extracted map"-shaped frames
(16x72x96 sparse planes) -- see the paper's experiment section for the
environments these replace.
"""
from __future__ import annotations

import numpy as np

MASTER_SEED = 201209849

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)

# stream ids (one per kind of array)
S_OBS, S_REW, S_DONE, S_PARAM, S_PERM, S_VAL, S_MISC = 1, 2, 3, 4, 5, 6, 7


def _mix(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (z ^ (z >> _U64(30))) * _M1
        z = (z ^ (z >> _U64(27))) * _M2
        return z ^ (z >> _U64(31))


def bits64(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit words: word i = hash(seed, stream, offset + i)."""
    with np.errstate(over="ignore"):
        base = _mix(np.array([(seed * 0x2545F4914F6CDD1D + stream) & 0xFFFFFFFFFFFFFFFF], dtype=_U64))[0]
        idx = np.arange(offset, offset + n, dtype=_U64)
        return _mix(base + (idx + _U64(1)) * _GOLDEN)


def uniform01(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """float64 uniforms in [0,1) with 53 random bits."""
    return (bits64(seed, stream, n, offset) >> _U64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """float64 standard normals (Box-Muller on two counter streams)."""
    u1 = uniform01(seed, stream, n, 2 * offset)
    u2 = uniform01(seed, stream + 1000, n, 2 * offset)
    return np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * np.pi * u2)


def randint(seed: int, stream: int, n: int, lo: int, hi: int, offset: int = 0) -> np.ndarray:
    """int64 uniform integers in [lo, hi]."""
    span = hi - lo + 1
    return (bits64(seed, stream, n, offset) % _U64(span)).astype(np.int64) + lo


# ----------------------------------------------------------------------------
# observations
# ----------------------------------------------------------------------------

def obs_uniform(seed: int, count: int, C: int = 4, H: int = 84, W: int = 84) -> np.ndarray:
    """uint8 [count, C, H, W], i.i.d. uniform 0..255 (tiny-A2C config)."""
    n = count * C * H * W
    return (bits64(seed, S_OBS, n) >> _U64(56)).astype(np.uint8).reshape(count, C, H, W)


def obs_atari(seed: int, T: int, N: int, C: int = 4, H: int = 84, W: int = 84) -> np.ndarray:
    """uint8 [T, N, C, H, W] pixel-correlated frame stacks.

    Per environment a base image is a clamped raster random walk (start
    U{0..255}, steps U{-8..8}).  Raw frame f is the base image rolled by an
    accumulated (dx, dy) drift in {-1,0,1}^2 per frame plus +-2 noise.  The
    observation at step t stacks raw frames t..t+C-1, so channel c at step t
    equals channel c+1 at step t-1.
    """
    out = np.empty((T, N, C, H, W), dtype=np.uint8)
    nraw = T + C - 1
    for e in range(N):
        es = seed * 1315423911 + e * 2654435761 + 17
        steps = randint(es, S_OBS, H * W, -8, 8)
        start = int(randint(es, S_OBS + 1, 1, 0, 255)[0])
        # raster walk, one image row at a time: each row continues from the clipped end of the previous one
        walk = np.empty(H * W, dtype=np.int64)
        v = start
        st = steps.reshape(H, W)
        for r in range(H):
            row = np.cumsum(st[r]) + v
            row = np.clip(row, 0, 255)
            walk[r * W:(r + 1) * W] = row
            v = int(row[-1])
        base = walk.reshape(H, W)
        drift = randint(es, S_OBS + 2, 2 * nraw, -1, 1).reshape(nraw, 2)
        pos = np.cumsum(drift, axis=0)
        raw = np.empty((nraw, H, W), dtype=np.uint8)
        for f in range(nraw):
            img = np.roll(base, (int(pos[f, 0]), int(pos[f, 1])), axis=(0, 1))
            noise = randint(es, S_OBS + 3, H * W, -2, 2, offset=f * H * W).reshape(H, W)
            raw[f] = np.clip(img + noise, 0, 255).astype(np.uint8)
        for t in range(T):
            out[t, e] = raw[t:t + C]
    return out


def obs_football(seed: int, T: int, N: int, frames: int = 4, planes: int = 4, H: int = 72, W: int = 96,
                 density: float = 0.02) -> np.ndarray:
    """uint8 [T, N, frames*planes, H, W]: stacked sparse planes, value 255 where set.

    Each plane holds round(density*H*W) points doing a lazy random walk, so
    consecutive frames are correlated and about `density` of pixels are 255.
    Channel index = frame*planes + plane; the stack at step t holds raw
    frames t..t+frames-1.
    """
    npts = int(round(density * H * W))
    nraw = T + frames - 1
    out = np.zeros((T, N, frames * planes, H, W), dtype=np.uint8)
    for e in range(N):
        raw = np.zeros((nraw, planes, H, W), dtype=np.uint8)
        for p in range(planes):
            es = seed * 40503 + e * 2654435761 + p * 97 + 5
            y0 = randint(es, S_OBS, npts, 0, H - 1)
            x0 = randint(es, S_OBS + 1, npts, 0, W - 1)
            dy = randint(es, S_OBS + 2, npts * nraw, -1, 1).reshape(nraw, npts)
            dx = randint(es, S_OBS + 3, npts * nraw, -1, 1).reshape(nraw, npts)
            ys = (y0[None, :] + np.cumsum(dy, axis=0)) % H
            xs = (x0[None, :] + np.cumsum(dx, axis=0)) % W
            for f in range(nraw):
                raw[f, p, ys[f], xs[f]] = 255
        for t in range(T):
            out[t, e] = raw[t:t + frames].reshape(frames * planes, H, W)
    return out


# ----------------------------------------------------------------------------
# rewards / dones / values
# ----------------------------------------------------------------------------

def rewards_ternary(seed: int, T: int, N: int, p_nonzero: float = 0.1) -> np.ndarray:
    """float32 [T,N] in {-1,0,1}; P(-1) = P(+1) = p_nonzero/2."""
    u = uniform01(seed, S_REW, T * N)
    r = np.zeros(T * N, dtype=np.float32)
    r[u < p_nonzero / 2] = -1.0
    r[u >= 1.0 - p_nonzero / 2] = 1.0
    return r.reshape(T, N)


def rewards_score_clipped(seed: int, T: int, N: int) -> np.ndarray:
    """Raw integer score (0 w.p. 0.9 else uniform in -10..10 without 0), clipped to [-1,1]."""
    u = uniform01(seed, S_REW, T * N)
    mag = randint(seed, S_REW + 1, T * N, 1, 10)
    sgn = np.where(bits64(seed, S_REW + 2, T * N) & _U64(1), 1, -1)
    raw = np.where(u < 0.9, 0, mag * sgn)
    return np.clip(raw, -1, 1).astype(np.float32).reshape(T, N)


def dones_bernoulli(seed: int, T: int, N: int, p: float) -> np.ndarray:
    return (uniform01(seed, S_DONE, T * N) < p).astype(np.uint8).reshape(T, N)


def normal_f32(seed: int, stream: int, shape) -> np.ndarray:
    n = int(np.prod(shape))
    return normal(seed, stream, n).astype(np.float32).reshape(shape)


# ----------------------------------------------------------------------------
# network shapes and initial weights (an *input* of the method, not part of it)
# ----------------------------------------------------------------------------

def conv_out(size: int, k: int, s: int) -> int:
    return (size - k) // s + 1


def param_shapes(C: int, H: int, W: int, A: int, convs=((32, 8, 4), (64, 4, 2), (64, 3, 1)), hidden: int = 512):
    """List of (name, shape) in flat packing order: per conv w,b; fc w,b; pi w,b; v w,b."""
    shapes = []
    cin, h, w = C, H, W
    for i, (co, k, s) in enumerate(convs):
        shapes.append((f"conv{i + 1}.w", (co, cin, k, k)))
        shapes.append((f"conv{i + 1}.b", (co,)))
        cin, h, w = co, conv_out(h, k, s), conv_out(w, k, s)
    F = cin * h * w
    shapes += [("fc.w", (hidden, F)), ("fc.b", (hidden,)), ("pi.w", (A, hidden)), ("pi.b", (A,)),
               ("v.w", (1, hidden)), ("v.b", (1,))]
    return shapes


def param_count(C: int, H: int, W: int, A: int, **kw) -> int:
    return sum(int(np.prod(s)) for _, s in param_shapes(C, H, W, A, **kw))


def init_params(seed: int, C: int, H: int, W: int, A: int, bias_scale: float = 0.0, **kw) -> np.ndarray:
    """float32 flat vector: He-normal N(0, 2/fan_in) weights; biases zero (or small normal if bias_scale>0)."""
    parts = []
    for i, (name, shp) in enumerate(param_shapes(C, H, W, A, **kw)):
        n = int(np.prod(shp))
        if name.endswith(".w"):
            fan_in = int(np.prod(shp[1:]))
            parts.append(normal(seed, S_PARAM + 10 * i, n) * np.sqrt(2.0 / fan_in))
        else:
            parts.append(normal(seed, S_PARAM + 10 * i, n) * bias_scale)
    return np.concatenate(parts).astype(np.float32)


def split_params(flat: np.ndarray, C: int, H: int, W: int, A: int, **kw) -> dict:
    out, off = {}, 0
    for name, shp in param_shapes(C, H, W, A, **kw):
        n = int(np.prod(shp))
        out[name] = flat[off:off + n].reshape(shp)
        off += n
    assert off == flat.size
    return out


def permutation(seed: int, n: int, epoch: int = 0) -> np.ndarray:
    """int32 permutation of 0..n-1 (argsort of counter-hash keys; ties impossible in practice)."""
    keys = bits64(seed, S_PERM + 100 * epoch, n)
    return np.argsort(keys, kind="stable").astype(np.int32)
