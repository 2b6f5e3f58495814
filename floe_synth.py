"""Seeded synthetic inputs for the FloE decode path (shared by the tests, the benchmark and the smoke run).

This module holds NO arithmetic of the method itself: it only draws reproducible pseudo-random
tensors with the shapes and value distributions of the paper's workloads (Mixtral-shaped SwiGLU
experts, Sec. 4.1 / Table 1 and App. F give d=4096, f=14336) and lays them out in the channel-major
and compact [gate | down] layouts (Sec. 3.4.2) that both the CPU oracle and the HIP library read.

Generator: counter-based SplitMix64 (Steele, Lea, Flood 2014 finaliser) -> Box-Muller.
Element n of stream `key` never depends on how many other elements were drawn, so every tensor can be
regenerated alone, in chunks, or in parallel with identical bits.  Values are drawn in float64 and
rounded ONCE to fp16 (round-to-nearest-even); oracle and GPU receive the same fp16 bit patterns.
"""
from __future__ import annotations

import concurrent.futures as _fut
import os

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 18  # pairs per work item (keeps every temporary cache-resident)

# tensor kinds (part of the stream key)
KIND_W_GATE, KIND_W_UP, KIND_W_DOWN, KIND_X, KIND_ROUTER, KIND_MISC = 1, 2, 3, 4, 5, 6


def _mix_inplace(z: np.ndarray) -> np.ndarray:
    """SplitMix64 output function applied in place to a uint64 array."""
    t = z >> np.uint64(30)
    z ^= t
    z *= _M1
    np.right_shift(z, np.uint64(27), out=t)
    z ^= t
    z *= _M2
    np.right_shift(z, np.uint64(31), out=t)
    z ^= t
    return z


def _mix_scalar(z: int) -> int:
    m = (1 << 64) - 1
    z &= m
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    return z ^ (z >> 31)


def stream_key(seed: int, config: int, kind: int, layer: int = 0, expert: int = 0, token: int = 0) -> int:
    """Hash (seed, config id, tensor kind, layer, expert, token) into a 64-bit stream key."""
    k = _mix_scalar(seed + 0x9E3779B97F4A7C15)
    for part in (config, kind, layer, expert, token):
        k = _mix_scalar(k ^ _mix_scalar((part + 1) * 0x9E3779B97F4A7C15))
    return k


def raw_u64(key: int, start: int, count: int) -> np.ndarray:
    """Outputs start..start+count-1 of stream `key`: mix(key + (n+1)*gamma) (wrapping 64-bit)."""
    with np.errstate(over="ignore"):
        n = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        n *= _GAMMA
        n += np.uint64(key)
        return _mix_inplace(n)


def _normal_pairs(key: int, p0: int, p1: int, out: np.ndarray) -> None:
    """Fill out[2*p0 : 2*p1] with N(0,1) draws: pair p uses outputs 2p and 2p+1 of the stream."""
    with np.errstate(over="ignore"):
        u = raw_u64(key, 2 * p0, 2 * (p1 - p0))
    a = (u[0::2] >> np.uint64(11)).astype(np.float64)
    b = (u[1::2] >> np.uint64(11)).astype(np.float64)
    a += 1.0
    a *= 2.0 ** -53          # (0, 1]
    b *= 2.0 ** -53 * 2.0 * np.pi  # [0, 2pi)
    np.log(a, out=a)
    a *= -2.0
    np.sqrt(a, out=a)
    seg = out[2 * p0: 2 * p1]
    seg[0::2] = a * np.cos(b)
    seg[1::2] = a * np.sin(b)


def normal(key: int, count: int, sigma: float = 1.0, workers: int | None = None) -> np.ndarray:
    """`count` draws of N(0, sigma^2) as float64 (element n is a pure function of (key, n))."""
    npairs = (count + 1) // 2
    out = np.empty(2 * npairs, dtype=np.float64)
    spans = [(p, min(p + _CHUNK, npairs)) for p in range(0, npairs, _CHUNK)]
    if workers is None:
        workers = min(8, os.cpu_count() or 1)
    if len(spans) > 1 and workers > 1:
        with _fut.ThreadPoolExecutor(workers) as ex:
            list(ex.map(lambda s: _normal_pairs(key, s[0], s[1], out), spans))
    else:
        for p0, p1 in spans:
            _normal_pairs(key, p0, p1, out)
    out = out[:count]
    if sigma != 1.0:
        out *= sigma
    return out


def normal_f16(key: int, shape, sigma: float = 1.0) -> np.ndarray:
    """N(0, sigma^2) rounded once to fp16 (RNE), C-contiguous array of `shape`."""
    n = int(np.prod(shape))
    return normal(key, n, sigma).astype(np.float16).reshape(shape)


# --------------------------------------------------------------------------------------------
# Workload recipes (benchmark configs; weights ~ N(0, 0.02^2), activations ~ N(0, 1))
# --------------------------------------------------------------------------------------------
W_SIGMA = 0.02


def expert_weights(seed: int, config: int, d: int, f: int, layer: int = 0, expert: int = 0):
    """One SwiGLU expert in channel-major form.

    Returns (w_up_cm [f][d], gd [f][2][d]) as fp16: row j of w_up_cm is column j of W_up
    (Eq. 1 uses x as a row vector, W_up in R^{d x f}); gd[j][0] is column j of W_gate and gd[j][1]
    is row j of W_down, i.e. the co-located compact chunk of channel j (Sec. 3.4.2).
    """
    w_up = normal_f16(stream_key(seed, config, KIND_W_UP, layer, expert), (f, d), W_SIGMA)
    gd = np.empty((f, 2, d), dtype=np.float16)
    gd[:, 0, :] = normal_f16(stream_key(seed, config, KIND_W_GATE, layer, expert), (f, d), W_SIGMA)
    gd[:, 1, :] = normal_f16(stream_key(seed, config, KIND_W_DOWN, layer, expert), (f, d), W_SIGMA)
    return w_up, gd


def tokens(seed: int, config: int, T: int, d: int, layer: int = 0) -> np.ndarray:
    """T hidden states x ~ N(0,1) as fp16 [T][d]; token t is its own stream."""
    x = np.empty((T, d), dtype=np.float16)
    for t in range(T):
        x[t] = normal_f16(stream_key(seed, config, KIND_X, layer, 0, t), (d,), 1.0)
    return x


def router_weights(seed: int, config: int, n_experts: int, d: int, layer: int = 0) -> np.ndarray:
    """Router matrix, channel-major [n_experts][d] fp16 ~ N(0, 0.02^2)."""
    return normal_f16(stream_key(seed, config, KIND_ROUTER, layer), (n_experts, d), W_SIGMA)


def random_channel_subset(seed: int, config: int, f: int, count: int, salt: int = 0) -> np.ndarray:
    """`count` distinct channel ids in ascending order (for the transfer experiment of Sec. 4.1)."""
    u = raw_u64(stream_key(seed, config, KIND_MISC, salt), 0, f)
    order = np.argsort(u, kind="stable")
    return np.sort(order[:count]).astype(np.int32)
