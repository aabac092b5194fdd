"""Seeded synthetic inputs for the fused projection + cross-entropy path.

This module holds none of the method's arithmetic: it only makes the arrays
(hidden states, vocabulary weights, integer targets) that both the HIP path
and the CPU oracle are handed, so that they see identical bytes.  It imports
neither of them.

Generator.  Counter based, so any element can be produced on its own and the
values do not depend on a library's random stream:

    key(seed, stream) = mix(mix(seed) + stream)
    word(j)           = mix(key + (j + 1) * 0x9E3779B97F4A7C15)     (splitmix64)
    u1 = (hi32(word) + 1) / 2^32  in (0, 1],   u2 = lo32(word) / 2^32
    normal pair j     = sqrt(-2 ln u1) * (cos 2 pi u2, sin 2 pi u2)  (Box-Muller)

element 2j takes the cosine, 2j+1 the sine.  Values are formed in fp64, cast
to fp32 and, for bf16 tensors, rounded once to bf16 (round to nearest even)
on the host; bf16 tensors are carried as uint16 bit patterns.

The five workloads are the benchmark shapes this build is measured on
(they stand in for the activations, weights and token streams of the named
model shapes; the paper's own evaluation, Table 1, is likewise a pure shape
sweep on synthetic data).  Targets are uniform over [0, V) or a truncated
Zipf law on ranks 1..V (pmf proportional to rank^-s, token id = rank - 1,
drawn by inverse CDF); ignored rows are exactly round(frac * N) rows chosen
by a seeded ranking and set to ``ignore_index``.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

STREAM_H, STREAM_W, STREAM_Y, STREAM_MASK = 1, 2, 3, 4


def _mix(z):
    """splitmix64 output function on a uint64 array (wrap-around arithmetic)."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed, stream):
    with np.errstate(over="ignore"):
        k = _mix(np.array([seed], dtype=np.uint64) + _GOLD)
        return _mix(k + np.uint64(stream) + _GOLD)[0]


def words(seed, stream, start, count):
    """64-bit words start .. start+count-1 of the (seed, stream) sequence."""
    with np.errstate(over="ignore"):
        j = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        return _mix(_key(seed, stream) + j * _GOLD)


def _normal_pairs(seed, stream, pair_start, pair_count):
    w = words(seed, stream, pair_start, pair_count)
    u1 = ((w >> np.uint64(32)).astype(np.float64) + 1.0) * (1.0 / 4294967296.0)
    u2 = (w & np.uint64(0xFFFFFFFF)).astype(np.float64) * (1.0 / 4294967296.0)
    r = np.sqrt(-2.0 * np.log(u1))
    th = (2.0 * np.pi) * u2
    out = np.empty(2 * pair_count, dtype=np.float32)
    out[0::2] = r * np.cos(th)
    out[1::2] = r * np.sin(th)
    return out


def normal_f32(seed, stream, n, std=1.0, threads=None):
    """n values ~ N(0, std^2) as fp32."""
    n_pairs = (n + 1) // 2
    chunk = 1 << 19
    out = np.empty(2 * n_pairs, dtype=np.float32)

    def work(p0):
        p1 = min(n_pairs, p0 + chunk)
        v = _normal_pairs(seed, stream, p0, p1 - p0)
        if std != 1.0:
            v *= np.float32(std)
        out[2 * p0:2 * p1] = v

    starts = range(0, n_pairs, chunk)
    threads = threads or min(16, os.cpu_count() or 1)
    if threads > 1 and n_pairs > chunk:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, starts))
    else:
        for p0 in starts:
            work(p0)
    return out[:n]


def f32_to_bf16_bits(x):
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def uniform01(seed, stream, n):
    """n values in [0, 1) with 53 random bits."""
    return (words(seed, stream, 0, n) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def targets_uniform(seed, n, V):
    w = words(seed, STREAM_Y, 0, n) >> np.uint64(32)
    return ((w * np.uint64(V)) >> np.uint64(32)).astype(np.int64)


def targets_zipf(seed, n, V, s):
    pmf = np.arange(1, V + 1, dtype=np.float64) ** (-float(s))
    cdf = np.cumsum(pmf)
    cdf /= cdf[-1]
    ids = np.searchsorted(cdf, uniform01(seed, STREAM_Y, n), side="right")
    return np.minimum(ids, V - 1).astype(np.int64)


def ignored_rows(seed, n, frac):
    """Exactly round(frac * n) row indices, chosen by ranking a seeded word per row."""
    k = int(round(frac * n))
    if k == 0:
        return np.empty(0, dtype=np.int64)
    order = np.argsort(words(seed, STREAM_MASK, 0, n), kind="stable")
    return np.sort(order[:k]).astype(np.int64)


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    d: int
    V: int
    dtype: str              # "f32" or "bf16": storage type of H, W, dH, dW
    targets: str            # "uniform" or "zipf"
    zipf_s: float = 0.0
    ignore_frac: float = 0.0
    reduction: str = "mean"
    seed: int = 0
    h_std: float = 1.0
    w_std: float = 0.02
    ignore_index: int = -100

    @property
    def naive_logits_bytes(self):
        return self.N * self.V * 4


WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", 256, 256, 4096, "f32", "uniform", ignore_frac=0.05, seed=1001),
    "gpt2_small": Workload("gpt2_small", 4096, 768, 50257, "bf16", "zipf", zipf_s=1.1, seed=1002),
    "llama3_8b": Workload("llama3_8b", 8192, 4096, 128256, "bf16", "uniform", ignore_frac=0.10, seed=1003),
    "large_vocab": Workload("large_vocab", 8192, 3072, 256000, "bf16", "zipf", zipf_s=1.05,
                            reduction="sum", seed=1004),
    "long_seq": Workload("long_seq", 131072, 4096, 128256, "bf16", "uniform", ignore_frac=0.02, seed=1005),
}


def make_targets(wl: Workload):
    if wl.targets == "uniform":
        y = targets_uniform(wl.seed, wl.N, wl.V)
    elif wl.targets == "zipf":
        y = targets_zipf(wl.seed, wl.N, wl.V, wl.zipf_s)
    else:
        raise ValueError(wl.targets)
    y[ignored_rows(wl.seed, wl.N, wl.ignore_frac)] = wl.ignore_index
    return y


def make_inputs(wl: Workload):
    """Arrays of one workload.

    Returns a dict with ``y`` (int64[N]) and, for "f32", ``H``/``W`` as fp32
    arrays; for "bf16", ``H``/``W`` as uint16 bit patterns of shape [N,d] /
    [V,d] (widen with ``to_f64``).
    """
    H = normal_f32(wl.seed, STREAM_H, wl.N * wl.d, wl.h_std).reshape(wl.N, wl.d)
    W = normal_f32(wl.seed, STREAM_W, wl.V * wl.d, wl.w_std).reshape(wl.V, wl.d)
    if wl.dtype == "bf16":
        H, W = f32_to_bf16_bits(H), f32_to_bf16_bits(W)
    elif wl.dtype != "f32":
        raise ValueError(wl.dtype)
    return dict(H=H, W=W, y=make_targets(wl))


def to_f64(a):
    """Exact fp64 image of a stored tensor (fp32 array or bf16 bit patterns)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)
