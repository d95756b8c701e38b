"""Seeded synthetic inputs: token streams and initial weights.

This module holds no arithmetic of the language model itself.  It only draws
random numbers: a counter-based 64-bit generator, a Zipf rank sampler working on
integer thresholds, sentence lengths, and the initial weight matrices.  Both the
CPU oracle's tests and the HIP path's tests/bench consume these arrays, so that
the two sides always see identical inputs.

Stand-in for the paper's corpora (Sec. 2.1 and Sec. 5.1: news/Wikipedia text
with a 64k-class vocabulary, a sentence marker every ~20-25 words, contiguous
text whose between-sentence context is kept): a Zipf-like unigram law over V ids
with id 0 reserved for the sentence marker where the configuration names one.
"""
from __future__ import annotations

import hashlib
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _chunked(n: int, fill, step: int = 1 << 22) -> None:
    """fill(a, m) for every chunk [a, a+m) of range(n).  Element i is a pure function of (seed, i), so the
    chunks are independent: large arrays are filled by a few threads (numpy releases the interpreter lock
    inside its loops); the result does not depend on the number of threads."""
    starts = range(0, n, step)
    workers = min(16, os.cpu_count() or 1, len(starts))
    if workers <= 1:
        for a in starts:
            fill(a, min(step, n - a))
        return
    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(lambda a: fill(a, min(step, n - a)), starts))


def counter_u64(seed: int, start: int, count: int) -> np.ndarray:
    """u[i] = mix64(seed + (start+i+1)*golden): a pure function of (seed, index).

    The mixer is the public SplitMix64 finaliser (xor-shift / multiply rounds).
    """
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _thresholds(weights: np.ndarray) -> np.ndarray:
    """Integer CDF thresholds thr[r] = floor(cdf_r * 2^64), last entry 2^64-1."""
    cdf = np.cumsum(weights.astype(np.float64))
    cdf /= cdf[-1]
    # cdf*2^64 overflows uint64 when cdf == 1.0; clip just below and pin the end.
    scaled = np.minimum(cdf * 18446744073709551616.0, 18446744073709549568.0)
    thr = scaled.astype(np.uint64)
    thr[-1] = np.uint64(0xFFFFFFFFFFFFFFFF)
    return thr


def zipf_thresholds(R: int, s: float) -> np.ndarray:
    return _thresholds(np.arange(1, R + 1, dtype=np.float64) ** (-s))


def poisson_thresholds(lam: float) -> np.ndarray:
    kmax = int(lam + 12.0 * np.sqrt(lam) + 20)
    k = np.arange(0, kmax + 1, dtype=np.float64)
    from math import lgamma
    logp = -lam + k * np.log(lam) - np.array([lgamma(v + 1.0) for v in k])
    return _thresholds(np.exp(logp))


def sample_from_thresholds(thr: np.ndarray, u: np.ndarray) -> np.ndarray:
    """index = #{r : thr[r] <= u}, by binary search on integers only."""
    idx = np.searchsorted(thr, u, side="right")
    return np.minimum(idx, len(thr) - 1).astype(np.int64)


def zipf_tokens(N: int, V: int, s: float, seed: int, sentence_lambda: float | None = None,
                markov_contexts: int = 0) -> np.ndarray:
    """N token ids in [0, V).

    sentence_lambda=None: id = rank-1 over R=V ranks.
    sentence_lambda=lam : words take ids 1..V-1 (R=V-1 ranks); id 0 is emitted after
    every max(1, Poisson(lam)) words; N counts the markers too.
    markov_contexts=K>0 : with probability 1/2 a word is relabelled by an affine map
    chosen by a hash of the two preceding latent ranks (gives the stream structure
    beyond unigram statistics while keeping a Zipf-like marginal).
    """
    if sentence_lambda is None:
        R = V
        base = 0
    else:
        R = V - 1
        base = 1
    thr = zipf_thresholds(R, s)
    tok = np.empty(N, dtype=np.int32)

    def fill(a, n):
        tok[a:a + n] = sample_from_thresholds(thr, counter_u64(seed, a, n)) + base
    _chunked(N, fill)
    if markov_contexts > 0:
        K = markov_contexts
        rng_a = counter_u64(seed ^ 0xA5A5A5A5, 0, K)
        a_k = (rng_a % np.uint64(V)).astype(np.int64)
        # make a_k coprime to V = 2^a 5^b style sizes: force odd and not a multiple of 5
        a_k |= 1
        a_k[a_k % 5 == 0] += 2
        c_k = (counter_u64(seed ^ 0x5A5A5A5A, 0, K) % np.uint64(V)).astype(np.int64)
        lat = tok.astype(np.int64) - base
        p1 = np.concatenate([[0], lat[:-1]])
        p2 = np.concatenate([[0, 0], lat[:-2]])
        ctx = ((p1 * 1000003 + p2 * 7919 + 12345) % K).astype(np.int64)
        coin = (counter_u64(seed ^ 0x0C0FFEE0, 0, N) >> np.uint64(63)).astype(bool)
        relab = (a_k[ctx] * lat + c_k[ctx]) % R
        lat = np.where(coin, relab, lat)
        tok = (lat + base).astype(np.int32)
    if sentence_lambda is not None:
        pthr = poisson_thresholds(sentence_lambda)
        nsent = int(N / max(1.0, sentence_lambda * 0.5)) + 16
        lens = np.maximum(1, sample_from_thresholds(pthr, counter_u64(seed ^ 0x53454E54, 0, nsent)))
        ends = np.cumsum(lens + 1) - 1
        ends = ends[ends < N]
        tok[ends] = 0
    return tok


def _uniform01(seed: int, start: int, count: int) -> np.ndarray:
    return ((counter_u64(seed, start, count) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def uniform_weights(shape, lo: float, hi: float, seed: int) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)

    def fill(a, m):
        out[a:a + m] = (lo + (hi - lo) * _uniform01(seed, a, m)).astype(np.float32)
    _chunked(n, fill)
    return out.reshape(shape)


def normal_weights(shape, std: float, seed: int) -> np.ndarray:
    """Box-Muller on pairs of counter words, fp64 then stored as fp32."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)

    def fill(a, m):
        u1 = _uniform01(seed, 2 * a, m)
        u2 = _uniform01(seed ^ 0x7777777, 2 * a, m)
        out[a:a + m] = (std * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    _chunked(n, fill)
    return out.reshape(shape)


@dataclass(frozen=True)
class Config:
    name: str
    V: int
    H: int
    B: int
    T: int
    N: int
    zipf_s: float
    sentence_lambda: float | None
    markov_contexts: int
    init: str            # "uniform" or "normal"
    init_scale: float
    lr: float
    precision: str       # "fp32" or "bf16"
    data_seed: int
    weight_seed: int


CONFIGS = {
    "cfg1": Config("cfg1", 1000, 64, 4, 8, 10_000, 1.1, None, 0, "uniform", 0.1, 0.1, "fp32", 0x5EED0001, 0x5EED1001),
    "cfg2": Config("cfg2", 10_000, 256, 32, 10, 1_000_000, 1.1, 20.0, 0, "uniform", 0.1, 0.1, "fp32", 0x5EED0002, 0x5EED1002),
    "cfg3": Config("cfg3", 64_000, 1024, 128, 20, 20_000_000, 1.05, 25.0, 0, "normal", 0.02, 0.05, "bf16", 0x5EED0003, 0x5EED1003),
    "cfg4": Config("cfg4", 100_000, 2048, 128, 20, 50_000_000, 1.0, None, 4096, "normal", 0.02, 0.02, "bf16", 0x5EED0004, 0x5EED1004),
    "cfg5": Config("cfg5", 100_000, 4096, 256, 32, 100_000_000, 1.0, 25.0, 0, "normal", 0.01, 0.01, "bf16", 0x5EED0005, 0x5EED1005),
    # the word-prediction model of Sec. 5.4 (vocabulary 10K, nstate 1024; the 512-unit layers are COMPRESSED_P)
    "wp10k": Config("wp10k", 10_000, 1024, 128, 20, 5_000_000, 1.05, 25.0, 0, "normal", 0.02, 0.05, "bf16", 0x5EED0006, 0x5EED1006),
}
COMPRESSED_P = 512


def make_tokens(cfg: Config, N: int | None = None) -> np.ndarray:
    return zipf_tokens(cfg.N if N is None else N, cfg.V, cfg.zipf_s, cfg.data_seed,
                       cfg.sentence_lambda, cfg.markov_contexts)


def make_weights(V: int, H: int, init: str, scale: float, seed: int):
    """Returns fp32 (E[V][H], U[H][H], Wo[V][H], b[V]); b is zero."""
    f = (lambda shp, sd: uniform_weights(shp, -scale, scale, sd)) if init == "uniform" \
        else (lambda shp, sd: normal_weights(shp, scale, sd))
    E = f((V, H), seed + 11)
    U = f((H, H), seed + 22)
    Wo = f((V, H), seed + 33)
    b = np.zeros(V, dtype=np.float32)
    return E, U, Wo, b


def make_compressed_weights(V: int, H: int, P: int, init: str, scale: float, seed: int):
    """Returns fp32 (E[V][P], A[H][P], U[H][H], C[P][H], b[V]) of the compressed architecture; b is zero."""
    f = (lambda shp, sd: uniform_weights(shp, -scale, scale, sd)) if init == "uniform" \
        else (lambda shp, sd: normal_weights(shp, scale, sd))
    return f((V, P), seed + 11), f((H, P), seed + 44), f((H, H), seed + 22), f((P, H), seed + 55), \
        np.zeros(V, dtype=np.float32)


def unigram_noise(tok: np.ndarray, V: int):
    """Noise distribution for a contrastive criterion: the add-one-smoothed unigram of a token array.

    Returns (lnq[V] float32, thr[V] uint64): log-probabilities as both sides consume them, and the
    integer thresholds noise words are drawn with."""
    counts = np.bincount(tok, minlength=V).astype(np.float64) + 1.0
    q = counts / counts.sum()
    return np.log(q).astype(np.float32), _thresholds(q)


def noise_words(thr: np.ndarray, K: int, seed: int, window: int) -> np.ndarray:
    """K noise ids for window number `window`, drawn i.i.d. from the thresholds' distribution: draw j
    of window k is a pure function of (seed, k*K + j)."""
    u = counter_u64(seed, window * K, K)
    return sample_from_thresholds(thr, u).astype(np.int32)


def sha256_of(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
