"""Seeded synthetic inputs for the LSH beam-search decode step.

This module only *draws numbers*: embedding matrices, permutation windows, top-frequent word
lists and per-step hidden states, with the shapes and distributions of the five benchmark
configurations (plus the paper-scale banding).  It holds none of the method's arithmetic (no hashing, no tables, no softmax),
so both the CPU oracle's tests and the HIP path's tests can consume the same bytes without
sharing any code of the method itself.

The paper's own workloads (trained LSTM translation models, Table 6) cannot be reproduced
without its corpora; these inputs keep the shapes of Table 1's model (d=1000, V=40000, beam 12)
and the beam sizes of Table 8, with clustered embeddings so that bucket sizes are skewed the way
real embeddings skew them.

Randomness: numpy's Philox counter-based generator keyed by (seed, stream id); every array is a
pure function of (config name, seed).
"""
from __future__ import annotations

import dataclasses

import numpy as np

F32 = 0
BF16 = 1


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    d: int            # hidden size
    V: int            # vocabulary
    S: int            # sentences per call
    B: int            # beams per sentence
    K: int            # WTA window
    P: int            # permutations (codes per vector)
    W: int            # bands
    T: int            # top-frequent words merged into every candidate list
    n_centres: int
    centre_std: float  # std of a cluster centre coordinate
    noise_std: float   # std of the per-word noise around its centre
    h_scale: float     # H = h_scale * E[w] + N(0, h_noise_std^2)
    h_noise_std: float
    steps: int
    e_dtype: int = F32
    uniform_row_frac: float = 0.0   # fraction of H rows drawn iid uniform (low-overlap buckets)
    zipf_s: float = 1.1
    threshold: int = 1              # t of Eq. 10

    @property
    def R(self) -> int:
        return self.S * self.B

    @property
    def u(self) -> int:
        return self.P // self.W


def _cfg(name, d, V, S, B, K, P, W, T, nc, steps, h_scale, *, tiny=False, e_dtype=F32, uni=0.0,
         t=1):
    if tiny:
        return Config(name, d, V, S, B, K, P, W, T, nc, 1.0, 0.3, 1.0, 0.2, steps, e_dtype, uni,
                      threshold=t)
    sd = 1.0 / np.sqrt(d)
    return Config(name, d, V, S, B, K, P, W, T, nc, sd, 0.3 * sd, h_scale, 0.3 * sd, steps,
                  e_dtype, uni, threshold=t)


CONFIGS = {
    "tiny": _cfg("tiny", 64, 1000, 1, 4, 8, 16, 4, 50, 32, 20, 1.0, tiny=True),
    "paper": _cfg("paper", 1000, 40000, 1, 12, 8, 32, 8, 1000, 1000, 50, 0.8),
    "batched": _cfg("batched", 1000, 40000, 32, 10, 8, 32, 8, 1000, 1000, 50, 0.8),
    "widebeam": _cfg("widebeam", 1000, 100000, 4, 50, 16, 48, 12, 2000, 2000, 40, 0.7),
    "largevocab": _cfg("largevocab", 1024, 200000, 64, 10, 8, 64, 16, 2000, 4000, 30, 0.8,
                       e_dtype=BF16, uni=0.10),
    # the paper's own banding {K, u, W} = {8, 3, 500} (Table 1's setting) with a hit threshold
    "paperscale": _cfg("paperscale", 1000, 40000, 1, 12, 8, 1500, 500, 1000, 1000, 20, 0.8, t=5),
}

_STREAMS = {"centres": 1, "noise": 2, "perms": 3, "targets": 4, "hnoise": 5, "uniform": 6,
            "unimask": 7}


def _rng(seed: int, stream: str) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, _STREAMS[stream]]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the 16-bit patterns as uint16."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_embeddings(cfg: Config, seed: int = 0) -> np.ndarray:
    """[V, d] fp32, or the uint16 bf16 bit patterns when cfg.e_dtype == BF16.
    Word j belongs to cluster j mod n_centres."""
    centres = _rng(seed, "centres").standard_normal((cfg.n_centres, cfg.d), dtype=np.float32)
    centres *= np.float32(cfg.centre_std)
    rng = _rng(seed, "noise")
    E = np.empty((cfg.V, cfg.d), dtype=np.float32)
    chunk = 16384
    for lo in range(0, cfg.V, chunk):
        hi = min(cfg.V, lo + chunk)
        blk = rng.standard_normal((hi - lo, cfg.d), dtype=np.float32)
        blk *= np.float32(cfg.noise_std)
        blk += centres[np.arange(lo, hi) % cfg.n_centres]
        E[lo:hi] = blk
    if cfg.e_dtype == BF16:
        return f32_to_bf16_bits(E)
    return E


def embeddings_as_f32(cfg: Config, E: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(E) if cfg.e_dtype == BF16 else E


def make_perms(cfg: Config, seed: int = 0) -> np.ndarray:
    """int32 [P, K]: row p holds the first K entries of a random permutation of 0..d-1."""
    rng = _rng(seed, "perms")
    out = np.empty((cfg.P, cfg.K), dtype=np.int32)
    for p in range(cfg.P):
        out[p] = rng.permutation(cfg.d)[: cfg.K]
    return out


def make_topfreq(cfg: Config) -> np.ndarray:
    """Word id = Zipf rank - 1, so the T most frequent words are ids 0..T-1."""
    return np.arange(cfg.T, dtype=np.int32)


def zipf_targets(cfg: Config, n: int, rng: np.random.Generator) -> np.ndarray:
    """n word ids with P(rank r) proportional to r^-s, truncated to V (inverse-CDF sampling)."""
    w = np.arange(1, cfg.V + 1, dtype=np.float64) ** (-cfg.zipf_s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    ids = np.searchsorted(cdf, rng.random(n), side="left")
    return np.minimum(ids, cfg.V - 1).astype(np.int64)


def make_hidden(cfg: Config, E: np.ndarray, seed: int = 0, steps: int | None = None) -> np.ndarray:
    """fp32 [steps, R, d]: H = h_scale * E[w] + noise, w Zipf-distributed; a fraction
    uniform_row_frac of the rows is replaced by iid uniform values of the same variance."""
    steps = cfg.steps if steps is None else steps
    n = steps * cfg.R
    w = zipf_targets(cfg, n, _rng(seed, "targets"))
    rows = embeddings_as_f32(cfg, E[w]) if cfg.e_dtype == BF16 else E[w]
    H = rows.astype(np.float32) * np.float32(cfg.h_scale)
    H += _rng(seed, "hnoise").standard_normal((n, cfg.d), dtype=np.float32) * np.float32(
        cfg.h_noise_std)
    if cfg.uniform_row_frac > 0.0:
        mask = _rng(seed, "unimask").random(n) < cfg.uniform_row_frac
        a = np.float32(np.sqrt(3.0) * cfg.centre_std)
        U = _rng(seed, "uniform").random((int(mask.sum()), cfg.d), dtype=np.float32)
        H[mask] = (U * np.float32(2.0) - np.float32(1.0)) * a
    return np.ascontiguousarray(H.reshape(steps, cfg.R, cfg.d))


def make_all(cfg: Config, seed: int = 0, steps: int | None = None):
    E = make_embeddings(cfg, seed)
    return E, make_perms(cfg, seed), make_topfreq(cfg), make_hidden(cfg, E, seed, steps)
