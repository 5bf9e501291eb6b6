"""Seeded synthetic inputs for SBO dictionary learning (test/bench inputs only).

This module only *draws inputs*: planted unions of orthonormal bases, sparse
single-block signals, additive noise and random initial dictionaries.  It holds
none of the method's arithmetic (no coding, grouping, accumulation or SVD
update) and is the one module that both the CPU oracle's tests and the HIP
path's tests/bench may share.

The workloads stand in for the paper's 8x8 image-patch training sets
(Section 4: p = 64, m in the tens of thousands, s0 = 4..12, K = 8..64); the
images themselves are not used.

Layouts
-------
Y : (m, p) float32, signal-major  (row i = signal y_i; equals column-major p x m)
D : (K, p, p) float32, atom-major (D[j, k, :] = atom k of Q_j = column k of Q_j)
"""
from __future__ import annotations

import dataclasses
import numpy as np

BASE_SEED = 14124944 * 10


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    number: int          # 1-based index used to derive the seed
    p: int
    K: int
    m: int
    s0: int
    iters: int
    snr_db: float | None  # None = noiseless
    coef: str = "normal"  # "normal" | "normal_x_uniform"
    zipf_s: float | None = None


CONFIGS = {
    "tiny": Config("tiny", 1, p=16, K=4, m=1024, s0=3, iters=5, snr_db=None),
    "patch8": Config("patch8", 2, p=64, K=16, m=16384, s0=6, iters=10, snr_db=20.0),
    "headline": Config("headline", 3, p=64, K=32, m=262144, s0=8, iters=10, snr_db=20.0,
                       coef="normal_x_uniform"),
    "patch16": Config("patch16", 4, p=256, K=16, m=131072, s0=12, iters=5, snr_db=25.0),
    "skew": Config("skew", 5, p=64, K=128, m=1048576, s0=6, iters=5, snr_db=20.0, zipf_s=1.1),
}


def random_onb(rng: np.random.Generator, p: int) -> np.ndarray:
    """One Haar-distributed orthonormal basis, fp64, as a p x p matrix whose
    columns are the atoms (QR of a Gaussian matrix, signs fixed so diag(R) > 0)."""
    a = rng.standard_normal((p, p))
    q, r = np.linalg.qr(a)
    s = np.sign(np.diag(r))
    s[s == 0] = 1.0
    return q * s[None, :]


def random_dictionary(rng: np.random.Generator, K: int, p: int) -> np.ndarray:
    """K random orthonormal bases, fp64, atom-major (K, p, p)."""
    return np.stack([random_onb(rng, p).T.copy() for _ in range(K)])


def _random_supports(rng: np.random.Generator, m: int, p: int, s0: int) -> np.ndarray:
    """Uniformly random s0-subsets of {0..p-1}, one per signal, ascending."""
    out = np.empty((m, s0), dtype=np.int32)
    step = 65536
    for a in range(0, m, step):
        b = min(m, a + step)
        keys = rng.random((b - a, p))
        idx = np.argpartition(keys, s0 - 1, axis=1)[:, :s0]
        out[a:b] = np.sort(idx, axis=1)
    return out


@dataclasses.dataclass
class Problem:
    cfg: Config
    Y: np.ndarray          # (m, p) float32
    D_planted: np.ndarray  # (K, p, p) float32 atom-major
    D_init: np.ndarray     # (K, p, p) float32 atom-major
    blk: np.ndarray        # (m,) int32 planted block
    supp: np.ndarray       # (m, s0) int32 planted support, ascending
    coef: np.ndarray       # (m, s0) float64 planted coefficients
    Y64: np.ndarray | None = None          # unrounded clean+noise signals (small configs only)
    D_planted64: np.ndarray | None = None  # unrounded planted dictionary


def generate(cfg: Config, m: int | None = None, keep_fp64: bool = False,
             seed_offset: int = 0) -> Problem:
    """Draw one problem instance.  `m` overrides the number of signals (a prefix
    of a longer stream is NOT the same draw; the override simply draws fewer)."""
    m = cfg.m if m is None else int(m)
    p, K, s0 = cfg.p, cfg.K, cfg.s0
    rng = np.random.default_rng(BASE_SEED + cfg.number + 1000 * seed_offset)
    rng_init = np.random.default_rng(BASE_SEED + cfg.number + 5 + 1000 * seed_offset)

    Dp = random_dictionary(rng, K, p)                       # fp64 atom-major
    if cfg.zipf_s is None:
        blk = rng.integers(0, K, size=m).astype(np.int32)
    else:
        w = (np.arange(K) + 1.0) ** (-cfg.zipf_s)
        blk = rng.choice(K, size=m, p=w / w.sum()).astype(np.int32)
    supp = _random_supports(rng, m, p, s0)
    coef = rng.standard_normal((m, s0))
    if cfg.coef == "normal_x_uniform":
        coef = coef * rng.uniform(0.5, 2.0, size=(m, s0))

    Y = np.empty((m, p), dtype=np.float64)
    step = 32768
    for a in range(0, m, step):
        b = min(m, a + step)
        atoms = Dp[blk[a:b, None], supp[a:b]]               # (n, s0, p)
        Y[a:b] = np.einsum("nt,ntd->nd", coef[a:b], atoms)
    if cfg.snr_db is not None:
        noise = rng.standard_normal((m, p))
        scale = np.sqrt((Y ** 2).sum() / ((noise ** 2).sum() * 10.0 ** (cfg.snr_db / 10.0)))
        Y += scale * noise

    D_init = random_dictionary(rng_init, K, p)
    return Problem(cfg=cfg, Y=Y.astype(np.float32), D_planted=Dp.astype(np.float32),
                   D_init=D_init.astype(np.float32), blk=blk, supp=supp, coef=coef,
                   Y64=Y if keep_fp64 else None, D_planted64=Dp if keep_fp64 else None)


def custom(name: str, p: int, K: int, m: int, s0: int, snr_db: float | None = 20.0,
           number: int = 99, **kw) -> Config:
    """A config outside the five named ones (ragged sizes, edge cases)."""
    return Config(name, number, p=p, K=K, m=m, s0=s0, iters=kw.pop("iters", 3), snr_db=snr_db, **kw)
