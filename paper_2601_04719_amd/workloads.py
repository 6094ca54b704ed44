"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and shapes them; it holds none of the
quantization method's arithmetic, so both the CPU oracle's tests and the HIP
library's tests may feed from it.  numpy only (no torch, no GPU).

Recipe (all draws from numpy Generator(PCG64(SeedSequence([seed, cfg, tensor,
stream, chunk]))); data are drawn in float64, multiplied by the per-channel
spread, then rounded once to float32):

  cfg 1  [1024 x 64]        x = z*s_d, z~N(0,1), s_d = exp(U(ln .1, ln 2));   16 N(0,1) queries
  cfg 2  [32768 x 128]      same law, 4 distinct outlier channels x20;        64 queries
  cfg 3  [8,32,4096,128]    z*s[h,d], s = exp(U(ln .05, ln 4)) per (h,d),
                            shared by the 8 batch entries; tensors K (0), V (1)
  cfg 4  [16384 x 8192]     t_4 * s_d, s_d = exp(U(ln .1, ln 2));             64 queries
  cfg 5  [131072 x 8192]    t_3 * s_d, 82 channels (1 %) identically +0.0

Rows are generated in fixed-size chunks (CHUNK_ELEMS elements, whole rows) so
any row range can be produced without the rest and the bytes do not depend on
the number of worker threads.
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
import math
import os

import numpy as np

CHUNK_ELEMS = 1 << 21

STREAM_SPREAD = 0
STREAM_SPECIAL = 1
STREAM_DATA = 2
STREAM_QUERIES = 3


@dataclass(frozen=True)
class Config:
    cfg: int
    batch: int          # leading B*H (1 for a plain matrix)
    N: int              # tokens
    D: int              # channels
    law: str            # "normal" or "t"
    nu: float           # Student-t degrees of freedom (0 for normal)
    spread_lo: float
    spread_hi: float
    n_queries: int
    heads: int = 1      # cfg 3: spread drawn per (head, channel), shared over B
    n_outlier: int = 0  # channels multiplied by 20
    n_zero: int = 0     # channels forced to +0.0

    @property
    def elements(self):
        return self.batch * self.N * self.D

    @property
    def name(self):
        if self.batch == 1:
            return "cfg%d[%dx%d]" % (self.cfg, self.N, self.D)
        return "cfg%d[%dx%dx%d]" % (self.cfg, self.batch, self.N, self.D)


CONFIGS = {
    1: Config(1, 1, 1024, 64, "normal", 0.0, 0.1, 2.0, 16),
    2: Config(2, 1, 32768, 128, "normal", 0.0, 0.1, 2.0, 64, n_outlier=4),
    3: Config(3, 8 * 32, 4096, 128, "normal", 0.0, 0.05, 4.0, 0, heads=32),
    4: Config(4, 1, 16384, 8192, "t", 4.0, 0.1, 2.0, 64),
    5: Config(5, 1, 131072, 8192, "t", 3.0, 0.1, 2.0, 0, n_zero=82),
}


def _rng(seed, cfg, tensor, stream, chunk=0):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(
        [int(seed), int(cfg), int(tensor), int(stream), int(chunk)])))


def channel_spread(c: Config, seed=0, tensor=0):
    """Per-slab, per-channel standard-deviation-like multiplier, float64 [batch, D]."""
    r = _rng(seed, c.cfg, tensor, STREAM_SPREAD)
    lo, hi = math.log(c.spread_lo), math.log(c.spread_hi)
    per_head = np.exp(r.uniform(lo, hi, size=(c.heads, c.D)))
    reps = c.batch // c.heads
    spread = np.tile(per_head, (reps, 1))          # slab index = b*heads + h
    r2 = _rng(seed, c.cfg, tensor, STREAM_SPECIAL)
    if c.n_outlier:
        ch = r2.choice(c.D, size=c.n_outlier, replace=False)
        spread[:, ch] *= 20.0
    if c.n_zero:
        ch = r2.choice(c.D, size=c.n_zero, replace=False)
        spread[:, ch] = 0.0
    return spread


def special_channels(c: Config, seed=0, tensor=0):
    """Indices of the outlier (x20) or all-zero channels of a configuration."""
    r2 = _rng(seed, c.cfg, tensor, STREAM_SPECIAL)
    n = c.n_outlier or c.n_zero
    if not n:
        return np.zeros(0, dtype=np.int64)
    return np.sort(r2.choice(c.D, size=n, replace=False))


def chunk_rows(c: Config):
    """Rows per generation chunk (chunks never straddle slabs)."""
    return max(1, min(c.N, CHUNK_ELEMS // c.D))


def _fill_chunk(c, seed, tensor, slab, chunk_in_slab, spread_row, out):
    """out: float32 view [rows, D] of one chunk."""
    chunks_per_slab = -(-c.N // chunk_rows(c))
    r = _rng(seed, c.cfg, tensor, STREAM_DATA, slab * chunks_per_slab + chunk_in_slab)
    if c.law == "normal":
        z = r.standard_normal(size=out.shape)
    else:
        z = r.standard_t(c.nu, size=out.shape)
    z *= spread_row[None, :]
    if c.n_zero:
        z[:, spread_row == 0.0] = 0.0       # +0.0, never -0.0
    out[...] = z                             # one rounding float64 -> float32


def generate(cfg, seed=0, tensor=0, slabs=None, rows=None, out=None, threads=None):
    """Float32 data of a configuration, shape [n_slabs, n_rows, D].

    slabs: (start, stop) slab range, default all; rows: (start, stop) row range
    inside each slab, default all, start must be a multiple of chunk_rows(c).
    """
    c = CONFIGS[cfg] if not isinstance(cfg, Config) else cfg
    s0, s1 = slabs if slabs is not None else (0, c.batch)
    r0, r1 = rows if rows is not None else (0, c.N)
    cr = chunk_rows(c)
    if r0 % cr:
        raise ValueError("row start must be a multiple of %d" % cr)
    if not (0 <= s0 <= s1 <= c.batch and 0 <= r0 <= r1 <= c.N):
        raise ValueError("range outside the configuration")
    shape = (s1 - s0, r1 - r0, c.D)
    if out is None:
        out = np.empty(shape, dtype=np.float32)
    elif out.shape != shape or out.dtype != np.float32 or not out.flags.c_contiguous:
        raise ValueError("out must be C-contiguous float32 of shape %r" % (shape,))
    spread = channel_spread(c, seed, tensor)
    jobs = []
    for s in range(s0, s1):
        for r in range(r0, r1, cr):
            jobs.append((s, r // cr, out[s - s0, r - r0:min(r + cr, r1) - r0]))

    def run(job):
        s, ch, view = job
        if view.shape[0] == cr or ch * cr + view.shape[0] == c.N:
            _fill_chunk(c, seed, tensor, s, ch, spread[s], view)
        else:                                   # partial chunk: draw whole, keep head
            full = np.empty((min(cr, c.N - ch * cr), c.D), dtype=np.float32)
            _fill_chunk(c, seed, tensor, s, ch, spread[s], full)
            view[...] = full[:view.shape[0]]

    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    if threads <= 1 or len(jobs) <= 1:
        for j in jobs:
            run(j)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(run, jobs))
    return out


def queries(cfg, seed=0, n=None):
    """Normal(0,1) float32 queries [Q, D] of a configuration."""
    c = CONFIGS[cfg] if not isinstance(cfg, Config) else cfg
    q = c.n_queries if n is None else n
    r = _rng(seed, c.cfg, 0, STREAM_QUERIES)
    return r.standard_normal(size=(q, c.D)).astype(np.float32)


# The paper's own benchmark shapes (Tests, "Test configurations"): (tokens T, head dimension D).
PAPER_SHAPES = {
    "Small": (2048, 128), "Medium": (16384, 256), "Large": (65536, 256), "Very Large": (131072, 256),
    "Realistic Small": (131072, 1024), "Realistic Medium": (131072, 2048),
    "Realistic Large": (131072, 4096), "Realistic V. Large": (131072, 8192),
}


def uniform_matrix(N, D, seed=0, lo=-1.0, hi=1.0, stream=0, threads=None):
    """The paper's own fill (Evaluation, "Reconstruction Error": inputs in [-1, 1]): float32 [N, D],
    drawn in row chunks of about CHUNK_ELEMS elements so that large shapes can use several threads."""
    out = np.empty((N, D), dtype=np.float32)
    cr = max(1, CHUNK_ELEMS // D)
    jobs = list(range(0, N, cr))

    def run(r0):
        r = _rng(seed, 100, D, stream, r0 // cr)
        out[r0:r0 + cr] = r.uniform(lo, hi, size=(min(cr, N - r0), D))

    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    if threads <= 1 or len(jobs) <= 1:
        for j in jobs:
            run(j)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(run, jobs))
    return out
