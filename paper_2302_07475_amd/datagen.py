"""Seeded synthetic inputs for the S3GD-MV hot path.

This module only draws random numbers and shapes them into gradient-like
tensors.  It contains none of the method's arithmetic (no selection, no sign
coding, no vote, no update) so that both the HIP path and the CPU checker can
consume exactly the same bytes without sharing any logic.

The paper trains a CNN (N = 5e5) on MNIST and ResNet-56 (N = 8.5e5) on
CIFAR-10 with M in {1, 5, 10, 50, 100} workers and sparsity K/N in
{1, 0.5, 0.1, 0.05, 0.01, 0.001}, IID and one-class-per-worker non-IID
(Section 4, "Settings").  Neither the datasets nor trained models are
available here; the five recipes below stand in for the local stochastic
gradients g_m of Algorithm 1:

  C1  i.i.d. N(0,1)                                   (correctness size)
  C2  IID workers: shared mean + per-layer-scaled noise (ResNet-18 sized)
  C3  non-IID workers: per-worker mean + Laplace noise, 10 steps
  C4  heavy tails (Student-t, 3 d.o.f.), 5 % exact zeros, values on a
      2^-12 grid so that many magnitudes tie at the K-th threshold
  C5  1.2e9 coordinates, per-4096-block worker means, even M (vote ties)

Every random stream is numpy's counter-based Philox generator seeded from
SeedSequence([BASE_SEED, config, field, step, worker, chunk]); a chunk is 2^22
coordinates.  Chunks are therefore independent of how they are scheduled over
threads.  Values are drawn and combined in fp64 and rounded to fp32 once.
"N(a, b)" always means standard deviation b.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 230207475
CHUNK = 1 << 22
SHARED = 0xFFFFFFFF  # "worker" id of streams that every worker shares
ANY_STEP = 0xFFFFFFFF  # "step" id of streams that do not change over steps

# stream fields
_F_NOISE, _F_SHARED_MEAN, _F_WORKER_MEAN, _F_LAYER_SCALE, _F_ZERO_MASK, _F_BLOCK_MEAN, _F_X0 = range(7)


@dataclass(frozen=True)
class Config:
    name: str
    cid: int  # seeds the streams; kept when a config is scaled down
    recipe: str  # "c1" .. "c5"
    M: int
    N: int
    K: int
    steps: int = 1
    lr: float = 1e-3

    def scaled(self, M: int | None = None, N: int | None = None, K: int | None = None,
               steps: int | None = None) -> "Config":
        """Same recipe and seeds at another shape (parity tests use small shapes)."""
        return replace(self, name=self.name + "-scaled", M=M or self.M, N=N or self.N,
                       K=self.K if K is None else K, steps=steps or self.steps)


C1 = Config("C1", 1, "c1", 3, 10_000, 100)
C2 = Config("C2", 2, "c2", 16, 11_200_000, 112_000)
C3 = Config("C3", 3, "c3", 32, 25_600_000, 25_600, steps=10)
C4 = Config("C4", 4, "c4", 8, 124_000_000, 1_240_000)
C5 = Config("C5", 5, "c5", 4, 1_200_000_000, 1_200_000)
CONFIGS = {c.name: c for c in (C1, C2, C3, C4, C5)}

N_LAYERS_C2 = 60
BLOCK_C5 = 4096


def _rng(cid: int, field: int, step: int, worker: int, chunk: int) -> np.random.Generator:
    ss = np.random.SeedSequence([BASE_SEED, cid, field, step, worker, chunk])
    return np.random.Generator(np.random.Philox(ss))


def n_chunks(N: int) -> int:
    return (N + CHUNK - 1) // CHUNK


def _span(N: int, j: int) -> tuple[int, int]:
    lo = j * CHUNK
    return lo, min(N, lo + CHUNK)


def layer_scales_c2(cfg: Config) -> np.ndarray:
    """Per-layer noise std of recipe C2: 10^U(-4,-1), one per contiguous layer block."""
    u = _rng(cfg.cid, _F_LAYER_SCALE, ANY_STEP, SHARED, 0).uniform(-4.0, -1.0, N_LAYERS_C2)
    return 10.0 ** u


def _layer_of(cfg: Config, lo: int, hi: int) -> np.ndarray:
    width = max(1, cfg.N // N_LAYERS_C2)
    return np.minimum(np.arange(lo, hi, dtype=np.int64) // width, N_LAYERS_C2 - 1)


def grad_chunk(cfg: Config, step: int, m: int, j: int) -> np.ndarray:
    """fp32 values of worker m's gradient on coordinates [j*CHUNK, min(N,(j+1)*CHUNK))."""
    lo, hi = _span(cfg.N, j)
    n = hi - lo
    c = cfg.cid
    if cfg.recipe == "c1":
        v = _rng(c, _F_NOISE, step, m, j).standard_normal(n)
    elif cfg.recipe == "c2":
        mu = 0.1 * _rng(c, _F_SHARED_MEAN, ANY_STEP, SHARED, j).standard_normal(n)
        eps = _rng(c, _F_NOISE, step, m, j).standard_normal(n)
        v = mu + layer_scales_c2(cfg)[_layer_of(cfg, lo, hi)] * eps
    elif cfg.recipe == "c3":
        mu = 0.1 * _rng(c, _F_SHARED_MEAN, ANY_STEP, SHARED, j).standard_normal(n)
        nu = 0.5 * _rng(c, _F_WORKER_MEAN, ANY_STEP, m, j).standard_normal(n)
        v = mu + nu + _rng(c, _F_NOISE, step, m, j).laplace(0.0, 1.0, n)
    elif cfg.recipe == "c4":
        t = _rng(c, _F_NOISE, step, m, j).standard_t(3.0, n)
        zero = _rng(c, _F_ZERO_MASK, step, m, j).random(n) < 0.05
        t[zero] = 0.0
        v = np.rint(t * 4096.0) / 4096.0
    elif cfg.recipe == "c5":
        assert CHUNK % BLOCK_C5 == 0
        nb = (n + BLOCK_C5 - 1) // BLOCK_C5
        mu_b = 0.2 * _rng(c, _F_BLOCK_MEAN, ANY_STEP, m, j).standard_normal(nb)
        v = np.repeat(mu_b, BLOCK_C5)[:n] + _rng(c, _F_NOISE, step, m, j).standard_normal(n)
    else:
        raise ValueError(cfg.recipe)
    return v.astype(np.float32)


def x0_chunk(cfg: Config, j: int) -> np.ndarray:
    lo, hi = _span(cfg.N, j)
    return (0.01 * _rng(cfg.cid, _F_X0, ANY_STEP, SHARED, j).standard_normal(hi - lo)).astype(np.float32)


def default_threads() -> int:
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        avail = os.cpu_count() or 1
    return max(1, min(16, avail))


def _run(jobs, threads):
    threads = threads or default_threads()
    if threads == 1 or len(jobs) == 1:
        for fn in jobs:
            fn()
        return
    with ThreadPoolExecutor(threads) as ex:
        for f in [ex.submit(fn) for fn in jobs]:
            f.result()


def gradients(cfg: Config, step: int = 0, out: np.ndarray | None = None, threads: int | None = None,
              rows: list[int] | None = None) -> np.ndarray:
    """[M, N] fp32 gradients of one step (or only the listed rows, in that order)."""
    rows = list(range(cfg.M)) if rows is None else rows
    if out is None:
        out = np.empty((len(rows), cfg.N), dtype=np.float32)
    assert out.shape == (len(rows), cfg.N) and out.dtype == np.float32

    def job(r, m, j):
        lo, hi = _span(cfg.N, j)
        out[r, lo:hi] = grad_chunk(cfg, step, m, j)

    jobs = [(lambda r=r, m=m, j=j: job(r, m, j)) for r, m in enumerate(rows) for j in range(n_chunks(cfg.N))]
    _run(jobs, threads)
    return out


def params(cfg: Config, out: np.ndarray | None = None, threads: int | None = None) -> np.ndarray:
    """[N] fp32 initial model x^0 = 0.01 * z."""
    if out is None:
        out = np.empty(cfg.N, dtype=np.float32)

    def job(j):
        lo, hi = _span(cfg.N, j)
        out[lo:hi] = x0_chunk(cfg, j)

    _run([(lambda j=j: job(j)) for j in range(n_chunks(cfg.N))], threads)
    return out


def lr32(cfg: Config) -> np.float32:
    return np.float32(cfg.lr)


def to_device(cfg: Config, step: int = 0, device: str = "cuda:0", threads: int | None = None, want_x: bool = True):
    """(g, x): the [M, N] gradients of one step and x^0 as device tensors, generated chunk by
    chunk on host threads and copied straight into device memory (the host never holds the whole
    tensor).  The bytes are those of gradients() / params()."""
    import torch

    g = torch.empty((cfg.M, cfg.N), dtype=torch.float32, device=device)
    x = torch.empty((cfg.N,), dtype=torch.float32, device=device) if want_x else None

    def gjob(m, j):
        lo = j * CHUNK
        c = grad_chunk(cfg, step, m, j)
        g[m, lo:lo + c.shape[0]].copy_(torch.from_numpy(c))

    def xjob(j):
        lo = j * CHUNK
        c = x0_chunk(cfg, j)
        x[lo:lo + c.shape[0]].copy_(torch.from_numpy(c))

    jobs = [(lambda m=m, j=j: gjob(m, j)) for m in range(cfg.M) for j in range(n_chunks(cfg.N))]
    if want_x:
        jobs += [(lambda j=j: xjob(j)) for j in range(n_chunks(cfg.N))]
    _run(jobs, threads)
    torch.cuda.synchronize()
    return g, x
