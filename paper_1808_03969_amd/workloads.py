"""The five benchmark configurations as synthetic workloads, built on the GPU.

Each configuration names a data distribution (from ``synth``), the PQ parameters, the coarse
quantiser size and the query batch.  ``build()`` generates the database chunk by chunk on the
GPU, encodes it with the library, and builds the index with the library's own reconfigure
(code-space clustering + posting lists); nothing here touches the CPU oracle.
"""
from __future__ import annotations

import time
from dataclasses import dataclass

import numpy as np
import torch

import synth

from . import binding as rii


@dataclass(frozen=True)
class Config:
    name: str
    N: int
    D: int
    M: int
    K: int          # coarse centres (0: none)
    Q: int
    topk: int
    kind: str       # "gaussian" | "sift" | "mixture"
    train_rows: int
    c: int          # configuration number (seeds are 1000+c, 2000+c, ...)


CONFIGS = {
    "c1": Config("c1_tiny_linear", 10_000, 128, 8, 0, 100, 10, "gaussian", 5_000, 1),
    "c2": Config("c2_sift_shaped", 1_000_000, 128, 16, 1_000, 10_000, 100, "sift", 100_000, 2),
    "c3": Config("c3_sift_subset", 1_000_000, 128, 16, 1_000, 1_000, 100, "sift", 100_000, 3),
    "c4": Config("c4_deep_shaped", 10_000_000, 96, 16, 4_096, 10_000, 100, "mixture", 100_000, 4),
    "c5": Config("c5_billion_shard", 100_000_000, 96, 32, 16_384, 10_000, 100, "mixture", 100_000, 5),
}


def rows(cfg: Config, seed: int, r0: int, r1: int, device, shift: float = 0.0) -> torch.Tensor:
    if cfg.kind == "gaussian":
        return synth.gaussian(seed, r0, r1, cfg.D, device)
    if cfg.kind == "sift":
        return synth.sift_like(seed, r0, r1, cfg.D, device)
    return synth.mixture(seed, r0, r1, cfg.D, shift=shift, means_seed=1000 + cfg.c, device=device)


def build(cfg: Config, device="cuda", coarse_iters: int = 3, chunk: int = 2_000_000, log=None, N: int | None = None,
          Q: int | None = None):
    """Returns a dict: index, cb (numpy), q (device [Q][D]), timings.  ``N``/``Q`` override the sizes."""
    N = cfg.N if N is None else N
    Q = cfg.Q if Q is None else Q
    say = log or (lambda *a: None)
    t = {}
    t0 = time.time()
    train = rows(cfg, 3000 + cfg.c, 0, min(cfg.train_rows, max(N, 256)), device).cpu().numpy()
    cb = rii.rii_train_codebooks(train, cfg.M, iters=20, seed=4000 + cfg.c)
    t["train_codebooks_s"] = time.time() - t0
    say(f"codebooks trained on {len(train)} rows in {t['train_codebooks_s']:.1f}s")
    index = rii.Index(cb)
    t0 = time.time()
    for r0 in range(0, N, chunk):
        r1 = min(N, r0 + chunk)
        x = rows(cfg, 1000 + cfg.c, r0, r1, device)
        index.add(rii.rii_encode_device(index, x))
        del x
    torch.cuda.synchronize()
    t["generate_encode_s"] = time.time() - t0
    say(f"{N} vectors generated and encoded in {t['generate_encode_s']:.1f}s")
    if cfg.K:
        t0 = time.time()
        index.reconfigure(cfg.K, iters=coarse_iters, seed=4000 + cfg.c)
        t["reconfigure_s"] = time.time() - t0
        say(f"K={cfg.K} coarse centres + posting lists in {t['reconfigure_s']:.1f}s")
    q = rows(cfg, 2000 + cfg.c, 0, Q, device)
    return dict(cfg=cfg, N=N, Q=Q, index=index, cb=cb, q=q, timings=t)


def subsets(cfg: Config, N: int, Q: int, S: int, device="cuda"):
    """Sorted uniform target-identifier subsets of size S for Q queries (CSR, on `device`)."""
    return synth.subset_batch(5000 + cfg.c, N, [S] * Q, device)
