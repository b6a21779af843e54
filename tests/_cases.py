"""Shared builders for the parity tests: seeded stacks per benchmark configuration."""
from __future__ import annotations

import functools

import numpy as np

from oracle import bitstack_oracle as O
from workloads import synth as W


@functools.lru_cache(maxsize=None)
def true_stack(config: int, out: int, inn: int, n: int, method: str = "full", iters: int = 10) -> O.Stack:
    """Real IAVD of a seeded synthetic weight (configs 1 and 2)."""
    cfg = W.CONFIGS[config]
    rng = W.rng_for(config, 0)
    Wt = W.dense_weight(rng, out, inn, cfg["sigma_w"], cfg["fp16_weights"])
    s = W.column_scales(rng, inn)
    kw = dict(method=method)
    if method == "subspace":
        kw.update(iters=iters, rng=W.rng_for(config, 1))
    return O.iavd(Wt, s, n, 16, **kw)


@functools.lru_cache(maxsize=4)
def synth_stack(config: int, out: int, inn: int, n: int, tag: int = 0) -> O.Stack:
    """Random blocks with the documented magnitude profile (configs 3-5)."""
    cfg = W.CONFIGS[config]
    rng = W.rng_for(config, 10 + tag, out, inn)
    s = W.column_scales(rng, inn)
    S, U, V = W.synthetic_blocks(rng, out, inn, n, 16, s, cfg["sigma_w"])
    return O.Stack(S, U, V, s)


def acts(config: int, batch: int, inn: int, tag: int = 0) -> np.ndarray:
    return W.activations(W.rng_for(config, 100 + tag, batch, inn), batch, inn)
