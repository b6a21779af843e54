"""Seeded synthetic workloads with the shapes and value distributions of the
five benchmark configurations (orientation: weight is out x in, y = W x).

Only random draws live here; decomposition, packing and the forward pass are
implemented separately by the CPU oracle and by the HIP library.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 2410_23918 * 10  # + config index

# (out, in) of the seven linears of one Llama-3-8B-shaped decoder layer
# (hidden 4096, MLP 14336, grouped-query kv width 1024).
LLAMA3_8B_LINEARS = (
    ("q_proj", 4096, 4096),
    ("k_proj", 1024, 4096),
    ("v_proj", 1024, 4096),
    ("o_proj", 4096, 4096),
    ("gate_proj", 14336, 4096),
    ("up_proj", 14336, 4096),
    ("down_proj", 4096, 14336),
)

CONFIGS = {
    1: dict(name="linear512", shapes=[(512, 512)], sigma_w=0.02, n=4, k=16, batches=[1], fp16_weights=False),
    2: dict(name="llama3_8b_attn_proj", shapes=[(4096, 4096)], sigma_w=0.02, n=16, k=16, batches=[1], fp16_weights=True),
    3: dict(name="llama3_8b_mlp", shapes=[(14336, 4096), (4096, 14336)], sigma_w=0.02, n=16, k=16, batches=[1, 4, 16], fp16_weights=True),
    4: dict(name="llama3_8b_decoder", shapes=[(o, i) for _, o, i in LLAMA3_8B_LINEARS], layers=32, sigma_w=0.02, n=24, k=16, n_loaded_range=(8, 24), batches=[1], fp16_weights=True),
    5: dict(name="llama3_70b_mlp_prefill", shapes=[(28672, 8192)], sigma_w=0.015, n=16, k=16, batches=[2048], fp16_weights=True),
}


def rng_for(config: int, *stream: int) -> np.random.Generator:
    """Independent PCG64 stream for (config, sub-stream ids)."""
    ss = np.random.SeedSequence([BASE_SEED + int(config), *[int(v) for v in stream]])
    return np.random.Generator(np.random.PCG64(ss))


def dense_weight(rng: np.random.Generator, out: int, inn: int, sigma: float, fp16: bool) -> np.ndarray:
    """W ~ N(0, sigma^2), float32; optionally rounded to fp16 values first."""
    w = rng.standard_normal((out, inn), dtype=np.float32) * np.float32(sigma)
    if fp16:
        w = w.astype(np.float16).astype(np.float32)
    return w


def column_scales(rng: np.random.Generator, inn: int) -> np.ndarray:
    """Activation-aware scales, one per input channel: s ~ LogNormal(0, 0.5), float32."""
    return np.exp(0.5 * rng.standard_normal(inn)).astype(np.float32)


def activations(rng: np.random.Generator, batch: int, inn: int) -> np.ndarray:
    """x ~ N(0,1) rounded to fp16, shape (batch, in)."""
    return rng.standard_normal((batch, inn), dtype=np.float32).astype(np.float16)


# Magnitude profile of the factors of block i, measured on a true decomposition
# (k = 16) of a 1024 x 1024 N(0, 0.02^2) matrix with LogNormal(0, 0.5) column
# scales: mean of the single-signed leading column of U (V's leading column is
# the same times the column scale), and standard deviation of columns 1..15.
_LEAD = (0.144, 0.107, 0.079, 0.060, 0.047, 0.038, 0.032, 0.028, 0.025, 0.023,
         0.021, 0.020, 0.0186, 0.0174, 0.0163, 0.0154)
_TAIL = (0.039, 0.027, 0.020, 0.0165, 0.0144, 0.0130, 0.0119, 0.0110, 0.0103,
         0.0096, 0.0090, 0.0085, 0.0080, 0.0076, 0.0072, 0.0068)


def _profile(tab, n: int) -> np.ndarray:
    v = list(tab)
    while len(v) < n:                      # geometric continuation past block 15
        v.append(v[-1] * v[-1] / v[-2])
    return np.asarray(v[:n], dtype=np.float64)


def synthetic_blocks(rng: np.random.Generator, out: int, inn: int, n: int, k: int,
                     s: np.ndarray, sigma_w: float):
    """Random residual blocks with realistic structure, for timing and parity at
    shapes where a true decomposition is too slow.

    Signs are fair coin flips.  The magnitude factors mimic what a rank-k SVD of
    an entrywise non-negative matrix returns: column 0 of U and V is strictly
    positive (Perron vector) and carries most of the energy, columns 1..k-1 are
    zero-mean; V follows the column scales s, as the column norms of the scaled
    weight do; magnitudes shrink from block to block as in a true decomposition
    and scale with sigma_w.  Returns (sign_pm1 int8 [n,out,in], U fp16
    [n,out,k], V fp16 [n,in,k]).
    """
    lead = _profile(_LEAD, n) * np.sqrt(sigma_w / 0.02)
    # bulk singular values scale like (sqrt(out)+sqrt(in)), entries like 1/sqrt(dim)
    tail = _profile(_TAIL, n) * np.sqrt(sigma_w / 0.02) * (1024.0 / np.sqrt(float(out) * inn)) ** 0.25
    s64 = np.asarray(s, dtype=np.float64)
    sn = s64 / np.sqrt((s64 * s64).mean())
    S = np.empty((n, out, inn), dtype=np.int8)
    U = np.empty((n, out, k), dtype=np.float16)
    V = np.empty((n, inn, k), dtype=np.float16)
    for i in range(n):
        S[i] = (rng.integers(0, 2, size=(out, inn), dtype=np.int8) << 1) - 1
        Ui = np.empty((out, k)); Vi = np.empty((inn, k))
        Ui[:, 0] = np.abs(lead[i] * (1.0 + 0.08 * rng.standard_normal(out)))
        Vi[:, 0] = np.abs(lead[i] * sn * (1.0 + 0.08 * rng.standard_normal(inn)))
        Ui[:, 1:] = tail[i] * rng.standard_normal((out, k - 1))
        Vi[:, 1:] = tail[i] * sn[:, None] * rng.standard_normal((inn, k - 1))
        U[i] = Ui.astype(np.float16)
        V[i] = Vi.astype(np.float16)
    return S, U, V


def llama3_8b_layer_shapes():
    return [(name, o, i) for name, o, i in LLAMA3_8B_LINEARS]


def variable_n_loaded(rng: np.random.Generator, count: int, lo: int = 8, hi: int = 24) -> np.ndarray:
    """Per-matrix number of loaded blocks, uniform on [lo, hi] inclusive."""
    return rng.integers(lo, hi + 1, size=count).astype(np.int32)
