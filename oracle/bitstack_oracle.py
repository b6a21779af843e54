"""CPU oracle for the BitStack linear layer (arxiv 2410.23918).

TEST INFRASTRUCTURE ONLY.  This module is the plain, slow, obviously-correct
reference the HIP library is compared with.  It shares no code with the HIP
path and must never be imported by the product package; only tests/, the
smoke check and the benchmark's cpu_baseline leg may use it.

Orientation.  The paper writes X (p x m), W (m x n), Y = X W, with the scale
vector s running over the m input channels (rows of W).  This file uses the
transposed, PyTorch-linear orientation: W_t = W^T is (out x in), y = W_t x,
and s scales the *columns* of W_t.  Paper -> here: A' (m x k) -> V (in x k),
B' (n x k) -> U (out x k), W_sign -> S = W_sign^T.

Everything is evaluated in float64 unless a step of the paper fixes a storage
precision (the magnitude factors are kept in fp16, Section 2.1.2).

Parity pins (tests/test_oracle_*.py, none of which re-types these formulas):
  block_bytes            the printed residual-block size table (Appendix, k=16)
  pack_signs/unpack      per-bit brute force, popcount, +-0 handling
  rank_k_factors         Eckart-Young error and the sqrt(sigma) split, both
                         against LAPACK's full SVD
  avd_block / iavd       |R - S.M| = ||R| - M|, Perron sign pattern, monotone
                         error, exact recovery at full rank, scale covariance
  forward_dense          brute-force triple loop, the factored form, linearity,
                         per-block additivity, closed-form rank-1 case
  relative_error and its two companions (rms_relative_error,
  damped_elementwise_error): hand-computed examples (different row maxima, a
                         zero reference row, a negative peak), scale invariance
  Exact y values: parity unpinned by the paper (it prints no worked example);
  pinned only through the invariants above.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


# --------------------------------------------------------------------------
# Section "Discussion on minimal transmission units", Eq. (9)
# --------------------------------------------------------------------------
def block_bits(out: int, inn: int, k: int) -> int:
    """Size of one residual block in bits: one bit per weight for the packed
    sign matrix plus 16 bits for each entry of the two rank-k factor
    matrices (Eq. 9: delta_W = m n + 16 k (m + n))."""
    return out * inn + 16 * k * (out + inn)


def block_bytes(out: int, inn: int, k: int) -> int:
    bits = block_bits(out, inn, k)
    assert bits % 8 == 0
    return bits // 8


# --------------------------------------------------------------------------
# Sign packing.  The paper only says the +-1 matrix is packed into a
# GPU-supported integer type (Section 2.1.2, Fig. 3).  Canonical interchange
# format chosen here: uint32, row-major [out][in/32], bit b of word w is
# column 32 w + b, bit value 1 <=> sign +1.  sign(0) := +1 (also for -0.0) so
# that the sign matrix holds only +-1 as the paper requires.
# --------------------------------------------------------------------------
def sign_pm1(residual: np.ndarray) -> np.ndarray:
    """+1 where residual >= 0 (including both zeros), -1 elsewhere; int8."""
    r = np.asarray(residual)
    return np.where(r >= 0, 1, -1).astype(np.int8)


def pack_signs(sign: np.ndarray) -> np.ndarray:
    """(out, in) array of +-1 -> (out, in/32) uint32 canonical words."""
    s = np.asarray(sign)
    out, inn = s.shape
    if inn % 32:
        raise ValueError("in must be a multiple of 32 for the canonical packing")
    if not np.all((s == 1) | (s == -1)):
        raise ValueError("sign matrix must hold only +1/-1")
    # bit b of byte q <-> column 8 q + b; four consecutive bytes, least significant
    # first, form one word
    by = np.packbits(s > 0, axis=1, bitorder="little")
    return np.ascontiguousarray(by).view("<u4").astype(np.uint32)


def unpack_signs(words: np.ndarray, inn: int) -> np.ndarray:
    """Inverse of pack_signs: (out, in/32) uint32 -> (out, in) int8 of +-1."""
    w = np.asarray(words, dtype=np.uint32)
    out = w.shape[0]
    bits = (w[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & np.uint32(1)
    return (bits.reshape(out, inn).astype(np.int8) * 2 - 1).astype(np.int8)


# --------------------------------------------------------------------------
# Eq. (3): activation-aware scale from calibration activations
# --------------------------------------------------------------------------
def scales_from_activations(X: np.ndarray) -> np.ndarray:
    """s_j = l2 norm of input channel j over the calibration rows of X (p x in).
    (The paper's Eq. 3 indexes the norms 1..n although X has m channels; the
    reading taken is one entry per input channel.)"""
    X = np.asarray(X, dtype=np.float64)
    return np.sqrt((X * X).sum(axis=0))


def _check_scales(s: np.ndarray) -> np.ndarray:
    s = np.asarray(s, dtype=np.float64)
    if not np.all(np.isfinite(s)) or not np.all(s > 0):
        raise ValueError("scales must be finite and > 0")
    return s


# --------------------------------------------------------------------------
# Eq. (1)-(2): rank-k SVD with the sqrt(sigma) split
# --------------------------------------------------------------------------
def rank_k_factors(M: np.ndarray, k: int, method: str = "full", iters: int = 40,
                   oversample: int = 16, rng: np.random.Generator | None = None):
    """Top-k singular triplets of M (out x in) split symmetrically:
    U = [sqrt(s_r) p_r], V = [sqrt(s_r) q_r] so that U V^T is the rank-k
    truncation of M (Eq. 2).  Returns (U (out x k), V (in x k), sigma (k,)).

    method="full" calls LAPACK on the whole matrix.  method="subspace" runs a
    block power (subspace) iteration with k+oversample columns followed by a
    Rayleigh-Ritz step: any method returning the leading triplets is a valid
    reading of "SVD"; the two are cross-checked in the tests."""
    M = np.asarray(M, dtype=np.float64)
    out, inn = M.shape
    k = int(k)
    if not 1 <= k <= min(out, inn):
        raise ValueError("k out of range")
    if method == "full":
        P, sig, Qt = np.linalg.svd(M, full_matrices=False)
        P, sig, Q = P[:, :k], sig[:k], Qt[:k].T
    elif method == "subspace":
        rng = rng or np.random.default_rng(0)
        b = min(k + oversample, min(out, inn))
        Q = np.linalg.qr(rng.standard_normal((inn, b)))[0]
        for _ in range(iters):
            Z = np.linalg.qr(M @ Q)[0]
            Q = np.linalg.qr(M.T @ Z)[0]
        Bm = M @ Q                                   # out x b
        Pb, sig, Wt = np.linalg.svd(Bm, full_matrices=False)
        P, sig, Q = Pb[:, :k], sig[:k], (Q @ Wt.T)[:, :k]
    else:
        raise ValueError(method)
    root = np.sqrt(sig)
    return P * root[None, :], Q * root[None, :], sig


# --------------------------------------------------------------------------
# Eq. (5): absolute value decomposition of one (residual) matrix
# --------------------------------------------------------------------------
def avd_block(R: np.ndarray, k: int, round_fp16: bool = True, **svd_kw):
    """One residual block of R: S = sign(R), (U, V) = rank-k factors of |R|.
    With round_fp16 the factors are rounded to fp16 (the stored precision,
    Section 2.1.2) and returned as float16 arrays."""
    R = np.asarray(R, dtype=np.float64)
    S = sign_pm1(R)
    U, V, _ = rank_k_factors(np.abs(R), k, **svd_kw)
    if round_fp16:
        U = U.astype(np.float16)
        V = V.astype(np.float16)
    return S, U, V


def block_dense(S: np.ndarray, U: np.ndarray, V: np.ndarray) -> np.ndarray:
    """S (.) (U V^T) in float64 (Eq. 5)."""
    return S.astype(np.float64) * (U.astype(np.float64) @ V.astype(np.float64).T)


@dataclass
class Stack:
    """A weight stack: n residual blocks of one (out x in) matrix plus s."""
    S: np.ndarray          # int8  [n, out, in], entries +-1
    U: np.ndarray          # fp16 (or float64 when unrounded) [n, out, k]
    V: np.ndarray          # fp16 (or float64 when unrounded) [n, in, k]
    s: np.ndarray          # float32/float64 [in]

    @property
    def n(self): return self.S.shape[0]
    @property
    def out(self): return self.S.shape[1]
    @property
    def inn(self): return self.S.shape[2]
    @property
    def k(self): return self.U.shape[2]

    def sign_words(self) -> np.ndarray:
        return np.stack([pack_signs(self.S[i]) for i in range(self.n)])


# --------------------------------------------------------------------------
# Eq. (4) + Eq. (6)-(8), Algorithm 1 lines 1-23: scaling then iterative AVD
# --------------------------------------------------------------------------
def iavd(W_t: np.ndarray, s: np.ndarray, n: int, k: int, round_fp16: bool = True,
         **svd_kw) -> Stack:
    """Decompose W_t (out x in) into n residual blocks.

    R_0 = W_t diag(s)            (column j times s_j: Eq. 4, Alg. 1 line 5)
    for i = 0..n-1:
        S_i, U_i, V_i = AVD(R_i)              (Eq. 5, Eq. 7)
        R_{i+1} = R_i - S_i (.) (U_i V_i^T)   (Eq. 6)
    The residual update uses the factors as stored (fp16-rounded when
    round_fp16): what is subtracted is what inference will add back."""
    W_t = np.asarray(W_t, dtype=np.float64)
    s = _check_scales(s)
    out, inn = W_t.shape
    if s.shape != (inn,):
        raise ValueError("s must have one entry per input channel")
    R = W_t * s[None, :]
    Ss, Us, Vs = [], [], []
    for _ in range(n):
        S, U, V = avd_block(R, k, round_fp16=round_fp16, **svd_kw)
        R = R - block_dense(S, U, V)
        Ss.append(S); Us.append(U); Vs.append(V)
    dt = np.float16 if round_fp16 else np.float64
    return Stack(np.stack(Ss) if n else np.zeros((0, out, inn), np.int8),
                 np.stack(Us).astype(dt) if n else np.zeros((0, out, k), dt),
                 np.stack(Vs).astype(dt) if n else np.zeros((0, inn, k), dt),
                 np.asarray(s))


def reconstruct_scaled(stack: Stack, n_loaded: int) -> np.ndarray:
    """W'_scaled = sum_{i < n_loaded} S_i (.) (U_i V_i^T)  (Eq. 8); zero matrix
    for n_loaded = 0 (W_iavd^(0) = 0)."""
    if not 0 <= n_loaded <= stack.n:
        raise ValueError("n_loaded out of range")
    Wp = np.zeros((stack.out, stack.inn), dtype=np.float64)
    for i in range(n_loaded):
        Wp += block_dense(stack.S[i], stack.U[i], stack.V[i])
    return Wp


# --------------------------------------------------------------------------
# Forward pass: Y = X diag(1/s) W_iavd  (Eq. 4 with Eq. 8)
# --------------------------------------------------------------------------
def forward_dense(stack: Stack, x: np.ndarray, n_loaded: int) -> np.ndarray:
    """Dense reconstruct-then-matmul.  x: (batch, in); returns (batch, out)
    float64: y_b = W' (x_b / s)."""
    x = np.asarray(x, dtype=np.float64)
    s = _check_scales(stack.s)
    Wp = reconstruct_scaled(stack, n_loaded)
    xp = x / s[None, :]
    return xp @ Wp.T


def forward_factored(stack: Stack, x: np.ndarray, n_loaded: int) -> np.ndarray:
    """Same result through the per-rank identity
    (S (.) u v^T) x = u (.) (S (v (.) x)), never forming U V^T."""
    x = np.asarray(x, dtype=np.float64)
    s = _check_scales(stack.s)
    if not 0 <= n_loaded <= stack.n:
        raise ValueError("n_loaded out of range")
    xp = x / s[None, :]
    y = np.zeros((x.shape[0], stack.out), dtype=np.float64)
    for i in range(n_loaded):
        S = stack.S[i].astype(np.float64)
        U = stack.U[i].astype(np.float64)
        V = stack.V[i].astype(np.float64)
        for b in range(x.shape[0]):
            T = V * xp[b][:, None]          # in x k
            Z = S @ T                        # out x k
            y[b] += (U * Z).sum(axis=1)
    return y


def forward_rows(stack: Stack, x: np.ndarray, n_loaded: int, rows: np.ndarray) -> np.ndarray:
    """forward_dense restricted to a subset of output rows (for spot checks at
    shapes where the full product is too slow).  Returns (batch, len(rows))."""
    x = np.asarray(x, dtype=np.float64)
    s = _check_scales(stack.s)
    rows = np.asarray(rows)
    xp = x / s[None, :]
    Wp = np.zeros((len(rows), stack.inn), dtype=np.float64)
    for i in range(n_loaded):
        Wp += stack.S[i][rows].astype(np.float64) * (
            stack.U[i][rows].astype(np.float64) @ stack.V[i].astype(np.float64).T)
    return xp @ Wp.T


def relative_error(y: np.ndarray, y_ref: np.ndarray) -> float:
    """Parity metric: per token row max_o |y - y_ref| / max_o |y_ref|, worst row."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    num = np.abs(y - y_ref).max(axis=-1)
    den = np.abs(y_ref).max(axis=-1)
    den = np.where(den == 0, 1.0, den)
    return float((num / den).max())


def rms_relative_error(y: np.ndarray, y_ref: np.ndarray) -> float:
    """Companion figure to relative_error: per token row
    sqrt(mean_o (y - y_ref)^2) / sqrt(mean_o y_ref^2), worst row."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    num = np.sqrt(((y - y_ref) ** 2).mean(axis=-1))
    den = np.sqrt((y_ref ** 2).mean(axis=-1))
    den = np.where(den == 0, 1.0, den)
    return float((num / den).max())


def damped_elementwise_error(y: np.ndarray, y_ref: np.ndarray, damping: float = 1e-3) -> float:
    """Companion figure to relative_error that also constrains small outputs:
    max over elements of |y - y_ref| / (|y_ref| + damping * max_o |y_ref|), per token
    row, worst row.  (A pure element-wise relative error is meaningless next to the
    zeros of y_ref.)"""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    peak = np.abs(y_ref).max(axis=-1, keepdims=True)
    peak = np.where(peak == 0, 1.0, peak)
    return float((np.abs(y - y_ref) / (np.abs(y_ref) + damping * peak)).max())

