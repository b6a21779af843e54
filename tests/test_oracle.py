"""Pins for the CPU oracle.  None of these re-type the oracle's formulas: each
checks it against something fixed by the paper or by mathematics (printed table
values, LAPACK's SVD, brute force, closed forms, invariants)."""
import os

import numpy as np
import pytest

from oracle import bitstack_oracle as O
from workloads import synth as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- Eq. (9) + table
def _table():
    rows = []
    with open(os.path.join(GOLD, "residual_block_sizes.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            rows.append((p[0], int(p[1]), int(p[2]), int(p[3]), [float(v) for v in p[4:]]))
    return rows


def test_block_bytes_matches_printed_table():
    for name, hidden, mlp, kv, printed in _table():
        shapes = [(hidden, hidden), (kv, hidden), (kv, hidden), (hidden, hidden),
                  (mlp, hidden), (mlp, hidden), (hidden, mlp)]
        for (o, i), mb in zip(shapes, printed):
            got = O.block_bytes(o, i, 16) / 2 ** 20
            # printed to two decimals (half-up or half-even both within 0.005 + eps)
            assert abs(got - mb) <= 0.005 + 1e-9, (name, o, i, got, mb)


def test_block_is_about_one_bit_per_parameter():
    # "approximately 1 bit per parameter when k << min(m, n)"
    assert O.block_bits(4096, 4096, 16) / (4096 * 4096) == pytest.approx(1.125)
    assert O.block_bits(4096, 14336, 16) == O.block_bits(14336, 4096, 16)  # symmetric in m, n


# ---------------------------------------------------------------- sign packing
def test_sign_of_zero_and_negative_zero_is_plus_one():
    r = np.array([[0.0, -0.0, 1e-30, -1e-30, np.inf, -np.inf]])
    assert O.sign_pm1(r).tolist() == [[1, 1, 1, -1, 1, -1]]


def test_pack_signs_bruteforce_bits():
    rng = np.random.default_rng(1)
    S = rng.choice(np.array([-1, 1], dtype=np.int8), size=(5, 96))
    words = O.pack_signs(S)
    assert words.dtype == np.uint32 and words.shape == (5, 3)
    for o in range(5):
        for j in range(96):
            bit = (int(words[o, j // 32]) >> (j % 32)) & 1
            assert bit == (1 if S[o, j] == 1 else 0)
    assert np.array_equal(O.unpack_signs(words, 96), S)


def test_pack_signs_known_words():
    S = -np.ones((1, 64), dtype=np.int8)
    S[0, 0] = 1; S[0, 31] = 1; S[0, 33] = 1
    assert O.pack_signs(S).tolist() == [[0x80000001, 0x00000002]]


def test_popcount_equals_number_of_nonnegative():
    rng = np.random.default_rng(2)
    R = rng.standard_normal((64, 256)).astype(np.float32)
    R[rng.random(R.shape) < 0.05] = 0.0
    words = O.pack_signs(O.sign_pm1(R))
    pop = sum(bin(int(w)).count("1") for w in words.ravel())
    assert pop == int((R >= 0).sum())


def test_pack_rejects_zero_entries():
    S = np.ones((2, 32), dtype=np.int8); S[0, 3] = 0
    with pytest.raises(ValueError):
        O.pack_signs(S)


# ---------------------------------------------------------------- rank-k step
@pytest.mark.parametrize("shape", [(48, 32), (32, 80)])
def test_rank_k_eckart_young_and_sqrt_split(shape):
    rng = np.random.default_rng(3)
    M = np.abs(rng.standard_normal(shape))
    k = 5
    U, V, sig = O.rank_k_factors(M, k)
    full = np.linalg.svd(M, compute_uv=False)
    assert np.allclose(sig, full[:k])
    # error of the best rank-k approximation = tail of the spectrum
    err2 = np.linalg.norm(M - U @ V.T) ** 2
    assert err2 == pytest.approx((full[k:] ** 2).sum(), rel=1e-10)
    # symmetric split: both factor Gram matrices equal diag(sigma)
    assert np.allclose(U.T @ U, np.diag(full[:k]), atol=1e-10)
    assert np.allclose(V.T @ V, np.diag(full[:k]), atol=1e-10)


def test_subspace_iteration_agrees_with_lapack():
    rng = W.rng_for(1, 77)
    M = np.abs(W.dense_weight(rng, 256, 384, 0.02, False).astype(np.float64) * W.column_scales(rng, 384))
    Uf, Vf, sf = O.rank_k_factors(M, 16, method="full")
    Us, Vs, ss = O.rank_k_factors(M, 16, method="subspace", iters=60)
    assert np.allclose(sf, ss, rtol=1e-6)
    # compare the approximation error, which is unique (near-degenerate
    # singular subspaces make U V^T itself ill-conditioned)
    ef = np.linalg.norm(M - Uf @ Vf.T); es = np.linalg.norm(M - Us @ Vs.T)
    assert es == pytest.approx(ef, rel=1e-5)


# ---------------------------------------------------------------- AVD block
def test_sign_times_magnitude_identity_and_perron():
    rng = np.random.default_rng(4)
    R = rng.standard_normal((40, 64)) * 0.02
    S, U, V = O.avd_block(R, 4, round_fp16=False)
    assert set(np.unique(S).tolist()) <= {-1, 1}
    M = U @ V.T
    # |S| = 1 entrywise  =>  ||R - S.M||_F = || |R| - M ||_F for any M
    assert np.linalg.norm(R - O.block_dense(S, U, V)) == pytest.approx(np.linalg.norm(np.abs(R) - M), rel=1e-12)
    # |R| is entrywise non-negative: its leading singular vectors are single-signed
    assert np.all(U[:, 0] > 0) or np.all(U[:, 0] < 0)
    assert np.all(V[:, 0] > 0) or np.all(V[:, 0] < 0)
    assert np.sign(U[0, 0]) == np.sign(V[0, 0])


def test_rank1_closed_form_is_exact_in_one_block():
    rng = np.random.default_rng(5)
    a = rng.uniform(0.5, 2.0, 24); b = rng.uniform(0.5, 2.0, 32)
    Sg = rng.choice([-1.0, 1.0], size=(24, 32))
    Wt = Sg * np.outer(a, b)
    st = O.iavd(Wt, np.ones(32), n=1, k=1, round_fp16=False)
    assert np.allclose(O.reconstruct_scaled(st, 1), Wt, rtol=1e-12, atol=1e-14)
    x = rng.standard_normal((2, 32))
    assert np.allclose(O.forward_dense(st, x, 1), x @ Wt.T, rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- IAVD
def _cfg1(n=4, k=16, fp16=True, out=512, inn=512):
    rng = W.rng_for(1, 0)
    Wt = W.dense_weight(rng, out, inn, 0.02, False)
    s = W.column_scales(rng, inn)
    return Wt, s, O.iavd(Wt, s, n, k, round_fp16=fp16)


def test_error_is_non_increasing_and_zero_blocks_is_zero():
    Wt, s, st = _cfg1(n=6)
    R0 = Wt.astype(np.float64) * s[None, :]
    errs = [np.linalg.norm(R0 - O.reconstruct_scaled(st, m)) for m in range(7)]
    assert errs[0] == pytest.approx(np.linalg.norm(R0))
    assert np.all(np.diff(errs) < 0)
    assert not O.reconstruct_scaled(st, 0).any()
    x = W.activations(W.rng_for(1, 1), 3, 512)
    assert not O.forward_dense(st, x, 0).any()


def test_first_block_error_follows_eckart_young():
    # ratio^2 = 1 - sum_{r<=k} sigma_r^2 / ||R||^2 with sigma from LAPACK on |R0|
    rng = W.rng_for(1, 5)
    Wt = W.dense_weight(rng, 96, 128, 0.02, False); s = W.column_scales(rng, 128)
    R0 = Wt.astype(np.float64) * s
    st = O.iavd(Wt, s, 1, 8, round_fp16=False)
    sig = np.linalg.svd(np.abs(R0), compute_uv=False)
    want = np.sqrt(1 - (sig[:8] ** 2).sum() / (R0 ** 2).sum())
    got = np.linalg.norm(R0 - O.reconstruct_scaled(st, 1)) / np.linalg.norm(R0)
    assert got == pytest.approx(want, rel=1e-10)


def test_one_full_rank_block_recovers_weight_exactly():
    rng = W.rng_for(1, 2)
    Wt = W.dense_weight(rng, 48, 64, 0.02, False)
    s = W.column_scales(rng, 64)
    st = O.iavd(Wt, s, n=1, k=48, round_fp16=False)
    R0 = Wt.astype(np.float64) * s
    assert np.allclose(O.reconstruct_scaled(st, 1), R0, rtol=0, atol=1e-13 * np.abs(R0).max() * 48)
    # and the scaling cancels in the forward pass: y = W x   (Eq. 4)
    x = rng.standard_normal((2, 64))
    assert np.allclose(O.forward_dense(st, x, 1), x @ Wt.astype(np.float64).T, rtol=1e-10, atol=1e-12)


def test_scale_covariance():
    # s -> c s : scaled residuals scale by c, factors by sqrt(c), y is unchanged
    rng = W.rng_for(1, 3)
    Wt = W.dense_weight(rng, 64, 96, 0.02, False); s = W.column_scales(rng, 96)
    a = O.iavd(Wt, s, 3, 4, round_fp16=False)
    b = O.iavd(Wt, 4.0 * s, 3, 4, round_fp16=False)
    assert np.array_equal(a.S, b.S)
    for i in range(3):
        assert np.allclose(b.U[i] @ b.V[i].T, 4.0 * (a.U[i] @ a.V[i].T), rtol=1e-8)
        assert np.allclose(np.linalg.norm(b.U[i], axis=0), 2.0 * np.linalg.norm(a.U[i], axis=0), rtol=1e-8)
    x = rng.standard_normal((2, 96))
    assert np.allclose(O.forward_dense(a, x, 3), O.forward_dense(b, x, 3), rtol=1e-8)


def test_unit_scales_reduce_to_plain_iavd_and_bad_scales_raise():
    rng = W.rng_for(1, 4)
    Wt = W.dense_weight(rng, 32, 64, 0.02, False)
    st = O.iavd(Wt, np.ones(64), 2, 4, round_fp16=False)
    S0, U0, V0 = O.avd_block(Wt.astype(np.float64), 4, round_fp16=False)
    assert np.array_equal(st.S[0], S0) and np.allclose(st.U[0] @ st.V[0].T, U0 @ V0.T)
    for bad in (0.0, -1.0, np.nan, np.inf):
        s = np.ones(64); s[5] = bad
        with pytest.raises(ValueError):
            O.iavd(Wt, s, 1, 4)


def test_stored_factors_are_fp16_and_update_uses_them():
    Wt, s, st = _cfg1(n=2)
    assert st.U.dtype == np.float16 and st.V.dtype == np.float16
    R0 = Wt.astype(np.float64) * s
    R1 = R0 - O.block_dense(st.S[0], st.U[0], st.V[0])
    assert np.array_equal(st.S[1], O.sign_pm1(R1))


def test_scales_from_activations_is_channel_l2_norm():
    X = np.array([[3.0, 0.0, 1.0], [4.0, 2.0, 1.0]])
    assert np.allclose(O.scales_from_activations(X), [5.0, 2.0, np.sqrt(2.0)])


# ---------------------------------------------------------------- forward
def test_forward_bruteforce_tiny():
    rng = np.random.default_rng(6)
    out, inn, k, n = 6, 32, 2, 3
    S = rng.choice(np.array([-1, 1], dtype=np.int8), size=(n, out, inn))
    U = rng.standard_normal((n, out, k)).astype(np.float16)
    V = rng.standard_normal((n, inn, k)).astype(np.float16)
    s = rng.uniform(0.5, 2.0, inn).astype(np.float32)
    x = rng.standard_normal((2, inn)).astype(np.float16)
    st = O.Stack(S, U, V, s)
    for nl in range(n + 1):
        want = np.zeros((2, out))
        for b in range(2):
            for o in range(out):
                acc = 0.0
                for j in range(inn):
                    w = 0.0
                    for i in range(nl):
                        m = 0.0
                        for r in range(k):
                            m += float(U[i, o, r]) * float(V[i, j, r])
                        w += float(S[i, o, j]) * m
                    acc += w * (float(x[b, j]) / float(s[j]))
                want[b, o] = acc
        assert np.allclose(O.forward_dense(st, x, nl), want, rtol=1e-12, atol=1e-12)
        assert np.allclose(O.forward_factored(st, x, nl), want, rtol=1e-12, atol=1e-12)


def test_dense_equals_factored_linearity_additivity_cfg1():
    Wt, s, st = _cfg1()
    rng = W.rng_for(1, 1)
    x = W.activations(rng, 2, 512)
    yd = O.forward_dense(st, x, 4); yf = O.forward_factored(st, x, 4)
    assert O.relative_error(yf, yd) < 1e-12
    # linear in x
    x2 = W.activations(rng, 2, 512)
    lhs = O.forward_dense(st, 2.0 * x.astype(np.float64) - 3.0 * x2.astype(np.float64), 4)
    assert np.allclose(lhs, 2.0 * yd - 3.0 * O.forward_dense(st, x2, 4), rtol=1e-10, atol=1e-12)
    # loading one more block adds exactly that block's contribution
    only3 = O.Stack(st.S[3:4], st.U[3:4], st.V[3:4], st.s)
    assert np.allclose(yd - O.forward_dense(st, x, 3), O.forward_dense(only3, x, 1), rtol=1e-9, atol=1e-12)
    # spot rows agree with the full product
    rows = np.array([0, 17, 511])
    assert np.allclose(O.forward_rows(st, x, 4, rows), yd[:, rows], rtol=1e-12, atol=1e-14)
    # more blocks -> closer to the unscaled dense layer (forward compatibility)
    y_true = x.astype(np.float64) @ Wt.astype(np.float64).T
    e = [O.relative_error(O.forward_dense(st, x, m), y_true) for m in range(1, 5)]
    assert e[3] < e[0]


def test_synthetic_blocks_have_the_documented_structure():
    rng = W.rng_for(3, 9)
    s = W.column_scales(rng, 256)
    S, U, V = W.synthetic_blocks(rng, 64, 256, 3, 16, s, 0.02)
    assert set(np.unique(S).tolist()) == {-1, 1}
    assert U.dtype == np.float16 and V.dtype == np.float16
    assert np.all(U[:, :, 0].astype(float) > 0) and np.all(V[:, :, 0].astype(float) > 0)
    m0 = np.abs(U[0].astype(float) @ V[0].astype(float).T).mean()
    m2 = np.abs(U[2].astype(float) @ V[2].astype(float).T).mean()
    assert m2 < m0


# ---------------------------------------------------------------------------
# The parity metric itself (the reading of "maximum relative error 2e-3": per
# token row max |y - y_ref| / max |y_ref|), pinned on values worked out by hand.
# ---------------------------------------------------------------------------
def test_relative_error_hand_examples():
    ref = np.array([[1.0, -4.0, 2.0],        # peak 4 (negative entry)
                    [0.5, 0.25, -0.125]])    # peak 0.5
    y = np.array([[1.0, -4.0, 2.2],          # largest deviation 0.2  -> 0.2 / 4   = 0.05
                  [0.5, 0.30, -0.125]])      # largest deviation 0.05 -> 0.05 / 0.5 = 0.1
    assert O.relative_error(y, ref) == pytest.approx(0.1, rel=1e-12)
    # every row is judged against its own peak: swapping the deviations changes the figure
    y2 = np.array([[1.0, -4.0, 2.05], [0.5, 0.45, -0.125]])   # 0.0125 and 0.4
    assert O.relative_error(y2, ref) == pytest.approx(0.4, rel=1e-12)
    # one row only, deviation at the (negative) peak itself
    assert O.relative_error(np.array([[1.0, -3.0, 2.0]]), ref[:1]) == pytest.approx(0.25, rel=1e-12)
    # a zero reference row: the deviation itself (denominator 1), not a division by zero
    z = np.zeros((1, 3))
    assert O.relative_error(np.array([[0.0, 0.0, 0.0]]), z) == 0.0
    assert O.relative_error(np.array([[0.0, -0.25, 0.0]]), z) == pytest.approx(0.25, rel=1e-12)
    # 1-D inputs are one row; exact match is zero; a common factor on both cancels
    assert O.relative_error(ref[0], ref[0]) == 0.0
    assert O.relative_error(7.0 * y, 7.0 * ref) == pytest.approx(0.1, rel=1e-12)
    # not symmetric in its arguments: the reference supplies the denominator
    assert O.relative_error(ref, y) == pytest.approx(0.05 / 0.5, rel=1e-12)
    assert O.relative_error(np.array([[8.0, 0.0]]), np.array([[4.0, 0.0]])) == pytest.approx(1.0)
    assert O.relative_error(np.array([[4.0, 0.0]]), np.array([[8.0, 0.0]])) == pytest.approx(0.5)


def test_companion_error_figures_hand_examples():
    ref = np.array([[3.0, -4.0], [0.0, 2.0]])
    y = np.array([[3.0, -3.0], [0.1, 2.0]])
    # rms: row 0 sqrt(0.5) / sqrt(12.5) = 0.2; row 1 sqrt(0.005) / sqrt(2) = 0.05
    assert O.rms_relative_error(y, ref) == pytest.approx(0.2, rel=1e-12)
    # damped element-wise, damping 0.5: row 0 -> 1 / (4 + 2) = 1/6; row 1 -> 0.1 / (0 + 1) = 0.1
    assert O.damped_elementwise_error(y, ref, damping=0.5) == pytest.approx(1.0 / 6.0, rel=1e-12)
    # default damping 1e-3: the small reference entry dominates: 0.1 / (0 + 0.002) = 50
    assert O.damped_elementwise_error(y, ref) == pytest.approx(50.0, rel=1e-12)
    assert O.rms_relative_error(ref, ref) == 0.0 and O.damped_elementwise_error(ref, ref) == 0.0
    assert O.rms_relative_error(np.array([[0.0, 0.5]]), np.zeros((1, 2))) == pytest.approx(np.sqrt(0.125))

