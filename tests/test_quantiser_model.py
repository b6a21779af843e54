"""CPU model of the decode kernel's panel arithmetic against the oracle: the 16-bit fixed-point
panel with class pre-division, and the finer scale of quiet steps (a step = the 32 columns of one
column class in one 256-column chunk) next to loud ones.  It pins the scheme itself, independent
of any GPU: with a few activation channels far above the rest -- the case activation-aware
scaling (Eq. 3-4) exists for -- the error of y stays well inside the 2e-3 parity bound, and it
would not without the per-step scale.  Written from the scheme's description, in numpy; shares
no code with the kernels."""
import numpy as np
import pytest

from oracle import bitstack_oracle as O
from workloads import synth as W

K_QMAX = 32512.0          # |code| <= 127 * 256


def _model_forward(st, x16, n, range_cols, per_step, fp16_arith=False):
    """y by the fixed-point scheme; per_step: quiet steps quantised 2^e finer, e in {0, 2, 3}."""
    inn = st.inn
    xs = (x16.astype(np.float32) * (np.float32(1.0) / st.s.astype(np.float32))).astype(np.float32)
    col = np.arange(inn)
    tc = (col % 8) & 3                                    # class weight of a column's sign byte: 2^(t mod 4)
    step_of = (col // 256) * 8 + (col % 8)                # (chunk, class)
    y = np.zeros(st.out)
    for b in range(n):
        V = st.V[b].astype(np.float32)
        U = st.U[b].astype(np.float64)
        S = st.S[b].astype(np.float64)
        for c0 in range(0, inn, range_cols):
            sl = slice(c0, min(inn, c0 + range_cols))
            T = (V[sl] * xs[sl, None]).astype(np.float64)
            amax = np.abs(T).max()
            if amax == 0.0:
                continue
            e = np.zeros(T.shape[0])
            if per_step:
                steps = step_of[sl]
                smax = np.zeros(steps.max() + 1)
                np.maximum.at(smax, steps, np.abs(T).max(axis=1))
                ratio = amax / np.maximum(smax[steps], 1e-300)
                fl = np.floor(np.log2(ratio))
                e = np.where(fl >= 2, np.minimum(fl, 3), 0.0)
            scale = np.exp2(e - tc[sl])[:, None] * (K_QMAX / amax)
            if fp16_arith:
                # x/s * scale rounded to fp16, product and rounding offset in fp16 as the packed quantiser does
                xf = (xs[sl].astype(np.float64) * scale[:, 0] / 32767.0).astype(np.float16).astype(np.float64)
                p = (V[sl].astype(np.float64) * xf[:, None]).astype(np.float16).astype(np.float64)
                code = np.rint(np.clip(p, -1, 1) * 32767.0)
            else:
                code = np.rint(np.clip(T * scale, -K_QMAX, K_QMAX))
            assert np.abs(code).max() <= 32767
            Tq = code / scale                               # what the integer sums stand for
            y += (U * (S[:, sl] @ Tq)).sum(axis=1)
    return y


def _case(out, inn, n, seed):
    rng = W.rng_for(3, seed, out, inn)
    s = W.column_scales(rng, inn)
    S, U, V = W.synthetic_blocks(rng, out, inn, n, 16, s, 0.02)
    return O.Stack(S, U, V, s), W.activations(W.rng_for(3, 100 + seed, 1, inn), 1, inn).astype(np.float32)


@pytest.mark.parametrize("channels,factor", [(1, 30.0), (1, 100.0), (1, 1000.0), (4, 100.0), (4, 1000.0), (32, 30.0), (32, 100.0)])
def test_outlier_channels_keep_parity_with_the_per_step_scale(channels, factor):
    st, x = _case(1024, 2048, 4, 5)
    idx = W.rng_for(3, 77, channels).choice(st.inn, channels, replace=False)
    x[0, idx] *= factor
    x16 = np.clip(x, -60000, 60000).astype(np.float16)
    ref = O.forward_dense(st, x16, st.n)
    for range_cols in (2048, 1024):
        with_steps = O.relative_error(_model_forward(st, x16[0], st.n, range_cols, True)[None], ref)
        without = O.relative_error(_model_forward(st, x16[0], st.n, range_cols, False)[None], ref)
        print(f"{channels} channel(s) x {factor:g}, ranges of {range_cols} columns: {with_steps:.2e} with the per-step scale, "
              f"{without:.2e} without")
        assert with_steps <= 1.0e-3
        assert with_steps <= without * 1.0001
    if factor >= 100.0 and channels <= 4:
        assert without > 2.0 * with_steps          # the scheme is what keeps these cases inside the bound


def test_plain_activations_both_arithmetics():
    st, x = _case(1024, 2048, 4, 6)
    x16 = x.astype(np.float16)
    ref = O.forward_dense(st, x16, st.n)
    e32 = O.relative_error(_model_forward(st, x16[0], st.n, 2048, True)[None], ref)
    e16 = O.relative_error(_model_forward(st, x16[0], st.n, 2048, True, fp16_arith=True)[None], ref)
    print(f"plain activations: {e32:.2e} (exact products), {e16:.2e} (fp16 products)")
    assert e32 <= 2.5e-4 and e32 < e16 <= 8.0e-4
