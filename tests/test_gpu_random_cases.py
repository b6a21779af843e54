"""Seeded random shapes, stack heights, batch sizes and entry points against the oracle: the
launchers pick tile heights, column splits, tokens per decode launch and kernels from the
arguments, and this walks through combinations the hand-picked cases do not name."""
from __future__ import annotations

import numpy as np
import pytest

from oracle import bitstack_oracle as O
from workloads import synth as W

pytestmark = pytest.mark.gpu
TOL = 2e-3   # max |y - y_ref| / max |y_ref| per token row


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2410_23918_amd as B
    B.lib()
    return B


@pytest.mark.parametrize("seed,cases,big", [(11, 30, False), (12, 16, True)])
def test_random_shapes_batches_and_entry_points(B, seed, cases, big):
    import torch
    rng = np.random.default_rng(seed)
    for case in range(cases):
        out = int(rng.integers(1, 140 if big else 70)) * 32
        inn = int(rng.integers(1, 11)) * 256
        n = int(rng.integers(1, 13 if big else 7))
        max_batch = int(rng.choice([2, 5, 33, 64, 100, 600, 2100] if big else [1, 3, 16, 64, 65, 200, 300]))
        batch = int(rng.integers(1, max_batch + 1))
        nl = int(rng.integers(0, n + 1))
        mode = str(rng.choice(["auto", "decode", "panel", "scratch", "materialised"]))
        if mode == "decode" and batch > 9:
            batch = int(rng.integers(1, 10))
        f32 = bool(rng.integers(0, 2))
        print(f"seed {seed} case {case}: {out}x{inn} n={n} max_batch={max_batch} batch={batch} n_loaded={nl} "
              f"{mode} {'f32' if f32 else 'f16'}", flush=True)
        r = W.rng_for(3, 1000 * seed + case, out, inn)
        s = W.column_scales(r, inn)
        S, U, V = W.synthetic_blocks(r, out, inn, n, 16, s, 0.02)
        st = O.Stack(S, U, V, s)
        ps = B.PackedStack(st.sign_words(), st.U, st.V, st.s, max_batch=max_batch)
        x = W.activations(W.rng_for(3, 2000 * seed + case, batch, inn), batch, inn)
        xd = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
        dt = torch.float32 if f32 else torch.float16
        ws = torch.empty(B.dense_bytes(out, inn), dtype=torch.uint8, device="cuda:0")
        if mode == "auto":
            y = ps.linear_batched(xd, nl, out_dtype=dt)
        elif mode == "decode":
            y = ps.linear_batched(xd, nl, out_dtype=dt, kernel=B.KERNEL_DECODE)
        elif mode == "panel":
            y = ps.linear_batched(xd, nl, out_dtype=dt, kernel=B.KERNEL_PANEL)
        elif mode == "scratch":
            y = ps.linear_batched_ws(xd, nl, workspace=ws, out_dtype=dt)
        else:
            y = ps.linear_materialised(xd, nl, ws, out_dtype=dt)
        torch.cuda.synchronize()
        y = y.float().cpu().numpy().astype(np.float64)
        assert y.shape == (batch, out)
        if nl == 0:
            assert not y.any()
        else:
            err = O.relative_error(y, O.forward_dense(st, x, nl))
            print(f"   rel err {err:.2e}", flush=True)
            assert err <= TOL
        ps.release()
