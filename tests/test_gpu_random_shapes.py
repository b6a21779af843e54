"""Seeded random walk over the forward calls: shape, stack height, loaded prefix, batch, output
type and entry point are drawn per case (out a multiple of 32 up to 4448, in a multiple of 256 up
to 2560, up to 12 blocks, batches up to 700, prefixes including the empty one), and every result is
compared with the oracle's dense forward under the parity bound.  The fixed-shape tests aim at known
tile edges; this one covers the combinations nobody listed."""
from __future__ import annotations

import numpy as np
import pytest

from oracle import bitstack_oracle as O
from workloads import synth as W

pytestmark = pytest.mark.gpu
TOL = 2e-3
CASES = 48
MODES = ("library's choice", "decode kernel", "batch kernels", "library's choice with a scratch",
         "materialised, caller's scratch", "materialised, image's scratch")


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2410_23918_amd as B
    B.lib()
    return B


def _draw(rng):
    out = int(rng.integers(1, 140)) * 32
    inn = int(rng.integers(1, 11)) * 256
    n = int(rng.integers(1, 13))
    max_batch = int(rng.choice([2, 5, 33, 64, 100, 300, 700]))
    batch = int(rng.integers(1, max_batch + 1))
    n_loaded = int(rng.integers(0, n + 1))
    mode = int(rng.integers(0, len(MODES)))
    if mode == 1 and batch > 9:                 # the decode kernel takes tokens one to four per launch
        batch = int(rng.integers(1, 10))
    if mode == 5:                               # needs the activation scratch of an image packed for many tokens:
        max_batch = max(max_batch, 1024)        # at least 1024 rows of the dense weight fit it
    f32 = bool(rng.integers(0, 2))
    tile = int(rng.integers(0, 4))              # dense product's output tile on the materialising paths (0: its own choice)
    return out, inn, n, max_batch, batch, n_loaded, mode, f32, tile


def test_random_shapes_and_entry_points(B):
    import torch
    rng = np.random.default_rng(2410_23918)
    worst = 0.0
    for case in range(CASES):
        out, inn, n, max_batch, batch, n_loaded, mode, f32, tile = _draw(rng)
        dt = torch.float32 if f32 else torch.float16
        print(f"case {case}: {out}x{inn} n={n} max_batch={max_batch} batch={batch} n_loaded={n_loaded} "
              f"{'f32' if f32 else 'f16'} {MODES[mode]} tile={tile}", flush=True)
        r = W.rng_for(3, 1000 + case, out, inn)
        s = W.column_scales(r, inn)
        S, U, V = W.synthetic_blocks(r, out, inn, n, 16, s, 0.02)
        st = O.Stack(S, U, V, s)
        ps = B.PackedStack(st.sign_words(), st.U, st.V, st.s, max_batch=max_batch)
        x = W.activations(W.rng_for(3, 2000 + case, batch, inn), batch, inn)
        xd = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
        ws = torch.empty(B.dense_bytes(out, inn), dtype=torch.uint8, device="cuda:0")
        B.set_option(B.OPT_DENSE_TILE, tile)
        try:
            if mode == 0:
                y = ps.linear_batched(xd, n_loaded, out_dtype=dt)
            elif mode == 1:
                y = ps.linear_batched(xd, n_loaded, out_dtype=dt, kernel=B.KERNEL_DECODE)
            elif mode == 2:
                y = ps.linear_batched(xd, n_loaded, out_dtype=dt, kernel=B.KERNEL_PANEL)
            elif mode == 3:
                y = ps.linear_batched_ws(xd, n_loaded, workspace=ws, out_dtype=dt)
            elif mode == 4:
                y = ps.linear_materialised(xd, n_loaded, ws, out_dtype=dt)
            else:
                y = ps.linear_batched(xd, n_loaded, out_dtype=dt, kernel=B.KERNEL_MATERIALISE)
            torch.cuda.synchronize()
        finally:
            B.set_option(B.OPT_DENSE_TILE, 0)
        assert y.shape == (batch, out) and y.dtype == dt
        y = y.float().cpu().numpy().astype(np.float64)
        if n_loaded == 0:
            assert not y.any(), case
        else:
            err = O.relative_error(y, O.forward_dense(st, x, n_loaded))
            print(f"   rel err {err:.2e}", flush=True)
            worst = max(worst, err)
            assert err <= TOL, (case, err)
        ps.release()
    print(f"worst of {CASES} cases: {worst:.2e}", flush=True)
