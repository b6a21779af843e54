"""Bounded stress of the split accumulation (partial rows in the workspace, one arrival counter per
row slab, the last workgroup to arrive adds the rows up): many calls back to back on one handle,
alternating the number of loaded blocks and the work split, each output compared bit for bit with
the first one its combination produced.  The sums are taken in a fixed order, so any difference
means a partial row was read before it was written or a counter was left non-zero."""
from __future__ import annotations

import itertools

import numpy as np
import pytest

from oracle import bitstack_oracle as O

from _cases import acts, synth_stack

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2410_23918_amd as B
    B.lib()
    return B


def _reset(B):
    for opt in (B.OPT_DECODE_TILES, B.OPT_DECODE_KS_CHUNKS, B.OPT_DECODE_BGROUPS, B.OPT_DECODE_EARLY):
        B.set_option(opt, 0)


def test_decode_split_accumulation_ten_thousand_calls(B):
    import torch
    out, inn, n = 2048, 4096, 8
    st = synth_stack(3, out, inn, n)
    ps = B.PackedStack(st.sign_words(), st.U, st.V, st.s)
    x = acts(3, 1, inn, tag=5)
    xd = torch.from_numpy(x[0]).to("cuda:0")
    combos = [c for c in itertools.product((8, 3, 5, 1), (0, 1, 2, 4, 8), (0, 2, 4, 16))
              if c[1] <= max(c[0], 1)]
    first, refused = {}, 0
    order = np.random.default_rng(5).integers(0, len(combos), size=10000)
    y = torch.empty(out, dtype=torch.float16, device="cuda:0")
    try:
        for call, ci in enumerate(order):
            nl, bg, ksc = combos[ci]
            B.set_option(B.OPT_DECODE_BGROUPS, bg)
            B.set_option(B.OPT_DECODE_KS_CHUNKS, ksc)
            try:
                ps.linear(xd, nl, y=y)
            except B.BitStackError:
                # finer than the stack's workspace was sized for: refused before anything is
                # enqueued, every time
                assert first.setdefault(ci, None) is None
                refused += 1
                continue
            if ci not in first:
                first[ci] = y.clone()
                ref = O.forward_dense(st, x, nl)
                err = O.relative_error(first[ci].float().cpu().numpy().astype(np.float64)[None], ref)
                assert err <= TOL, (combos[ci], err)
            elif first[ci] is None:
                pytest.fail(f"call {call}: {combos[ci]} was refused before and is served now")
            elif not torch.equal(y, first[ci]):
                bad = int((y != first[ci]).sum())
                pytest.fail(f"call {call}: n_loaded={nl} bgroups={bg} ks_chunks={ksc}: {bad} of {out} outputs "
                            f"differ from the first result of this combination")
    finally:
        _reset(B)
    assert len(first) == len(combos)
    served = sum(v is not None for v in first.values())
    print(f"{served} of {len(combos)} combinations served, {refused} calls refused", flush=True)
    assert served >= len(combos) // 2


def test_batch_kernel_column_split_three_thousand_calls(B):
    import torch
    out, inn, n, batch = 256, 4096, 6, 8      # few row tiles, long rows: the small-batch kernel splits the columns
    st = synth_stack(3, out, inn, n)
    ps = B.PackedStack(st.sign_words(), st.U, st.V, st.s, max_batch=batch)
    x = acts(3, batch, inn, tag=6)
    xd = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
    first = {}
    order = np.random.default_rng(6).integers(1, n + 1, size=3000)
    y = torch.empty((batch, out), dtype=torch.float16, device="cuda:0")
    for call, nl in enumerate(order):
        nl = int(nl)
        ps.linear_batched(xd, nl, y=y, kernel=B.KERNEL_PANEL)
        if nl not in first:
            first[nl] = y.clone()
            ref = O.forward_dense(st, x, nl)
            err = O.relative_error(first[nl].float().cpu().numpy().astype(np.float64), ref)
            assert err <= TOL, (nl, err)
        elif not torch.equal(y, first[nl]):
            bad = int((y != first[nl]).sum())
            pytest.fail(f"call {call}: n_loaded={nl}: {bad} of {batch * out} outputs differ from the first result")
