"""Block manager on the device: several stacks of different shapes under one byte budget that
rises and falls (Section 2.2-2.3).  After every change each stack holds exactly the prefix the
universal stack and the budget give it, the byte count is Eq. 9's, and every stack's forward pass
matches the oracle's forward over that prefix."""
from __future__ import annotations

import numpy as np
import pytest

from oracle import bitstack_oracle as O
from workloads import synth as W

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


def test_budget_rises_and_falls_every_stack_matches_the_oracle_prefix(B):
    import torch
    dev = "cuda:0"
    shapes = [(512, 512, 4), (1056, 768, 4), (256, 1024, 3), (2048, 2048, 4)]   # (out, in, blocks)
    stacks, packed, xs = [], [], []
    for si, (out, inn, n) in enumerate(shapes):
        rng = W.rng_for(3, 40 + si, out, inn)
        s = W.column_scales(rng, inn)
        S, U, V = W.synthetic_blocks(rng, out, inn, n, 16, s, 0.02)
        st = O.Stack(S, U, V, s)
        stacks.append(st)
        packed.append(B.PackedStack.empty(out, inn, n, st.s))
        xs.append(W.activations(W.rng_for(3, 140 + si, 1, inn), 1, inn))
    mgr = B.BlockManager(packed)
    for si, st in enumerate(stacks):
        sw = st.sign_words()
        for b in range(st.n):
            mgr.stage_block(si, b, sw[b], st.U[b], st.V[b])
    # the universal stack: level by level, inside a level by a seeded stand-in for the importance scores
    rng = np.random.default_rng(8)
    order = []
    for level in range(4):
        members = [si for si, sh in enumerate(shapes) if sh[2] > level]
        rng.shuffle(members)
        order += members
    # a skip across levels is refused, and so is a budget before every block on the way is staged
    bad = list(order)
    bad[0], bad[len(shapes)] = bad[len(shapes)], bad[0]
    if bad != order and B.order_check([sh[2] for sh in shapes], bad) != 0:
        with pytest.raises(B.BitStackError):
            mgr.set_order(bad)
    mgr.set_order(order)
    bb = [B.block_bytes(out, inn, 16) for out, inn, _ in shapes]
    prefix = np.concatenate([[0], np.cumsum([bb[s] for s in order])])
    total = int(prefix[-1])
    budgets = [0, total, total // 2, total // 3, int(prefix[5]), int(prefix[5]) - 1, total + 7, bb[order[0]], 0,
               int(prefix[9]) + 1, total]
    xd = [torch.from_numpy(x[0]).to(dev) for x in xs]
    pos_before = 0
    for budget in budgets:
        up, down = mgr.set_budget(budget)
        pos = mgr.position
        want = int(np.searchsorted(prefix, budget, side="right")) - 1
        assert pos == want
        assert mgr.resident_bytes == prefix[pos] <= budget
        assert pos == len(order) or mgr.resident_bytes + bb[order[pos]] > budget
        assert (up, down) == (max(0, pos - pos_before), max(0, pos_before - pos))
        pos_before = pos
        heights = [order[:pos].count(si) for si in range(len(shapes))]
        unfinished = [h for h, sh in zip(heights, shapes) if h < sh[2]]
        assert not unfinished or max(heights) - min(unfinished) <= 1    # heights differ by at most one block
        assert sum(p.resident_bytes for p in packed) == mgr.resident_bytes
        for si, st in enumerate(stacks):
            nl = mgr.n_loaded(si)
            assert nl == heights[si] == packed[si].resident_blocks
            y = packed[si].linear(xd[si], nl)
            torch.cuda.synchronize()
            yv = y.float().cpu().numpy().astype(np.float64)[None]
            if nl == 0:
                assert not yv.any()
                continue
            err = O.relative_error(yv, O.forward_dense(st, xs[si], nl))
            print(f"budget {budget}: stack {si} {st.out}x{st.inn} n_loaded={nl}: {err:.2e}", flush=True)
            assert err <= TOL
    mgr.release()
