"""CPU-only checks of the block manager's host logic: the validity rule of the universal stack
(Section 2.3: no stack takes block i+1 before every stack has block i) and the byte accounting
against a budget (Eq. 9 per block, loading stops at the first block that does not fit)."""
import numpy as np

import paper_2410_23918_amd as B

E_RANGE, E_ARG = -3, -8


def _codes():
    L = B.lib()
    assert B.strerror(E_RANGE).startswith("n_loaded") and "selector" in B.strerror(E_ARG)
    return L


def _level_order(rng, slots):
    """A valid universal stack: level i holds, in random order, every stack that has a block i."""
    order = []
    for i in range(max(slots)):
        level = [s for s, n in enumerate(slots) if n > i]
        rng.shuffle(level)
        order += level
    return order


def test_order_check_accepts_levels_and_rejects_level_skips():
    _codes()
    rng = np.random.default_rng(3)
    for slots in ([4, 4, 4], [3, 5, 1, 4], [1], [2, 2, 2, 2, 2, 2, 2]):
        order = _level_order(rng, slots)
        assert B.order_check(slots, order) == 0
        for cut in range(len(order) + 1):             # a prefix of a valid order is valid
            assert B.order_check(slots, order[:cut]) == 0
    # stack 0 takes its second block while stack 2 still lacks its first
    assert B.order_check([2, 2, 2], [0, 1, 0, 2, 1, 2]) == E_ARG
    # an exhausted stack does not hold the others back
    assert B.order_check([1, 3], [1, 0, 1, 1]) == 0
    assert B.order_check([1, 3], [1, 1, 0, 1]) == E_ARG
    # more entries for a stack than it has blocks; a stack index out of range
    assert B.order_check([1, 1], [0, 1, 0]) == E_RANGE
    assert B.order_check([2, 2], [0, 2]) == E_RANGE
    assert B.order_check([2, 2], [0, -1]) == E_RANGE


def test_budget_position_counts_eq9_bytes_exactly():
    # the block sizes of one decoder layer of the 8B model (q, k, v, o, gate, up, down), k = 16
    shapes = [(4096, 4096), (1024, 4096), (1024, 4096), (4096, 4096), (14336, 4096), (14336, 4096), (4096, 14336)]
    bb = [B.block_bytes(o, i, 16) for o, i in shapes]
    assert bb[0] == 2359296 and bb[1] == 688128 and bb[4] == 7929856 and bb[6] == 7929856
    assert min(bb) == 688128                      # 0.66 MB: the smallest unit that moves in that model
    rng = np.random.default_rng(4)
    slots = [6] * len(shapes)
    order = _level_order(rng, slots)
    prefix = np.concatenate([[0], np.cumsum([bb[s] for s in order])])
    assert prefix[-1] == 6 * sum(bb)
    budgets = [0, 1, bb[order[0]] - 1, bb[order[0]], int(prefix[-1]) - 1, int(prefix[-1]), int(prefix[-1]) + 5, 2 ** 40]
    budgets += [int(v) for v in rng.integers(0, prefix[-1] + 1000, size=200)]
    budgets += [int(p) for p in prefix] + [int(p) - 1 for p in prefix[1:]] + [int(p) + 1 for p in prefix]
    last = None
    for budget in sorted(budgets):
        pos, tot = B.budget_position(bb, order, budget)
        want = int(np.searchsorted(prefix, budget, side="right")) - 1     # brute force: longest prefix that fits
        assert pos == want and tot == prefix[pos]
        assert tot <= budget and (pos == len(order) or tot + bb[order[pos]] > budget)
        assert last is None or pos >= last                                # monotone in the budget
        last = pos
    # nothing is skipped: a small block behind a large one that does not fit stays out
    pos, tot = B.budget_position([100, 10], [0, 1], 50)
    assert (pos, tot) == (0, 0)
