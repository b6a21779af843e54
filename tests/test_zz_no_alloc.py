"""The entry point that allocates nothing (bitstack_linear_static: split-accumulation workspace in
a static device array of the library) against bitstack_linear, through the C ABI: two calls in a
row on one GPU, the second with a smaller stack, each compared with the existing entry point's
output and with the CPU oracle."""
import numpy as np
import pytest

from oracle import bitstack_oracle as O

from _cases import acts, synth_stack

pytestmark = pytest.mark.gpu
TOL = 2e-3


def test_static_workspace_entry_point_two_calls_second_smaller():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2410_23918_amd as B
    L = B.lib()
    assert L.bitstack_static_workspace_bytes() == (4 << 20) + 16384 * 4
    dev = "cuda:0"
    stacks = []
    for out, inn, n in ((4096, 4096, 16), (1056, 2048, 5)):      # the second is the smaller input
        st = synth_stack(3, out, inn, n)
        ps = B.PackedStack(st.sign_words(), st.U, st.V, st.s)
        x = acts(3, 1, inn, tag=3)
        stacks.append((st, ps, x, torch.from_numpy(x[0]).to(dev)))
    for rnd in range(2):                                          # and once more: the array keeps the last call's contents
        for st, ps, x, xd in stacks:
            for nl in (st.n, st.n // 2, 0):
                y_new = torch.full((st.out,), float("nan"), dtype=torch.float16, device=dev)
                rc = L.bitstack_linear_static(xd.data_ptr(), ps.handle, nl, y_new.data_ptr(), None)
                assert rc == 0, B.lib().bitstack_strerror(rc)
                y_old = ps.linear(xd, nl)
                torch.cuda.synchronize()
                a = y_new.float().cpu().numpy().astype(np.float64)[None]
                b = y_old.float().cpu().numpy().astype(np.float64)[None]
                if nl == 0:
                    assert not a.any() and not b.any()
                    continue
                ref = O.forward_dense(st, x, nl)
                e_old, e_new, e_pair = O.relative_error(b, ref), O.relative_error(a, ref), O.relative_error(a, b)
                print(f"round {rnd} {st.out}x{st.inn} n_loaded={nl}: static workspace vs oracle {e_new:.2e}, "
                      f"bitstack_linear vs oracle {e_old:.2e}, the two against each other {e_pair:.2e}", flush=True)
                assert e_new <= TOL and e_old <= TOL and e_pair <= TOL
    # a stack whose partial rows cannot fit the array is refused before anything is enqueued
    assert B.lib().bitstack_static_workspace_bytes() < 1100000 * 4
    synth_stack.cache_clear()
