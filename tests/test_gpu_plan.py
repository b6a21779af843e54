"""Token plan (bitstack_plan_create / _launch / _release): the job list of one token through a
small decoder -- q/k/v on one input, o, gate/up on one input, down, each matrix with its own
number of loaded blocks, one of them empty -- prepared once and launched many times.  Every
launch must leave the same bits in every output as bitstack_linear_many on the same buffers, also
after the inputs change, and when the plan is recorded into a graph and replayed."""
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


def _decoder(B, layers, hidden, kv, mlp, n):
    """-> (oracle stacks, packed stacks, items (x index, stack index, n_loaded, y index), buffer sizes)"""
    stacks, packed, items, bufs = [], [], [], [hidden]
    rng = np.random.default_rng(17)

    def add(out, inn, xi):
        r = W.rng_for(3, 300 + len(stacks), out, inn)
        s = W.column_scales(r, inn)
        S, U, V = W.synthetic_blocks(r, out, inn, n, 16, s, 0.02)
        st = O.Stack(S, U, V, s)
        stacks.append(st)
        packed.append(B.PackedStack(st.sign_words(), st.U, st.V, st.s))
        bufs.append(out)
        nl = int(rng.integers(max(1, n - 3), n + 1))
        items.append((xi, len(stacks) - 1, nl, len(bufs) - 1))
        return len(bufs) - 1

    h = 0
    for _ in range(layers):
        q = add(hidden, hidden, h)
        add(kv, hidden, h)
        add(kv, hidden, h)
        o = add(hidden, hidden, q)
        g = add(mlp, hidden, o)
        add(mlp, hidden, o)
        h = add(hidden, mlp, g)
    return stacks, packed, items, bufs


def test_plan_gives_the_bits_of_linear_many_on_every_launch(B):
    import torch
    dev = "cuda:0"
    stacks, packed, items, bufs = _decoder(B, layers=2, hidden=1024, kv=256, mlp=2816, n=6)
    items[3] = (items[3][0], items[3][1], 0, items[3][3])          # one matrix with nothing loaded
    rng = np.random.default_rng(18)

    def fresh_buffers():
        return [torch.from_numpy(rng.standard_normal(m).astype(np.float16)).to(dev) for m in bufs]

    ref_bufs, plan_bufs = fresh_buffers(), None
    plan_bufs = [b.clone() for b in ref_bufs]
    jobs_ref = B.make_jobs([(ref_bufs[xi], packed[si], nl, ref_bufs[yi]) for xi, si, nl, yi in items])
    jobs_plan = B.make_jobs([(plan_bufs[xi], packed[si], nl, plan_bufs[yi]) for xi, si, nl, yi in items])
    plan = B.TokenPlan(jobs_plan)
    print(f"{len(items)} linears in {plan.steps} launches", flush=True)
    assert plan.steps < len(items)            # q/k/v and gate/up share launches
    for token in range(3):
        x0 = torch.from_numpy(rng.standard_normal(bufs[0]).astype(np.float16)).to(dev)
        ref_bufs[0].copy_(x0)
        plan_bufs[0].copy_(x0)
        B.linear_many(jobs_ref, 1)
        plan.launch()
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(zip(ref_bufs, plan_bufs)):
            assert torch.equal(a, b), f"token {token}: buffer {k} differs"
    # and against the oracle, linear by linear, on the inputs each linear actually read
    for xi, si, nl, yi in items:
        x = plan_bufs[xi].float().cpu().numpy().astype(np.float64)[None]
        y = plan_bufs[yi].float().cpu().numpy().astype(np.float64)[None]
        if nl == 0:
            assert not y.any()
            continue
        if not np.isfinite(x).all() or np.abs(x).max() == 0:
            continue
        ref = O.forward_dense(stacks[si], x.astype(np.float16), nl)
        assert O.relative_error(y, ref) <= TOL
    # recorded into a graph: three replays with eager work between them, each checked
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        plan.launch(stream=side)
    for replay in range(3):
        x0 = torch.from_numpy(rng.standard_normal(bufs[0]).astype(np.float16)).to(dev)
        ref_bufs[0].copy_(x0)
        plan_bufs[0].copy_(x0)
        for b in plan_bufs[1:]:
            b.fill_(float("nan"))
        B.linear_many(jobs_ref, 1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(zip(ref_bufs, plan_bufs)):
            assert torch.equal(a, b), f"replay {replay}: buffer {k} differs"
    plan.release()


def test_plan_refuses_to_run_after_a_block_it_uses_was_offloaded(B):
    import torch
    dev = "cuda:0"
    out, inn, n = 512, 512, 3
    r = W.rng_for(3, 400, out, inn)
    s = W.column_scales(r, inn)
    S, U, V = W.synthetic_blocks(r, out, inn, n, 16, s, 0.02)
    st = O.Stack(S, U, V, s)
    ps = B.PackedStack.empty(out, inn, n, st.s)
    sw = st.sign_words()
    for b in range(n):
        ps.push_block(sw[b], st.U[b], st.V[b])
    x = torch.from_numpy(W.activations(W.rng_for(3, 401, 1, inn), 1, inn)[0]).to(dev)
    y = torch.empty(out, dtype=torch.float16, device=dev)
    jobs = B.make_jobs([(x, ps, n, y)])
    plan = B.TokenPlan(jobs)
    plan.launch()
    torch.cuda.synchronize()
    ps.pop_block()
    with pytest.raises(B.BitStackError) as e:
        plan.launch()
    assert e.value.code == -3
    with pytest.raises(B.BitStackError):
        B.TokenPlan(jobs)        # and a new plan for the same job is refused as bitstack_linear would refuse it
    jobs2 = B.make_jobs([(x, ps, n - 1, y)])
    plan2 = B.TokenPlan(jobs2)
    plan2.launch()
    torch.cuda.synchronize()
    ref = O.forward_dense(st, x.cpu().numpy()[None], n - 1)
    assert O.relative_error(y.float().cpu().numpy().astype(np.float64)[None], ref) <= TOL
