#!/usr/bin/env python3
"""Benchmark of the BitStack linear-layer forward path on one MI355X.

Metric: effective block-stream GB/s (and % of the 8 TB/s HBM peak) of batch-1
decode through a 4096x4096 Llama-3-8B-shaped projection held as n = 16 loaded
residual blocks (k = 16): value = n * block_bytes / time per call, block_bytes =
(out*in + 16*k*(out+in)) / 8 (the paper's residual-block size formula).

A step is one call of bitstack_linear (the whole hot path: activation scaling,
panel staging, sign-stream contraction, U epilogue, cross-block accumulation) on
inputs resident in HBM.  Steps rotate over enough separately packed copies of the
stack that the working set exceeds the 256 MB last-level cache.

Prints ONE JSON line on stdout; a per-shape table goes to stderr with --table.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Blocks:
    """Seeded synthetic stack for the benchmark (workloads.synth): coin-flip signs and fp16
    factors with the magnitude profile of a real decomposition.  The kernels' work does not
    depend on the values; parity on a true decomposition of this shape is a test."""

    def __init__(self, out, inn, n, config):
        from workloads import synth as W
        cfg = W.CONFIGS[config]
        rng = W.rng_for(config, 10, out, inn)
        self.s = W.column_scales(rng, inn)
        self.S, self.U, self.V = W.synthetic_blocks(rng, out, inn, n, 16, self.s, cfg["sigma_w"])

    def sign_words(self):
        """Canonical packing: bit b of word w of a row = (S[row, 32 w + b] > 0)."""
        n, out, inn = self.S.shape
        bits = np.packbits(self.S > 0, axis=-1, bitorder="little")
        return np.ascontiguousarray(bits).view("<u4").reshape(n, out, inn // 32)


_stack_cache = {}


def build_stack(out, inn, n, config: int):
    """Generated once per shape (the MLP shapes serve the batch-1 and the batch tables)."""
    key = (out, inn, n, config)
    if key not in _stack_cache:
        if len(_stack_cache) >= 2:
            _stack_cache.pop(next(iter(_stack_cache)))
        _stack_cache[key] = Blocks(out, inn, n, config)
    return _stack_cache[key]


def time_calls(B, torch, jobs, steps, warmup):
    """Whole-job time of `steps` calls (events on the stream the kernels run on)."""
    per = len(jobs._keepalive)
    B.linear_many(jobs, max(1, (warmup + per - 1) // per))
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    reps, tail = divmod(steps, per)
    e0.record()
    if reps:
        B.linear_many(jobs, reps)
    if tail:
        B.linear_many(B.make_jobs(jobs._keepalive[:tail]), 1)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3  # seconds


def kernel_durations(B, torch, items, steps):
    """Average duration of one launch: an event pair around every call."""
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for i in range(steps):
        x, ps, nl, y = items[i % len(items)]
        evs[i][0].record()
        ps.linear(x, nl, y)
        evs[i][1].record()
    torch.cuda.synchronize()
    d = np.array([a.elapsed_time(b) for a, b in evs]) * 1e-3
    return float(d.mean()), float(np.median(d)), float(d.min())


def cpu_baseline(blocks, x, n_loaded, block_stream_bytes, y_gpu, budget_s=12.0):
    """The oracle's dense reconstruct-then-matmul, as it stands, on the host cores; the only
    place where this script touches the oracle.  Also compares the timed GPU outputs with it."""
    from oracle import bitstack_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([int(p.get("num_threads", 1)) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    stack = O.Stack(blocks.S, blocks.U, blocks.V, blocks.s)
    t0 = time.perf_counter()
    calls = 0
    while True:
        ref = O.forward_dense(stack, x, n_loaded)
        calls += 1
        el = time.perf_counter() - t0
        if el >= budget_s or calls >= 16:
            break
    per = el / calls
    err = max(O.relative_error(y[None], ref) for y in y_gpu)
    log(f"[bench] max relative error of the timed GPU outputs vs oracle: {err:.2e}")
    assert err <= 2e-3, err
    return {
        "value": round(block_stream_bytes / per / 1e9, 4),
        "unit": "GB/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"{calls} full calls of oracle.forward_dense (fp64 reconstruct-then-matmul) on the same "
                  f"4096x4096, n=16 stack and x; {per * 1e3:.0f} ms per call",
        "max_rel_err_gpu_vs_oracle": float(f"{err:.3e}"),
    }


def read_ceiling(B, torch, dev):
    """Achievable HBM read rate of this machine: a plain 128-bit read stream (k_stream_read) over
    buffers of the sizes the decode figures are quoted on, rotating over enough distinct buffers
    that the stream comes from HBM."""
    out = {}
    sink = torch.zeros(64, dtype=torch.uint8, device=dev)
    for label, nbytes in (("38MiB", 38 << 20), ("128MiB", 128 << 20), ("1GiB", 1 << 30)):
        copies = max(2, int((768 << 20) // nbytes) + 1)
        bufs = [torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(copies)]
        for b in bufs:
            B.probe_read(b, sink, 4096)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 6
        e0.record()
        for _ in range(reps):
            for b in bufs:
                B.probe_read(b, sink, 4096)
        e1.record()
        torch.cuda.synchronize()
        gbs = nbytes * copies * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
        out[label] = round(gbs, 1)
        log(f"[bench] read probe, {label} buffers x {copies}: {gbs:.0f} GB/s ({gbs / HBM_PEAK_GBS * 100:.1f}% of 8 TB/s)")
        del bufs
    return out


def mlp_table(B, torch, dev, n, ceiling):
    """Config 3 at batch 1 (plus the 1024x4096 k/v projection shape): one call = one launch,
    rotating over packed copies."""
    from workloads import synth as W
    rows = []
    for (o, i) in [(14336, 4096), (4096, 14336), (1024, 4096)]:
        s2 = build_stack(o, i, n, 3)
        copies = max(2, min(16, int(700e6 // (n * B.block_bytes(o, i))) + 1))
        sw2 = s2.sign_words()
        pst = [B.PackedStack(sw2, s2.U, s2.V, s2.s) for _ in range(copies)]
        x2 = torch.from_numpy(W.activations(W.rng_for(3, 100, 1, i), 1, i)[0]).to(dev)
        x2c = [x2.clone() for _ in range(copies)]   # one launch per call: shared inputs would be merged
        y2 = [torch.empty(o, dtype=torch.float16, device=dev) for _ in range(copies)]
        j2 = B.make_jobs([(x2c[k], pst[k], n, y2[k]) for k in range(copies)])
        B.linear_many(j2, 40)     # the device has idled while the host built the stack: back to full clocks first
        torch.cuda.synchronize()
        t = time_calls(B, torch, j2, copies * 40, copies) / (copies * 40)
        bb = n * B.block_bytes(o, i)
        gbs = bb / t / 1e9
        log(f"[bench] {o}x{i} n={n} batch 1: {t * 1e6:.2f} us/call, {gbs:.0f} GB/s "
            f"({gbs / HBM_PEAK_GBS * 100:.1f}% of 8 TB/s)")
        row = {"shape": f"{o}x{i}", "batch": 1, "n_loaded": n, "us_per_call": round(t * 1e6, 2), "GBps": round(gbs, 1),
               "pct_of_hbm_peak": round(gbs / HBM_PEAK_GBS * 100, 2)}
        if ceiling:
            row["pct_of_read_ceiling"] = round(gbs / ceiling["128MiB"] * 100, 1)
        rows.append(row)
        del pst, j2
    return rows


def batch_table(B, torch, dev, n):
    """Batch path (row a6): forced batch kernels at the MLP shapes of configs 3 and 5, one packed
    copy each, inputs resident; for the prefill-sized batches also the materialising path
    (restore to a dense fp16 scratch, then the dense product).  Useful FLOP/s = 2 * out * in *
    tokens / time."""
    from workloads import synth as W

    def timed(fn, reps):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    rows = []
    names = {B.KERNEL_DECODE: "decode kernel, up to four tokens per launch", B.KERNEL_PANEL: None,
             B.KERNEL_MATERIALISE: "restore + k_gemm in row slabs through the image's own activation scratch"}
    for cfg, (o, i), batches in ((3, (14336, 4096), (4, 16, 64, 512, 2048)), (3, (4096, 14336), (4, 16)),
                                 (5, (28672, 8192), (128, 2048))):
        st = build_stack(o, i, n, cfg)
        ps = B.PackedStack(st.sign_words(), st.U, st.V, st.s, max_batch=max(batches))
        del st
        wd = torch.empty((o, i), dtype=torch.float16, device=dev) if max(batches) > 64 else None
        for b in batches:
            x = torch.from_numpy(W.activations(W.rng_for(cfg, 100, b, i), b, i)).to(dev)
            y = torch.empty((b, o), dtype=torch.float16, device=dev)
            # the library's own choice of kernel (no scratch buffer lent)
            us = timed(lambda: ps.linear_batched(x, n, y=y), 10 if b <= 64 else 3)
            tf = 2.0 * o * i * b / us / 1e6
            kern = names[B.choose_kernel(o, i, n, max(batches), b, n)] or (
                "k_fused" if b <= 32 else "k_fused or k_xpack + k_tile, the launcher's estimate" if b <= 64
                else "k_xpack + k_tile")
            log(f"[bench] batch path {o}x{i} n={n} tokens={b} ({kern}): {us:.1f} us, {tf:.1f} useful TFLOP/s")
            rows.append({"shape": f"{o}x{i}", "tokens": b, "kernel": kern, "us": round(us, 1),
                         "useful_TFLOPs": round(tf, 2)})
            if B.choose_kernel(o, i, n, max(batches), b, n) == B.KERNEL_MATERIALISE:
                # the kernel that rebuilds weight tiles on chip, for comparison
                ut = timed(lambda: ps.linear_batched(x, n, y=y, kernel=B.KERNEL_PANEL), 3)
                tft = 2.0 * o * i * b / ut / 1e6
                log(f"[bench] batch path {o}x{i} n={n} tokens={b} (k_xpack + k_tile, forced): {ut:.1f} us, "
                    f"{tft:.1f} useful TFLOP/s")
                rows.append({"shape": f"{o}x{i}", "tokens": b, "kernel": "k_xpack + k_tile (forced)", "us": round(ut, 1),
                             "useful_TFLOPs": round(tft, 2)})
            if b > 64:
                y2 = torch.empty_like(y)
                um = timed(lambda: ps.linear_materialised(x, n, wd, y=y2), 3)
                ur = timed(lambda: ps.restore_weight(n, wd), 3)
                tfm = 2.0 * o * i * b / um / 1e6
                diff = (y2.float() - y.float()).abs().max().item() / y.float().abs().max().item()
                log(f"[bench] materialising path {o}x{i} n={n} tokens={b} (k_tile<restore> + k_gemm): "
                    f"{um:.1f} us ({ur:.1f} us of it restoring), {tfm:.1f} useful TFLOP/s; "
                    f"max |difference| to the batch kernel / max |y| = {diff:.1e}")
                rows.append({"shape": f"{o}x{i}", "tokens": b, "kernel": "restore + k_gemm", "us": round(um, 1),
                             "restore_us": round(ur, 1), "useful_TFLOPs": round(tfm, 2)})
                if b >= 512:
                    # the same through a scratch of 128 MiB (a slab of rows at a time, the scratch stays in
                    # the last-level cache): what a caller gets who lends one small buffer for all stacks
                    slab = wd.view(-1)[: (128 << 20) // 2]
                    y3 = torch.empty_like(y)
                    usl = timed(lambda: ps.linear_materialised(x, n, slab, y=y3), 3)
                    tfs = 2.0 * o * i * b / usl / 1e6
                    # (the product's output tile is chosen per slab, so the last bits may differ)
                    dslab = (y3.float() - y2.float()).abs().max().item() / y2.float().abs().max().item()
                    log(f"[bench] materialising path in row slabs, 128 MiB scratch, {o}x{i} n={n} tokens={b}: "
                        f"{usl:.1f} us, {tfs:.1f} useful TFLOP/s; max |difference| to the full scratch / max |y| = {dslab:.1e}")
                    rows.append({"shape": f"{o}x{i}", "tokens": b, "kernel": "restore + k_gemm in row slabs, 128 MiB scratch",
                                 "us": round(usl, 1), "useful_TFLOPs": round(tfs, 2), "max_diff_to_full_scratch": dslab})
        del ps, wd
    return rows


def decompose_table(B, torch, dev, iterations=16):
    """The decomposition on the device (bitstack_decompose): time per residual block at the 4096x4096
    and 14336x4096 shapes.  Bytes per block as the kernels move them: the fp32 residual is read by
    the sign packing, by the conversion to bf16 (which writes |R| and its transpose), by the
    Rayleigh-Ritz product, and read and written by the residual update (5 x 4 bytes per element);
    the 2 * iterations + 1 tall products of the power rounds read one bf16 copy each."""
    from workloads import synth as W
    rows = []
    for cfg, (o, i), nblk in ((2, (4096, 4096), 4), (3, (14336, 4096), 2)):
        c = W.CONFIGS[cfg]
        rng = W.rng_for(cfg, 0)
        Wt = W.dense_weight(rng, o, i, c["sigma_w"], c["fp16_weights"])
        s = W.column_scales(rng, i)
        Wd = torch.from_numpy(np.ascontiguousarray(Wt, dtype=np.float32)).to(dev)
        B.decompose(Wd, s, 1, iterations=iterations)          # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sw, U, V = B.decompose(Wd, s, nblk, iterations=iterations)   # synchronises before returning
        ms = (time.perf_counter() - t0) * 1e3 / nblk
        bytes_per_block = (5 * 4 + (2 + 2 * iterations + 1) * 2) * o * i
        gbs = bytes_per_block / ms / 1e6
        log(f"[bench] decomposition on the device {o}x{i}, {iterations} iterations: {ms:.1f} ms per block, "
            f"{gbs:.0f} GB/s of residual traffic, fp32 and bf16 passes ({gbs / HBM_PEAK_GBS * 100:.1f}% of 8 TB/s)")
        rows.append({"shape": f"{o}x{i}", "iterations": iterations, "ms_per_block": round(ms, 2),
                     "residual_GBs": round(gbs, 1)})
        del Wd, sw, U, V
    return rows


def decoder_token(B, torch, dev, layers=32, n_pack=24):
    """Config 4: one token through 7 linears x 32 layers, per-matrix n_loaded ~ U{8..24}.
    One layer's seven stacks are generated on the host; every layer gets its own packed
    device copy (distinct memory is what the HBM stream sees)."""
    from workloads import synth as W
    shapes = W.llama3_8b_layer_shapes()
    nl = W.variable_n_loaded(W.rng_for(4, 0), layers * len(shapes))
    t0 = time.time()
    host = []
    for m, (name, o, i) in enumerate(shapes):
        st = build_stack(o, i, n_pack, 4)
        host.append((st.sign_words(), st.U, st.V, st.s))
    packed = [[B.PackedStack(*host[m]) for m in range(len(shapes))] for _ in range(layers)]
    log(f"[bench] decoder: generated and packed {layers * len(shapes)} stacks (n={n_pack}) in {time.time() - t0:.0f} s")
    # inputs as a decoder layer has them: q/k/v read one vector, o another, gate/up a third, down a
    # fourth (the native loop merges only calls that read the same vector: 4 launches per layer)
    def vec(width, tag):
        return torch.from_numpy(W.activations(W.rng_for(4, 100 + tag, 1, width), 1, width)[0]).to(dev)
    x_of = {"q_proj": vec(4096, 0), "o_proj": vec(4096, 1), "gate_proj": vec(4096, 2), "down_proj": vec(14336, 3)}
    x_of["k_proj"] = x_of["v_proj"] = x_of["q_proj"]
    x_of["up_proj"] = x_of["gate_proj"]
    items, total_bytes = [], 0
    for l in range(layers):
        for m, (name, o, i) in enumerate(shapes):
            n_l = int(nl[l * len(shapes) + m])
            y = torch.empty(o, dtype=torch.float16, device=dev)
            items.append((x_of[name], packed[l][m], n_l, y))
            total_bytes += n_l * B.block_bytes(o, i)
    jobs = B.make_jobs(items)
    B.linear_many(jobs, 2)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    reps = 5
    e0.record()
    B.linear_many(jobs, reps)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    gbs = total_bytes / ms / 1e6
    log(f"[bench] decoder token: {len(items)} linears, {total_bytes / 1e9:.2f} GB of blocks, {ms:.3f} ms/token, "
        f"{gbs:.0f} GB/s ({gbs / HBM_PEAK_GBS * 100:.1f}% of 8 TB/s)")
    # the same token through a plan made once (grouping, work splits and argument blocks are not
    # recomputed per token); its outputs must be the native loop's, bit for bit
    ms_plan, plan_steps = None, None
    try:
        want = [it[3].clone() for it in items]
        for it in items:
            it[3].zero_()
        plan = B.TokenPlan(jobs)
        plan_steps = plan.steps
        plan.launch()
        torch.cuda.synchronize()
        assert all(torch.equal(a, it[3]) for a, it in zip(want, items)), "plan launch differs from bitstack_linear_many"
        for _ in range(2):   # the comparison above left the device idle: same warm-up as the native loop had
            plan.launch()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            plan.launch()
        e1.record()
        torch.cuda.synchronize()
        ms_plan = e0.elapsed_time(e1) / reps
        log(f"[bench] decoder token through a plan ({plan_steps} launches): {ms_plan:.3f} ms/token, "
            f"{total_bytes / ms_plan / 1e6:.0f} GB/s")
        plan.release()
    except Exception as ex:
        log(f"[bench] decoder token plan variant skipped: {type(ex).__name__}: {ex}")
    # the same token as one captured graph (the launches carry no memset nodes); replayed with
    # eager work between replays and compared with the eager outputs
    ms_graph = None
    try:
        eager = [it[3].clone() for it in items[:14]]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            B.linear_many(jobs, 1, stream=side)
        torch.cuda.current_stream().wait_stream(side)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            B.linear_many(jobs, 1, stream=torch.cuda.current_stream())
        for _ in range(3):
            for it in items[:14]:
                it[3].zero_()
            g.replay()
            torch.cuda.synchronize()
            assert all(torch.equal(a, it[3]) for a, it in zip(eager, items[:14])), "graph replay differs from eager"
        for _ in range(2):
            g.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        ms_graph = e0.elapsed_time(e1) / reps
        log(f"[bench] decoder token as one graph: {ms_graph:.3f} ms/token, {total_bytes / ms_graph / 1e6:.0f} GB/s")
    except Exception as ex:  # graphs are a side measurement
        log(f"[bench] decoder token graph variant skipped: {type(ex).__name__}: {ex}")
    return {"linears": len(items), "block_stream_bytes": total_bytes, "ms_per_token": round(ms, 4),
            "GBps": round(gbs, 1), "pct_of_hbm_peak": round(gbs / HBM_PEAK_GBS * 100, 2),
            "n_loaded": "U{8..24} per matrix, seeded", "launches_per_layer": 4,
            "ms_per_token_graph": None if ms_graph is None else round(ms_graph, 4),
            "ms_per_token_plan": None if ms_plan is None else round(ms_plan, 4), "plan_launches": plan_steps}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=960)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--batch-table", action="store_true",
                    help="with --headline-only: also the batch kernels of configs 3 and 5 (they are timed by default otherwise)")
    ap.add_argument("--copies", type=int, default=16, help="separately packed copies to rotate over")
    ap.add_argument("--table", action="store_true", help="(kept for compatibility: the MLP shapes are timed by default)")
    ap.add_argument("--decoder", action="store_true",
                    help="with --headline-only: also the decoder token of config 4 (timed by default otherwise)")
    ap.add_argument("--decompose", action="store_true",
                    help="also time the decomposition on the device (4096x4096 and 14336x4096)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--headline-only", action="store_true",
                    help="only config 2 (the headline figure): skips the same-buffer and merged-launch variants, the "
                         "read probe and configs 3, 4 and 5, so that a profiler run sees only the headline's launches")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a 256 MiB read probe and a 256 MiB device copy (known sizes that scale the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build targets one GPU; run with --gpus 1 "
                 "(the path would shard by output rows, one slice of every block per GPU)")

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    import paper_2410_23918_amd as B
    from workloads import synth as W

    B.lib()
    dev = "cuda:0"
    out, inn, n = 4096, 4096, 16
    t0 = time.time()
    st = build_stack(out, inn, n, 2)
    log(f"[bench] generated {n} blocks of {out}x{inn} on the host in {time.time() - t0:.1f} s")
    sw = st.sign_words()
    stacks = [B.PackedStack(sw, st.U, st.V, st.s) for _ in range(args.copies)]
    xh = W.activations(W.rng_for(2, 100), 1, inn)
    x = torch.from_numpy(xh[0]).to(dev)
    ys = [torch.empty(out, dtype=torch.float16, device=dev) for _ in range(args.copies)]
    # every call gets its own copy of x: consecutive jobs that share the input pointer would be
    # merged into one launch by the native loop, and a step here is one call = one launch
    xcs = [x.clone() for _ in range(args.copies)]
    items = [(xcs[i], stacks[i], n, ys[i]) for i in range(args.copies)]
    jobs = B.make_jobs(items)
    bytes_per_call = n * B.block_bytes(out, inn)

    # outputs of the calls being timed, kept for the comparison in the CPU leg
    B.linear_many(jobs, 1)
    torch.cuda.synchronize()
    y_gpu = [y.float().cpu().numpy().astype(np.float64) for y in ys]
    # set-up, not measurement: the device leaves its idle power state only after some milliseconds of
    # work (the first ~100 calls after an idle period run 5-10 % slower than the ones that follow),
    # so the stacks are walked a few dozen times before the --warmup steps and the timed steps
    B.linear_many(jobs, 40)
    torch.cuda.synchronize()

    steps = max(1, args.steps)   # exactly as asked: whole rotations over the copies, then the remainder
    total = time_calls(B, torch, jobs, steps, args.warmup)
    sec_per_step = total / steps
    value = bytes_per_call / sec_per_step / 1e9
    kmean, kmed, kmin = kernel_durations(B, torch, items, min(steps, 480))
    log(f"[bench] {steps} calls: {sec_per_step * 1e6:.2f} us/call back to back; per-launch events: "
        f"mean {kmean * 1e6:.2f} us, median {kmed * 1e6:.2f} us, min {kmin * 1e6:.2f} us")
    merged = None
    if not args.headline_only:
        # same-buffer (cache-warm) number, labelled
        warm = time_calls(B, torch, B.make_jobs(items[:1]), 200, 20) / 200
        log(f"[bench] same buffer every call (last-level-cache warm): {warm * 1e6:.2f} us/call, "
            f"{bytes_per_call / warm / 1e9:.0f} GB/s")

        # the same calls with one shared x: the native loop merges up to four same-input calls per
        # launch (the q/k/v pattern of a decoder layer); reported beside the headline, not as it
        merged_jobs = B.make_jobs([(x, stacks[i], n, ys[i]) for i in range(args.copies)])
        merged = time_calls(B, torch, merged_jobs, steps, args.warmup) / steps
        log(f"[bench] same calls sharing one x (merged four per launch): {merged * 1e6:.2f} us/call, "
            f"{bytes_per_call / merged / 1e9:.0f} GB/s")

    if args.calibrate:
        nb = 256 << 20
        src = torch.empty(nb, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        sink = torch.zeros(64, dtype=torch.uint8, device=dev)
        for _ in range(4):
            B.probe_read(src, sink, 4096)      # k_stream_read: reads 256 MiB, writes nothing
            dst.copy_(src)                     # elementwise copy: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        log("[bench] calibration kernels done: k_stream_read and a 256 MiB device copy, 4 times each")

    extra = {}
    ceiling = None
    if not args.headline_only:
        ceiling = read_ceiling(B, torch, dev)
        extra["read_ceiling_GBps"] = ceiling
        extra["pct_of_read_ceiling"] = round(value / ceiling["38MiB"] * 100, 1)
        merged_jobs = None
        del stacks, jobs, items
        extra["config3_mlp_batch1"] = mlp_table(B, torch, dev, n, ceiling)
        extra["config3_5_batch_path"] = batch_table(B, torch, dev, n)
        extra["config4_decoder_token"] = decoder_token(B, torch, dev)
        if ceiling:
            extra["config4_decoder_token"]["pct_of_read_ceiling"] = round(
                extra["config4_decoder_token"]["GBps"] / ceiling["1GiB"] * 100, 1)
    else:
        # a profiler run of one table: the headline's launches plus that table's
        if args.batch_table or args.decoder:
            del stacks, jobs, items
        if args.batch_table:
            extra["config3_5_batch_path"] = batch_table(B, torch, dev, n)
        if args.decoder:
            extra["config4_decoder_token"] = decoder_token(B, torch, dev)
    if args.decompose:
        extra["decomposition"] = decompose_table(B, torch, dev)

    result = {
        "metric": "effective block-stream GB/s, batch-1 decode, n=16 k=16, Llama-3-8B 4096x4096 projection",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 matrix-core contraction of 1-bit signs with a 16-bit fixed-point panel, fp32 accumulate "
                 "(fp16 in, fp16 out)",
        "data": "synthetic",
        "config": {
            "workload": "configs[1]: 4096x4096, n=16 blocks of sign bits + rank-16 fp16 U,V (seeded synthetic "
                        "blocks with a decomposition's magnitude profile, s~LogNormal(0,0.5)), batch-1 decode, "
                        "x~N(0,1) fp16",
            "copies_rotated": args.copies,
            "block_stream_bytes_per_call": bytes_per_call,
            "pct_of_hbm_peak": round(value / HBM_PEAK_GBS * 100, 2),
            "merged_same_input_calls": None if merged is None else {
                "calls_per_launch": 4, "us_per_call": round(merged * 1e6, 3),
                "GBps": round(bytes_per_call / merged / 1e9, 1)},
        },
        "roofline": {
            "bound": "hbm",
            "achieved": round(bytes_per_call / sec_per_step / 1e9, 2),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(bytes_per_call / sec_per_step / 1e9 / HBM_PEAK_GBS, 4),
            "traffic": TRAFFIC_BYTES_PER_LAUNCH,
            "kernel": "k_decode<2, 2> (512 rows x 2048 columns x 1 block per workgroup)",
            "avg_launch_us": round(sec_per_step * 1e6, 3),
            "avg_launch_us_event_pairs": round(kmean * 1e6, 3),
        },
    }
    result["config"].update(extra)
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(st, xh, n, bytes_per_call, y_gpu)
    print(json.dumps(result), flush=True)


# HBM bytes per launch of the decode kernel on this workload from rocprofv3 --pmc
# (FETCH_SIZE + WRITE_SIZE, scaled by a read kernel and a copy of known size); see
# profiles/decode_4096x4096_n16_pmc.txt (39.14 MB fetched + 0.54 MB written; algorithmic 37.75 MB).
TRAFFIC_BYTES_PER_LAUNCH = 39682000

if __name__ == "__main__":
    main()
