#!/usr/bin/env python3
"""Benchmark of the gradient-compression hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic gradients:
W workers' compress calls (error-feedback accumulate, top-k, int8 codes, residual
write-back) followed by one decompress_sum of the W compressed buffers. Inputs are
resident in HBM when a timed interval starts; where one GPU cannot hold all W
workers' gradients at once (the 7B workload), each worker's gradient and residual
are regenerated in place between the timed intervals, and a step's time is the sum
of its W compress intervals and its decompress_sum interval.

Prints ONE JSON line: metric / value / unit (GB/s of gradient processed, whole job), ms_per_step,
config (workload, sizes, per-phase times, variants), roofline (the streaming kernel k_main:
algorithmic 12 B/element over its HIP-event time, against the 8 TB/s HBM peak, with the measured
traffic from the committed counter summary), kernels (per-kernel HIP-event times of one extra step)
and cpu_baseline (the CPU oracle on a bounded sample of the same workload).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", type=int, default=5, choices=[1, 2, 3, 4, 5],
                    help="benchmark workload (default 5: the 7B fp32 gradient the metric is quoted on)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink n (for quick checks; invalid as a result)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="library tuning knob (gc_set_option), e.g. item_len=16384")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device-to-device copy of 4 GiB three times: the reference that "
                         "scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--verify", action="store_true", help="check invariants of the last step on the device")
    return ap.parse_args()


class Timer:
    """Accumulates device time of intervals on the current stream with event pairs."""

    def __init__(self, torch):
        self.torch = torch
        self.pairs = []

    def __enter__(self):
        a = self.torch.cuda.Event(enable_timing=True)
        b = self.torch.cuda.Event(enable_timing=True)
        self.pairs.append((a, b))
        a.record()
        return self

    def __exit__(self, *exc):
        self.pairs[-1][1].record()

    def total_ms(self):
        self.torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in self.pairs)

    def reset(self):
        self.pairs = []


def place_streams(gc, torch, wl, ctx, k, scratch_buf, dev, free_bytes):
    """Where the two big operands of the streaming pass sit in HBM matters: the memory behaves as
    three equal address ranges (a third of the capacity each), and a pass whose gradient and
    residual lie in the same third runs ~6 % faster than one whose operands lie in different
    thirds (measured with 4 GB buffers along the whole address space; memory is handed out top-down
    in allocation order, but not always in one piece). A caller allocates these buffers once, so it
    can afford to look: one arena is allocated, (gradient, residual) pairs at 8 GB steps inside it
    are timed on one streaming pass each, and the fastest pair is used; the aggregate's output
    takes another piece of the arena. Returns (g, e, out, report)."""
    n = wl.n
    step = 1 << 31                                   # floats between candidate positions (8 GB)
    arena_floats = int(min(free_bytes - 60e9, 230e9) // 4)
    arena = torch.empty(arena_floats, dtype=torch.float32, device=dev)
    for i, a in enumerate(range(0, arena_floats, n)):  # realistic values everywhere
        piece = arena[a:min(a + n, arena_floats)]
        wl.residual0(i, dev, out=piece) if piece.numel() == n else piece.normal_(0.0, 1e-3)
    starts = [x for x in range(0, arena_floats - 2 * n + 1, step) if x + 3 * n <= arena_floats or x >= n]
    probe = []
    for x in starts:
        best = None
        for _ in range(2):
            ctx.profile_enable(2)
            gc.compress(ctx, arena[x:x + n], arena[x + n:x + 2 * n], k, wl.block, out=scratch_buf)
            gc.sync_status(ctx)
            ms = ctx.profile_read()["k_main"][0]
            ctx.profile_enable(0)
            best = ms if best is None else min(best, ms)
        probe.append(round(best, 2))
    x = starts[min(range(len(starts)), key=lambda j: probe[j])]
    o = x + 2 * n if x + 3 * n <= arena_floats else x - n  # the output: after the pair if it fits, else before
    report = {"k_main_ms_by_position_8GB_steps": probe, "position_used_GB": round(4 * x / 1e9, 1)}
    return arena[x:x + n], arena[x + n:x + 2 * n], arena[o:o + n], report


def run_flat(args, gc, inputs, torch, wl, ctx):
    """Workloads 1, 4, 5: one flat tensor per worker."""
    dev = "cuda:0"
    n, W, block = wl.n, wl.W, wl.block
    k = gc.k_from_density(n, wl.density)
    nsc = gc.num_scales(k, block)
    bufs = [gc.CompressedBuf.allocate(n, k, nsc, block, wl.index_bits, dev) for _ in range(W)]
    gbytes = 4 if wl.grad_dtype == "f32" else 2
    total_bytes = (gbytes + 8) * n
    free, _ = torch.cuda.mem_get_info()
    # keep every worker's residual resident when it fits (the error-feedback state of each
    # worker across steps); otherwise regenerate gradient and residual per worker in place
    resident = (W * 4 * n + 4 * n + gbytes * n * 2) < free * 0.8
    placement = None
    if resident or 3 * 4 * n + 60e9 > free:
        out = torch.empty(n, dtype=torch.float32, device=dev)
        g32 = torch.empty(n, dtype=torch.float32, device=dev)
        res = [wl.residual0(w, dev) for w in range(W)] if resident else [torch.empty(n, dtype=torch.float32, device=dev)]
    else:
        try:
            g32, e1, out, placement = place_streams(gc, torch, wl, ctx, k, bufs[0], dev, free)
        except torch.OutOfMemoryError:  # the arena did not fit in one piece: take the buffers as they come
            torch.cuda.empty_cache()
            out = torch.empty(n, dtype=torch.float32, device=dev)
            g32 = torch.empty(n, dtype=torch.float32, device=dev)
            e1 = torch.empty(n, dtype=torch.float32, device=dev)
            placement = {"arena": "allocation failed; operands placed in allocation order"}
        res = [e1]
    tc, td = Timer(torch), Timer(torch)
    nsteps = args.warmup + args.steps + 1  # the last, extra step records every kernel and is not timed
    for step in range(nsteps):
        if step == args.warmup:
            torch.cuda.synchronize()
            ctx.profile_enable(2)  # events around the streaming kernel only
            tc.reset()
            td.reset()
        if step == args.warmup + args.steps:
            ms_c, ms_d = tc.total_ms() / args.steps, td.total_ms() / args.steps
            main_prof = ctx.profile_read()["k_main"]
            ctx.profile_enable(1)
        for w in range(W):
            g = wl.grad(w, step, dev, out=g32)
            e = res[w] if resident else wl.residual0(w, dev, out=res[0])
            torch.cuda.synchronize()
            with tc:
                gc.compress(ctx, g, e, k, block, out=bufs[w])
        with td:
            gc.decompress_sum(ctx, bufs, n, out=out)
        gc.sync_status(ctx)
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    ctx.profile_enable(0)
    prof["k_main"] = main_prof
    stats = gc.last_stats(ctx)
    # the aggregation variants on the same buffers (outside the timed steps): staleness-damped
    # sum (Eq. 12) and the fused update of a parameter vector (Eq. 8-9); `out` doubles as theta
    tw, ta = Timer(torch), Timer(torch)
    for _ in range(2):
        tw.reset()
        ta.reset()
        with tw:
            gc.decompress_sum_weighted(ctx, bufs, [w % 4 for w in range(W)], n, out=out)
        with ta:
            gc.decompress_apply(ctx, bufs, out, 1.0 / W)
    variants = {"decompress_sum_weighted_ms": round(tw.total_ms(), 4), "decompress_apply_ms": round(ta.total_ms(), 4)}
    # the paper's own 1-bit value code (Eq. 10) on the last worker's inputs, same selection path
    sbuf = gc.CompressedBuf.allocate(n, k, nsc, block, wl.index_bits, dev, gc.GC_CODEC_SIGN1)
    ts_, tds = Timer(torch), Timer(torch)
    for _ in range(2):
        ts_.reset()
        tds.reset()
        with ts_:
            gc.compress(ctx, g, e, k, block, out=sbuf)
        with tds:
            gc.decompress_sum(ctx, [sbuf] * W, n, out=out)
    gc.sync_status(ctx)
    variants["compress_sign1_ms_per_worker"] = round(ts_.total_ms(), 4)
    variants["decompress_sum_sign1_ms"] = round(tds.total_ms(), 4)
    # the dense coders (every entry sent, no selection): Eq. 10 over the whole accumulated gradient
    dq = dsc = None
    t1, t2, t3 = Timer(torch), Timer(torch), Timer(torch)
    for _ in range(2):
        for t in (t1, t2, t3):
            t.reset()
        with t1:
            dq, dsc = gc.compress_dense(ctx, g, e, block, codec=gc.GC_CODEC_SIGN1, q=dq, scales=dsc)
        with t2:
            gc.decompress_sum_dense(ctx, [dq] * W, [dsc] * W, n, block, codec=gc.GC_CODEC_SIGN1, out=out)
    q8 = None
    for _ in range(2):
        t3.reset()
        with t3:
            q8, dsc = gc.compress_dense(ctx, g, e, block, codec=gc.GC_CODEC_INT8, q=q8, scales=dsc)
    gc.sync_status(ctx)
    del q8, dq
    variants["compress_dense_sign1_ms"] = round(t1.total_ms(), 4)
    variants["decompress_sum_dense_sign1_ms"] = round(t2.total_ms(), 4)
    variants["compress_dense_int8_ms"] = round(t3.total_ms(), 4)
    if n <= (1 << 24):
        # small, launch-bound workload: the same step captured once in a HIP graph and replayed
        # (the calls queue only kernels on the caller's stream once the shape has been seen)
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for w in range(W):
                    gc.compress(ctx, g, res[w] if resident else res[0], k, block, out=bufs[w])
                gc.decompress_sum(ctx, bufs, n, out=out)
        torch.cuda.current_stream().wait_stream(side)
        reps = 50
        tg = Timer(torch)
        for _ in range(2):
            tg.reset()
            with tg:
                for _ in range(reps):
                    graph.replay()
        gc.sync_status(ctx)
        variants["step_ms_hip_graph_replay"] = round(tg.total_ms() / reps, 4)
    info = {"n": n, "k": k, "block": block, "W": W, "index_bits": wl.index_bits, **variants,
            "compress_ms_per_worker": ms_c / W, "decompress_sum_ms": ms_d,
            "residuals_resident": resident, "fallback_tensors": stats["tensors_fallback"],
            "candidates_last_call": stats["candidates"]}
    if placement is not None:
        info["operand_placement"] = placement
    if args.verify:
        info["verify"] = verify_flat(gc, torch, wl, ctx, k, g32, res[0], out)
    return ms_c + ms_d, W * n * gbytes, prof, total_bytes, info


def verify_flat(gc, torch, wl, ctx, k, g32, e_buf, e0_buf):
    """Size-independent invariants of one compress call, checked on the device (in the bench's own
    buffers: gradient, residual, and the aggregate's output as the copy of the old residual)."""
    dev = "cuda:0"
    n = wl.n
    g = wl.grad(0, 0, dev, out=g32)
    e0 = wl.residual0(0, dev, out=e0_buf)
    e = e_buf.copy_(e0)
    buf = gc.compress(ctx, g, e, k, wl.block)
    gc.sync_status(ctx)
    idx = buf.indices.to(torch.int64)
    if wl.index_bits == 32:
        idx = idx & 0xFFFFFFFF
    ok = bool((idx[1:] > idx[:-1]).all()) and int(idx[-1]) < n and idx.numel() == k
    CH = 1 << 28
    thr = None
    kept_abs_min = None
    for a in range(0, n, CH):
        b = min(n, a + CH)
        acc = g[a:b].float() + e0[a:b]
        sel = idx[(idx >= a) & (idx < b)] - a
        keptv = acc[sel].abs()
        if keptv.numel():
            m = keptv.min()
            kept_abs_min = m if kept_abs_min is None else torch.minimum(kept_abs_min, m)
        mask = torch.ones(b - a, dtype=torch.bool, device=dev)
        mask[sel] = False
        ok = ok and bool(torch.equal(e[a:b][mask].view(torch.int32), acc[mask].view(torch.int32)))
        dropped_max = acc[mask].abs().max() if mask.any() else None
        if dropped_max is not None:
            thr = dropped_max if thr is None else torch.maximum(thr, dropped_max)
        del acc, mask
    ok = ok and (thr is None or bool(kept_abs_min >= thr))
    return ok


def run_multi(args, gc, inputs, torch, wl, ctx):
    """Workload 2: a list of tensors per worker, per-tensor top-k, one launch set per worker."""
    import numpy as np
    dev = "cuda:0"
    off = inputs.offsets_of(wl.sizes)
    n, W, block = wl.n, wl.W, wl.block
    ks = np.array([gc.k_from_density(int(s), wl.density) for s in wl.sizes], dtype=np.int64)
    ktot = int(ks.sum())
    stot = int(sum(gc.num_scales(int(x), block) for x in ks))
    bufs = [gc.CompressedBuf.allocate(n, ktot, stot, block, 32, dev) for _ in range(W)]
    out = torch.empty(n, dtype=torch.float32, device=dev)
    grads = [None] * W
    res = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(W)]
    tc, td = Timer(torch), Timer(torch)
    for step in range(args.warmup + args.steps + 1):  # last step: per-kernel recording, not timed
        if step == args.warmup:
            torch.cuda.synchronize()
            ctx.profile_enable(2)
            tc.reset()
            td.reset()
        if step == args.warmup + args.steps:
            ms_c, ms_d = tc.total_ms() / args.steps, td.total_ms() / args.steps
            main_prof = ctx.profile_read()["k_main"]
            ctx.profile_enable(1)
        for w in range(W):
            grads[w] = wl.grad(w, step, dev, out=grads[w])
        torch.cuda.synchronize()
        with tc:
            for w in range(W):
                gc.compress_multi(ctx, grads[w], res[w], off, ks, block, out=bufs[w])
        with td:
            gc.decompress_sum_multi(ctx, bufs, ks, n, out=out)
        gc.sync_status(ctx)
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    ctx.profile_enable(0)
    prof["k_main"] = main_prof
    stats = gc.last_stats(ctx)
    info = {"n": n, "k": ktot, "tensors": len(wl.sizes), "block": block, "W": W,
            "compress_ms_per_worker": ms_c / W, "decompress_sum_ms": ms_d,
            "fallback_tensors": stats["tensors_fallback"], "note": wl.note}
    return ms_c + ms_d, W * n * 4, prof, 12 * n, info


def run_recsys(args, gc, inputs, torch, wl, ctx):
    """Workload 3: per worker a 100M dense tower gradient plus a row-sparse embedding gradient
    (touched rows of a 10M x 128 table). The embedding step is gc_compress_rows on a table-shaped
    residual per worker (8 x 5.12 GB); its buffers carry table positions and are aggregated over the
    union of the workers' touched rows (gc_decompress_sum_rows). The dense 10M x 128 aggregate and
    the in-place update of the table are timed beside it."""
    dev = "cuda:0"
    W, block, n = wl.W, wl.block, wl.n
    k = gc.k_from_density(n, wl.density)
    ctx_e = gc.Context(0)  # the embedding tensors have per-worker sizes: keep their plans apart
    R, D = 10_000_000, 128
    n_table = R * D
    rows, vals, kv = [], [], []
    for w in range(W):
        r, v = inputs.embedding_rows_workload(w, dev)
        rows.append(torch.from_numpy(r).to(dev))
        vals.append(v)
        kv.append(gc.k_from_density(v.numel(), wl.density))
    g = [None] * W
    res = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(W)]
    res_t = [torch.zeros(R, D, dtype=torch.float32, device=dev) for _ in range(W)]
    bufs = [gc.CompressedBuf.allocate(n, k, gc.num_scales(k, block), block, 32, dev) for _ in range(W)]
    bufs_e = [gc.CompressedBuf.allocate(n_table, kv[w], gc.num_scales(kv[w], block), block, 32, dev)
              for w in range(W)]
    out = torch.empty(n, dtype=torch.float32, device=dev)
    out_t = torch.empty(n_table, dtype=torch.float32, device=dev)
    # the embedding aggregate is formed over the union of the workers' touched rows (index
    # bookkeeping of the harness, untimed: the row sets are inputs)
    urows = torch.unique(torch.cat(rows))
    out_u = torch.empty((urows.numel(), D), dtype=torch.float32, device=dev)
    tc, td = Timer(torch), Timer(torch)
    for step in range(args.warmup + args.steps + 1):  # last step: per-kernel recording, not timed
        if step == args.warmup:
            torch.cuda.synchronize()
            ctx.profile_enable(2)
            tc.reset()
            td.reset()
        if step == args.warmup + args.steps:
            ms_c, ms_d = tc.total_ms() / args.steps, td.total_ms() / args.steps
            main_prof = ctx.profile_read()["k_main"]
            ctx.profile_enable(1)
        for w in range(W):
            g[w] = wl.grad(w, step, dev, out=g[w])
        torch.cuda.synchronize()
        with tc:
            for w in range(W):
                gc.compress(ctx, g[w], res[w], k, block, out=bufs[w])
                gc.compress_rows(ctx_e, vals[w], res_t[w], rows[w], kv[w], block, out=bufs_e[w])
        with td:
            gc.decompress_sum(ctx, bufs, n, out=out)
            gc.decompress_sum_rows(ctx, bufs_e, urows, D, out=out_u)
        gc.sync_status(ctx)
        gc.sync_status(ctx_e)
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    ctx.profile_enable(0)
    prof["k_main"] = main_prof
    # the same aggregate as a dense 10M x 128 table, and applied to the table in place (Eq. 8-9)
    ta, tt = Timer(torch), Timer(torch)
    for _ in range(2):
        ta.reset()
        tt.reset()
        with tt:
            gc.decompress_sum(ctx, bufs_e, n_table, out=out_t)
        with ta:
            gc.decompress_apply(ctx, bufs_e, out_t, 1.0 / W)
    gc.sync_status(ctx)
    nv = sum(v.numel() for v in vals)
    info = {"n": n, "k": k, "block": block, "W": W, "embedding_values_total": nv,
            "union_rows": int(urows.numel()), "decompress_sum_dense_table_ms": round(tt.total_ms(), 4),
            "decompress_apply_table_ms": round(ta.total_ms(), 4),
            "embedding_rows_per_worker": [int(r.numel()) for r in rows],
            "compress_ms_per_worker": ms_c / W, "decompress_sum_ms": ms_d,
            "fallback_tensors": gc.last_stats(ctx)["tensors_fallback"], "note": wl.note}
    ctx_e.destroy()
    # k_main launches in `prof` are the tower's only (the embedding calls ran on the second context)
    return ms_c + ms_d, (W * n + nv) * 4, prof, 12 * n, info


def cpu_baseline(inputs, wl_config):
    """The CPU oracle, as it stands, timed on a bounded sample of the same workload."""
    import numpy as np
    from oracle import gc_oracle
    gc_oracle.build()
    n, W = 1 << 27, 16
    if wl_config == 1:
        n, W = 1 << 20, 1
    wl = inputs.workload(wl_config)
    wl.n = n
    if wl.sizes is not None:  # multi-tensor workload: time its flat equivalent
        wl.sizes = None
    k = gc_oracle.k_from_density(n, wl.density)
    refs = []
    t_total = 0.0
    for w in range(W):
        g = wl.grad(w, 0, "cpu")
        gnp = inputs.bf16_bits(g) if g.dtype != __import__("torch").float32 else g.numpy()
        e = wl.residual0(w, "cpu").numpy()
        t0 = time.perf_counter()
        rc, idx, q, s = gc_oracle.compress(gnp, e, k, wl.block)
        t_total += time.perf_counter() - t0
        assert rc == 0
        refs.append((idx, q, s))
    t0 = time.perf_counter()
    rc, _ = gc_oracle.decompress_sum(refs, n, wl.block)
    t_total += time.perf_counter() - t0
    gbytes = 4 if wl.grad_dtype == "f32" else 2
    return {"value": W * n * gbytes / t_total / 1e9, "unit": "GB/s of gradient processed", "cores": 1,
            "kind": "oracle",
            "sample": f"{W} workers x {n} elements of the same distribution, density {wl.density}, "
                      f"block {wl.block}: compress x{W} + decompress_sum(W={W}), {t_total:.1f} s on one thread "
                      f"(host has {os.cpu_count()} logical cores)"}


def read_traffic(name):
    """HBM bytes per k_main launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE),
    kept as a small text file under profiles/ next to the profile it came from."""
    path = os.path.join(ROOT, "profiles", f"k_main_{name}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the aggregation is a local reduction over W "
              "buffers in one GPU's HBM); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2506_17551_amd as gc
    from paper_2506_17551_amd import inputs
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_copy:
        nbytes = 4 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").fill_(3)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"bytes_read_per_copy": nbytes, "bytes_written_per_copy": nbytes,
                                             "copies": 3}}))
        return
    wl = inputs.workload(args.workload, args.scale)
    ctx = gc.Context(0)
    for opt in args.option:
        name, val = opt.split("=")
        ctx.set_option(name, int(val))
    t_wall = time.time()
    if args.workload == 3:
        ms_step, grad_bytes, prof, main_bytes, info = run_recsys(args, gc, inputs, torch, wl, ctx)
    elif wl.sizes is not None:
        ms_step, grad_bytes, prof, main_bytes, info = run_multi(args, gc, inputs, torch, wl, ctx)
    else:
        ms_step, grad_bytes, prof, main_bytes, info = run_flat(args, gc, inputs, torch, wl, ctx)
    wall = time.time() - t_wall
    value = grad_bytes / (ms_step * 1e-3) / 1e9
    km_ms, km_n = prof.get("k_main", (0.0, 0))
    km_avg = km_ms / max(km_n, 1)
    achieved = main_bytes / (km_avg * 1e-3) / 1e9 if km_avg > 0 else 0.0
    kernels = {name: {"ms_total": round(ms, 4), "launches": cnt, "ms_avg": round(ms / cnt, 5)}
               for name, (ms, cnt) in prof.items() if cnt}
    result = {
        "metric": "compress+decompress_sum GB/s of gradient processed and % of MI355X HBM peak",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if wl.grad_dtype == "f32" else "bf16->f32",
        "data": "synthetic",
        "config": {"workload": wl.name + ("" if args.scale >= 1.0 else f" (scaled x{args.scale}: not a result)"),
                   **info,
                   "timed_region": "sum over the step of W compress intervals + 1 decompress_sum interval "
                                   "(HIP events on the launch stream); per-worker input generation is untimed",
                   "pct_hbm_peak_whole_path_algorithmic": round(
                       100.0 * ((main_bytes * info["W"] + 4 * wl.n) / (ms_step * 1e-3) / 1e9) / HBM_PEAK_GBS, 2),
                   "wall_s_including_generation": round(wall, 1)},
        "roofline": {"bound": "hbm", "kernel": "k_main", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": read_traffic(wl.name) if args.scale >= 1.0 else None,
                     "algorithmic_bytes_per_launch": main_bytes, "avg_launch_ms": round(km_avg, 5),
                     "launches": km_n},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(inputs, args.workload)
    ctx.destroy()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
