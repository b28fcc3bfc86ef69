#!/usr/bin/env python3
"""Benchmark of the gradient-compression hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic gradients:
W workers' compress calls (error-feedback accumulate, top-k, int8 codes, residual
write-back) followed by one decompress_sum of the W compressed buffers. Inputs are
resident in HBM when a timed interval starts; where one GPU cannot hold all W
workers' gradients at once (the 7B workload), each worker's gradient and residual
are regenerated in place between the timed intervals, and a step's time is the sum
of its W compress intervals and its decompress_sum interval.

Prints ONE JSON line. The headline (metric / value / ms_per_step / roofline / cpu_baseline) is the
7B fp32 workload the metric is quoted on; `config.workloads` carries the same figures for all five
synthetic workloads (run in the same process, each with its own oracle baseline), so that one line
holds the whole report:
  value               GB/s of gradient processed = W * n * sizeof(grad) / step time
  roofline            the streaming kernel k_main: algorithmic 12 B/element over its HIP-event time
                      against the 8 TB/s HBM peak, with the operands where a placement probe put
                      them AND where plain allocation puts them
  roofline_decompress the aggregate (k_dec_fused up to 32 workers, else k_dec_pack +
                      k_dec_tiles): 4 n + W (k (index + code) + scales) bytes over the time of the
                      whole gc_decompress_sum call
  copy_ceiling        a plain device copy of the same size in the same run
  cpu_baseline        the CPU oracle on a bounded sample: one thread, and its W compress calls spread
                      one per core
`--workload N` runs only workload N with full detail.
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
DEV = "cuda:0"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", type=int, default=0, choices=[0, 1, 2, 3, 4, 5],
                    help="0 (default): all five workloads, headline on workload 5 (the 7B fp32 gradient the "
                         "metric is quoted on); N: only workload N")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink n (for quick checks; invalid as a result)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the timings of the widened rows (weighted sum, fused apply, sign code, dense coders)")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="library tuning knob (gc_set_option), e.g. main_lds_pad=32768")
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


def pair_bytes(k, nscales, index_bits):
    """Bytes of one worker's compressed buffer: k (index, code) pairs and the block scales."""
    return k * (index_bits // 8 + 1) + 4 * nscales


def copy_ceiling(torch, dst, src):
    """GB/s (read + written) of a plain device copy of the same size, in the same run."""
    t = Timer(torch)
    best = None
    for _ in range(3):
        t.reset()
        with t:
            dst.copy_(src)
        ms = t.total_ms()
        best = ms if best is None else min(best, ms)
    return 2 * src.numel() * src.element_size() / (best * 1e-3) / 1e9


def k_main_allocation_order(gc, torch, wl, ctx, k, scratch_buf):
    """The streaming pass with the operands where plain allocation puts them (what a caller gets who
    allocates gradient and residual one after the other and does not look): average of 3 passes."""
    g = wl.grad(0, 0, DEV)
    e = wl.residual0(0, DEV)
    ms = []
    for _ in range(4):
        ctx.profile_enable(2)
        gc.compress(ctx, g, e, k, wl.block, out=scratch_buf)
        gc.sync_status(ctx)
        ms.append(ctx.profile_read()["k_main"][0])
        ctx.profile_enable(0)
    del g, e
    torch.cuda.empty_cache()
    return sum(ms[1:]) / 3


def place_streams(gc, torch, wl, ctx, k, scratch_buf, free_bytes):
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
    arena = torch.empty(arena_floats, dtype=torch.float32, device=DEV)
    for i, a in enumerate(range(0, arena_floats, n)):  # realistic values everywhere
        piece = arena[a:min(a + n, arena_floats)]
        wl.residual0(i, DEV, out=piece) if piece.numel() == n else piece.normal_(0.0, 1e-3)
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
    report = {"k_main_ms_by_position_8GB_steps": probe, "position_used_GB": round(4 * x / 1e9, 1),
              "k_main_ms_median_position": sorted(probe)[len(probe) // 2]}
    return arena[x:x + n], arena[x + n:x + 2 * n], arena[o:o + n], report


def run_flat(args, gc, inputs, torch, wl, ctx, steps, warmup, detail):
    """Workloads 1, 4, 5: one flat tensor per worker."""
    n, W, block = wl.n, wl.W, wl.block
    k = gc.k_from_density(n, wl.density)
    nsc = gc.num_scales(k, block)
    bufs = [gc.CompressedBuf.allocate(n, k, nsc, block, wl.index_bits, DEV) for _ in range(W)]
    gbytes = 4 if wl.grad_dtype == "f32" else 2
    free, _ = torch.cuda.mem_get_info()
    # keep every worker's residual resident when it fits (the error-feedback state of each
    # worker across steps); otherwise regenerate gradient and residual per worker in place
    resident = (W * 4 * n + 4 * n + gbytes * n * 2) < free * 0.8
    placement = None
    unplaced_ms = None
    if resident or 3 * 4 * n + 60e9 > free:
        out = torch.empty(n, dtype=torch.float32, device=DEV)
        g32 = torch.empty(n, dtype=torch.float32, device=DEV)
        res = [wl.residual0(w, DEV) for w in range(W)] if resident else [torch.empty(n, dtype=torch.float32, device=DEV)]
    else:
        unplaced_ms = k_main_allocation_order(gc, torch, wl, ctx, k, bufs[0])
        free, _ = torch.cuda.mem_get_info()
        try:
            g32, e1, out, placement = place_streams(gc, torch, wl, ctx, k, bufs[0], free)
        except torch.OutOfMemoryError:  # the arena did not fit in one piece: take the buffers as they come
            torch.cuda.empty_cache()
            out = torch.empty(n, dtype=torch.float32, device=DEV)
            g32 = torch.empty(n, dtype=torch.float32, device=DEV)
            e1 = torch.empty(n, dtype=torch.float32, device=DEV)
            placement = {"arena": "allocation failed; operands placed in allocation order"}
        res = [e1]
    tc, td = Timer(torch), Timer(torch)
    nsteps = warmup + steps + 1  # the last, extra step records every kernel and is not timed
    for step in range(nsteps):
        if step == warmup:
            torch.cuda.synchronize()
            ctx.profile_enable(2)  # events around the streaming kernel only
            tc.reset()
            td.reset()
        if step == warmup + steps:
            ms_c, ms_d = tc.total_ms() / steps, td.total_ms() / steps
            main_prof = ctx.profile_read()["k_main"]
            ctx.profile_enable(1)
        for w in range(W):
            g = wl.grad(w, step, DEV, out=g32)
            e = res[w] if resident else wl.residual0(w, DEV, out=res[0])
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
    variants = {}
    if detail and not args.no_variants:
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
        sbuf = gc.CompressedBuf.allocate(n, k, nsc, block, wl.index_bits, DEV, gc.GC_CODEC_SIGN1)
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
        # (the calls queue only kernels on the caller's stream once the workspace is sized)
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
    ceiling = copy_ceiling(torch, out, g32 if g32.dtype == out.dtype else out.clone())
    info = {"n": n, "k": k, "block": block, "W": W, "index_bits": wl.index_bits, **variants,
            "compress_ms_per_worker": ms_c / W, "decompress_sum_ms": ms_d,
            "residuals_resident": resident, "fallback_tensors": stats["tensors_fallback"],
            "candidates_last_call": stats["candidates"]}
    if placement is not None:
        info["operand_placement"] = placement
    if args.verify:
        info["verify"] = verify_flat(gc, torch, wl, ctx, k, g32, res[0], out)
    cbytes = (gbytes + 8) * n + pair_bytes(k, nsc, wl.index_bits)
    dbytes = 4 * n + W * pair_bytes(k, nsc, wl.index_bits)
    return {"ms_c": ms_c, "ms_d": ms_d, "grad_bytes": W * n * gbytes, "prof": prof, "main_bytes": (gbytes + 8) * n,
            "compress_bytes": cbytes, "dec_bytes": dbytes, "info": info, "unplaced_ms": unplaced_ms,
            "copy_ceiling": ceiling, "W": W}


def verify_flat(gc, torch, wl, ctx, k, g32, e_buf, e0_buf):
    """Size-independent invariants of one compress call, checked on the device (in the bench's own
    buffers: gradient, residual, and the aggregate's output as the copy of the old residual)."""
    n = wl.n
    g = wl.grad(0, 0, DEV, out=g32)
    e0 = wl.residual0(0, DEV, out=e0_buf)
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
        mask = torch.ones(b - a, dtype=torch.bool, device=DEV)
        mask[sel] = False
        ok = ok and bool(torch.equal(e[a:b][mask].view(torch.int32), acc[mask].view(torch.int32)))
        dropped_max = acc[mask].abs().max() if mask.any() else None
        if dropped_max is not None:
            thr = dropped_max if thr is None else torch.maximum(thr, dropped_max)
        del acc, mask
    ok = ok and (thr is None or bool(kept_abs_min >= thr))
    return ok


def run_multi(args, gc, inputs, torch, wl, ctx, steps, warmup, detail):
    """Workload 2: a list of tensors per worker, per-tensor top-k, one launch set per worker."""
    import numpy as np
    off = inputs.offsets_of(wl.sizes)
    n, W, block = wl.n, wl.W, wl.block
    ks = np.array([gc.k_from_density(int(s), wl.density) for s in wl.sizes], dtype=np.int64)
    ktot = int(ks.sum())
    stot = int(sum(gc.num_scales(int(x), block) for x in ks))
    ctx.reserve(n, ktot, len(wl.sizes), W)
    bufs = [gc.CompressedBuf.allocate(n, ktot, stot, block, 32, DEV) for _ in range(W)]
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    grads = [None] * W
    res = [torch.zeros(n, dtype=torch.float32, device=DEV) for _ in range(W)]
    tc, td = Timer(torch), Timer(torch)
    for step in range(warmup + steps + 1):  # last step: per-kernel recording, not timed
        if step == warmup:
            torch.cuda.synchronize()
            ctx.profile_enable(2)
            tc.reset()
            td.reset()
        if step == warmup + steps:
            ms_c, ms_d = tc.total_ms() / steps, td.total_ms() / steps
            main_prof = ctx.profile_read()["k_main"]
            ctx.profile_enable(1)
        for w in range(W):
            grads[w] = wl.grad(w, step, DEV, out=grads[w])
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
    ceiling = copy_ceiling(torch, out, grads[0])
    info = {"n": n, "k": ktot, "tensors": len(wl.sizes), "block": block, "W": W,
            "compress_ms_per_worker": ms_c / W, "decompress_sum_ms": ms_d,
            "fallback_tensors": stats["tensors_fallback"], "note": wl.note}
    return {"ms_c": ms_c, "ms_d": ms_d, "grad_bytes": W * n * 4, "prof": prof, "main_bytes": 12 * n,
            "compress_bytes": 12 * n + pair_bytes(ktot, stot, 32), "dec_bytes": 4 * n + W * pair_bytes(ktot, stot, 32),
            "info": info, "unplaced_ms": None, "copy_ceiling": ceiling, "W": W}


def run_recsys(args, gc, inputs, torch, wl, ctx, steps, warmup, detail):
    """Workload 3: per worker a 100M dense tower gradient plus a row-sparse embedding gradient
    (touched rows of a 10M x 128 table). The embedding step is gc_compress_rows on a table-shaped
    residual per worker (8 x 5.12 GB); every (worker, step) draws its own batch of lookups, so the
    number of touched rows - the shape of the call - changes every step, as it does in training.
    Its buffers carry table positions and are aggregated over the union of the workers' touched rows
    (gc_decompress_sum_rows). The dense 10M x 128 aggregate and the in-place update of the table are
    timed beside it."""
    W, block, n = wl.W, wl.block, wl.n
    k = gc.k_from_density(n, wl.density)
    ctx_e = gc.Context(0)  # the embedding step has its own context (its own workspace)
    R, D = 10_000_000, 128
    n_table = R * D
    nsteps = warmup + steps + 1
    rows, vals, kv, bufs_e, urows, out_u = {}, {}, {}, {}, [], []
    for step in range(nsteps):           # inputs of every step, resident before anything is timed
        for w in range(W):
            r, v = inputs.embedding_rows_workload(w, DEV, step=step)
            rows[w, step] = torch.from_numpy(r).to(DEV)
            vals[w, step] = v
            kv[w, step] = gc.k_from_density(v.numel(), wl.density)
            bufs_e[w, step] = gc.CompressedBuf.allocate(n_table, kv[w, step], gc.num_scales(kv[w, step], block),
                                                         block, 32, DEV)
        # the embedding aggregate is formed over the union of the workers' touched rows (index
        # bookkeeping of the harness, untimed: the row sets are inputs)
        urows.append(torch.unique(torch.cat([rows[w, step] for w in range(W)])))
        out_u.append(torch.empty((urows[-1].numel(), D), dtype=torch.float32, device=DEV))
    max_vals = max(v.numel() for v in vals.values())
    ctx_e.reserve(max_vals, max(kv.values()), 1, W)      # sized once: no call below allocates or waits
    ctx.reserve(n, k, 1, W)
    g = [None] * W
    res = [torch.zeros(n, dtype=torch.float32, device=DEV) for _ in range(W)]
    res_t = [torch.zeros(R, D, dtype=torch.float32, device=DEV) for _ in range(W)]
    bufs = [gc.CompressedBuf.allocate(n, k, gc.num_scales(k, block), block, 32, DEV) for _ in range(W)]
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    tc, td = Timer(torch), Timer(torch)
    nv_timed = 0
    for step in range(nsteps):  # last step: per-kernel recording, not timed
        if step == warmup:
            torch.cuda.synchronize()
            ctx.profile_enable(2)
            tc.reset()
            td.reset()
        if step == warmup + steps:
            ms_c, ms_d = tc.total_ms() / steps, td.total_ms() / steps
            main_prof = ctx.profile_read()["k_main"]
            ctx.profile_enable(1)
        for w in range(W):
            g[w] = wl.grad(w, step, DEV, out=g[w])
        torch.cuda.synchronize()
        be = [bufs_e[w, step] for w in range(W)]
        with tc:
            for w in range(W):
                gc.compress(ctx, g[w], res[w], k, block, out=bufs[w])
                gc.compress_rows(ctx_e, vals[w, step], res_t[w], rows[w, step], kv[w, step], block, out=be[w])
        with td:
            gc.decompress_sum(ctx, bufs, n, out=out)
            gc.decompress_sum_rows(ctx_e, be, urows[step], D, out=out_u[step])
        gc.sync_status(ctx)
        gc.sync_status(ctx_e)
        if warmup <= step < warmup + steps:
            nv_timed += sum(vals[w, step].numel() for w in range(W))
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    ctx.profile_enable(0)
    prof["k_main"] = main_prof
    last = nsteps - 1
    be = [bufs_e[w, last] for w in range(W)]
    info = {"n": n, "k": k, "block": block, "W": W, "embedding_values_per_step": nv_timed // steps,
            "union_rows_last_step": int(urows[last].numel()),
            "embedding_rows_per_worker_last_step": [int(rows[w, last].numel()) for w in range(W)],
            "embedding_rows_change_every_step": True,
            "compress_ms_per_worker": ms_c / W, "decompress_sum_ms": ms_d,
            "fallback_tensors": gc.last_stats(ctx)["tensors_fallback"], "note": wl.note}
    if detail and not args.no_variants:
        # the same aggregate as a dense 10M x 128 table, and applied to the table in place (Eq. 8-9)
        out_t = torch.empty(n_table, dtype=torch.float32, device=DEV)
        ta, tt = Timer(torch), Timer(torch)
        for _ in range(2):
            ta.reset()
            tt.reset()
            with tt:
                gc.decompress_sum(ctx, be, n_table, out=out_t)
            with ta:
                gc.decompress_apply(ctx, be, out_t, 1.0 / W)
        gc.sync_status(ctx)
        info["decompress_sum_dense_table_ms"] = round(tt.total_ms(), 4)
        info["decompress_apply_table_ms"] = round(ta.total_ms(), 4)
        del out_t
    ceiling = copy_ceiling(torch, out, g[0])
    ctx_e.destroy()
    nv = nv_timed // steps                       # embedding values per step, all workers
    ke = sum(kv[w, last] for w in range(W))
    se = sum(gc.num_scales(kv[w, last], block) for w in range(W))
    nsc = gc.num_scales(k, block)
    cbytes = 12 * n + pair_bytes(k, nsc, 32) + (12 * nv + pair_bytes(ke, se, 32)) // W
    dbytes = 4 * n + W * pair_bytes(k, nsc, 32) + 4 * int(urows[last].numel()) * D + pair_bytes(ke, se, 32)
    # k_main launches in `prof` are the tower's only (the embedding calls ran on the second context)
    return {"ms_c": ms_c, "ms_d": ms_d, "grad_bytes": (W * n + nv) * 4, "prof": prof, "main_bytes": 12 * n,
            "compress_bytes": cbytes, "dec_bytes": dbytes, "info": info, "unplaced_ms": None,
            "copy_ceiling": ceiling, "W": W}


# ------------------------------------------------------------------------------------ CPU oracle
def _host_cores():
    try:
        c = len(os.sched_getaffinity(0))
    except AttributeError:
        c = os.cpu_count() or 1
    return max(1, min(c, 16))            # a one-GPU machine's share of the host is 16 cores


def cpu_baseline(inputs, torch, config, headline):
    """The CPU oracle, as it stands, timed on a bounded sample of the same workload: the W compress
    calls one after the other and the decompress_sum on ONE thread; for the headline workload also
    with the W compress calls spread one per core (the oracle itself stays single-threaded)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import gc_oracle
    gc_oracle.build()
    gen_dev = DEV if torch.cuda.is_available() else "cpu"     # draw on the GPU, copy to the host: only the oracle is timed
    wl = inputs.workload(config)
    samples = {1: (1 << 20, 1, 3), 2: (None, 2, 1), 3: (1 << 24, 2, 1), 4: (1 << 25, 4, 1),
               5: ((1 << 27, 16, 1) if headline else (1 << 25, 4, 1))}
    n, W, nsteps = samples[config]
    gbytes = 4 if wl.grad_dtype == "f32" else 2
    t_total = 0.0
    if config == 2:
        wl = inputs.workload(2, scale=0.25)
        n = wl.n
        off = inputs.offsets_of(wl.sizes)
        ks = np.array([gc_oracle.k_from_density(int(s), wl.density) for s in wl.sizes], dtype=np.int64)
        refs = []
        for w in range(W):
            g = wl.grad(w, 0, gen_dev).cpu().numpy()
            e = np.zeros(n, np.float32)
            t0 = time.perf_counter()
            rc, idx, q, s = gc_oracle.compress_multi(g, e, off, ks, wl.block)
            t_total += time.perf_counter() - t0
            assert rc == 0
            refs.append((idx, q, s))
        t0 = time.perf_counter()
        rc, _ = gc_oracle.decompress_sum(refs, n, wl.block, ktensor=ks)
        t_total += time.perf_counter() - t0
        what = f"{W} workers x the 148 tensor shapes at a quarter of their size ({n} elements)"
        value = W * n * gbytes / t_total / 1e9
        return {"value": value, "unit": "GB/s of gradient processed", "cores": 1, "kind": "oracle",
                "sample": f"{what}, density {wl.density}, block {wl.block}: compress_multi x{W} + decompress_sum, "
                          f"{t_total:.1f} s on one thread"}
    wl.n = n
    k = gc_oracle.k_from_density(n, wl.density)
    gs, es = [], []
    for w in range(W):
        g = wl.grad(w, 0, gen_dev)
        gs.append(inputs.bf16_bits(g) if g.dtype != torch.float32 else g.cpu().numpy())
        es.append(wl.residual0(w, gen_dev).cpu().numpy())
    multi = None
    if headline and W > 1:
        cores = min(W, _host_cores())
        e2 = [e.copy() for e in es]
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=cores) as pool:        # ctypes releases the GIL during the call
            list(pool.map(lambda w: gc_oracle.compress(gs[w], e2[w], k, wl.block), range(W)))
        t_par = time.perf_counter() - t0
        del e2
    refs = []
    t_comp = 0.0
    for step in range(nsteps):
        for w in range(W):
            g = gs[w] if step == 0 else wl.grad(w, step, gen_dev).cpu().numpy()
            t0 = time.perf_counter()
            rc, idx, q, s = gc_oracle.compress(g, es[w], k, wl.block)
            t_comp += time.perf_counter() - t0
            assert rc == 0
            if step == nsteps - 1:
                refs.append((idx, q, s))
    t0 = time.perf_counter()
    rc, _ = gc_oracle.decompress_sum(refs, n, wl.block)
    t_dec = (time.perf_counter() - t0) * nsteps
    t_total = t_comp + t_dec
    if config == 3:   # the row-sparse embedding step of one worker's batch, on its touched rows
        rows, vals = inputs.embedding_rows_workload(0, "cpu")
        kv = gc_oracle.k_from_density(vals.numel(), wl.density)
        table = np.zeros((rows.size, 128), np.float32)
        t0 = time.perf_counter()
        rc, idx, q, s = gc_oracle.compress_rows(vals.numpy(), table, np.arange(rows.size, dtype=np.int64), kv, wl.block)
        rc2, _ = gc_oracle.decompress_sum_rows([(idx, q, s)], np.arange(rows.size, dtype=np.int64), 128, wl.block)
        t_total += (time.perf_counter() - t0) * W
        assert rc == 0 and rc2 == 0
        extra_bytes = W * vals.numel() * 4
    else:
        extra_bytes = 0
    processed = nsteps * W * n * gbytes + extra_bytes
    out = {"value": processed / t_total / 1e9, "unit": "GB/s of gradient processed", "cores": 1, "kind": "oracle",
           "sample": f"{W} workers x {n} elements of the same distribution" + (f" x {nsteps} steps" if nsteps > 1 else "")
                     + (" + each worker's embedding rows" if config == 3 else "")
                     + f", density {wl.density}, block {wl.block}: compress x{W} + decompress_sum(W={W}), "
                       f"{t_total:.1f} s on one thread (host share: {_host_cores()} cores)"}
    if headline and W > 1:
        out["multi_core"] = {"value": W * n * gbytes / (t_par + t_dec) / 1e9, "unit": "GB/s of gradient processed",
                             "cores": cores,
                             "how": f"the {W} compress calls spread one per core over {cores} threads ({t_par:.1f} s), "
                                    f"decompress_sum on one ({t_dec:.1f} s)"}
    return out


def read_traffic(kernel, name):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE), kept as a small
    text file under profiles/ next to the profile it came from; None if there is no such file."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{name}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def run_one(args, gc, inputs, torch, config, steps, warmup, detail):
    wl = inputs.workload(config, args.scale)
    ctx = gc.Context(0)
    for opt in args.option:
        name, val = opt.split("=")
        ctx.set_option(name, int(val))
    t_wall = time.time()
    if config == 3:
        r = run_recsys(args, gc, inputs, torch, wl, ctx, steps, warmup, detail)
    elif wl.sizes is not None:
        r = run_multi(args, gc, inputs, torch, wl, ctx, steps, warmup, detail)
    else:
        r = run_flat(args, gc, inputs, torch, wl, ctx, steps, warmup, detail)
    r["wall_s"] = time.time() - t_wall
    ctx.destroy()
    torch.cuda.empty_cache()
    ms_step = r["ms_c"] + r["ms_d"]
    W = r["W"]
    km_ms, km_n = r["prof"].get("k_main", (0.0, 0))
    km_avg = km_ms / max(km_n, 1)
    r.update({
        "wl": wl, "ms_step": ms_step, "steps": steps, "warmup": warmup,
        "value": r["grad_bytes"] / (ms_step * 1e-3) / 1e9,
        "km_avg": km_avg, "km_n": km_n,
        "km_achieved": r["main_bytes"] / (km_avg * 1e-3) / 1e9 if km_avg > 0 else 0.0,
        "dec_achieved": r["dec_bytes"] / (r["ms_d"] * 1e-3) / 1e9,
        "path_achieved": (W * r["compress_bytes"] + r["dec_bytes"]) / (ms_step * 1e-3) / 1e9,
    })
    return r


def workload_record(r, cpu):
    """The short form of one workload's result for `config.workloads`."""
    rec = {"workload": r["wl"].name, "config": r["wl"].config, "W": r["W"], "steps": r["steps"],
           "value_GBps_gradient": round(r["value"], 2), "ms_per_step": round(r["ms_step"], 4),
           "compress_ms_per_worker": round(r["ms_c"] / r["W"], 4), "decompress_sum_ms": round(r["ms_d"], 4),
           "pct_hbm_peak_whole_path_algorithmic": round(100.0 * r["path_achieved"] / HBM_PEAK_GBS, 2),
           "k_main_ms": round(r["km_avg"], 5), "k_main_frac_of_peak": round(r["km_achieved"] / HBM_PEAK_GBS, 4),
           "decompress_frac_of_peak": round(r["dec_achieved"] / HBM_PEAK_GBS, 4),
           "copy_ceiling_GBps": round(r["copy_ceiling"], 1)}
    if cpu is not None:
        rec["cpu_oracle_GBps"] = round(cpu["value"], 4)
        rec["cpu_oracle_cores"] = cpu["cores"]
        rec["cpu_oracle_sample"] = cpu["sample"]
    return rec


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
        src = torch.empty(nbytes, dtype=torch.uint8, device=DEV).fill_(3)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"bytes_read_per_copy": nbytes, "bytes_written_per_copy": nbytes,
                                             "copies": 3}}))
        return
    head = args.workload if args.workload else 5
    others = [] if args.workload else [1, 2, 3, 4]
    records = []
    for c in others:          # the other four workloads first (short runs), then the headline
        r = run_one(args, gc, inputs, torch, c, max(1, min(args.steps, 5)), 1, detail=False)
        cpu = None if args.no_cpu_baseline else cpu_baseline(inputs, torch, c, headline=False)
        records.append(workload_record(r, cpu))
        del r
    r = run_one(args, gc, inputs, torch, head, args.steps, args.warmup, detail=True)
    cpu = None if args.no_cpu_baseline else cpu_baseline(inputs, torch, head, headline=True)
    records.append(workload_record(r, cpu))
    records.sort(key=lambda x: x["config"])
    wl, W, ms_step = r["wl"], r["W"], r["ms_step"]
    full = args.scale >= 1.0
    kernels = {name: {"ms_total": round(ms, 4), "launches": cnt, "ms_avg": round(ms / cnt, 5)}
               for name, (ms, cnt) in r["prof"].items() if cnt}
    roofline = {"bound": "hbm", "kernel": "k_main", "achieved": round(r["km_achieved"], 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(r["km_achieved"] / HBM_PEAK_GBS, 4),
                "traffic": read_traffic("k_main", wl.name) if full else None,
                "traffic_source": "profiles/ (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                                  "calibrated on a plain copy; not counted in this run)",
                "algorithmic_bytes_per_launch": r["main_bytes"], "avg_launch_ms": round(r["km_avg"], 5),
                "launches": r["km_n"]}
    if roofline["traffic"]:
        # the counted bytes over this run's kernel time: what the HBM pins actually carried
        roofline["frac_counted_traffic"] = round(roofline["traffic"] / (r["km_avg"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    extra = {}
    if r["unplaced_ms"]:
        # the headline figure has the operands where the placement probe put them; a caller that
        # allocates them one after the other gets this instead
        un = r["unplaced_ms"]
        un_step = ms_step + W * (un - r["km_avg"])
        roofline["operands"] = "placed by the probe (config.operand_placement)"
        roofline["allocation_order"] = {
            "avg_launch_ms": round(un, 5), "achieved": round(r["main_bytes"] / (un * 1e-3) / 1e9, 1),
            "frac": round(r["main_bytes"] / (un * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "ms_per_step_derived": round(un_step, 4),
            "value_GBps_derived": round(r["grad_bytes"] / (un_step * 1e-3) / 1e9, 2),
            "pct_hbm_peak_whole_path_derived": round(
                100.0 * (W * r["compress_bytes"] + r["dec_bytes"]) / (un_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
            "how": "k_main timed on operands taken from plain allocations before the arena existed; the step "
                   "figures substitute that k_main time into the measured step"}
    dec_traffic = read_traffic("k_dec", wl.name) if full else None
    result = {
        "metric": "compress+decompress_sum GB/s of gradient processed and % of MI355X HBM peak",
        "value": round(r["value"], 2),
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
        "config": {"workload": wl.name + ("" if full else f" (scaled x{args.scale}: not a result)"),
                   **r["info"],
                   "timed_region": "sum over the step of W compress intervals + 1 decompress_sum interval "
                                   "(HIP events on the launch stream); per-worker input generation is untimed",
                   "pct_hbm_peak_whole_path_algorithmic": round(100.0 * r["path_achieved"] / HBM_PEAK_GBS, 2),
                   "copy_ceiling_GBps": round(r["copy_ceiling"], 1),
                   "wall_s_including_generation": round(r["wall_s"], 1),
                   "workloads": records},
        "roofline": roofline,
        "roofline_decompress": {"bound": "hbm",
                                "kernel": ("k_dec_fused" if "k_dec_fused" in kernels and "k_dec_tiles" not in kernels
                                           else "k_dec_pack + k_dec_tiles") + " (one gc_decompress_sum call)",
                                "achieved": round(r["dec_achieved"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                "frac": round(r["dec_achieved"] / HBM_PEAK_GBS, 4), "traffic": dec_traffic,
                                "traffic_source": roofline["traffic_source"],
                                "algorithmic_bytes_per_launch": r["dec_bytes"],
                                "avg_launch_ms": round(r["ms_d"], 5), "launches": r["steps"]},
        "kernels": kernels,
        **extra,
    }
    if dec_traffic:
        result["roofline_decompress"]["frac_counted_traffic"] = round(
            dec_traffic / (r["ms_d"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result))


if __name__ == "__main__":
    main()
