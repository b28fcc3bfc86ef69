"""Row-sparse step (gc_compress_rows: touched rows of an embedding table, residual kept in the shape
of the table) against the CPU oracle: table positions, codes, scales and the whole residual table
must be bit-exact, and rows that were not touched must not change."""
import numpy as np
import pytest
import torch

from paper_2506_17551_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def gc():
    import paper_2506_17551_amd as gc_mod
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return gc_mod


@pytest.fixture(scope="module")
def ctx(gc):
    c = gc.Context(0)
    yield c
    c.destroy()


def bits(a):
    return a.view(np.uint32)


def _np_grad(g):
    return inputs.bf16_bits(g) if g.dtype == torch.bfloat16 else g.cpu().numpy()


def pick_rows(R, U, seed):
    rng = np.random.Generator(np.random.Philox(key=seed))
    return np.sort(rng.choice(R, size=U, replace=False)).astype(np.int64)


def check_rows(gc, ctx, oracle, vals_cpu, table_cpu, rows, k, block, index_bits=None, codec=0, tag=""):
    """One step on both sides from the same bytes; table_cpu (R, D) is the residual before the step.
    Returns (gpu buf, oracle triple, new table)."""
    R, D = table_cpu.shape
    print(f"[case] rows {tag} R={R} D={D} U={rows.size} k={k} block={block} bits={index_bits} codec={codec} "
          f"dtype={vals_cpu.dtype}", flush=True)
    ib = index_bits if index_bits is not None else (64 if R * D > (1 << 32) else 32)
    t_ref = table_cpu.numpy().copy()
    rc, idx, q, s = oracle.compress_rows(_np_grad(vals_cpu), t_ref, rows, k, block, index_bits=ib, codec=codec)
    assert rc == 0
    table = table_cpu.to(DEV).clone()
    buf = gc.compress_rows(ctx, vals_cpu.to(DEV), table, torch.from_numpy(rows).to(DEV), k, block,
                           index_bits=ib, codec=codec)
    gc.sync_status(ctx)
    assert np.array_equal(buf.indices_numpy(), idx), f"{tag}: table positions differ"
    assert np.array_equal(buf.q.cpu().numpy(), q), f"{tag}: codes differ"
    assert np.array_equal(bits(buf.scales.cpu().numpy()), bits(s)), f"{tag}: scales differ"
    assert np.array_equal(bits(table.cpu().numpy()), bits(t_ref)), f"{tag}: residual tables differ"
    return buf, (idx, q, s), torch.from_numpy(t_ref)


@pytest.mark.parametrize("D", [1, 3, 4, 64, 128, 130])
@pytest.mark.parametrize("codec", [0, 1])
def test_rows_shapes(gc, ctx, oracle, D, codec):
    R, U = 5000, 777
    rows = pick_rows(R, U, 10 + D)
    vals = inputs.normal(U * D, 0.01, 100 + D)
    table = inputs.normal(R * D, 0.01, 200 + D).reshape(R, D)
    k = gc.k_from_density(U * D, 0.01)
    check_rows(gc, ctx, oracle, vals, table, rows, k, 256, codec=codec, tag="shapes")
    check_rows(gc, ctx, oracle, vals, table, rows, k, 256, index_bits=64, codec=codec, tag="shapes 64-bit")


def test_rows_chain_of_steps_and_aggregate(gc, ctx, oracle):
    """Four chained steps of two workers on one table shape, a different row set every step (rows
    touched earlier keep their residual until they are touched again); the aggregate of the two
    workers' buffers after every step."""
    R, D, block = 200_000, 128, 256
    tables = [torch.zeros(R, D), torch.zeros(R, D)]
    for step in range(4):
        bufs, refs = [], []
        for w in range(2):
            U = 15_000 + 1000 * w + 37 * step
            rows = inputs.zipf_unique_rows(4 * U, R, 1.1, inputs.seed_for(3, w, step, 1))
            vals = inputs.normal(rows.size * D, 0.01, inputs.seed_for(3, w, step, 2))
            k = gc.k_from_density(rows.size * D, 0.01)
            buf, ref, tables[w] = check_rows(gc, ctx, oracle, vals, tables[w], rows, k, block, tag=f"chain {step}/{w}")
            bufs.append(buf)
            refs.append(ref)
        out = gc.decompress_sum(ctx, bufs, R * D)
        torch.cuda.synchronize()
        rc, want = oracle.decompress_sum(refs, R * D, block)
        assert rc == 0 and np.array_equal(bits(out.cpu().numpy()), bits(want))


def test_rows_every_entry_kept_and_bf16(gc, ctx, oracle):
    R, D, U = 3000, 32, 100
    rows = pick_rows(R, U, 5)
    vals = inputs.student_t3(U * D, 1e-3, 6).to(torch.bfloat16)
    table = inputs.normal(R * D, 1e-3, 7).reshape(R, D)
    check_rows(gc, ctx, oracle, vals, table, rows, U * D, 64, tag="all kept bf16")
    check_rows(gc, ctx, oracle, vals, table, rows, 17, 64, tag="bf16")


def test_rows_all_rows_touched_equals_flat_compress(gc, ctx):
    R, D, k, block = 4000, 64, 2000, 128
    g = inputs.normal(R * D, 1.0, 31).to(DEV)
    e1 = inputs.normal(R * D, 1.0, 32).to(DEV)
    e2 = e1.clone().reshape(R, D)
    flat = gc.compress(ctx, g, e1, k, block)
    rowed = gc.compress_rows(ctx, g, e2, torch.arange(R, device=DEV), k, block)
    gc.sync_status(ctx)
    assert torch.equal(flat.indices, rowed.indices) and torch.equal(flat.q, rowed.q)
    assert torch.equal(flat.scales.view(torch.int32), rowed.scales.view(torch.int32))
    assert torch.equal(e1.view(torch.int32), e2.reshape(-1).view(torch.int32))


def test_rows_config3_embedding_table(gc, ctx, oracle):
    """Config 3's embedding gradient at its real shape: a 10M x 128 residual table (5.12 GB), two
    workers' Zipf row sets. The oracle runs on the same rows renumbered 0..U-1 (only touched rows
    matter by definition), and the untouched part of the table is checked on the device."""
    R, D, block = 10_000_000, 128, 256
    free, _ = torch.cuda.mem_get_info()
    if free < 16 * (1 << 30):
        pytest.skip("needs ~16 GB of free HBM")
    table = torch.empty(R, D, device=DEV)
    inputs.normal(R * D, 0.01, 77, DEV, out=table.view(-1))
    before = table.clone()
    bufs, refs = [], []
    for w in range(2):
        rows, vals = inputs.embedding_rows_workload(w, "cpu")
        U = rows.size
        k = gc.k_from_density(U * D, 0.01)
        rows_d = torch.from_numpy(rows).to(DEV)
        small = before[rows_d].cpu().numpy().copy()              # the touched rows, renumbered
        rc, idx, q, s = oracle.compress_rows(vals.numpy(), small, np.arange(U, dtype=np.int64), k, block)
        assert rc == 0
        buf = gc.compress_rows(ctx, vals.to(DEV), table, rows_d, k, block)
        gc.sync_status(ctx)
        assert buf.index_bits == 32 and R * D < (1 << 32)
        c = idx.astype(np.int64)
        want_pos = rows[c // D] * D + c % D
        assert np.array_equal(buf.indices_numpy().astype(np.int64), want_pos)
        assert np.array_equal(buf.q.cpu().numpy(), q)
        assert np.array_equal(bits(buf.scales.cpu().numpy()), bits(s))
        assert np.array_equal(bits(table[rows_d].cpu().numpy()), bits(small))
        mask = torch.ones(R, dtype=torch.bool, device=DEV)
        mask[rows_d] = False
        assert torch.equal(table[mask].view(torch.int32), before[mask].view(torch.int32)), "an untouched row changed"
        del mask
        before[rows_d] = table[rows_d]
        bufs.append(buf)
        refs.append((want_pos.astype(np.uint64), q, s))
    # the aggregate of the two workers over the table; the oracle on the union of positions
    out = gc.decompress_sum(ctx, bufs, R * D)
    torch.cuda.synchronize()
    union = np.unique(np.concatenate([r[0] for r in refs]))
    comp = [(np.searchsorted(union, r[0]).astype(np.uint32), r[1], r[2]) for r in refs]
    rc, want = oracle.decompress_sum(comp, union.size, block)
    got = out[torch.from_numpy(union.astype(np.int64)).to(DEV)].cpu().numpy()
    assert rc == 0 and np.array_equal(bits(got), bits(want))
    assert int(torch.count_nonzero(out)) == int(np.count_nonzero(want))


def test_rows_bad_ids_are_reported_not_dereferenced(gc, ctx):
    from paper_2506_17551_amd import binding
    R, D = 1000, 8
    vals = inputs.normal(3 * D, 1.0, 1).to(DEV)
    gc.sync_status(ctx)
    for bad in ([5, 5, 9], [7, 3, 9], [1, 2, 1000], [-4, 2, 3], [1, 2, 1 << 40]):
        table = inputs.normal(R * D, 1.0, 2).to(DEV).reshape(R, D)
        keep = table.clone()
        gc.compress_rows(ctx, vals, table, torch.tensor(bad, dtype=torch.int64, device=DEV), 4, 4)
        assert gc.sync_status(ctx, raise_on_error=False) == binding.GC_ERR_INVALID_ARG
        good = [r for i, r in enumerate(bad) if 0 <= r < R and (i == 0 or bad[i - 1] < r)]
        mask = torch.ones(R, dtype=torch.bool, device=DEV)
        mask[torch.tensor(good, dtype=torch.int64, device=DEV)] = False
        assert torch.equal(table[mask].view(torch.int32), keep[mask].view(torch.int32))
        assert gc.sync_status(ctx, raise_on_error=False) == binding.GC_OK
    table = torch.zeros(R, D, device=DEV)
    rows = torch.tensor([1, 2, 3], dtype=torch.int64, device=DEV)
    for kwargs, status in [(dict(k=0), binding.GC_ERR_INVALID_ARG), (dict(k=3 * D + 1), binding.GC_ERR_INVALID_ARG),
                           (dict(k=4, block=0), binding.GC_ERR_INVALID_ARG)]:
        with pytest.raises(binding.GradCompError) as ei:
            gc.compress_rows(ctx, vals, table, rows, kwargs.get("k", 4), kwargs.get("block", 4))
        assert ei.value.status == status
    assert torch.count_nonzero(table).item() == 0


@pytest.mark.parametrize("codec", [0, 1])
def test_rows_aggregate_over_the_union_of_rows(gc, ctx, oracle, codec):
    """gc_decompress_sum_rows: five workers with overlapping Zipf row sets on one table shape; the
    output over the union of rows (plus two listed rows nobody touched) against the oracle, with
    and without staleness, and against the dense aggregate gathered at those rows."""
    R, D, block, W = 300_000, 128, 256, 5
    bufs, refs, touched = [], [], []
    for w in range(W):
        rows = inputs.zipf_unique_rows(30_000, R, 1.1, inputs.seed_for(3, w, 7, 1))
        vals = inputs.normal(rows.size * D, 0.01, inputs.seed_for(3, w, 7, 2))
        k = gc.k_from_density(rows.size * D, 0.01)
        buf, ref, _ = check_rows(gc, ctx, oracle, vals, torch.zeros(R, D), rows, k, block, codec=codec, tag=f"agg w{w}")
        bufs.append(buf)
        refs.append(ref)
        touched.append(rows)
    urows = np.union1d(np.concatenate(touched), np.array([R - 2, R - 1]))
    ur = torch.from_numpy(urows).to(DEV)
    stale = [0, 1, 4, 0, 2]
    out = gc.decompress_sum_rows(ctx, bufs, ur, D)
    outw = gc.decompress_sum_rows(ctx, bufs, ur, D, staleness=stale)
    dense = gc.decompress_sum(ctx, bufs, R * D)
    gc.sync_status(ctx)
    rc, want = oracle.decompress_sum_rows(refs, urows, D, block, codec=codec)
    rc2, wantw = oracle.decompress_sum_rows(refs, urows, D, block, staleness=stale, codec=codec)
    assert rc == 0 and rc2 == 0
    assert np.array_equal(bits(out.cpu().numpy()), bits(want))
    assert np.array_equal(bits(outw.cpu().numpy()), bits(wantw))
    assert torch.equal(dense.reshape(R, D)[ur].view(torch.int32), out.view(torch.int32))
    assert int(torch.count_nonzero(dense)) == int(torch.count_nonzero(out))


def test_rows_aggregate_reports_a_missing_row(gc, ctx):
    from paper_2506_17551_amd import binding
    R, D = 1000, 8
    rows = torch.tensor([3, 10, 500], dtype=torch.int64, device=DEV)
    vals = inputs.normal(3 * D, 1.0, 5).to(DEV)
    buf = gc.compress_rows(ctx, vals, torch.zeros(R, D, device=DEV), rows, 6, 4)
    gc.sync_status(ctx)
    for listed in ([3, 10], [10, 500, 900], [0, 1, 2]):
        ur = torch.tensor(listed, dtype=torch.int64, device=DEV)
        out = gc.decompress_sum_rows(ctx, [buf], ur, D)
        assert gc.sync_status(ctx, raise_on_error=False) == binding.GC_ERR_INVALID_ARG
        assert out.shape == (len(listed), D)
    out = gc.decompress_sum_rows(ctx, [buf], rows, D)
    assert gc.sync_status(ctx, raise_on_error=False) == binding.GC_OK
    with pytest.raises(binding.GradCompError) as ei:
        gc.decompress_sum_rows(ctx, [buf] * 65, rows, D)
    assert ei.value.status == binding.GC_ERR_UNSUPPORTED


def test_rows_size_products_are_checked_without_overflow(gc, ctx):
    """U * D, R * D and Ru * D beyond 64 bits are refused by the size checks, before any launch
    (the pointers only need to be non-null and aligned: nothing is dereferenced)."""
    import ctypes
    from paper_2506_17551_amd import binding
    L = binding.lib()
    vals = torch.zeros(64, device=DEV)
    rows = torch.zeros(8, dtype=torch.int64, device=DEV)
    buf = gc.CompressedBuf.allocate(64, 4, 1, 4, 64, DEV)
    raw = buf.struct()
    for U, D, R in [(1 << 33, 1 << 31, 1 << 40), (1 << 20, 1 << 44, 1 << 20), (2, 1 << 31, 1 << 33), (1 << 32, 1 << 32, 1 << 32)]:
        st = L.gc_compress_rows(ctx.handle, vals.data_ptr(), 0, vals.data_ptr(), rows.data_ptr(), U, D, R, 4, 4,
                                ctypes.byref(raw), None)
        assert st == binding.GC_ERR_UNSUPPORTED, (U, D, R, st)
    arr = (type(raw) * 1)(raw)
    for Ru, D in [(1 << 32, 1 << 32), (1 << 40, 1 << 30), (3, 1 << 62), (1 << 16, 1 << 16)]:
        st = L.gc_decompress_sum_rows(ctx.handle, arr, 1, rows.data_ptr(), Ru, D, None, vals.data_ptr(), None)
        assert st == binding.GC_ERR_UNSUPPORTED, (Ru, D, st)
    assert gc.sync_status(ctx, raise_on_error=False) == binding.GC_OK


def test_rows_steps_with_changing_row_counts_inside_one_capture(gc, oracle):
    """After gc_reserve a call only queues kernels, whatever its shape: 50 gc_compress_rows calls whose
    touched-row count differs every time (as an embedding gradient's does), each followed by
    gc_decompress_sum_rows, are recorded in ONE stream capture - a host wait, a copy from pageable
    memory or an allocation inside it would fail the capture. The replayed results equal the eager
    ones, which are checked against the oracle."""
    R, D, block, steps = 60_000, 64, 64, 50
    rng = np.random.default_rng(5)
    us = [int(u) for u in rng.integers(40, 3000, size=steps)]
    assert len(set(us)) > 40
    rows = [np.sort(rng.choice(R, size=u, replace=False)).astype(np.int64) for u in us]
    rows_d = [torch.from_numpy(r).to(DEV) for r in rows]
    vals = [inputs.normal(u * D, 0.01, inputs.seed_for(3, 0, s, 5)).to(DEV) for s, u in enumerate(us)]
    ks = [gc.k_from_density(u * D, 0.01) for u in us]
    table0 = inputs.normal(R * D, 0.002, 99).reshape(R, D)

    def fresh_bufs():
        return [gc.CompressedBuf.allocate(R * D, k, gc.num_scales(k, block), block, 32, DEV) for k in ks]

    def run_all(ctx, table, bufs, outs):
        for s in range(steps):
            gc.compress_rows(ctx, vals[s], table, rows_d[s], ks[s], block, out=bufs[s])
            gc.decompress_sum_rows(ctx, [bufs[s]], rows_d[s], D, out=outs[s])

    # eager, on a context that grows as it goes; the oracle follows step by step
    ctx_a = gc.Context(0)
    table_a = table0.to(DEV).clone()
    bufs_a, outs_a = fresh_bufs(), [torch.empty(u, D, device=DEV) for u in us]
    run_all(ctx_a, table_a, bufs_a, outs_a)
    gc.sync_status(ctx_a)
    table_ref = table0.numpy().copy()
    for s in range(steps):
        rc, idx, q, sc = oracle.compress_rows(vals[s].cpu().numpy(), table_ref, rows[s], ks[s], block, index_bits=32)
        assert rc == 0
        assert np.array_equal(bufs_a[s].indices_numpy(), idx) and np.array_equal(bufs_a[s].q.cpu().numpy(), q), s
        assert np.array_equal(bits(bufs_a[s].scales.cpu().numpy()), bits(sc)), s
        rc, want = oracle.decompress_sum_rows([(idx, q, sc)], rows[s], D, block)
        assert rc == 0 and np.array_equal(bits(outs_a[s].cpu().numpy()), bits(want)), s
    assert np.array_equal(bits(table_a.cpu().numpy()), bits(table_ref))
    ctx_a.destroy()

    # captured, on a fresh context that has only been told the bounds
    ctx_b = gc.Context(0)
    ctx_b.reserve(3000 * D, max(ks), 1, 1)
    table_b = table0.to(DEV).clone()
    bufs_b, outs_b = fresh_bufs(), [torch.full((u, D), float("nan"), device=DEV) for u in us]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run_all(ctx_b, table_b, bufs_b, outs_b)
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    assert gc.sync_status(ctx_b, raise_on_error=False) == 0
    for s in range(steps):
        assert torch.equal(bufs_b[s].indices, bufs_a[s].indices) and torch.equal(bufs_b[s].q, bufs_a[s].q), s
        assert torch.equal(bufs_b[s].scales.view(torch.int32), bufs_a[s].scales.view(torch.int32)), s
        assert torch.equal(outs_b[s].view(torch.int32), outs_a[s].view(torch.int32)), s
    assert torch.equal(table_b.view(torch.int32), table_a.view(torch.int32))
    ctx_b.destroy()
