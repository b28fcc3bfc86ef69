"""gc_decompress_sum_static (the entry point that allocates nothing) against gc_decompress_sum,
through the C ABI: same aggregate bit for bit, on two calls in a row that share the static scratch
array, the second with a smaller input; and sizes beyond the array are refused."""
import numpy as np
import pytest
import torch

from paper_2506_17551_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _workers(gc, ctx, n, density, block, W, seed0):
    k = gc.k_from_density(n, density)
    bufs = []
    for w in range(W):
        g = inputs.normal(n, 1.0, inputs.seed_for(77, w, seed0), DEV)
        e = inputs.normal(n, 0.3, inputs.seed_for(77, w, seed0, 0, 1), DEV)
        bufs.append(gc.compress(ctx, g, e, k, block))
    gc.sync_status(ctx)
    return bufs


def test_static_entry_point_matches_decompress_sum_twice_in_a_row():
    import paper_2506_17551_amd as gc
    assert torch.cuda.is_available()
    ctx = gc.Context(0)
    # first call: several ranges of tiles, a ragged tail, 5 workers; second call: smaller in every way
    cases = [(3_000_017, 0.01, 256, 5, 0), (70_001, 0.02, 64, 2, 1)]
    prepared = []
    for n, density, block, W, seed0 in cases:
        bufs = _workers(gc, ctx, n, density, block, W, seed0)
        want = gc.decompress_sum(ctx, bufs, n)
        got = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
        prepared.append((n, bufs, want, got))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for n, bufs, want, got in prepared:       # back to back, nothing in between
        print(f"[case] static aggregate n={n} W={len(bufs)} k={bufs[0].k}", flush=True)
        gc.decompress_sum_static(ctx, bufs, n, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for n, bufs, want, got in prepared:
        assert torch.equal(got.view(torch.int32), want.view(torch.int32)), f"n={n}"
    # and the first, larger case once more after the smaller one
    n, bufs, want, got = prepared[0]
    got.fill_(float("nan"))
    gc.decompress_sum_static(ctx, bufs, n, got)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int32), want.view(torch.int32))
    ctx.destroy()


def test_static_entry_point_refuses_what_does_not_fit():
    import paper_2506_17551_amd as gc
    from paper_2506_17551_amd import binding
    ctx = gc.Context(0)
    n, k = 1 << 24, 5_000_000                  # 5M pairs: 40 MB of records > 32 MiB
    idx = torch.arange(k, dtype=torch.int32, device=DEV)
    buf = gc.CompressedBuf(idx, torch.ones(k, dtype=torch.int8, device=DEV),
                           torch.ones(gc.num_scales(k, 256), dtype=torch.float32, device=DEV), n, k, 256, 32)
    out = torch.zeros(n, dtype=torch.float32, device=DEV)
    with pytest.raises(gc.GradCompError) as ei:
        gc.decompress_sum_static(ctx, [buf], n, out)
    assert ei.value.status == binding.GC_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert int(torch.count_nonzero(out)) == 0  # nothing was written
    ctx.destroy()
