"""Dense codes with error feedback (every entry sent, no indices; with the 1-bit code this is the
quantizer of Eq. 10 on the whole accumulated gradient, residual per Eq. 11) against the CPU oracle.
The oracle has no dense routine of its own: by definition the dense coder equals the sparse one with
k = n, so the oracle's compress(k = n) and its decompress_sum over the indices 0..n-1 are the
reference. Codes, scales and residuals must be bit-exact."""
import numpy as np
import pytest
import torch

from paper_2506_17551_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
INT8, SIGN1 = 0, 1


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


def check_dense(gc, ctx, oracle, g_cpu, e_cpu, block, codec, tag="", shift=0):
    """One dense step on both sides from the same bytes. shift > 0 places every device array
    `shift` elements into a larger allocation (unaligned base pointers)."""
    n = g_cpu.numel()
    print(f"[case] dense {tag} n={n} block={block} codec={codec} dtype={g_cpu.dtype} shift={shift}", flush=True)
    e_ref = e_cpu.numpy().copy()
    rc, idx, q_ref, s_ref = oracle.compress(_np_grad(g_cpu), e_ref, n, block, codec=codec)
    assert rc == 0 and np.array_equal(idx, np.arange(n, dtype=np.uint32))
    if shift:
        g = torch.zeros(n + shift, dtype=g_cpu.dtype, device=DEV)[shift:]
        g.copy_(g_cpu)
        e = torch.zeros(n + shift, dtype=torch.float32, device=DEV)[shift:]
        e.copy_(e_cpu)
        nq = gc.num_code_bytes(n, block, codec)
        q_all = torch.full((nq + shift + 8,), 0x5A, dtype=torch.int8, device=DEV)
        q = q_all[shift:shift + nq]
    else:
        g, e, q, q_all = g_cpu.to(DEV), e_cpu.to(DEV).clone(), None, None
    q, s = gc.compress_dense(ctx, g, e, block, codec=codec, q=q)
    gc.sync_status(ctx)
    assert q.numel() == q_ref.size and s.numel() == s_ref.size
    assert np.array_equal(q.cpu().numpy(), q_ref), f"{tag}: codes differ"
    assert np.array_equal(bits(s.cpu().numpy()), bits(s_ref)), f"{tag}: scales differ"
    assert np.array_equal(bits(e.cpu().numpy()), bits(e_ref)), f"{tag}: residuals differ"
    if q_all is not None:  # nothing written outside the code bytes
        guard = torch.cat([q_all[:shift], q_all[shift + q.numel():]]).cpu().numpy()
        assert np.all(guard == 0x5A)
    return (q, s), (idx, q_ref, s_ref), torch.from_numpy(e_ref)


@pytest.mark.parametrize("codec", [INT8, SIGN1])
@pytest.mark.parametrize("block", [1, 3, 8, 12, 64, 255, 256, 1000, 1024, 1025, 2048, 4096, 5000, 8192])
def test_dense_blocks(gc, ctx, oracle, codec, block):
    n = 300_007
    g = inputs.outlier_mixture(n, 1e-3, 0.01, 100.0, block)
    e = inputs.normal(n, 1e-3, block + 1)
    check_dense(gc, ctx, oracle, g, e, block, codec, tag="blocks")


@pytest.mark.parametrize("codec", [INT8, SIGN1])
@pytest.mark.parametrize("n", [1, 2, 7, 8, 9, 255, 256, 257, 1023, 4097, 65537, 1 << 20, (1 << 20) + 13])
def test_dense_ragged_sizes(gc, ctx, oracle, codec, n):
    g = inputs.normal(n, 1.0, n)
    e = inputs.normal(n, 0.5, n + 1)
    check_dense(gc, ctx, oracle, g, e, 256, codec, tag="ragged")
    check_dense(gc, ctx, oracle, g, e, 2048, codec, tag="ragged")


@pytest.mark.parametrize("codec", [INT8, SIGN1])
@pytest.mark.parametrize("shift", [1, 2, 3])
@pytest.mark.parametrize("block", [64, 1024, 2048, 2050])
def test_dense_unaligned_pointers(gc, ctx, oracle, codec, shift, block):
    n = 70_001
    g = inputs.normal(n, 1.0, 3 * shift)
    e = inputs.normal(n, 1.0, 3 * shift + 1)
    check_dense(gc, ctx, oracle, g, e, block, codec, tag="unaligned", shift=shift)


@pytest.mark.parametrize("codec", [INT8, SIGN1])
def test_dense_bf16_gradient(gc, ctx, oracle, codec):
    n = 500_003
    g = inputs.student_t3(n, 1e-3, 11).to(torch.bfloat16)
    e = inputs.normal(n, 1e-3, 12)
    check_dense(gc, ctx, oracle, g, e, 1024, codec, tag="bf16")
    check_dense(gc, ctx, oracle, g, e, 1024, codec, tag="bf16", shift=1)


@pytest.mark.parametrize("codec", [INT8, SIGN1])
def test_dense_error_feedback_chain_and_aggregate(gc, ctx, oracle, codec):
    """Three chained steps of two workers; after every step the aggregate of the two code streams."""
    n, block = 200_003, 2048
    e = [torch.zeros(n), torch.zeros(n)]
    for step in range(3):
        gpu, ref = [], []
        for w in range(2):
            g = inputs.outlier_mixture(n, 1e-3, 0.01, 100.0, 100 + 10 * step + w)
            got, want, e[w] = check_dense(gc, ctx, oracle, g, e[w], block, codec, tag=f"chain step {step} w {w}")
            gpu.append(got)
            ref.append(want)
        out = gc.decompress_sum_dense(ctx, [p[0] for p in gpu], [p[1] for p in gpu], n, block, codec=codec)
        torch.cuda.synchronize()
        rc, want = oracle.decompress_sum(ref, n, block, codec=codec)
        assert rc == 0 and np.array_equal(bits(out.cpu().numpy()), bits(want))


@pytest.mark.parametrize("codec", [INT8, SIGN1])
@pytest.mark.parametrize("block,n", [(256, 100_000), (6, 50_001), (2048, 1_000_003)])
def test_dense_aggregate_weighted_and_apply(gc, ctx, oracle, codec, block, n):
    W = 5
    qs, ss, refs = [], [], []
    for w in range(W):
        g = inputs.normal(n, 1.0, 40 + w)
        got, want, _ = check_dense(gc, ctx, oracle, g, torch.zeros(n), block, codec, tag=f"agg w {w}")
        qs.append(got[0]); ss.append(got[1]); refs.append(want)
    stale = [0, 3, 1, 0, 7]
    out = gc.decompress_sum_dense(ctx, qs, ss, n, block, codec=codec)
    outw = gc.decompress_sum_dense(ctx, qs, ss, n, block, codec=codec, staleness=stale)
    out0 = gc.decompress_sum_dense(ctx, qs, ss, n, block, codec=codec, staleness=[0] * W)
    theta0 = inputs.normal(n, 1.0, 77)
    theta = gc.decompress_apply_dense(ctx, qs, ss, theta0.to(DEV), 0.03125 / W, block, codec=codec, staleness=stale)
    torch.cuda.synchronize()
    rc, want = oracle.decompress_sum(refs, n, block, codec=codec)
    rc2, wantw = oracle.decompress_sum(refs, n, block, staleness=stale, codec=codec)
    assert rc == 0 and rc2 == 0
    assert np.array_equal(bits(out.cpu().numpy()), bits(want))
    assert np.array_equal(bits(out0.cpu().numpy()), bits(want))      # staleness 0 == plain sum
    assert np.array_equal(bits(outw.cpu().numpy()), bits(wantw))
    th = theta0.numpy().copy()
    assert oracle.apply(th, wantw, np.float32(0.03125 / W)) == 0
    assert np.array_equal(bits(theta.cpu().numpy()), bits(th))


def test_dense_equals_sparse_with_every_entry_kept(gc, ctx):
    """gc_compress with k = n takes the same coder and adds the index list 0..n-1."""
    n, block = 123_457, 512
    g = inputs.normal(n, 1.0, 1).to(DEV)
    for codec in (INT8, SIGN1):
        e1 = inputs.normal(n, 1.0, 2).to(DEV)
        e2 = e1.clone()
        q, s = gc.compress_dense(ctx, g, e1, block, codec=codec)
        for ib in (32, 64):
            e3 = e2.clone()
            buf = gc.compress(ctx, g, e3, n, block, index_bits=ib, codec=codec)
            gc.sync_status(ctx)
            assert gc.last_stats(ctx)["tensors"] == 1
            assert np.array_equal(buf.indices_numpy(), np.arange(n, dtype=buf.indices_numpy().dtype))
            assert torch.equal(buf.q, q) and torch.equal(buf.scales.view(torch.int32), s.view(torch.int32))
            assert torch.equal(e3.view(torch.int32), e1.view(torch.int32))


def test_dense_argument_errors_and_nonfinite(gc, ctx):
    from paper_2506_17551_amd import binding
    n = 10_000
    g = torch.ones(n, device=DEV)
    e = torch.zeros(n, device=DEV)
    with pytest.raises(binding.GradCompError) as ei:
        gc.compress_dense(ctx, g, e, 8193, codec=SIGN1)
    assert ei.value.status == binding.GC_ERR_UNSUPPORTED
    with pytest.raises(binding.GradCompError) as ei:
        gc.compress_dense(ctx, g, e, 0, codec=SIGN1)
    assert ei.value.status == binding.GC_ERR_INVALID_ARG
    with pytest.raises(binding.GradCompError) as ei:
        gc.compress_dense(ctx, g, e, 64, codec=7)
    assert ei.value.status == binding.GC_ERR_INVALID_ARG
    assert torch.count_nonzero(e).item() == 0          # argument errors write nothing
    q, s = gc.compress_dense(ctx, g, e, 64, codec=SIGN1)
    with pytest.raises(binding.GradCompError) as ei:
        gc.decompress_sum_dense(ctx, [q] * 65, [s] * 65, n, 64, codec=SIGN1)
    assert ei.value.status == binding.GC_ERR_UNSUPPORTED
    with pytest.raises(binding.GradCompError) as ei:
        gc.decompress_sum_dense(ctx, [q], [s], n, 64, codec=SIGN1, staleness=[-1])
    assert ei.value.status == binding.GC_ERR_INVALID_ARG
    gc.sync_status(ctx)
    g[5000] = float("inf")
    gc.compress_dense(ctx, g, torch.zeros(n, device=DEV), 64, codec=INT8)
    assert gc.sync_status(ctx, raise_on_error=False) == binding.GC_ERR_NONFINITE
    assert gc.sync_status(ctx, raise_on_error=False) == binding.GC_OK
