"""Host logic of the synthetic workloads (no GPU): shapes, k per tensor, seeds."""
import numpy as np

from paper_2506_17551_amd import inputs


def test_decoder_shape_list():
    shapes = inputs.decoder_125m_shapes()
    assert len(shapes) == 148
    assert sum(s for _, s in shapes) == 124_439_808
    sizes = sorted(set(s for _, s in shapes))
    assert sizes == [768, 2304, 3072, 589824, 786432, 1769472, 2359296, 38597376]


def test_workload_sizes(oracle):
    w = inputs.workload(5)
    assert (w.n, w.block, w.W, w.index_bits) == (7_000_000_000, 2048, 16, 64)
    assert oracle.k_from_density(w.n, w.density) == 7_000_000
    w = inputs.workload(4)
    assert (w.n, w.block, w.W, w.grad_dtype) == (1_300_000_000, 1024, 16, "bf16")
    w = inputs.workload(2)
    ks = [oracle.k_from_density(s, w.density) for s in w.sizes]
    assert sum(ks) == 124_503
    assert sum((k + 255) // 256 for k in ks) == 613
    w = inputs.workload(1)
    assert (w.n, oracle.k_from_density(w.n, w.density), w.steps) == (1 << 20, 10486, 3)
    assert inputs.workload(5, scale=0.001).index_bits == 32


def test_streams_are_independent_and_reproducible():
    a = inputs.workload(1).grad(0, 0, "cpu")
    b = inputs.workload(1).grad(0, 0, "cpu")
    c = inputs.workload(1).grad(0, 1, "cpu")
    assert np.array_equal(a.numpy(), b.numpy()) and not np.array_equal(a.numpy(), c.numpy())
    m = inputs.outlier_mixture(200000, 1e-3, 0.01, 100.0, 5).numpy()
    frac = (np.abs(m) > 0.01).mean()          # nearly all of these are outliers
    assert 0.008 < frac < 0.011
    rows = inputs.zipf_unique_rows(65536, 10_000_000, 1.1, 3)
    assert np.all(np.diff(rows) > 0) and 15000 < rows.size < 26000
