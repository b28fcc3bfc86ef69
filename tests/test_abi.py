"""Host-only checks of the C ABI: the library loads, exports every function the header
declares, and its pure host functions follow the k rule. No compute call is made."""
import ctypes
import os
import re

from tests.conftest import ROOT, read_golden


def _declared():
    text = open(os.path.join(ROOT, "include", "gradcomp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gc_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2506_17551_amd import binding
    L = binding.lib()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


def test_host_functions():
    import paper_2506_17551_amd as gc
    for n, d, k in read_golden("k_rule.txt")["rows"]:
        assert gc.k_from_density(int(n), float(d)) == int(k)
    assert gc.num_scales(10486, 256) == 41
    assert gc.num_scales(7_000_000, 2048) == 3418
    assert gc.num_scales(1, 2048) == 1
    assert gc.num_scales(0, 4) == 0
    from paper_2506_17551_amd import binding
    assert binding._status_string(0) == "ok"
    assert "non-finite" in binding._status_string(4)


def test_product_does_not_touch_the_oracle():
    """The product package must not import, load or mention the oracle."""
    pkg = os.path.join(ROOT, "paper_2506_17551_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "gc_oracle" not in src and "import oracle" not in src and "from oracle" not in src, f


def test_code_bytes_table():
    """gc_num_code_bytes (pure host) against the hand-worked table."""
    import paper_2506_17551_amd as gc
    for k, block, codec, want in read_golden("code_bytes.txt")["rows"]:
        assert gc.num_code_bytes(int(k), int(block), int(codec)) == int(want), (k, block, codec)
    assert gc.num_code_bytes(10, 4, 7) == 0          # unknown code


def test_error_paths_that_need_no_device():
    """Argument errors that every entry point reports before it touches HIP: a null context, null
    output pointers of the pure functions. No kernel is launched and no device is needed."""
    from paper_2506_17551_amd import binding
    L = binding.lib()
    INV = binding.GC_ERR_INVALID_ARG
    buf = binding._GcBuf()
    stats = binding._GcStats()
    ms, cnt = ctypes.c_double(), ctypes.c_int64()
    assert L.gc_create(None, 0) == INV
    assert L.gc_destroy(None) == INV
    assert L.gc_compress(None, 1, 0, 1, 16, 1, 4, ctypes.byref(buf), None) == INV
    assert L.gc_compress_multi(None, 1, 0, 1, 1, 1, 1, 4, ctypes.byref(buf), None) == INV
    assert L.gc_decompress_sum(None, ctypes.byref(buf), 1, 1, 16, None) == INV
    assert L.gc_decompress_sum_static(None, ctypes.byref(buf), 1, 1, 16, None) == INV
    assert L.gc_decompress_sum_multi(None, ctypes.byref(buf), 1, 1, 1, 1, 16, None) == INV
    assert L.gc_decompress_sum_weighted(None, ctypes.byref(buf), 1, None, 0, 1, 1, 16, None) == INV
    assert L.gc_decompress_apply(None, ctypes.byref(buf), 1, None, 0, None, 1, 0.5, 16, None) == INV
    assert L.gc_compress_rows(None, 1, 0, 1, 1, 1, 1, 1, 1, 1, ctypes.byref(buf), None) == INV
    assert L.gc_decompress_sum_rows(None, ctypes.byref(buf), 1, 1, 1, 1, None, 1, None) == INV
    assert L.gc_compress_dense(None, 1, 0, 1, 16, 4, 0, 1, 1, None) == INV
    assert L.gc_decompress_sum_dense(None, 1, 1, 1, 4, 0, None, 1, 16, None) == INV
    assert L.gc_decompress_apply_dense(None, 1, 1, 1, 4, 0, None, 1, 0.5, 16, None) == INV
    assert L.gc_sync_status(None, None) == INV
    assert L.gc_last_stats(None, ctypes.byref(stats)) == INV
    assert L.gc_profile_enable(None, 1) == INV
    assert L.gc_profile_read(None, 0, ctypes.byref(ms), ctypes.byref(cnt)) == INV
    assert L.gc_set_option(None, b"main_lds_pad", 0) == INV
    assert L.gc_profile_num_kernels() >= 18
    assert L.gc_profile_kernel_name(-1) == b"" and L.gc_profile_kernel_name(10 ** 6) == b""
    names = {L.gc_profile_kernel_name(i).decode() for i in range(L.gc_profile_num_kernels())}
    assert {"k_main", "k_dec_tiles", "k_quant"} <= names
    for code in range(6):
        assert binding._status_string(code) not in ("", "unknown status")
    assert binding._status_string(99) == "unknown status"
    # pure host size rules at their edges
    import paper_2506_17551_amd as gc
    assert gc.k_from_density(0, 0.5) == 0 and gc.k_from_density(10, 0.0) == 1 and gc.k_from_density(10, 2.0) == 10
    assert gc.k_from_density(10, float("nan")) == 1
    assert gc.num_scales(5, 0) == 0 and gc.num_scales(-3, 4) == 0
