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
