"""Host-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad shapes before touching the GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"^\s*(?:int|void|const char\*)\s+(\w+)\s*\(", text, flags=re.M)


@pytest.fixture(scope="module")
def lib():
    from paper_2209_15203_amd import binding
    if not os.path.exists(binding.lib_path()):
        from paper_2209_15203_amd import build
        build.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    """The contract (bts.h), the testing aids (bts_testing.h) and the measurement instrument
    (bts_probe.h, a library of its own): each library exports exactly what its header
    declares, and the binding lists the same names."""
    from paper_2209_15203_amd import binding
    contract = declared_symbols("bts.h")
    aids = declared_symbols("bts_testing.h")
    probe = declared_symbols("bts_probe.h")
    assert len(contract) >= 12 and len(aids) >= 5 and probe == ["bts_hbm_probe"]
    for n in contract + aids:
        assert hasattr(lib, n), n
    assert sorted(contract) == sorted(binding.EXPORTS)
    assert sorted(aids) == sorted(binding.TESTING_EXPORTS)
    plib = binding.load_probe_library()
    for n in probe:
        assert hasattr(plib, n), n
    assert probe == binding.PROBE_EXPORTS
    assert not hasattr(lib, "bts_hbm_probe"), "the probe is not part of the product library"


def test_create_rejects_bad_shapes_without_a_gpu(lib):
    h = C.c_void_p()
    bad = [(0, 100, 1, 1), (-3, 100, 1, 1), (4, 0, 0, 0), (4, 1 << 32, 1, 1), (4, 100, 101, 1),
           (4, 100, 1, 101), (70000, 100, 1, 1)]
    for N, d, ku, kd in bad:
        assert lib.bts_create(C.byref(h), N, d, ku, kd, None) == -1
        assert not h.value
    assert lib.bts_create(None, 4, 100, 1, 1, None) == -1


def test_null_context_is_rejected(lib):
    assert lib.topk_compress(None, None, None, 0.0, None, None) == -1
    assert lib.sparse_aggregate(None, None, None, None, None, None) == -1
    assert lib.downlink_topk(None, None, None, None) == -1
    assert lib.sparse_sgd_update(None, None, None, 0, 0.0, None) == -1
    assert lib.bidir_step(None, None, None, None, None, None, 0.0, 0.0, None, None, None, None,
                          None) == -1
    lib.bts_destroy(None)


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2209_15203_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libbts.so")
    with pytest.raises(binding.BtsError):
        binding.load_library()


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the headers must compile as C99 without any HIP or C++."""
    import subprocess
    src = tmp_path / "t.c"
    src.write_text('#include "bts.h"\n#include "bts_testing.h"\n#include "bts_probe.h"\n'
                   'int main(void) { return BTS_OK; }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror",
                    "-I", os.path.join(ROOT, "include"), "-fsyntax-only", str(src)], check=True)
