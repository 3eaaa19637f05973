"""The C-ABI library loads and exports every function the header declares (no GPU compute here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fastardiff.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b(?:int|float|const char\s*\*)\s+(\w+)\s*\(", src)
    return sorted(set(names))


def test_header_declares_the_four_named_entry_points():
    names = declared_functions()
    for n in ("spec_round_init", "spec_verify", "entropy_prefilter", "diffhead_decode"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    for n in declared_functions():
        assert hasattr(lib.lib, n), n
    assert sorted(lib.EXPORTS) == declared_functions()


def test_struct_sizes_match_the_header(lib):
    # 10 int32 + 2 float + 4 int32; 6 int32 + 3 float + 1 int32; 2 tf + head + 7 int32 + 1 float
    assert C.sizeof(lib.TfCfg) == 16 * 4
    assert C.sizeof(lib.HeadCfg) == 10 * 4
    assert C.sizeof(lib.RoundCfg) == 2 * 64 + 40 + 8 * 4
    assert C.sizeof(lib.Tensor) == 8 + 8 + 8 + 4 + 4


def test_host_only_paths(lib):
    assert lib.entropy_threshold(7.12, 0.0) == pytest.approx(0.3 * 7.12, rel=1e-6)
    assert lib.entropy_threshold(2.0, 0.816496580927726) == pytest.approx(0.5183503419072274, rel=1e-6)
    # argument errors are reported before any HIP call
    out = C.c_void_p()
    assert lib.lib.spec_round_init(None, None, 0, None, C.byref(out)) == -1
    assert lib.lib.spec_round_destroy(None) == -1
    assert lib.lib.spec_kv_commit(None, 0, None, 0) == -1
    assert lib.lib.spec_last_error(None) == b"null context"


def test_oracle_and_product_do_not_import_each_other():
    for pkg, banned in (("oracle", "paper_2512_08537_amd"), ("paper_2512_08537_amd", "oracle"), ("synth", "oracle"),
                        ("synth", "paper_2512_08537_amd")):
        d = os.path.join(ROOT, pkg)
        for dirpath, _, files in os.walk(d):
            for f in files:
                if f.endswith((".py", ".hip", ".h")):
                    text = open(os.path.join(dirpath, f)).read()
                    assert not re.search(r"^\s*(from|import)\s+" + banned, text, flags=re.M), (pkg, f)
