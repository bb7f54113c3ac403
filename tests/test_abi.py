"""The C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "distshap.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ds_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_what_the_binding_uses():
    from paper_2506_22668_amd import EXPORTED_SYMBOLS
    assert sorted(EXPORTED_SYMBOLS) == _declared()


def test_library_exports_every_declared_symbol():
    from paper_2506_22668_amd import library_path
    if not os.path.exists(library_path()):
        from paper_2506_22668_amd.build import build_library
        build_library(verbose=False)
    lib = ctypes.CDLL(library_path())
    for name in _declared():
        assert hasattr(lib, name), name


def test_host_only_calls_work_without_a_gpu():
    from paper_2506_22668_amd import binding
    lib = binding.load_library()
    assert b"gfx950" in lib.ds_version()
    assert binding.sample_plan(12, 4096) == (4096, True)
    assert binding.sample_plan(24, 1 << 24) == (1 << 24, True)
    assert binding.sample_plan(25, 1 << 26) == (1 << 26, False)
    assert binding.sample_plan(1000, 20001) == (20000, False)
    with pytest.raises(binding.DistShapError):
        binding.sample_plan(-1, 10)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2506_22668_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no oracle", ""), f


def test_host_plan_tables_equal_the_oracle_bit_for_bit():
    import numpy as np
    from oracle import sampling
    from paper_2506_22668_amd import binding
    for n, ns in [(2, 4), (12, 4096), (24, 1 << 24), (25, 1000), (30, 25000), (1010, 20000), (4097, 131),
                  (99981, 200000), (1000175, 400000)]:
        b, wtab = binding.plan_tables(n, ns)
        plan = sampling.allocation(n, ns)
        assert np.array_equal(wtab.view(np.uint32), plan["wtab"].view(np.uint32)), (n, ns)
        if not plan["enumerate"]:
            assert np.array_equal(b, plan["b"]), (n, ns)
    with pytest.raises(binding.DistShapError):
        binding.plan_tables(1, 10)
    with pytest.raises(binding.DistShapError):
        binding.plan_tables(100, 3)


def test_host_plan_tables_with_saturated_classes_equal_the_oracle():
    import numpy as np
    from oracle import sampling
    from paper_2506_22668_amd import binding
    for n, ns in [(30, 25000), (200, 3000), (12, 1000), (9, 510), (1010, 20000), (99981, 200000), (333, 70000)]:
        b, wtab, upto = binding.plan_tables(n, ns, binding.Options(saturate=1))
        plan = sampling.allocation(n, ns, saturate=True)
        assert upto == plan["enum_upto"], (n, ns)
        assert np.array_equal(b, plan["b"]), (n, ns)
        assert np.array_equal(wtab.view(np.uint32), plan["wtab"].view(np.uint32)), (n, ns)
    with pytest.raises(binding.DistShapError):
        binding.plan_tables(100, 1000, binding.Options(saturate=1, weighting=1))
