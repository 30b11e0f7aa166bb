"""Host-only checks of the C ABI: the library loads, exports every symbol that include/slide.h
declares, and rejects bad configurations without touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2201_12667_amd import slide, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(slide.LIB_PATH):
        from paper_2201_12667_amd import build
        build.build_hip()
    return slide.load_library()


def test_every_declared_symbol_is_exported(lib):
    with open(os.path.join(ROOT, "include", "slide.h")) as f:
        text = f.read()
    declared = set(re.findall(r"^(?:int|const char\*)\s+(slide_\w+)\s*\(", text, flags=re.M))
    assert declared == set(slide.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_config_struct_matches_header_size(lib):
    cfg = slide.config_from_workload(synth.config(0))
    req = slide.query_memory(cfg)            # would fail on a struct_size mismatch
    assert req.tables_bytes > 0 and req.workspace_bytes > 0


@pytest.mark.parametrize("i", range(5))
def test_memory_plan_of_the_benchmark_configurations(lib, i):
    wl = synth.config(i)
    req = slide.query_memory(slide.config_from_workload(wl))
    tables_floor = wl.L * (wl.num_buckets + 1 + wl.num_classes) * 4
    assert tables_floor <= req.tables_bytes < tables_floor + (1 << 20)
    assert req.tables_bytes + req.workspace_bytes < 100 * (1 << 30)     # far inside 288 GB of HBM


@pytest.mark.parametrize("field,value", [("hidden_dim", 30), ("hidden_dim", 4096), ("bucket_cap", 0),
                                         ("bucket_cap", 2048), ("K", 0), ("L", 0), ("dwta_bin", 3),
                                         ("max_batch", 0), ("max_batch", 5000), ("lr", 0.0), ("beta1", 1.0),
                                         ("hash_kind", 7), ("overflow_policy", 2), ("num_classes", 0),
                                         ("abi_version", 99), ("rebuild_every", -1)])
def test_bad_configurations_are_rejected_on_the_host(lib, field, value):
    cfg = slide.config_from_workload(synth.small(synth.HASH_DWTA))
    setattr(cfg, field, value)
    req = slide.slide_mem_req()
    assert lib.slide_query_memory(C.byref(cfg), C.byref(req)) == slide.SLIDE_EINVAL
    assert len(lib.slide_last_error(None)) > 0


def test_code_width_limit(lib):
    cfg = slide.config_from_workload(synth.small(synth.HASH_DWTA, K=9))       # 27 bits
    assert lib.slide_query_memory(C.byref(cfg), C.byref(slide.slide_mem_req())) == slide.SLIDE_EINVAL
