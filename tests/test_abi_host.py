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


def test_configurations_whose_lookup_kernel_cannot_fit_the_lds_are_rejected(lib):
    """The lookup kernel keeps 2L + H + (tiles per sample) words and K*L bytes in LDS besides a segment of
    the per-sample bitmap; a configuration that leaves no room for a segment is refused when the memory
    plan is asked for, not at the first launch."""
    req = slide.slide_mem_req()
    # very many tiles per sample: a huge layer with the small tiles of a 2048-sample batch
    cfg = slide.config_from_workload(synth.small(synth.HASH_DWTA, num_classes=(1 << 30) - 5, batch=2048, K=2, L=2))
    assert lib.slide_query_memory(C.byref(cfg), C.byref(req)) == slide.SLIDE_EINVAL
    assert b"LDS" in lib.slide_last_error(None)
    # very many tables
    cfg = slide.config_from_workload(synth.small(synth.HASH_SIMHASH, K=2, L=30000, num_classes=5000))
    assert lib.slide_query_memory(C.byref(cfg), C.byref(req)) == slide.SLIDE_EINVAL
    # the benchmark configurations are far inside the limit
    for i in range(9):
        assert lib.slide_query_memory(C.byref(slide.config_from_workload(synth.config(i))), C.byref(req)) == slide.SLIDE_OK


def test_buffers_smaller_than_the_memory_plan_are_refused_at_init(lib):
    """SLIDE_ENOMEM for a tables or workspace buffer below slide_query_memory's figures (checked on the
    host before anything touches a device: the pointers here are never dereferenced)."""
    wl = synth.small(synth.HASH_DWTA)
    cfg = slide.config_from_workload(wl)
    req = slide.query_memory(cfg)
    hp_arrays = synth.Generator(wl, 0).hash_params()
    import numpy as np
    perm = np.ascontiguousarray(hp_arrays["dwta_perm"], dtype=np.int32)
    hp = slide.slide_hash_params()
    hp.dwta_perm = perm.ctypes.data
    hp.dens_a, hp.dens_b, hp.prio_a, hp.prio_b = (hp_arrays[k] for k in ("dens_a", "dens_b", "prio_a", "prio_b"))
    fake = 0x10000                                        # aligned, non-NULL, never used
    for short_tables, short_ws in ((True, False), (False, True)):
        b = slide.slide_buffers()
        for n in ("W1", "b1", "W2", "b2", "mW1", "vW1", "mb1", "vb1", "mW2", "vW2", "mb2", "vb2", "tables", "workspace"):
            setattr(b, n, fake)
        b.tables_bytes = req.tables_bytes - (1 if short_tables else 0)
        b.workspace_bytes = req.workspace_bytes - (1 if short_ws else 0)
        ctx = C.c_void_p()
        rc = lib.slide_init(C.byref(cfg), C.byref(b), C.byref(hp), C.byref(ctx))
        assert rc == slide.SLIDE_ENOMEM and not ctx.value
        assert (b"tables" if short_tables else b"workspace") in lib.slide_last_error(None)
