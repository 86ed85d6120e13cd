"""Host-side checks of the C ABI that need no GPU: the libraries load, export
every symbol the headers under include/ declare, and the block partition is
validated before the device is touched."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

import paper_1905_10936_amd as ef

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ef_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    """include/ef.h is the boundary of Algorithm 4, include/ef_debug.h the tuning knobs (both in
    libef.so); include/ef_bench.h the bandwidth probes of libef_bench.so."""
    from paper_1905_10936_amd import bench_probe
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["ef.h", "ef_bench.h", "ef_debug.h"]
    for header, names, L in (("ef.h", ef.ABI_SYMBOLS, ef.lib()), ("ef_debug.h", ef.DEBUG_SYMBOLS, ef.lib()),
                             ("ef_bench.h", bench_probe.BENCH_SYMBOLS, bench_probe.lib())):
        declared = _declared_symbols(header)
        assert set(declared) == set(names), header
        for n in declared:
            assert getattr(L, n) is not None
    # the probes allocate and synchronise: they must stay out of the product library
    for n in bench_probe.BENCH_SYMBOLS:
        assert not hasattr(ef.lib(), n)


def test_built_libraries_are_not_older_than_their_sources():
    """The built libraries travel to the GPU machine as they are: a stale one would be what gets tested."""
    from paper_1905_10936_amd import build
    for lib in build.TARGETS:
        assert os.path.exists(lib) and not build.stale(lib), "%s is missing or older than its sources: rebuild" % lib


def test_sign_words_without_a_plan():
    assert ef.lib().ef_sign_words(None) == 0


@pytest.mark.parametrize("offs", [[0, 2, 2, 4], [1, 4], [0, 3, 2, 4], [0], [0, 0]])
def test_bad_partitions_are_rejected_before_any_gpu_call(offs):
    with pytest.raises(ef.EfError) as ei:
        ef.ef_plan_create(np.asarray(offs, dtype=np.int64), 2)
    assert ei.value.code == ef.EF_ERR_OFFSETS


def test_bad_worker_count_rejected():
    with pytest.raises(ef.EfError) as ei:
        ef.ef_plan_create(np.asarray([0, 4], dtype=np.int64), 0)
    assert ei.value.code == ef.EF_ERR_ARG
    with pytest.raises(ef.EfError) as ei:
        ef.ef_plan_create(np.asarray([0, 4], dtype=np.int64), ef.EF_MAX_WORKERS + 1)
    assert ei.value.code == ef.EF_ERR_ARG


def test_null_plan_pointer():
    L = ef.lib()
    offs = (ctypes.c_int64 * 2)(0, 4)
    assert L.ef_plan_create(None, offs, 1, 1, None) == ef.EF_ERR_NULL
    assert L.ef_plan_destroy(None) == ef.EF_ERR_NULL
    assert L.ef_apply(None, None, None, None, 0.1, None) == ef.EF_ERR_NULL


def test_strerror_texts():
    assert ef.ef_strerror(0) == "ok"
    assert "partition" in ef.ef_strerror(ef.EF_ERR_OFFSETS)
    assert "unknown" in ef.ef_strerror(-99)


@pytest.mark.skipif(torch.cuda.is_available(), reason="only meaningful without a GPU")
def test_no_gpu_is_a_loud_error_not_a_fallback():
    with pytest.raises(ef.EfError) as ei:
        ef.ef_plan_create(np.asarray([0, 4, 9], dtype=np.int64), 2)
    assert ei.value.code == ef.EF_ERR_HIP
