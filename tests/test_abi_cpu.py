"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/ef.h declares, and validates the block partition before
touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

import paper_1905_10936_amd as ef

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "ef.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ef_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ef.lib()
    names = _declared_symbols()
    assert set(names) == set(ef.ABI_SYMBOLS)
    for n in names:
        assert getattr(L, n) is not None


def test_sign_words():
    assert [ef.ef_sign_words(d) for d in (1, 63, 64, 65, 128, 1 << 28)] == [1, 1, 1, 2, 2, 1 << 22]


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
