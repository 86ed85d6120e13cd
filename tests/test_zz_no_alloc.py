"""ef_compressor_quality_static, the entry point that allocates nothing (its per-tile sums go to
a fixed array in the library's device image): through the C ABI it must give what
ef_compressor_quality gives, to that call's own bar against the oracle (1e-9 relative; the two
run the same kernels, so the bits are expected to be equal), on two calls in a row that share
the array, the second on a smaller input; and it must refuse inputs beyond its stated capacity.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_1905_10936_amd as ef

pytestmark = pytest.mark.gpu

TILE = 4096
MAX_TILE_VECTORS = 131072       # EF_QUALITY_STATIC_MAX_TILE_VECTORS of include/ef.h


def _offs(sizes):
    return np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))])


def _vectors(rng, n, d, offs):
    v = rng.standard_normal((n, d)).astype(np.float32)
    for b in range(0, len(offs) - 1, 3):            # some blocks with a very different scale
        v[:, offs[b]:offs[b + 1]] *= 10.0 ** rng.uniform(-3, 1)
    v[rng.random((n, d)) < 0.05] = 0.0
    return v


def _both(plan, v_host, pad):
    """(plan-scratch result, static-scratch result) for the rows of v_host, rows `pad` floats apart."""
    n, d = v_host.shape
    stride = (d + 3) // 4 * 4 + 4 * pad
    v = torch.zeros((n, stride), dtype=torch.float32, device="cuda")
    v[:, :d].copy_(torch.as_tensor(v_host))
    out_a = torch.full((n, 2), -1.0, dtype=torch.float64, device="cuda")
    out_b = torch.full((n, 2), -2.0, dtype=torch.float64, device="cuda")
    ef.ef_compressor_quality(plan, v, out_a)
    ef.ef_compressor_quality_static(plan, v, out_b)
    torch.cuda.synchronize()
    return out_a.cpu().numpy(), out_b.cpu().numpy()


def test_static_scratch_call_matches_the_allocating_one_twice_in_a_row():
    rng = np.random.default_rng(77)
    # first call: blocks from 1 element to 9 tiles, a ragged end, 3 vectors
    sizes1 = [1, 5, 64, 3 * TILE + 17, 700, 9 * TILE - 3, TILE, 2 * TILE + 1, 33, 40000, 11]
    # second call, smaller: fewer tiles, one vector, other block boundaries
    sizes2 = [2 * TILE + 5, 9, 3000, TILE - 9]
    for sizes, n in ((sizes1, 3), (sizes2, 1)):
        offs = _offs(sizes)
        d = int(offs[-1])
        plan = ef.Plan(offs, 4)
        v = _vectors(rng, n, d, offs)
        got_plan, got_static = _both(plan, v, pad=2)
        assert np.array_equal(got_plan.view(np.uint64), got_static.view(np.uint64)), (got_plan, got_static)
        for i in range(n):
            phi, delta = oracle.quality(np.ascontiguousarray(v[i]), offs)
            assert abs(got_static[i, 0] - phi) <= 1e-9 * phi and abs(got_static[i, 1] - delta) <= 1e-9 * delta
        plan.close()


def test_static_scratch_call_refuses_what_does_not_fit():
    """Capacity is tiles x vectors <= 131072: a layout of 2^26 + 4096 elements with 8 vectors is one
    tile per vector too many and is refused before anything is read; with 7 vectors it fits."""
    d = (MAX_TILE_VECTORS // 8 + 1) * TILE
    plan = ef.Plan(_offs([d]), 8)
    L = ef.lib()
    out = torch.zeros((8, 2), dtype=torch.float64, device="cuda")
    v = torch.zeros((7, d), dtype=torch.float32, device="cuda")
    v[:, ::7] = 1.0
    v[:, 1::2] -= 3.0
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.ef_compressor_quality_static(plan._h, 8, ctypes.c_void_p(v.data_ptr()), d, ctypes.c_void_p(out.data_ptr()), stream)
    assert rc == ef.EF_ERR_SIZE and "static scratch" in ef.ef_strerror(rc)
    out_a = torch.zeros((7, 2), dtype=torch.float64, device="cuda")
    ef.ef_compressor_quality(plan, v, out_a)
    ef.ef_compressor_quality_static(plan, v, out[:7])
    torch.cuda.synchronize()
    assert torch.equal(out_a, out[:7])
    plan.close()
