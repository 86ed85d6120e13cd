"""GPU parity on randomly drawn partitions: block sizes from several
distributions at once (single elements, sizes around multiples of the
4096-element tile, sizes around the one-pass limits chosen for the case), a
random number of workers, a random route for finishing multi-tile blocks, a
stepsize that changes every step.  Same bar as tests/test_parity_gpu.py.
"""
import numpy as np
import pytest

from tests.parity_util import F, GpuState, synced_step
from tests.test_parity_gpu import ROUTES

pytestmark = pytest.mark.gpu

TILE = 4096


def _random_sizes(rng):
    parts = []
    for _ in range(int(rng.integers(3, 9))):
        kind = rng.integers(0, 6)
        if kind == 0:        # runs of tiny blocks
            parts.append(rng.integers(1, 65, size=int(rng.integers(1, 400))))
        elif kind == 1:      # around a multiple of the tile
            k = int(rng.integers(1, 6))
            parts.append(np.array([k * TILE + int(rng.integers(-2, 3))]))
        elif kind == 2:      # exactly tile-aligned runs
            parts.append(np.full(int(rng.integers(1, 4)), TILE * int(rng.integers(1, 4))))
        elif kind == 3:      # medium blocks
            parts.append(rng.integers(65, 3 * TILE, size=int(rng.integers(1, 6))))
        elif kind == 4:      # one element
            parts.append(np.array([1]))
        else:                # a block of several tiles with a ragged end
            parts.append(np.array([int(rng.integers(2, 9)) * TILE + int(rng.integers(1, TILE))]))
    sizes = np.concatenate(parts).astype(np.int64)
    rng.shuffle(sizes)
    return sizes


@pytest.mark.parametrize("seed", range(36))
def test_random_layout(seed):
    rng = np.random.default_rng(1000 + seed)
    sizes = _random_sizes(rng)
    offs = np.concatenate([[0], np.cumsum(sizes)])
    d = int(offs[-1])
    M = int(rng.integers(1, 6))
    route = ROUTES[seed % len(ROUTES)]
    st = GpuState(offs, M, x0=rng.standard_normal(d).astype(F), route=route, pad=int(rng.integers(0, 3)),
                  fused=bool(seed % 3 == 0))
    if seed % 5 == 4:        # a one-pass limit in the middle of the block sizes present
        st.plan.tune(fuse_limit=int(rng.integers(1, 8)))
    mu = [0.9, 0.0, 0.5][seed % 3]
    eta_prev = 0.0
    for t in range(3):
        eta = float(rng.choice([0.4, 0.1, 0.05, 0.025]))
        g = rng.standard_normal((M, d)) * 10.0 ** rng.uniform(-3, 1)
        g[rng.random((M, d)) < 0.1] = 0.0
        st.set_grads(g.astype(F))
        synced_step(st, mu, eta_prev, eta, None, "seed %d (%s, M=%d, B=%d, d=%d) step %d" % (seed, route, M, len(sizes), d, t))
        eta_prev = eta
    st.plan.close()
