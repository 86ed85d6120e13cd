"""Seeded synthetic workloads: block layouts and gradient generators.

This module holds NO arithmetic of the method (no momentum, compressor,
residual or decode).  It only says where the blocks are and draws random
gradients, so that the CPU oracle and the HIP library can be fed identical
bits.  Both sides' tests and the benchmark import it; it imports neither.

The five named workloads follow the benchmark configurations: layer shapes of
ResNet-20 / ResNet-50 (the networks of the paper's Sections 4.1 and 4.2, one
block per parameter tensor as in Section 3.2), a flat 2^28 case, a skewed
block-size case and a transformer-like layout.  No dataset is involved: the
gradients are random draws with the stated distributions.
"""
import math

import numpy as np
import torch

BASE_SEED = 190510936


# ---------------------------------------------------------------- layouts ---

def _offsets(sizes):
    sizes = np.asarray(sizes, dtype=np.int64)
    offs = np.zeros(sizes.size + 1, dtype=np.int64)
    np.cumsum(sizes, out=offs[1:])
    return offs


def resnet20_sizes():
    """65 tensors, 272 474 elements: 3x3 stem, 3 stages x 3 basic blocks of two
    3x3 convs, 1x1 projections at the two stage changes, BN gamma/beta after
    every conv, fc 64x10 + bias."""
    sizes = []

    def conv(cin, cout, k):
        sizes.extend([k * k * cin * cout, cout, cout])

    conv(3, 16, 3)
    cin = 16
    for c in (16, 32, 64):
        for blk in range(3):
            conv(cin if blk == 0 else c, c, 3)
            conv(c, c, 3)
            if blk == 0 and cin != c:
                conv(cin, c, 1)
        cin = c
    sizes.extend([64 * 10, 10])
    return sizes


def resnet50_sizes():
    """161 tensors, 25 557 032 elements: 7x7 stem, [3,4,6,3] bottlenecks with
    a 1x1 projection in the first bottleneck of each stage, BN gamma/beta after
    every conv, fc 2048x1000 + bias."""
    sizes = []

    def conv(cin, cout, k):
        sizes.extend([k * k * cin * cout, cout, cout])

    conv(3, 64, 7)
    cin = 64
    for planes, n in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(n):
            conv(cin, planes, 1)
            conv(planes, planes, 3)
            conv(planes, planes * 4, 1)
            if blk == 0:
                conv(cin, planes * 4, 1)
            cin = planes * 4
    sizes.extend([2048 * 1000, 1000])
    return sizes


def transformer_sizes(layers=24, h=1024, ff=4096, vocab=50257):
    """289 tensors, 353 772 544 elements: embedding table, then per layer QKV,
    output and two MLP weights with biases and two LayerNorm gamma/beta."""
    sizes = [vocab * h]
    for _ in range(layers):
        sizes.extend([h * 3 * h, 3 * h, h * h, h, h * ff, ff, ff * h, h, h, h, h, h])
    return sizes


def skewed_sizes(n_small=1_000_000, n_big=4, big=8 * 1024 * 1024, seed=BASE_SEED + 4):
    """n_small blocks with sizes floor(exp(U(0, ln 65))) in [1, 64] and n_big
    blocks of `big` elements placed at seeded random positions among them."""
    rng = np.random.Generator(np.random.Philox(seed))
    small = np.floor(np.exp(rng.uniform(0.0, math.log(65.0), n_small))).astype(np.int64)
    small = np.clip(small, 1, 64)
    pos = np.sort(rng.choice(n_small + 1, size=n_big, replace=False))
    sizes = np.insert(small, pos, big)
    return sizes


def uniform_sizes(d, block):
    q, r = divmod(d, block)
    return [block] * q + ([r] if r else [])


# -------------------------------------------------------------- workloads ---

class Workload:
    """Block layout + hyper-parameters + seeded gradient generator."""

    def __init__(self, name, index, sizes, M, steps, dist, mu=0.9, eta=0.1, note=""):
        self.name = name
        self.index = index
        self.offsets = _offsets(sizes)
        self.d = int(self.offsets[-1])
        self.B = int(self.offsets.size - 1)
        self.M = M
        self.steps = steps
        self.mu = mu
        self.eta = eta
        self.dist = dist
        self.note = note
        self._sigma = {}

    def seed(self, step, worker):
        return BASE_SEED + 100_003 * self.index + 1_009 * step + worker

    def _per_element_sigma(self, device):
        """cfg 2: one sigma per tensor, log-uniform in [1e-4, 1e-1]."""
        key = str(device)
        if key not in self._sigma:
            rng = np.random.Generator(np.random.Philox(BASE_SEED + 7 * self.index))
            sig = np.power(10.0, rng.uniform(-4.0, -1.0, self.B)).astype(np.float32)
            sizes = torch.from_numpy(np.diff(self.offsets))
            s = torch.repeat_interleave(torch.from_numpy(sig), sizes)
            self._sigma[key] = s.to(device)
        return self._sigma[key]

    def grad(self, step, worker, device="cpu", out=None):
        """float32[d] gradient of `worker` at `step` (same bits for the same
        arguments and device type)."""
        dev = torch.device(device)
        gen = torch.Generator(device=dev)
        gen.manual_seed(self.seed(step, worker))
        d = self.d
        if out is None:
            out = torch.empty(d, dtype=torch.float32, device=dev)
        kind = self.dist[0]
        if kind == "normal":
            out.normal_(0.0, self.dist[1], generator=gen)
        elif kind == "normal_per_block":
            out.normal_(0.0, 1.0, generator=gen)
            out.mul_(self._per_element_sigma(dev))
        elif kind == "laplace_zeros":
            scale, pzero = self.dist[1], self.dist[2]
            u = torch.empty(d, dtype=torch.float32, device=dev)
            u.uniform_(-0.5, 0.5, generator=gen)
            out.copy_(-scale * torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.4999999)))
            u.uniform_(0.0, 1.0, generator=gen)
            out.masked_fill_(u < pzero, 0.0)
            del u
        elif kind == "student_t3":
            scale = self.dist[1]
            out.normal_(0.0, 1.0, generator=gen)
            chi = torch.zeros(d, dtype=torch.float32, device=dev)
            z = torch.empty(d, dtype=torch.float32, device=dev)
            for _ in range(3):
                z.normal_(0.0, 1.0, generator=gen)
                chi.addcmul_(z, z)
            del z
            out.div_(torch.sqrt(chi / 3.0).clamp_(min=1e-6)).mul_(scale)
            del chi
        else:
            raise ValueError(kind)
        return out

    def describe(self):
        return {"workload": self.name, "d": self.d, "B": self.B, "M": self.M, "mu": self.mu,
                "eta": self.eta, "steps": self.steps, "grad_dist": list(self.dist)}


def resnet20():
    return Workload("resnet20_like", 1, resnet20_sizes(), M=2, steps=5, dist=("normal", 0.1),
                    note="N(0, 1e-2) read as variance 1e-2")


def resnet50():
    return Workload("resnet50_like", 2, resnet50_sizes(), M=7, steps=3, dist=("normal_per_block",))


def flat(log2_d=28, log2_block=20, M=8, steps=10):
    d = 1 << log2_d
    return Workload("flat_2p%d_blocks_2p%d" % (log2_d, log2_block), 3,
                    uniform_sizes(d, 1 << log2_block), M=M, steps=steps, dist=("normal", 1.0))


def skewed(n_small=1_000_000, n_big=4, big=8 * 1024 * 1024):
    return Workload("skewed_blocks", 4, skewed_sizes(n_small, n_big, big), M=4, steps=3,
                    dist=("laplace_zeros", 1e-3, 0.05))


def transformer(layers=24):
    return Workload("transformer_like", 5, transformer_sizes(layers), M=16, steps=2,
                    dist=("student_t3", 1e-3))


def one_block(log2_d=28, M=8, steps=10):
    """The non-block compressor of Eq. (1) as a layout: B = 1, one scale for the whole vector."""
    d = 1 << log2_d
    return Workload("one_block_2p%d" % log2_d, 6, [d], M=M, steps=steps, dist=("normal", 1.0))


def odd_tiles(M=8, steps=10):
    """257 blocks of 255 x 4096 elements: every block holds an odd number of
    whole tiles, so fixed-size groups of tiles would straddle block ends."""
    return Workload("odd_tiles_257x255", 7, [255 * 4096] * 257, M=M, steps=steps, dist=("normal", 1.0))


def beyond_2p31(M=2, steps=2):
    """d a little above 2^31 elements, so that element, word and tile arithmetic must be 64-bit:
    2047 blocks of 2^20, one block that straddles element 2^31 and ends off the tile grid, 3000
    tiny blocks behind it, one medium block at the end (ragged last tile)."""
    rng = np.random.Generator(np.random.Philox(BASE_SEED + 8))
    tiny = np.clip(np.floor(np.exp(rng.uniform(0.0, np.log(65.0), 3000))), 1, 64).astype(np.int64)
    sizes = [1 << 20] * 2047 + [(1 << 20) + 3 * 4096 + 5] + [int(v) for v in tiny] + [10_000]
    return Workload("beyond_2p31", 8, sizes, M=M, steps=steps, dist=("normal", 1.0))


WORKLOADS = {
    "resnet20_like": resnet20,
    "resnet50_like": resnet50,
    "flat_2p28": flat,
    "skewed_blocks": skewed,
    "transformer_like": transformer,
    "one_block_2p28": one_block,
    "odd_tiles": odd_tiles,
    "beyond_2p31": beyond_2p31,
}


def get(name):
    return WORKLOADS[name]()
