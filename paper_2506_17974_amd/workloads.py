"""Seeded synthetic gradient workloads.

Input data only: this module holds none of the compressor's arithmetic.  It
serves both the HIP path (tests, bench) and the CPU oracle (tests), which is
the one thing the two are allowed to share.

The five workloads stand in for the gradients of the paper's experiments
(Section 5: ResNet-18 on CIFAR-10/100, MNIST, ImageNet); datasets and trained
weights are not available, so shapes, sizes and value distributions are
reproduced and the values are random.  A 2-D layer is (rows, cols) =
(C_out, C_in * k * k) for convolutions and (out, in) for linear layers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

BASE_SEED = 20250617


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                      # position in the benchmark's config list
    layers: Tuple[Tuple[int, int], ...]
    vectors: Tuple[int, ...]        # 1-D tensors sent uncompressed
    rank: int
    bits: int
    workers: int
    dist: str                       # "normal", "student_t3", "normal_outliers"
    scale: float
    steps: int = 1
    alpha: float = 255.0

    @property
    def elements_per_worker(self) -> int:
        return sum(r * c for r, c in self.layers)

    @property
    def gradient_bytes(self) -> int:
        """fp32 bytes of 2-D gradient entering one step, all workers."""
        return 4 * self.workers * self.elements_per_worker

    def layer_rank(self, l: int) -> int:
        r, c = self.layers[l]
        return min(self.rank, r, c)


def _resnet18_layers():
    L = [(64, 27)] + [(64, 576)] * 4 + [(128, 576)] + [(128, 1152)] * 3
    L += [(256, 1152)] + [(256, 2304)] * 3 + [(512, 2304)] + [(512, 4608)] * 3
    L += [(128, 64), (256, 128), (512, 256)] + [(10, 512)]
    return tuple(L)


def _resnet18_vectors():
    # BatchNorm weight + bias per normalised tensor, then the fc bias.
    bn = [64] + [64] * 4 + [128] * 4 + [128] + [256] * 4 + [256] + [512] * 4 + [512]
    v = []
    for c in bn:
        v += [c, c]
    return tuple(v + [10])


def _llm_layers(n_layers=32):
    per = [(4096, 4096)] * 4 + [(4096, 11008), (11008, 4096)]
    return tuple(per * n_layers)


def fc_256x128() -> Workload:
    return Workload("fc_256x128", 0, ((256, 128),), (), rank=2, bits=8, workers=2,
                    dist="normal", scale=1e-3, steps=1)


def small_cnn() -> Workload:
    return Workload("small_cnn", 1, ((32, 25), (64, 800), (1024, 3136), (10, 1024)),
                    (32, 64, 1024, 10), rank=4, bits=8, workers=4,
                    dist="normal", scale=1e-3, steps=10)


def resnet18(rank=4, bits=8) -> Workload:
    return Workload("resnet18", 2, _resnet18_layers(), _resnet18_vectors(), rank=rank,
                    bits=bits, workers=8, dist="student_t3", scale=1e-3)


def llm_stack(n_layers=32) -> Workload:
    return Workload("llm_stack", 3, _llm_layers(n_layers), (), rank=4, bits=8, workers=4,
                    dist="normal_outliers", scale=1e-4)


def sweep_8192(rank=4, bits=8, workers=16) -> Workload:
    return Workload("sweep_8192", 4, ((8192, 8192),), (), rank=rank, bits=bits,
                    workers=workers, dist="normal", scale=1e-3)


def scaled(w: Workload, **kw) -> Workload:
    """Copy of a workload with some fields replaced (e.g. fewer workers)."""
    d = dict(w.__dict__)
    d.update(kw)
    return Workload(**d)


# ----------------------------------------------------------------------------
# host generators (numpy, Philox keyed by (workload, step, tensor, worker))
# ----------------------------------------------------------------------------
def _rng(*key) -> np.random.Generator:
    ss = np.random.SeedSequence([BASE_SEED] + [int(k) for k in key])
    return np.random.Generator(np.random.Philox(ss))


def _draw(rng, dist, scale, shape) -> np.ndarray:
    if dist == "normal":
        return (rng.standard_normal(shape, dtype=np.float32) * np.float32(scale))
    if dist == "student_t3":
        return (rng.standard_t(3.0, size=shape) * scale).astype(np.float32)
    if dist == "normal_outliers":
        x = rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)
        mask = rng.random(shape, dtype=np.float32) < np.float32(0.01)
        x[mask] *= np.float32(100.0)
        return x
    raise ValueError(dist)


def gradient(w: Workload, step: int, layer: int, worker: int) -> np.ndarray:
    """fp32 gradient of 2-D layer `layer` on `worker` at `step`."""
    return _draw(_rng(w.index, 1, step, layer, worker), w.dist, w.scale, w.layers[layer])


def vector_gradient(w: Workload, step: int, vec: int, worker: int) -> np.ndarray:
    return _draw(_rng(w.index, 2, step, vec, worker), w.dist, w.scale, (w.vectors[vec],))


def initial_q(w: Workload, layer: int) -> np.ndarray:
    """Q_0 ~ N(0, 1), one matrix per layer shared by all workers (Algorithm 1,
    initialisation)."""
    rows, cols = w.layers[layer]
    return _rng(w.index, 3, layer).standard_normal((cols, w.layer_rank(layer)), dtype=np.float32)


def host_step_inputs(w: Workload, step: int) -> List[List[np.ndarray]]:
    """grads[worker][layer] for one step."""
    return [[gradient(w, step, l, k) for l in range(len(w.layers))] for k in range(w.workers)]


# ----------------------------------------------------------------------------
# device generator for the sets too large to build on the host
# ----------------------------------------------------------------------------
def device_gradient(w: Workload, step: int, layer: int, worker: int, device="cuda"):
    """Same distributions drawn with torch's generator on the device.  The
    values differ from the host generator's; whoever needs them on the host
    copies the tensor back."""
    import torch
    seed = int(np.random.SeedSequence([BASE_SEED, w.index, 4, step, layer, worker]).generate_state(1, np.uint64)[0] >> 1)
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    shape = w.layers[layer]
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if w.dist == "normal":
        return x.mul_(w.scale)
    if w.dist == "student_t3":
        chi = torch.zeros(shape, device=device, dtype=torch.float32)
        for _ in range(3):
            chi.add_(torch.randn(shape, generator=g, device=device, dtype=torch.float32).square_())
        return x.div_(chi.div_(3.0).sqrt_()).mul_(w.scale)
    if w.dist == "normal_outliers":
        x.mul_(w.scale)
        mask = torch.rand(shape, generator=g, device=device, dtype=torch.float32) < 0.01
        return torch.where(mask, x * 100.0, x)
    raise ValueError(w.dist)
