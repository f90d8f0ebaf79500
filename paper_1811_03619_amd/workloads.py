"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke
check.  This module holds *no* arithmetic of the method (no ring, no codec, no
update): only tensor shapes and random draws.  It imports neither the HIP
binding nor the oracle.

The tensors stand in for the gradients of the networks the paper trains
(MNIST-MLP 784-500-500-10 and AlexNet / ResNet on ImageNet, Sec. 4 "Datasets
and Deep Net Architecture"); the datasets themselves are not used: only the
per-layer shapes matter to the aggregation path.  VGG-16 and ResNet-50 shapes
are added by the workload list this project is measured on.

Law of every tensor: i.i.d. N(0, sigma^2) with sigma = 0.01 / sqrt(fan_in);
a bias (or batch-norm vector) takes the fan_in of the weight it follows.
Generator: numpy Philox (counter based), keyed by (seed, config, worker,
iteration, tensor index) so that any tensor can be regenerated alone.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: Tuple[int, ...]
    fan_in: int

    @property
    def numel(self) -> int:
        n = 1
        for s in self.shape:
            n *= s
        return n


def _conv(name, cout, cin, k) -> List[TensorSpec]:
    fi = cin * k * k
    return [TensorSpec(name + ".weight", (cout, cin, k, k), fi),
            TensorSpec(name + ".bias", (cout,), fi)]


def _fc(name, cout, cin) -> List[TensorSpec]:
    return [TensorSpec(name + ".weight", (cout, cin), cin),
            TensorSpec(name + ".bias", (cout,), cin)]


def mlp_tensors() -> List[TensorSpec]:
    """784-500-500-10 perceptron (Sec. 4, MNIST-MLP)."""
    return _fc("fc1", 500, 784) + _fc("fc2", 500, 500) + _fc("fc3", 10, 500)


def alexnet_tensors() -> List[TensorSpec]:
    """Two-tower AlexNet parameter shapes, 60,965,224 parameters."""
    t = []
    t += _conv("conv1", 96, 3, 11)
    t += _conv("conv2", 256, 48, 5)
    t += _conv("conv3", 384, 256, 3)
    t += _conv("conv4", 384, 192, 3)
    t += _conv("conv5", 256, 192, 3)
    t += _fc("fc6", 4096, 9216)
    t += _fc("fc7", 4096, 4096)
    t += _fc("fc8", 1000, 4096)
    return t


def vgg16_tensors() -> List[TensorSpec]:
    """VGG-16 (configuration D), 138,357,544 parameters."""
    t, cin = [], 3
    for i, cout in enumerate([64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512]):
        t += _conv(f"conv{i + 1}", cout, cin, 3)
        cin = cout
    t += _fc("fc14", 4096, 25088)
    t += _fc("fc15", 4096, 4096)
    t += _fc("fc16", 1000, 4096)
    return t


def resnet50_tensors() -> List[TensorSpec]:
    """ResNet-50: 7x7 stem, [3,4,6,3] bottleneck stages of width 64/128/256/512
    (1x1 -> 3x3 -> 1x1 x4), a batch-norm scale+bias pair after every conv, a
    1x1 projection in the first block of each stage, 1000-way classifier.
    161 tensors, 25,557,032 parameters; convolutions carry no bias."""
    t: List[TensorSpec] = []

    def conv_bn(name, cout, cin, k):
        fi = cin * k * k
        t.append(TensorSpec(name + ".conv", (cout, cin, k, k), fi))
        t.append(TensorSpec(name + ".bn.scale", (cout,), fi))
        t.append(TensorSpec(name + ".bn.bias", (cout,), fi))

    conv_bn("stem", 64, 3, 7)
    cin = 64
    for si, (blocks, width) in enumerate(zip([3, 4, 6, 3], [64, 128, 256, 512])):
        for bi in range(blocks):
            nm = f"s{si + 1}.b{bi + 1}"
            conv_bn(nm + ".a", width, cin, 1)
            conv_bn(nm + ".b", width, width, 3)
            conv_bn(nm + ".c", 4 * width, width, 1)
            if bi == 0:
                conv_bn(nm + ".proj", 4 * width, cin, 1)
            cin = 4 * width
    t += _fc("fc", 1000, 2048)
    return t


def flat_tensor(n: int) -> List[TensorSpec]:
    """One flat vector; fan_in chosen so that sigma^2 = 1e-3 (config 1)."""
    return [TensorSpec("flat", (n,), 0)]


CONFIG_NAMES = {
    1: "flat-1M",
    2: "mlp-784-500-500-10",
    3: "alexnet-61M",
    4: "vgg16-138M",
    5: "resnet50-25.6M",
}


def config_tensors(cfg: int) -> List[TensorSpec]:
    if cfg == 1:
        return flat_tensor(1 << 20)
    if cfg == 2:
        return mlp_tensors()
    if cfg == 3:
        return alexnet_tensors()
    if cfg == 4:
        return vgg16_tensors()
    if cfg == 5:
        return resnet50_tensors()
    raise ValueError(f"unknown config {cfg}")


def sigma_of(spec: TensorSpec) -> float:
    if spec.fan_in == 0:                    # config 1: variance 1e-3
        return float(np.sqrt(1e-3))
    return 0.01 / float(np.sqrt(spec.fan_in))


def _rng(seed: int, cfg: int, worker: int, iteration: int, tensor: int) -> np.random.Generator:
    key = (np.uint64(seed) << np.uint64(32)) ^ np.uint64(cfg)
    ctr = [np.uint64(worker), np.uint64(iteration), np.uint64(tensor), np.uint64(0)]
    return np.random.Generator(np.random.Philox(key=int(key), counter=[int(c) for c in ctr]))


def gaussian(n: int, sigma: float, seed: int, stream: Sequence[int] = (0, 0, 0, 0)) -> np.ndarray:
    """n i.i.d. N(0, sigma^2) values as fp32."""
    g = _rng(seed, stream[0], stream[1], stream[2], stream[3])
    x = g.standard_normal(n, dtype=np.float32)
    x *= np.float32(sigma)
    return x


def small_integers(n: int, lo: int, hi: int, seed: int, stream: Sequence[int] = (0, 0, 0, 0)) -> np.ndarray:
    """n integers uniform in [lo, hi] as fp32 (sums of a few of them are exact)."""
    g = _rng(seed, stream[0], stream[1], stream[2], stream[3])
    return g.integers(lo, hi, size=n, endpoint=True).astype(np.float32)


def gradient_tensors(cfg: int, worker: int, seed: int, iteration: int = 0) -> List[np.ndarray]:
    """Worker `worker`'s per-layer gradient tensors (flattened) for a config."""
    out = []
    for ti, spec in enumerate(config_tensors(cfg)):
        g = _rng(seed, cfg, worker, iteration, ti)
        x = g.standard_normal(spec.numel, dtype=np.float32)
        x *= np.float32(sigma_of(spec))
        out.append(x)
    return out


def flat_gradient(cfg: int, worker: int, seed: int, iteration: int = 0) -> np.ndarray:
    """All tensors of a config concatenated in declaration order."""
    return np.concatenate(gradient_tensors(cfg, worker, seed, iteration))


def scaled_config(cfg: int, shrink: int) -> List[TensorSpec]:
    """Same tensor list with every dimension > 16 divided by `shrink`
    (rounded up): keeps the tensor count and the size mix at a fraction of the
    volume, for parity cases the oracle finishes in seconds."""
    out = []
    for s in config_tensors(cfg):
        shp = tuple(d if d <= 16 else -(-d // shrink) for d in s.shape)
        out.append(TensorSpec(s.name, shp, s.fan_in))
    return out


def gradient_tensors_for(specs: Sequence[TensorSpec], tag: int, worker: int, seed: int,
                         iteration: int = 0) -> List[np.ndarray]:
    out = []
    for ti, spec in enumerate(specs):
        g = _rng(seed, tag, worker, iteration, ti)
        x = g.standard_normal(spec.numel, dtype=np.float32)
        x *= np.float32(sigma_of(spec))
        out.append(x)
    return out
