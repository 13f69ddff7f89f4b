"""Seeded synthetic workloads shaped like the CNNs the paper quantizes.

This module only *draws inputs*: layer shape tables (architecture facts) and
seeded value generators.  It holds none of the method's arithmetic, so that the
CPU oracle and the HIP path can both be fed from it without sharing code.

The paper evaluates on ImageNet CNNs with pretrained weights (Section 4); neither
is available here, so every tensor below is synthetic: the *shapes* are those of
the public architectures, the *values* are heavy-tailed per-channel draws.

Conventions
-----------
* A weight tensor is returned as a contiguous fp32 array ``[K, n]``: K output
  channel kernels of n = c*w*h elements each (Section 3.3, kernel-wise partition).
* A calibration activation tensor is returned flat, fp32 ``[N]`` (Section 3.7,
  one scale per layer).
* Every draw is made in fp64 with ``numpy.random.default_rng(seed)`` and cast to
  fp32;  ``seed = BASE_SEED + 1000*cfg + tensor_index`` (activations use
  ``tensor_index + 500``).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Iterator, List, Sequence, Tuple

import numpy as np

BASE_SEED = 190206822


# --------------------------------------------------------------------------
# shape tables
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class WeightShape:
    name: str
    K: int          # output channels = number of kernels
    n: int          # elements per kernel (cin/groups * kh * kw)


@dataclass(frozen=True)
class ActShape:
    name: str
    per_image: int  # elements per image of this layer's input

    def numel(self, batch: int) -> int:
        return self.per_image * batch


def resnet18_weights() -> List[WeightShape]:
    out = [WeightShape("conv1", 64, 3 * 49)]
    cin = 64
    for li, cout in enumerate((64, 128, 256, 512), start=1):
        for b in range(2):
            c_in_blk = cin if b == 0 else cout
            out.append(WeightShape(f"layer{li}.{b}.conv1", cout, c_in_blk * 9))
            out.append(WeightShape(f"layer{li}.{b}.conv2", cout, cout * 9))
            if b == 0 and c_in_blk != cout:
                out.append(WeightShape(f"layer{li}.{b}.downsample", cout, c_in_blk))
        cin = cout
    out.append(WeightShape("fc", 1000, 512))
    return out


def _resnet50_layers() -> Tuple[List[WeightShape], List[ActShape]]:
    """Weights of the 53 convolutions + fc, and the input of each (per image)."""
    w: List[WeightShape] = []
    a: List[ActShape] = []

    def add(name, cout, cin, k, hw_in):
        w.append(WeightShape(name, cout, cin * k * k))
        a.append(ActShape(name + ".in", cin * hw_in * hw_in))

    add("conv1", 64, 3, 7, 224)
    hw = 56                      # after stride-2 conv and stride-2 max-pool
    cin = 64
    for li, (width, nblk, stride) in enumerate(
            ((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)), start=1):
        cout = width * 4
        for b in range(nblk):
            s = stride if b == 0 else 1
            add(f"layer{li}.{b}.conv1", width, cin, 1, hw)
            add(f"layer{li}.{b}.conv2", width, width, 3, hw)      # stride s lives here
            hw_out = hw // s
            add(f"layer{li}.{b}.conv3", cout, width, 1, hw_out)
            if b == 0:
                add(f"layer{li}.{b}.downsample", cout, cin, 1, hw)
            cin = cout
            hw = hw_out
    w.append(WeightShape("fc", 1000, 2048))
    a.append(ActShape("fc.in", 2048))
    return w, a


def resnet50_weights() -> List[WeightShape]:
    return _resnet50_layers()[0]


def resnet50_activations() -> List[ActShape]:
    return _resnet50_layers()[1]


def _vgg16_layers() -> Tuple[List[WeightShape], List[ActShape]]:
    cfg = (64, 64, "M", 128, 128, "M", 256, 256, 256, "M", 512, 512, 512, "M", 512, 512, 512, "M")
    w: List[WeightShape] = []
    a: List[ActShape] = []
    cin, hw, i = 3, 224, 0
    for v in cfg:
        if v == "M":
            hw //= 2
            continue
        w.append(WeightShape(f"features.conv{i}", v, cin * 9))
        a.append(ActShape(f"features.conv{i}.in", cin * hw * hw))
        cin = v
        i += 1
    for name, cout, cin_fc in (("fc6", 4096, 512 * 7 * 7), ("fc7", 4096, 4096), ("fc8", 1000, 4096)):
        w.append(WeightShape(name, cout, cin_fc))
        a.append(ActShape(name + ".in", cin_fc))
    return w, a


def vgg16_weights() -> List[WeightShape]:
    return _vgg16_layers()[0]


def vgg16_activations() -> List[ActShape]:
    return _vgg16_layers()[1]


def mobilenetv2_weights() -> List[WeightShape]:
    out = [WeightShape("stem", 32, 27)]
    cin = 32
    settings = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
                (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1))
    bi = 0
    for t, c, reps, _s in settings:
        for _ in range(reps):
            hidden = cin * t
            if t != 1:
                out.append(WeightShape(f"block{bi}.expand", hidden, cin))
            out.append(WeightShape(f"block{bi}.depthwise", hidden, 9))
            out.append(WeightShape(f"block{bi}.project", c, hidden))
            cin = c
            bi += 1
    out.append(WeightShape("last_conv", 1280, 320))
    out.append(WeightShape("classifier", 1000, 1280))
    return out


# --------------------------------------------------------------------------
# value generators (one tensor at a time; all seeded)
# --------------------------------------------------------------------------
def _log_uniform(rng: np.random.Generator, lo: float, hi: float, size) -> np.ndarray:
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=size))


def seed_for(cfg: int, tensor_index: int, activation: bool = False) -> int:
    return BASE_SEED + 1000 * cfg + tensor_index + (500 if activation else 0)


def weights_normal_scaled(K: int, n: int, seed: int, std: float = 0.05,
                          lo: float = 0.25, hi: float = 4.0) -> np.ndarray:
    """N(0, std^2) with a per-channel factor log-uniform in [lo, hi] (config 1)."""
    rng = np.random.default_rng(seed)
    s = _log_uniform(rng, lo, hi, (K, 1))
    return np.ascontiguousarray((rng.normal(0.0, std, (K, n)) * s).astype(np.float32))


def weights_laplace(K: int, n: int, seed: int, lo: float, hi: float) -> np.ndarray:
    """Laplace(0, b_k), b_k log-uniform in [lo, hi] per channel (configs 2 and 5)."""
    rng = np.random.default_rng(seed)
    b = _log_uniform(rng, lo, hi, (K, 1))
    return np.ascontiguousarray((rng.laplace(0.0, 1.0, (K, n)) * b).astype(np.float32))


def weights_normal_outliers(K: int, n: int, seed: int, lo: float = 0.01, hi: float = 0.5,
                            p_out: float = 0.01, factor: float = 10.0) -> np.ndarray:
    """N(0, sigma_k^2), sigma_k log-uniform; each entry x10 with probability 1% (config 3)."""
    rng = np.random.default_rng(seed)
    sig = _log_uniform(rng, lo, hi, (K, 1))
    w = rng.normal(0.0, 1.0, (K, n)) * sig
    mask = rng.random((K, n)) < p_out
    w = np.where(mask, w * factor, w)
    return np.ascontiguousarray(w.astype(np.float32))


def weights_student_t(K: int, n: int, seed: int, nu: float = 4.0,
                      lo: float = 0.005, hi: float = 0.1) -> np.ndarray:
    """Student-t(nu) times a per-channel scale log-uniform in [lo, hi] (config 4)."""
    rng = np.random.default_rng(seed)
    c = _log_uniform(rng, lo, hi, (K, 1))
    return np.ascontiguousarray((rng.standard_t(nu, (K, n)) * c).astype(np.float32))


def _fill_blocks(N: int, draw: Callable[[np.random.Generator, int], np.ndarray],
                 seed: int, block: int = 1 << 22) -> np.ndarray:
    """Fill a flat fp32 array block by block so that peak host memory stays small."""
    rng = np.random.default_rng(seed)
    out = np.empty(N, dtype=np.float32)
    for s in range(0, N, block):
        e = min(N, s + block)
        out[s:e] = draw(rng, e - s)
    return out


def acts_relu_normal(N: int, seed: int) -> np.ndarray:
    """ReLU(N(0,1)) (configs 1 and 5)."""
    return _fill_blocks(N, lambda r, m: np.maximum(r.normal(0.0, 1.0, m), 0.0), seed)


def tiled_normal(N: int, seed: int, period: int = 16_000_057, relu: bool = False) -> np.ndarray:
    """N(0,1) values (optionally through ReLU) repeated with an odd period: fills the very large tensors of
    the maximum-size cases in seconds.  The period shares no factor with any power of two, so data
    addressed 2^k elements away from where it should be never looks the same."""
    base = np.random.default_rng(seed).standard_normal(period).astype(np.float32)
    if relu:
        base = np.maximum(base, np.float32(0.0))
    out = np.empty(N, dtype=np.float32)
    for s in range(0, N, period):
        e = min(N, s + period)
        out[s:e] = base[:e - s]
    return out


def acts_relu_student_t(N: int, seed: int, nu: float = 5.0) -> np.ndarray:
    """ReLU(Student-t(nu)) (config 4)."""
    return _fill_blocks(N, lambda r, m: np.maximum(r.standard_t(nu, m), 0.0), seed)


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    cfg: int
    name: str
    grid_points: int
    refine_iters: int
    weight_shapes: Sequence[WeightShape]
    act_shapes: Sequence[ActShape]
    act_batch: int
    residual: str                    # "none" | "top10pct" | "all"

    @property
    def weight_elements(self) -> int:
        return sum(s.K * s.n for s in self.weight_shapes)

    @property
    def act_elements(self) -> int:
        return sum(s.numel(self.act_batch) for s in self.act_shapes)

    def weight_tensor(self, i: int) -> np.ndarray:
        s = self.weight_shapes[i]
        sd = seed_for(self.cfg, i)
        if self.cfg == 1:
            return weights_normal_scaled(s.K, s.n, sd)
        if self.cfg == 2:
            return weights_laplace(s.K, s.n, sd, 0.005, 0.1)
        if self.cfg == 3:
            return weights_normal_outliers(s.K, s.n, sd)
        if self.cfg == 4:
            return weights_student_t(s.K, s.n, sd)
        if self.cfg == 5:
            return weights_laplace(s.K, s.n, sd, 0.001, 0.05)
        raise ValueError(self.cfg)

    def act_tensor(self, i: int) -> np.ndarray:
        s = self.act_shapes[i]
        sd = seed_for(self.cfg, i, activation=True)
        N = s.numel(self.act_batch)
        if self.cfg == 4:
            return acts_relu_student_t(N, sd)
        return acts_relu_normal(N, sd)

    def iter_weights(self) -> Iterator[Tuple[WeightShape, np.ndarray]]:
        for i, s in enumerate(self.weight_shapes):
            yield s, self.weight_tensor(i)


def config(cfg: int) -> Config:
    if cfg == 1:
        return Config(1, "single conv layer [64,64,3,3] + activations [8,64,32,32]", 128, 20,
                      (WeightShape("conv", 64, 576),), (ActShape("conv.in", 64 * 32 * 32),), 8, "none")
    if cfg == 2:
        return Config(2, "ResNet-18-shaped weights", 256, 20, tuple(resnet18_weights()), (), 0, "none")
    if cfg == 3:
        return Config(3, "MobileNetV2-shaped weights", 256, 20, tuple(mobilenetv2_weights()), (), 0, "none")
    if cfg == 4:
        return Config(4, "ResNet-50-shaped weights + batch-32 activations", 256, 20,
                      tuple(resnet50_weights()), tuple(resnet50_activations()), 32, "top10pct")
    if cfg == 5:
        return Config(5, "VGG-16-shaped weights + batch-16 activations", 512, 20,
                      tuple(vgg16_weights()), tuple(vgg16_activations()), 16, "all")
    raise ValueError(f"unknown config {cfg}")


# --------------------------------------------------------------------------
# small generic generators for tests
# --------------------------------------------------------------------------
def small_weights(K: int, n: int, seed: int, kind: str = "laplace") -> np.ndarray:
    if kind == "laplace":
        return weights_laplace(K, n, seed, 0.005, 0.1)
    if kind == "normal":
        return weights_normal_scaled(K, n, seed)
    if kind == "outliers":
        return weights_normal_outliers(K, n, seed)
    if kind == "student":
        return weights_student_t(K, n, seed)
    raise ValueError(kind)


def on_grid_tensor(K: int, n: int, seed: int, alpha0: float, qlo: int, qhi: int) -> Tuple[np.ndarray, np.ndarray]:
    """Integer codes in [qlo, qhi] (each row holds at least one qhi) times a power-of-two alpha0."""
    rng = np.random.default_rng(seed)
    q = rng.integers(qlo, qhi + 1, size=(K, n))
    q[np.arange(K), rng.integers(0, n, size=K)] = qhi
    return np.ascontiguousarray((q * alpha0).astype(np.float32)), q.astype(np.int32)
