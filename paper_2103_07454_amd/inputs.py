"""Seeded synthetic workloads for the EventGraD parameter path.

This module only *describes* inputs: parameter-tensor shape lists of the
networks the paper trains (Section 7: a residual network for 32x32 images;
its earlier proof of concept used a small MLP), the initial parameter values,
and the hyper-parameters of the five benchmark configurations.  It contains
none of the method's arithmetic (no norms, triggers, averaging, updates or
gradient generation), so the HIP path and the CPU test oracle may both be fed
from it without sharing code.

The tensors stand in for the paper's CIFAR-10 / ResNet-18 workload: shapes and
counts follow the architectures, values are synthetic and seeded.
Tensor order is the usual parameter registration order: convolution weight,
then batch-norm scale and shift; a block's projection shortcut after its main
path; classifier weight then bias.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

# ---------------------------------------------------------------------------
# tensor shape lists
# ---------------------------------------------------------------------------


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: Tuple[int, ...]
    fan_in: int
    kind: str  # "weight" | "bn_scale" | "bn_shift" | "bias"

    @property
    def numel(self) -> int:
        n = 1
        for s in self.shape:
            n *= s
        return n


def _conv(name, cin, cout, k):
    return TensorSpec(name + ".weight", (cout, cin, k, k), cin * k * k, "weight")


def _bn(name, c):
    return [TensorSpec(name + ".weight", (c,), c, "bn_scale"),
            TensorSpec(name + ".bias", (c,), c, "bn_shift")]


def _fc(name, fin, fout):
    return [TensorSpec(name + ".weight", (fout, fin), fin, "weight"),
            TensorSpec(name + ".bias", (fout,), fin, "bias")]


def mlp(sizes: Sequence[int] = (784, 128, 10)) -> List[TensorSpec]:
    out: List[TensorSpec] = []
    for i in range(len(sizes) - 1):
        out += _fc(f"fc{i + 1}", sizes[i], sizes[i + 1])
    return out


def _basic_stage(out, prefix, cin, cout, blocks, project_first):
    for b in range(blocks):
        name = f"{prefix}.{b}"
        c_in = cin if b == 0 else cout
        out.append(_conv(name + ".conv1", c_in, cout, 3))
        out += _bn(name + ".bn1", cout)
        out.append(_conv(name + ".conv2", cout, cout, 3))
        out += _bn(name + ".bn2", cout)
        if b == 0 and project_first:
            out.append(_conv(name + ".shortcut.0", c_in, cout, 1))
            out += _bn(name + ".shortcut.1", cout)


def resnet20(width: int = 16, classes: int = 10) -> List[TensorSpec]:
    """ResNet-20 for 32x32 inputs with 1x1 projection shortcuts (65 tensors)."""
    out: List[TensorSpec] = [_conv("conv1", 3, width, 3)]
    out += _bn("bn1", width)
    _basic_stage(out, "layer1", width, width, 3, False)
    _basic_stage(out, "layer2", width, 2 * width, 3, True)
    _basic_stage(out, "layer3", 2 * width, 4 * width, 3, True)
    out += _fc("fc", 4 * width, classes)
    return out


def resnet18(width: int = 64, classes: int = 10) -> List[TensorSpec]:
    """ResNet-18 for 32x32 inputs (3x3 stem), 62 tensors at any width."""
    out: List[TensorSpec] = [_conv("conv1", 3, width, 3)]
    out += _bn("bn1", width)
    _basic_stage(out, "layer1", width, width, 2, False)
    _basic_stage(out, "layer2", width, 2 * width, 2, True)
    _basic_stage(out, "layer3", 2 * width, 4 * width, 2, True)
    _basic_stage(out, "layer4", 4 * width, 8 * width, 2, True)
    out += _fc("fc", 8 * width, classes)
    return out


def resnet50(width: int = 64, classes: int = 1000) -> List[TensorSpec]:
    """ResNet-50 in its ImageNet form (7x7 stem, bottlenecks [3,4,6,3]), 161 tensors."""
    out: List[TensorSpec] = [_conv("conv1", 3, width, 7)]
    out += _bn("bn1", width)
    cin = width
    for s, blocks in enumerate((3, 4, 6, 3)):
        mid = width << s
        cout = 4 * mid
        for b in range(blocks):
            name = f"layer{s + 1}.{b}"
            c_in = cin if b == 0 else cout
            out.append(_conv(name + ".conv1", c_in, mid, 1))
            out += _bn(name + ".bn1", mid)
            out.append(_conv(name + ".conv2", mid, mid, 3))
            out += _bn(name + ".bn2", mid)
            out.append(_conv(name + ".conv3", mid, cout, 1))
            out += _bn(name + ".bn3", cout)
            if b == 0:
                out.append(_conv(name + ".downsample.0", c_in, cout, 1))
                out += _bn(name + ".downsample.1", cout)
        cin = cout
    out += _fc("fc", cin, classes)
    return out


def total_numel(tensors: Sequence[TensorSpec]) -> int:
    return sum(t.numel for t in tensors)


# ---------------------------------------------------------------------------
# initial parameters
# ---------------------------------------------------------------------------


def init_params(tensors: Sequence[TensorSpec], seed: int) -> np.ndarray:
    """Kaiming-normal weights (sigma = sqrt(2/fan_in)), batch-norm scale 1,
    shifts and biases 0.  Returns one replica's parameters, tensors
    concatenated without padding, float32."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    parts = []
    for t in tensors:
        if t.kind == "weight":
            w = rng.standard_normal(t.numel, dtype=np.float32)
            w *= np.float32(np.sqrt(2.0 / t.fan_in))
            parts.append(w)
        elif t.kind == "bn_scale":
            parts.append(np.ones(t.numel, dtype=np.float32))
        else:
            parts.append(np.zeros(t.numel, dtype=np.float32))
    return np.concatenate(parts)


def replicate(x0: np.ndarray, P: int) -> np.ndarray:
    """Common start for all P replicas (the analysis assumes one, Section 5)."""
    return np.ascontiguousarray(np.broadcast_to(x0, (P, x0.size)))


def distinct_params(n: int, P: int, seed: int, scale: float = 1.0) -> np.ndarray:
    """Per-replica different values, for tests of the averaging step."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    return (rng.standard_normal((P, n)) * scale).astype(np.float32)


def random_grads(P: int, n: int, seed: int, scale: float = 1.0) -> np.ndarray:
    """A caller-supplied gradient buffer (one iteration), for buffer-mode tests."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    return (rng.standard_normal((P, n)) * scale).astype(np.float32)


# ---------------------------------------------------------------------------
# benchmark configurations
# ---------------------------------------------------------------------------

THR_FIXED, THR_ADAPTIVE = 0, 1
DIST_GAUSS, DIST_STUDENT_T3 = 0, 1

DEFAULT_SEED = 210307454


@dataclass
class Workload:
    name: str
    P: int
    tensors: List[TensorSpec]
    iters: int
    lr: float = 0.05
    momentum: float = 0.9
    thr_mode: int = THR_ADAPTIVE
    thr_fixed: float = 0.0
    horizon: float = 1.0          # h = 1 in the paper's experiments (Section 7)
    delta_init: float = 0.0
    force_first: int = 1          # first event forced at k = 0 (Section 4)
    topk_ppm: int = 0             # Top-K share in parts per million (0 = whole tensors)
    dist: int = DIST_GAUSS
    sigma0: float = 0.01
    fan_in_scaling: int = 1       # sigma_l = sigma0 / sqrt(fan_in_l)
    decay: float = 1.0            # sigma decays as decay**k
    spike_prob: float = 0.0
    spike_gain: float = 1.0
    seed: int = DEFAULT_SEED

    @property
    def L(self) -> int:
        return len(self.tensors)

    @property
    def N(self) -> int:
        return total_numel(self.tensors)

    @property
    def layer_numel(self) -> np.ndarray:
        return np.array([t.numel for t in self.tensors], dtype=np.uint64)

    @property
    def layer_fan_in(self) -> np.ndarray:
        return np.array([t.fan_in for t in self.tensors], dtype=np.uint32)

    def x0(self) -> np.ndarray:
        return init_params(self.tensors, self.seed)

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def config(i: int, seed: int = DEFAULT_SEED) -> Workload:
    """The five benchmark configurations, numbered 1..5."""
    if i == 1:
        return Workload("cfg1_mlp_p4_fixed", 4, mlp(), 100, thr_mode=THR_FIXED,
                        thr_fixed=1e-3, sigma0=0.01, fan_in_scaling=0, decay=0.99,
                        seed=seed)
    if i == 2:
        return Workload("cfg2_resnet20_p8_adaptive", 8, resnet20(), 500, sigma0=0.02,
                        decay=0.995, seed=seed)
    if i == 3:
        return Workload("cfg3_resnet18_p16_adaptive_spikes", 16, resnet18(), 200,
                        sigma0=0.01, decay=0.995, spike_prob=0.1, spike_gain=5.0,
                        seed=seed)
    if i == 4:
        return Workload("cfg4_resnet50_p8_topk1pct_student_t", 8, resnet50(), 100,
                        sigma0=0.01, decay=1.0, dist=DIST_STUDENT_T3, topk_ppm=10_000,
                        seed=seed)
    if i == 5:
        return Workload("cfg5_resnet18_p64_topk10pct", 64, resnet18(), 100,
                        sigma0=0.01, decay=0.995, topk_ppm=100_000, seed=seed)
    raise ValueError(f"no configuration {i}")


def reduced(i: int, seed: int = DEFAULT_SEED) -> Workload:
    """Narrow-channel versions of configurations 3-5: same tensor count, ring
    size, trigger and send mode, small enough for a CPU oracle to run the full
    iteration count in seconds."""
    w = config(i, seed)
    if i == 3:
        return w.scaled(name=w.name + "_w8", tensors=resnet18(width=8))
    if i == 4:
        return w.scaled(name=w.name + "_w8", tensors=resnet50(width=8, classes=100))
    if i == 5:
        return w.scaled(name=w.name + "_w8", tensors=resnet18(width=8))
    return w
