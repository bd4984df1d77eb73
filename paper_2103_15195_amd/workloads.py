"""Seeded synthetic gradient workloads shaped like the paper's models.

This module holds ONLY input generation: tensor-shape lists of the five
benchmark configurations and the seeded random values that fill them.  It
contains none of the compression method's arithmetic, so both the test oracle
and the HIP path may be fed from it without sharing any of the method's code.

The paper (Section 5, "Workloads") trains ResNet50 / ResNet101 / Mask R-CNN on
CIFAR10 / ImageNet / COCO.  Those datasets are not needed here: the hot path
only sees gradient *tensors*, so the stand-in is a list of fp32 tensors with
the architectures' parameter shapes (161 tensors for ResNet50 and 314 for
ResNet101, as the caption of Figure 3 states) filled with seeded random
values.  Tensor lists are returned in gradient-ready order, i.e. the reverse of
forward order, which is the order wait-free back-propagation produces them in
(Section 2.2).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

Shape = Tuple[int, ...]


# --------------------------------------------------------------------------
# shape lists (forward order inside the helpers; reversed on return)
# --------------------------------------------------------------------------
def _bn(c: int) -> List[Shape]:
    return [(c,), (c,)]  # gamma, beta


def mlp_shapes() -> List[Shape]:
    """784-256-256-10 perceptron: weight and bias of three linear layers."""
    fwd = [(784, 256), (256,), (256, 256), (256,), (256, 10), (10,)]
    return fwd[::-1]


def resnet20_shapes() -> List[Shape]:
    """CIFAR ResNet-20: 3x3 stem, three stages of three basic blocks
    (16/32/64 channels), 1x1 projection shortcut with BN on the two
    down-sampling blocks, FC 64x10 with bias."""
    fwd: List[Shape] = [(16, 3, 3, 3)] + _bn(16)
    cin = 16
    for cout in (16, 32, 64):
        for b in range(3):
            fwd += [(cout, cin, 3, 3)] + _bn(cout)
            fwd += [(cout, cout, 3, 3)] + _bn(cout)
            if b == 0 and cin != cout:
                fwd += [(cout, cin, 1, 1)] + _bn(cout)
            cin = cout
    fwd += [(10, 64), (10,)]
    return fwd[::-1]


def _bottleneck_backbone(blocks: Sequence[int]) -> List[Shape]:
    fwd: List[Shape] = [(64, 3, 7, 7)] + _bn(64)
    cin = 64
    for stage, nb in enumerate(blocks):
        mid = 64 << stage
        cout = mid * 4
        for b in range(nb):
            fwd += [(mid, cin, 1, 1)] + _bn(mid)
            fwd += [(mid, mid, 3, 3)] + _bn(mid)
            fwd += [(cout, mid, 1, 1)] + _bn(cout)
            if b == 0:
                fwd += [(cout, cin, 1, 1)] + _bn(cout)
            cin = cout
    return fwd


def resnet50_shapes() -> List[Shape]:
    """ImageNet ResNet-50 (3-4-6-3 bottlenecks) with FC 2048x1000 + bias."""
    fwd = _bottleneck_backbone((3, 4, 6, 3)) + [(1000, 2048), (1000,)]
    return fwd[::-1]


def resnet101_shapes() -> List[Shape]:
    """ImageNet ResNet-101 (3-4-23-3 bottlenecks) with FC 2048x1000 + bias."""
    fwd = _bottleneck_backbone((3, 4, 23, 3)) + [(1000, 2048), (1000,)]
    return fwd[::-1]


def maskrcnn_shapes() -> List[Shape]:
    """Mask R-CNN with a ResNet-50-FPN backbone, 91 classes: backbone (BN
    affine parameters counted), FPN lateral 1x1 and output 3x3 256-channel
    convolutions, RPN head, two-FC box head (12544x1024, 1024x1024) with
    91/364-way predictors, four-conv mask head with 2x2 deconvolution and a
    91-way 1x1 predictor."""
    fwd = _bottleneck_backbone((3, 4, 6, 3))
    for cin in (256, 512, 1024, 2048):          # FPN lateral
        fwd += [(256, cin, 1, 1), (256,)]
    for _ in range(4):                          # FPN output
        fwd += [(256, 256, 3, 3), (256,)]
    fwd += [(256, 256, 3, 3), (256,), (3, 256, 1, 1), (3,), (12, 256, 1, 1), (12,)]  # RPN
    fwd += [(1024, 12544), (1024,), (1024, 1024), (1024,)]                         # box head
    fwd += [(91, 1024), (91,), (364, 1024), (364,)]                                # box predictors
    for _ in range(4):                          # mask head
        fwd += [(256, 256, 3, 3), (256,)]
    fwd += [(256, 256, 2, 2), (256,), (91, 256, 1, 1), (91,)]
    return fwd[::-1]


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    cfg: int                 # index into the benchmark configuration list
    name: str
    shapes: Tuple[Shape, ...]
    dist: str                # "normal_fixed" | "normal_loguniform" | "student_t3"
    workers: int
    ys: Tuple[int, ...]

    @property
    def numel(self) -> np.ndarray:
        return np.array([int(np.prod(s)) for s in self.shapes], dtype=np.int64)

    @property
    def total(self) -> int:
        return int(self.numel.sum())


def workload(cfg: int) -> Workload:
    if cfg == 0:
        return Workload(0, "mlp", tuple(mlp_shapes()), "normal_fixed", 4, (2,))
    if cfg == 1:
        return Workload(1, "resnet20", tuple(resnet20_shapes()), "normal_loguniform", 8, (1, 2, 4, 8, 16))
    if cfg == 2:
        return Workload(2, "resnet50", tuple(resnet50_shapes()), "normal_loguniform", 8, (1, 2, 3, 4))
    if cfg == 3:
        return Workload(3, "resnet101", tuple(resnet101_shapes()), "normal_loguniform", 16, (1, 2, 4))
    if cfg == 4:
        return Workload(4, "maskrcnn_r50fpn", tuple(maskrcnn_shapes()), "student_t3", 8, (1, 2, 4))
    raise ValueError(f"unknown workload config {cfg}")


def synthetic_workload(numel: Sequence[int], dist: str = "normal_loguniform", workers: int = 2,
                       cfg: int = 99, name: str = "custom") -> Workload:
    """A workload over an arbitrary list of tensor sizes (edge-case tests)."""
    return Workload(cfg, name, tuple((int(n),) for n in numel), dist, workers, (1,))


# --------------------------------------------------------------------------
# values
# --------------------------------------------------------------------------
def tensor_std(wl: Workload) -> np.ndarray:
    """Per-tensor standard deviation: a property of the model, shared by all
    workers and iterations.  Fixed 0.01 for the MLP; otherwise log-uniform in
    [1e-4, 1e-1]."""
    n = len(wl.shapes)
    if wl.dist == "normal_fixed":
        return np.full(n, 0.01, dtype=np.float64)
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([0, wl.cfg, 0xFFFF])))
    return 10.0 ** rng.uniform(-4.0, -1.0, size=n)


def gradients_flat(wl: Workload, worker: int, it: int, shared_fraction: float = 0.0) -> np.ndarray:
    """One worker's gradients as one flat fp32 vector (tensors in list order).

    Workers are independent by default; with shared_fraction = f the value is
    sqrt(f) * common + sqrt(1 - f) * private so that large entries overlap
    between workers (exercises index collisions in the sparse decompress)."""
    std = tensor_std(wl).astype(np.float32)
    numel = wl.numel
    total = int(numel.sum())

    def draw(seed_words) -> np.ndarray:
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence(seed_words)))
        if wl.dist == "student_t3":
            x = rng.standard_t(3.0, size=total).astype(np.float32)
        else:
            x = rng.standard_normal(size=total, dtype=np.float32)
        return x

    x = draw([0, wl.cfg, worker, it])
    if shared_fraction > 0.0:
        common = draw([0, wl.cfg, 0xC0FFEE, it])
        x = np.float32(np.sqrt(shared_fraction)) * common + np.float32(np.sqrt(1.0 - shared_fraction)) * x
    off = 0
    for t, n in enumerate(numel):
        x[off:off + int(n)] *= std[t]
        off += int(n)
    return x


def split(wl: Workload, flat: np.ndarray) -> List[np.ndarray]:
    """Views of a flat vector, one per tensor of the workload."""
    offs = np.concatenate([[0], np.cumsum(wl.numel)])
    return [flat[int(offs[t]):int(offs[t + 1])] for t in range(len(wl.shapes))]


def gradients(wl: Workload, worker: int, it: int, shared_fraction: float = 0.0) -> List[np.ndarray]:
    """One worker's fp32 gradient tensors (flattened, list order = wl.shapes)."""
    return split(wl, gradients_flat(wl, worker, it, shared_fraction))


# --------------------------------------------------------------------------
# inputs of the partition search (Section 4.3): a back-propagation timeline and
# the communication cost, from the figures the paper prints
# --------------------------------------------------------------------------
PAPER_ITERATION_S = 64e-3        # Section 3.3: one ResNet50 / CIFAR10 iteration on a V100
PAPER_COMM_S = 66e-3             # Section 3.3: communicating its 102 MB of fp32 gradients between two V100 over PCIe
PAPER_MESSAGE_S = 50e-6          # fixed cost per message (a launch plus a PCIe round trip; the paper gives B_g no value)
SENT_BYTES_PER_ELEM = {"fp16": 2.0, "qsgd": 1.0, "terngrad": 0.25, "efsign": 0.125, "signsgd": 0.125, "signum": 0.125,
                       "onebit": 0.125}


def sent_bytes_per_elem(algo: str, ratio_ppm: int) -> float:
    """Bytes a compressor sends per gradient element (Table 1's payloads; a sparsifier sends an index and a value per
    kept entry)."""
    return SENT_BYTES_PER_ELEM.get(algo, 8.0 * ratio_ppm * 1e-6)


def iteration_timeline(numel: Sequence[int], B_h_s: float, gamma_h_s: float, sent_bytes: float):
    """Inputs of the iteration-time model F (Section 4.3) for a tensor list.

    Returns (bwd, (fwd, B_h, gamma_h, B_g, gamma_g)): the forward pass takes a third of the paper's iteration and the
    back-propagation of a tensor a share of the rest proportional to its size; g(x) is linear (Assumption 5), its slope
    the paper's PCIe figure scaled to `sent_bytes` per element; h(x) = B_h_s + gamma_h_s x is the caller's (measured).
    """
    D = float(sum(int(m) for m in numel))
    bwd = [(2.0 / 3.0) * PAPER_ITERATION_S * (int(m) / D) for m in numel]
    gamma_g = PAPER_COMM_S / 25557032.0 * (sent_bytes / 4.0)
    return bwd, (PAPER_ITERATION_S / 3.0, float(B_h_s), float(gamma_h_s), PAPER_MESSAGE_S, gamma_g)
