"""The five benchmark configurations, as data (no arithmetic of the method).

Each stands in for a workload of the paper (ResNet-18 on CIFAR, ResNet-50 on
ImageNet; N and p as in its experiments) or extends it (ViT-B/16, a 1.1e9
parameter stress case).  Values are synthetic and seeded; no dataset or trained
weight is involved: the population-update path only moves or averages numbers.
"""
from dataclasses import dataclass, field
from typing import Callable, List, Sequence, Tuple

from . import layouts


@dataclass(frozen=True)
class WorkloadConfig:
    index: int                       # 1-based, as listed in the baseline file
    name: str
    N: int
    layout: Callable[[], List[layouts.Tensor]]
    init: str                        # "normal002" | "kaiming" | "trunc002"
    probs: Callable[[int], Sequence[float]]   # number of tensors -> p per tensor
    momentum: bool
    steps: int
    seed: int = 0
    data_seed: int = 1234
    p_sweep: Tuple[float, ...] = field(default_factory=tuple)   # config 4 only
    alpha: float = 0.99

    def tensors(self):
        return self.layout()

    @property
    def P(self) -> int:
        return sum(t.numel for t in self.layout())

    def segments(self, p_override: float = None):
        ts = self.layout()
        ps = [p_override] * len(ts) if p_override is not None else list(self.probs(len(ts)))
        return layouts.segments_of(ts, ps)


def _const(p):
    return lambda n: [p] * n


def _linear_005_0001(n):
    # p_s = 0.05 - 0.049 * s / (n - 1): 0.05 on the first segment, 0.001 on the last
    return [0.05 - 0.049 * s / (n - 1) for s in range(n)]


CONFIGS = [
    WorkloadConfig(1, "flat-2^20", 4, lambda: layouts.flat(1 << 20), "normal002", _const(0.01),
                   momentum=False, steps=1, data_seed=1235),
    WorkloadConfig(2, "resnet18-cifar10", 5, layouts.resnet18_cifar, "kaiming", _const(0.001),
                   momentum=False, steps=100, data_seed=1236),
    WorkloadConfig(3, "resnet50-imagenet", 10, layouts.resnet50_imagenet, "kaiming", _const(0.005),
                   momentum=True, steps=100, data_seed=1237),
    WorkloadConfig(4, "vit-b16", 20, layouts.vit_b16, "trunc002", _const(1e-3),
                   momentum=False, steps=20, data_seed=1238, p_sweep=(1e-4, 1e-3, 1e-2, 1e-1)),
    WorkloadConfig(5, "flat-1.1e9x200", 8, lambda: layouts.flat(1_100_000_000, 200), "normal002",
                   _linear_005_0001, momentum=True, steps=10, data_seed=1239),
]


def get_config(index: int) -> WorkloadConfig:
    return CONFIGS[index - 1]
