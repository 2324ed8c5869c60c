"""Seeded synthetic populations shaped like the paper's workloads.

This package holds tensor layouts and random input generators only: none of
the method's arithmetic (no shuffle, average, EMA, probability schedule or
random stream of the method) lives here.  It serves the tests, the benchmark
and the smoke check, on the oracle side and on the GPU side alike.
"""
from .layouts import Tensor, resnet18_cifar, resnet50_imagenet, vit_b16, flat, segments_of  # noqa: F401
from .configs import CONFIGS, WorkloadConfig, get_config  # noqa: F401
from .generate import host_population, device_population, distinct_population  # noqa: F401
