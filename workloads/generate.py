"""Seeded value generators for populations (inputs only, none of the method).

Init rules (one per config family):
  normal002 : every value ~ N(0, 0.02^2)
  kaiming   : conv weights ~ N(0, 2 / fan_out), fan_out = c_out * k * k;
              linear weights ~ N(0, 2 / fan_in); norm weights 1; norm biases
              and biases 0  (so constant tensors are identical across rows)
  trunc002  : weights and embeddings ~ N(0, 0.02^2) truncated at +-2 sigma;
              norm weights 1; biases 0
Momentum buffers ~ N(0, (1e-3)^2).  Each of the N rows is drawn independently.
"""
import math
from typing import Optional, Sequence, Tuple

import numpy as np

from .layouts import Tensor

MOMENTUM_STD = 1e-3


def _rule(t: Tensor, init: str):
    """-> ("normal", std) | ("trunc", std) | ("const", value)"""
    if init == "normal002" or t.kind == "flat":
        return ("normal", 0.02)
    if t.kind == "norm_w":
        return ("const", 1.0)
    if t.kind in ("norm_b", "bias"):
        return ("const", 0.0)
    if init == "kaiming":
        if t.kind == "conv":
            cout, _, kh, kw = t.shape
            return ("normal", math.sqrt(2.0 / (cout * kh * kw)))
        fan_in = t.shape[1]
        return ("normal", math.sqrt(2.0 / fan_in))
    if init == "trunc002":
        return ("trunc", 0.02)
    raise ValueError(init)


def host_population(tensors: Sequence[Tensor], N: int, init: str, seed: int,
                    momentum: bool = False) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """numpy float32 [N, P] (and momentum or None), generated on the host."""
    rng = np.random.default_rng(seed)
    P = sum(t.numel for t in tensors)
    pop = np.empty((N, P), dtype=np.float32)
    off = 0
    for t in tensors:
        kind, v = _rule(t, init)
        sl = pop[:, off:off + t.numel]
        if kind == "const":
            sl[...] = v
        elif kind == "normal":
            sl[...] = rng.standard_normal((N, t.numel), dtype=np.float32) * np.float32(v)
        else:
            x = rng.standard_normal((N, t.numel), dtype=np.float32)
            bad = np.abs(x) > 2.0
            while bad.any():
                x[bad] = rng.standard_normal(int(bad.sum()), dtype=np.float32)
                bad = np.abs(x) > 2.0
            sl[...] = x * np.float32(v)
        off += t.numel
    mom = None
    if momentum:
        mom = rng.standard_normal((N, P), dtype=np.float32) * np.float32(MOMENTUM_STD)
    return pop, mom


def device_population(tensors: Sequence[Tensor], N: int, init: str, seed: int,
                      momentum: bool = False, device: str = "cuda:0", out=None):
    """torch float32 [N, P] (and momentum or None) generated on the device with
    torch's own seeded generator, in place, tensor by tensor (no host copy).
    out: optional (params, momentum) [N, P] float32 device tensors to fill instead of
    allocating new ones (the values do not depend on where the buffers are)."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    P = sum(t.numel for t in tensors)
    if out is not None:
        pop = out[0]
        assert tuple(pop.shape) == (N, P) and pop.dtype == torch.float32 and pop.is_contiguous()
    else:
        pop = torch.empty((N, P), dtype=torch.float32, device=device)
    off = 0
    chunk = 1 << 26
    for t in tensors:
        kind, v = _rule(t, init)
        for a in range(off, off + t.numel, chunk):
            b = min(a + chunk, off + t.numel)
            sl = pop[:, a:b]
            if kind == "const":
                sl.fill_(v)
            elif kind == "normal":
                sl.normal_(0.0, v, generator=gen)
            else:
                sl.normal_(0.0, 1.0, generator=gen)
                for _ in range(64):
                    bad = sl.abs() > 2.0
                    nbad = int(bad.sum())
                    if nbad == 0:
                        break
                    sl[bad] = torch.empty(nbad, dtype=torch.float32, device=device).normal_(0.0, 1.0, generator=gen)
                sl.clamp_(-2.0, 2.0).mul_(v)
        off += t.numel
    mom = None
    if momentum:
        if out is not None:
            mom = out[1]
            assert tuple(mom.shape) == (N, P) and mom.dtype == torch.float32 and mom.is_contiguous()
        else:
            mom = torch.empty((N, P), dtype=torch.float32, device=device)
        for a in range(0, P, chunk):
            mom[:, a:min(a + chunk, P)].normal_(0.0, MOMENTUM_STD, generator=gen)
    return pop, mom


def distinct_population(N: int, P: int, base: int = 0x3F000000) -> np.ndarray:
    """float32 [N, P] whose N*P bit patterns are all distinct (pattern = base +
    n*P + g), so any misplaced value is visible in a bitwise compare."""
    assert base + N * P < 0x7F800000, "patterns must stay finite"
    bits = (np.arange(N * P, dtype=np.uint64) + np.uint64(base)).astype(np.uint32)
    return bits.view(np.float32).reshape(N, P).copy()
