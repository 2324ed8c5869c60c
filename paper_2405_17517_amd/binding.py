"""Thin ctypes binding of libwash_hip.so (declared in include/wash.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
torch is used for device memory and the current stream, nothing else.  If the
library has not been built the import of this module fails loudly; there is no
fallback implementation.
"""
import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwash_hip.so")
MAX_N = 32
OPT_TILE_COORDS = 1
OPT_STREAM_MIN_BYTES = 2
OPT_GAP_BLOCKS = 3
OPT_AVERAGE_CHUNKS = 4
OPT_DENSE = 5
OPT_SHUFFLE_BLOCKS_PER_CU = 6


class WashError(RuntimeError):
    pass


class Segment(ctypes.Structure):
    _fields_ = [("offset", ctypes.c_uint64), ("length", ctypes.c_uint64), ("p", ctypes.c_double)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2405_17517_amd.build, "
            "or __graft_entry__.build()). There is no CPU fallback.")
    L = ctypes.CDLL(LIB_PATH)
    u32, u64, vp = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_void_p
    L.wash_shuffle.argtypes = [vp, vp, u32, u64, vp, u32, u64, u64, vp, vp]
    L.wash_shuffle.restype = ctypes.c_int
    L.wash_shuffle_gap.argtypes = [vp, vp, u32, u64, vp, u32, u64, u64, vp, vp]
    L.wash_shuffle_gap.restype = ctypes.c_int
    L.wash_shuffle_states.argtypes = [vp, u32, u32, u64, vp, u32, u64, u64, ctypes.c_int, vp, vp]
    L.wash_shuffle_states.restype = ctypes.c_int
    L.wash_shuffle_device_step.argtypes = [vp, u32, u32, u64, vp, u32, u64, vp, ctypes.c_int, ctypes.c_int, vp, vp]
    L.wash_shuffle_device_step.restype = ctypes.c_int
    L.wash_average.argtypes = [vp, vp, u32, u64, vp]
    L.wash_average.restype = ctypes.c_int
    L.papa_ema.argtypes = [vp, u32, u64, ctypes.c_float, vp]
    L.papa_ema.restype = ctypes.c_int
    L.wash_consensus_sqdist.argtypes = [vp, u32, u64, u64, u64, vp, vp]
    L.wash_consensus_sqdist.restype = ctypes.c_int
    L.wash_consensus_sqdist_noalloc.argtypes = [vp, u32, u64, u64, u64, vp, vp]
    L.wash_consensus_sqdist_noalloc.restype = ctypes.c_int
    L.wash_weighted_average.argtypes = [vp, vp, vp, u32, u64, vp]
    L.wash_weighted_average.restype = ctypes.c_int
    L.wash_probe_scattered.argtypes = [vp, u64, ctypes.c_int, u32, u32, vp]
    L.wash_probe_scattered.restype = ctypes.c_int
    L.wash_copy_f32.argtypes = [vp, vp, u64, vp]
    L.wash_copy_f32.restype = ctypes.c_int
    L.wash_layer_probs.argtypes = [ctypes.c_double, u32, ctypes.c_int, vp]
    L.wash_layer_probs.restype = ctypes.c_int
    L.wash_strerror.argtypes = [ctypes.c_int]
    L.wash_strerror.restype = ctypes.c_char_p
    L.wash_last_error_detail.argtypes = []
    L.wash_last_error_detail.restype = ctypes.c_char_p
    L.wash_set_option.argtypes = [ctypes.c_int, ctypes.c_int64]
    L.wash_set_option.restype = ctypes.c_int
    L.wash_shutdown.argtypes = []
    L.wash_shutdown.restype = ctypes.c_int
    return L


_lib = _load()


def _check(rc: int, what: str):
    if rc != 0:
        msg = _lib.wash_strerror(rc).decode()
        detail = _lib.wash_last_error_detail().decode()
        raise WashError(f"{what}: {msg}" + (f" ({detail})" if detail else ""))


def _dev_pop(t: torch.Tensor, name: str) -> Tuple[int, int]:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.dim() == 2
            and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous float32 [N, P] tensor on the GPU")
    return t.shape[0], t.shape[1]


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


class SegmentList:
    """Host-side segment array, built once and reused across calls."""

    def __init__(self, segs: Sequence[Tuple[int, int, float]]):
        self.n = len(segs)
        self.array = (Segment * max(self.n, 1))()
        for k, (off, length, p) in enumerate(segs):
            self.array[k].offset, self.array[k].length, self.array[k].p = int(off), int(length), float(p)

    @property
    def ptr(self) -> int:
        return ctypes.addressof(self.array)


def wash_shuffle(params: torch.Tensor, momentum: Optional[torch.Tensor], segs, seed: int, step: int,
                 selected_count: Optional[torch.Tensor] = None) -> None:
    """In-place shuffling step (Eq. 3) on a device population; see wash.h."""
    _shuffle(_lib.wash_shuffle, "wash_shuffle", params, momentum, segs, seed, step, selected_count)


def wash_shuffle_gap(params: torch.Tensor, momentum: Optional[torch.Tensor], segs, seed: int, step: int,
                     selected_count: Optional[torch.Tensor] = None) -> None:
    """The same step on the gap-sampled mask stream (work proportional to p*P); see wash.h."""
    _shuffle(_lib.wash_shuffle_gap, "wash_shuffle_gap", params, momentum, segs, seed, step, selected_count)


def wash_shuffle_states(buffers: Sequence[torch.Tensor], segs, seed: int, step: int, gap_stream: bool = False,
                        selected_count: Optional[torch.Tensor] = None) -> None:
    """The shuffling step on the parameters (buffers[0]) and every optimizer state at once; see wash.h."""
    if len(buffers) == 0:
        raise TypeError("buffers: need at least the parameter population")
    N, P = _dev_pop(buffers[0], "buffers[0]")
    for k, b in enumerate(buffers[1:], 1):
        if _dev_pop(b, f"buffers[{k}]") != (N, P) or b.device != buffers[0].device:
            raise TypeError(f"buffers[{k}]: shape/device must match buffers[0]")
    ptrs = (ctypes.c_void_p * len(buffers))(*[b.data_ptr() for b in buffers])
    cnt_ptr = _count_ptr(selected_count, buffers[0])
    if not isinstance(segs, SegmentList):
        segs = SegmentList(segs)
    with torch.cuda.device(buffers[0].device):
        rc = _lib.wash_shuffle_states(ctypes.addressof(ptrs), len(buffers), N, P, segs.ptr, segs.n, seed, step,
                                      1 if gap_stream else 0, cnt_ptr, _stream(buffers[0]))
    _check(rc, "wash_shuffle_states")


def wash_shuffle_device_step(buffers: Sequence[torch.Tensor], segs, seed: int, step: torch.Tensor,
                             advance: bool = True, gap_stream: bool = False,
                             selected_count: Optional[torch.Tensor] = None) -> None:
    """The shuffling step with the step number read from a one-element int64 device tensor when the kernel runs
    (and incremented afterwards if `advance`), so that a captured HIP graph walks through the steps; see wash.h."""
    if len(buffers) == 0:
        raise TypeError("buffers: need at least the parameter population")
    N, P = _dev_pop(buffers[0], "buffers[0]")
    for k, b in enumerate(buffers[1:], 1):
        if _dev_pop(b, f"buffers[{k}]") != (N, P) or b.device != buffers[0].device:
            raise TypeError(f"buffers[{k}]: shape/device must match buffers[0]")
    if not (isinstance(step, torch.Tensor) and step.is_cuda and step.dtype == torch.int64 and step.numel() == 1
            and step.device == buffers[0].device):
        raise TypeError("step: need a one-element int64 tensor on the same GPU")
    ptrs = (ctypes.c_void_p * len(buffers))(*[b.data_ptr() for b in buffers])
    cnt_ptr = _count_ptr(selected_count, buffers[0])
    if not isinstance(segs, SegmentList):
        segs = SegmentList(segs)
    with torch.cuda.device(buffers[0].device):
        rc = _lib.wash_shuffle_device_step(ctypes.addressof(ptrs), len(buffers), N, P, segs.ptr, segs.n, seed,
                                           step.data_ptr(), 1 if advance else 0, 1 if gap_stream else 0, cnt_ptr,
                                           _stream(buffers[0]))
    _check(rc, "wash_shuffle_device_step")


def _count_ptr(selected_count, params):
    if selected_count is None:
        return None
    if not (selected_count.is_cuda and selected_count.dtype == torch.int64 and selected_count.numel() == 1
            and selected_count.device == params.device):
        raise TypeError("selected_count: need a one-element int64 tensor on the same GPU")
    return selected_count.data_ptr()


def _shuffle(fn, name, params, momentum, segs, seed, step, selected_count) -> None:
    N, P = _dev_pop(params, "params")
    mom_ptr = None
    if momentum is not None:
        if _dev_pop(momentum, "momentum") != (N, P) or momentum.device != params.device:
            raise TypeError("momentum: shape/device must match params")
        mom_ptr = momentum.data_ptr()
    cnt_ptr = _count_ptr(selected_count, params)
    if not isinstance(segs, SegmentList):
        segs = SegmentList(segs)
    with torch.cuda.device(params.device):
        rc = fn(params.data_ptr(), mom_ptr, N, P, segs.ptr, segs.n, seed, step, cnt_ptr, _stream(params))
    _check(rc, name)


def wash_average(params: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Uniform average over the population (Alg. 1 output); returns out [P]."""
    N, P = _dev_pop(params, "params")
    if out is None:
        out = torch.empty(P, dtype=torch.float32, device=params.device)
    elif not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() == P
              and out.device == params.device):
        raise TypeError("out: need a contiguous float32 [P] tensor on the same GPU")
    with torch.cuda.device(params.device):
        rc = _lib.wash_average(params.data_ptr(), out.data_ptr(), N, P, _stream(params))
    _check(rc, "wash_average")
    return out


def papa_ema(params: torch.Tensor, alpha: float) -> None:
    """In-place PAPA update (Eq. 1) on a device population."""
    N, P = _dev_pop(params, "params")
    with torch.cuda.device(params.device):
        rc = _lib.papa_ema(params.data_ptr(), N, P, float(alpha), _stream(params))
    _check(rc, "papa_ema")


def wash_consensus_sqdist(params: torch.Tensor, g_begin: int = 0, g_end: Optional[int] = None,
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """float64 [N] on the GPU: sum over the slice of (theta_n - mean)^2 (Eq. 2 / Eq. 5 quantity)."""
    N, P = _dev_pop(params, "params")
    if g_end is None:
        g_end = P
    if out is None:
        out = torch.empty(N, dtype=torch.float64, device=params.device)
    elif not (out.is_cuda and out.dtype == torch.float64 and out.is_contiguous() and out.numel() == N
              and out.device == params.device):
        raise TypeError("out: need a contiguous float64 [N] tensor on the same GPU")
    with torch.cuda.device(params.device):
        rc = _lib.wash_consensus_sqdist(params.data_ptr(), N, P, int(g_begin), int(g_end), out.data_ptr(),
                                        _stream(params))
    _check(rc, "wash_consensus_sqdist")
    return out


def wash_consensus_sqdist_noalloc(params: torch.Tensor, out: torch.Tensor, g_begin: int = 0,
                                  g_end: Optional[int] = None) -> torch.Tensor:
    """wash_consensus_sqdist without any allocation: the caller brings out (float64 [N]); see wash.h."""
    N, P = _dev_pop(params, "params")
    if g_end is None:
        g_end = P
    if not (isinstance(out, torch.Tensor) and out.is_cuda and out.dtype == torch.float64 and out.is_contiguous()
            and out.numel() == N and out.device == params.device):
        raise TypeError("out: need a contiguous float64 [N] tensor on the same GPU")
    with torch.cuda.device(params.device):
        rc = _lib.wash_consensus_sqdist_noalloc(params.data_ptr(), N, P, int(g_begin), int(g_end), out.data_ptr(),
                                                _stream(params))
    _check(rc, "wash_consensus_sqdist_noalloc")
    return out


def wash_weighted_average(params: torch.Tensor, weights: Sequence[float],
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out[g] = sum_n weights[n] * params[n][g] (fp64 accumulation); returns out [P]."""
    N, P = _dev_pop(params, "params")
    if len(weights) != N:
        raise TypeError("need one weight per model")
    w = (ctypes.c_double * N)(*[float(x) for x in weights])
    if out is None:
        out = torch.empty(P, dtype=torch.float32, device=params.device)
    elif not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() == P
              and out.device == params.device):
        raise TypeError("out: need a contiguous float32 [P] tensor on the same GPU")
    with torch.cuda.device(params.device):
        rc = _lib.wash_weighted_average(params.data_ptr(), ctypes.addressof(w), out.data_ptr(), N, P, _stream(params))
    _check(rc, "wash_weighted_average")
    return out


def wash_copy_f32(src: torch.Tensor, dst: torch.Tensor) -> None:
    """Plain streaming copy of a float32 buffer (bandwidth yardstick, see wash_bench.h)."""
    for t in (src, dst):
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
            raise TypeError("need contiguous float32 GPU tensors")
    if src.numel() != dst.numel() or src.device != dst.device:
        raise TypeError("src and dst must have the same size and device")
    with torch.cuda.device(src.device):
        rc = _lib.wash_copy_f32(src.data_ptr(), dst.data_ptr(), src.numel(), _stream(src))
    _check(rc, "wash_copy_f32")


def wash_probe_scattered(buf: torch.Tensor, mode: int, rounds: int, blocks: int) -> int:
    """Scattered access yardstick on a float32 buffer of a power-of-two number of 128-byte lines
    (see wash_bench.h); returns the number of places accessed (4-byte elements in modes 0 to 2, 64-byte
    pieces in mode 3)."""
    if not (buf.is_cuda and buf.dtype == torch.float32 and buf.is_contiguous()):
        raise TypeError("need a contiguous float32 GPU tensor")
    lines = buf.numel() // 32
    if lines * 32 != buf.numel():
        raise TypeError("buffer must be a whole number of 128-byte lines")
    with torch.cuda.device(buf.device):
        rc = _lib.wash_probe_scattered(buf.data_ptr(), lines, int(mode), int(rounds), int(blocks), _stream(buf))
    _check(rc, "wash_probe_scattered")
    return blocks * 256 * rounds * 8 // (4 if int(mode) == 3 else 1)


def wash_layer_probs(p: float, L: int, schedule: int = 0):
    """Eq. 6 (schedule 0) and its constant / increasing variants; list of L floats."""
    out = (ctypes.c_double * max(int(L), 1))()
    _check(_lib.wash_layer_probs(float(p), int(L), int(schedule), ctypes.addressof(out)), "wash_layer_probs")
    return [out[k] for k in range(L)]


def wash_set_option(option: int, value: int) -> None:
    _check(_lib.wash_set_option(int(option), int(value)), "wash_set_option")


def wash_shutdown() -> None:
    _check(_lib.wash_shutdown(), "wash_shutdown")


# raw entry points for tests of the C ABI itself (error paths, NULL arguments)
raw = _lib
