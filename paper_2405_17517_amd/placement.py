"""Where the [N, P] buffers of a population sit in HBM (MI355X).

How fast the DRAM takes the scattered accesses of the shuffling step (Eq. 3 moves single
values across the N rows), and the 2N interleaved row streams of the EMA, depends on the
physical place of the buffers.  Measured on MI355X, the physical address space under one
large allocation has two boundaries that matter, at 96 and at 192 GiB from its start
(three regions of 96 GiB), and a buffer that straddles one of them half and half is
served by the DRAM banks of two regions instead of one: a 1 GiB population shuffles 18 %
faster there (and nowhere else in a 262 GiB arena), a 6.5 GiB one (N = 20) 21 % faster
with its EMA 8 % faster; parameters and momentum of 32.8 GiB each take 14.2 ms per
shuffle back to back and 10.9 ms with each across one of the boundaries.  The average
alone prefers to sit inside one region (4 - 9 % slower across a boundary).  Virtual
addresses tell nothing about this, and the default allocator places buffers back to
back.

`place_population` therefore allocates ONE arena, finds the boundaries with a small probe
buffer moved over the arena in fine steps, tries positions for the buffers on a coarse
grid and centred on those boundaries, and keeps the fastest, timing the library's own
kernels (one pass of the hot path: shuffle, EMA, average) on the still uninitialised
memory.  It returns ordinary contiguous [N, P] float32 views: the layout every entry
point of the library expects is unchanged.  This module holds no arithmetic of the
method; torch is used for device memory and events only.
"""
from typing import Callable, List, Optional, Sequence, Tuple

import torch

from . import binding as _b

GiB = 1 << 30


def _timed(fn: Callable[[], None], reps: int) -> float:
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def _find_boundaries(arena: torch.Tensor, log: Optional[Callable[[str], None]]) -> List[int]:
    """Byte offsets in the arena around which a small population shuffles markedly faster than elsewhere:
    a [8, 2^24] probe buffer (512 MiB) is moved over the arena in steps of half its size and one shuffling
    step is timed at every position; positions more than 7 % below the median are dips, neighbouring dips
    are one boundary, at the middle of the fastest position."""
    n, cols = 8, 1 << 24
    size = n * cols * 4
    step = size // 2
    if arena.numel() < 8 * size:
        return []
    segs = _b.SegmentList([(0, cols, 0.02)])
    times = []
    k = [0]
    for off in range(0, arena.numel() - size + 1, step):
        buf = arena[off:off + size].view(torch.float32).view(n, cols)

        def probe():
            _b.wash_shuffle_states([buf], segs, 0, k[0])
            k[0] += 1

        times.append((off, _timed(probe, 3)))
    ordered = sorted(t for _, t in times)
    median = ordered[len(ordered) // 2]
    dips = [(off, t) for off, t in times if t < 0.93 * median]
    found: List[int] = []
    group: List[Tuple[int, float]] = []
    for off, t in dips + [(None, None)]:
        if group and (off is None or off - group[-1][0] > 2 * step):
            best = min(group, key=lambda x: x[1])
            found.append(best[0] + size // 2)
            group = []
        if off is not None:
            group.append((off, t))
    if log is not None:
        log(f"probe of {len(times)} positions, median {median * 1e3:.1f} us: faster across "
            + (", ".join(f"{b / GiB:.1f} GiB" for b in found) if found else "no position"))
    return found


def place_population(N: int, P: int, nbuf: int = 1, segs=None, device: str = "cuda:0",
                     arena_bytes: Optional[int] = None, reserve_bytes: int = 24 * GiB, grid_bytes: int = 8 * GiB,
                     reps: int = 2, log: Optional[Callable[[str], None]] = None,
                     offsets: Optional[Sequence[int]] = None,
                     boundaries: Optional[Sequence[int]] = None) -> Tuple[List[torch.Tensor], dict]:
    """nbuf uninitialised [N, P] float32 buffers (parameters first, then optimizer states) inside one arena,
    at the positions where one pass of the hot path (a shuffling step over all buffers, then the EMA and the
    average of the parameters) ran fastest.

      segs           the segment list the caller will shuffle with (list of (offset, length, p) or a
                     SegmentList); default: one segment with p = 0.02
      arena_bytes    size of the arena; default: the free device memory minus reserve_bytes
      grid_bytes     spacing of the candidate positions
      offsets        byte offsets found by an earlier call with the same arena size: the buffers are placed
                     there without probing
      boundaries     info["boundaries"] of an earlier call with the same arena size in this process: the
                     search for them is not repeated
    Returns (buffers, info); info holds the arena tensor (keep it alive as long as the buffers), the chosen
    offsets, the boundaries found, and the probe times in ms of every candidate.  The buffers are placed one
    after the other: the parameters where they alone are fastest, then each further buffer where the pass
    over all buffers placed so far is fastest.  Populations too small to matter (below 512 MiB per buffer)
    and arenas without room to move are placed back to back without probing."""
    dev = torch.device(device)
    buf_bytes = N * P * 4
    pitch = (buf_bytes + 255) // 256 * 256
    with torch.cuda.device(dev):
        torch.cuda.empty_cache()                    # blocks torch keeps cached count as used otherwise
        free, _ = torch.cuda.mem_get_info()
    if arena_bytes is None:
        arena_bytes = free - reserve_bytes
    arena_bytes = min(arena_bytes, free - (1 << 28))
    if arena_bytes < nbuf * pitch:
        raise MemoryError(f"{nbuf} buffers of {buf_bytes} bytes do not fit an arena of {arena_bytes} bytes")
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device=dev)
    if arena.data_ptr() % 256 != 0:
        raise RuntimeError("arena is not 256-byte aligned")

    def view(off: int) -> torch.Tensor:
        return arena[off:off + buf_bytes].view(torch.float32).view(N, P)

    info = {"arena": arena, "arena_bytes": arena_bytes, "offsets": [], "probes_ms": [], "tuned": False}
    if offsets is not None:
        offs = [int(o) for o in offsets]
        if len(offs) != nbuf or any(o % 256 != 0 or o < 0 or o + buf_bytes > arena_bytes for o in offs) or \
                any(a < b + pitch and b < a + pitch for i, a in enumerate(offs) for b in offs[:i]):
            raise ValueError("offsets do not fit this arena")
        info["offsets"], info["tuned"] = offs, True
        return [view(o) for o in offs], info
    candidates = list(range(0, arena_bytes - pitch + 1, grid_bytes))
    if buf_bytes < GiB // 2 or len(candidates) < 2 * nbuf + 1:
        offs = [k * pitch for k in range(nbuf)]
        info["offsets"] = offs
        return [view(o) for o in offs], info

    if segs is None:
        segs = [(0, P, 0.02)]
    if not isinstance(segs, _b.SegmentList):
        segs = _b.SegmentList(segs)
    arena.zero_()                                   # the probes move whatever is there: keep it finite
    # positions that put a boundary at the middle of the buffer join the coarse grid
    info["boundaries"] = [int(b) for b in boundaries] if boundaries is not None else _find_boundaries(arena, log)
    for b in info["boundaries"]:
        o = (b - buf_bytes // 2) // 256 * 256
        if 0 <= o <= arena_bytes - pitch and o not in candidates:
            candidates.append(o)
    candidates.sort()
    out = torch.empty(P, dtype=torch.float32, device=dev)
    step = [0]
    chosen: List[int] = []

    def overlaps(o: int) -> bool:
        return any(o < c + pitch and c < o + pitch for c in chosen)

    for k in range(nbuf):
        best, best_ms, table = None, float("inf"), []
        for o in candidates:
            if overlaps(o):
                continue
            bufs = [view(c) for c in chosen] + [view(o)]

            def probe():
                _b.wash_shuffle_states(bufs, segs, 0, step[0])
                step[0] += 1
                _b.papa_ema(bufs[0], 0.5)
                _b.wash_average(bufs[0], out)

            ms = _timed(probe, reps)
            table.append((o, ms))
            if ms < best_ms:
                best, best_ms = o, ms
        if best is None:
            raise MemoryError("no room left in the arena")
        chosen.append(best)
        info["probes_ms"].append(table)
        if log is not None:
            worst = max(ms for _, ms in table)
            log(f"buffer {k}: offset {best / GiB:.0f} GiB of the arena, step {best_ms:.2f} ms "
                f"(candidates {min(ms for _, ms in table):.2f} .. {worst:.2f} ms)")
    info["offsets"] = chosen
    info["tuned"] = True
    del out
    return [view(o) for o in chosen], info
