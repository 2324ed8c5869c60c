#!/usr/bin/env python3
"""Benchmark of the WASH population-update hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C] [--headline-only]

A "step" is one pass of the whole hot path over the population of the chosen
workload: one wash_shuffle (thresholds, mask, permutation, gather-permute-
scatter, plus momentum where the workload has it), one papa_ema and one
wash_average.  The default workload is the largest configuration, N = 8 models
of 1.1e9 parameters with momentum (70.4 GB resident in HBM).  Inputs are
resident in HBM before the timed region; timing uses HIP events on the stream
the kernels are launched on.

The LAST line of stdout is one short JSON object: value = coordinates decided
by wash_shuffle per second, ms_per_step = the whole pass, `roofline` for the
kernel with the longest duration plus one entry per kernel, and the CPU oracle
timed on a bounded sample of the same workload.  Everything else (per-kernel
medians, yardsticks, every other configuration with both mask streams, the
oracle timed on each configuration) goes to a side file (--detail PATH, an
empty PATH for none), and as progress lines to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def _median(xs):
    s = sorted(xs)
    return s[len(s) // 2]


def _expected_fraction(segs, P):
    return sum(length * p for _, length, p in segs) / P


def _expected_store_units(segs, N, bufs):
    """Expected number of distinct 64-byte half lines one shuffle launch writes: a half line holds 16
    coordinates of a row and is written if one of them is selected; of the N rows of a selected
    coordinate N - 1 change on average (a uniform permutation has one fixed point on average).
    Scattered stores cost the same per half line whatever their width (measured), so this count over
    the measured scattered-store rate is the time the memory system needs for the writes alone."""
    return sum(length / 16.0 * (1.0 - (1.0 - p) ** 16) for _, length, p in segs) * (N - 1) * bufs


class Timer:
    """HIP events on the current stream; elapsed() in ms after a synchronize."""

    def __init__(self, torch):
        self.torch = torch
        self.pairs = {}

    def record(self, key, fn):
        a = self.torch.cuda.Event(enable_timing=True)
        b = self.torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        self.pairs.setdefault(key, []).append((a, b))

    def ms(self, key):
        return [a.elapsed_time(b) for a, b in self.pairs.get(key, [])]


def kernel_rooflines(N, P, bufs, frac_selected, t_ms):
    """Algorithmic bytes per launch and achieved GB/s per kernel.
    shuffle: 2 * p * N * P * 4 B per buffer; average: (N + 1) * P * 4 B; EMA: 2 * N * P * 4 B."""
    alg = {
        "wash_shuffle": 2.0 * frac_selected * N * P * 4.0 * bufs,
        "wash_average": (N + 1.0) * P * 4.0,
        "papa_ema": 2.0 * N * P * 4.0,
    }
    out = {}
    for k, b in alg.items():
        if k in t_ms and t_ms[k] > 0:
            gbs = b / (t_ms[k] * 1e-3) / 1e9
            out[k] = {"bound": "hbm", "alg_bytes": b, "avg_us": t_ms[k] * 1e3, "achieved": gbs,
                      "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}
    return out


_PLACEMENT = {}      # per run of this script: arena size, and the buffer offsets found for each config


def run_config(torch, wash, cfg, steps, warmup, p_override=None, count=True, stream="v1", states=None, placement="tuned"):
    """Time the hot path on one workload. Returns a dict of measurements.
    placement: "tuned" = the buffers sit where wash.place_population found one step fastest (populations from
    512 MiB per buffer on); "default" = wherever torch's allocator puts them."""
    from workloads import device_population

    dev = "cuda:0"
    tensors = cfg.tensors()
    N, P = cfg.N, cfg.P
    segs_list = cfg.segments(p_override)
    segs = wash.SegmentList(segs_list)
    place_info, placed = None, None
    if placement == "tuned" and states is None and N * P * 4 >= (1 << 29):
        # one arena of a fixed size per run of this script, so that positions found once can be used again
        arena_bytes = _PLACEMENT.setdefault("arena_bytes", None)
        try:
            placed, place_info = wash.place_population(
                N, P, 2 if cfg.momentum else 1, segs, dev, arena_bytes=arena_bytes, offsets=_PLACEMENT.get(cfg.index),
                boundaries=_PLACEMENT.get("boundaries"),
                log=lambda m: print(f"[bench] placement, config {cfg.index}: {m}", file=sys.stderr, flush=True))
            _PLACEMENT["arena_bytes"] = place_info["arena_bytes"]
            _PLACEMENT[cfg.index] = place_info["offsets"]
            if "boundaries" in place_info:
                _PLACEMENT["boundaries"] = place_info["boundaries"]
        except (MemoryError, RuntimeError, ValueError) as exc:
            print(f"[bench] placement skipped ({exc}); buffers from the default allocator", file=sys.stderr, flush=True)
            placed, place_info = None, None
            torch.cuda.empty_cache()
    if placed is not None:
        pop, mom = device_population(tensors, N, cfg.init, cfg.data_seed, cfg.momentum, dev,
                                     out=(placed[0], placed[1] if cfg.momentum else None))
    else:
        pop, mom = device_population(tensors, N, cfg.init, cfg.data_seed, cfg.momentum, dev)
    bufs = 2 if cfg.momentum else 1
    state_bufs = None
    if states is not None:
        # WASH+Opt with `states` buffers in all (parameters + optimizer states), through wash_shuffle_states
        gen = torch.Generator(device=dev).manual_seed(cfg.data_seed + 77)
        state_bufs = [pop] + ([mom] if mom is not None else [])
        while len(state_bufs) < states:
            state_bufs.append(torch.randn(N, P, device=dev, generator=gen) * 1e-3)
        state_bufs = state_bufs[:states]
        bufs = states
    big = N * P * 4 > 8 * (1 << 30)
    # the EMA works on the population itself when that is huge or was placed (so that the placed buffer is
    # what is timed), else on a copy of its own
    ema_buf = pop if (big or placed is not None) else pop.clone()
    out = torch.empty(P, dtype=torch.float32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int64, device=dev)
    torch.cuda.synchronize()

    step_no = [0]

    shuffle_fn = wash.wash_shuffle if stream == "v1" else wash.wash_shuffle_gap

    def do_shuffle():
        if state_bufs is not None:
            wash.wash_shuffle_states(state_bufs, segs, cfg.seed, step_no[0], gap_stream=(stream == "gap"),
                                     selected_count=cnt if count else None)
        else:
            shuffle_fn(pop, mom, segs, cfg.seed, step_no[0], cnt if count else None)
        step_no[0] += 1

    def do_ema():
        wash.papa_ema(ema_buf, cfg.alpha)

    def do_avg():
        wash.wash_average(pop, out)

    for _ in range(warmup):
        do_shuffle()
        do_ema()
        do_avg()
    torch.cuda.synchronize()
    cnt.zero_()
    torch.cuda.synchronize()

    tm = Timer(torch)
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    t0.record()
    for _ in range(steps):
        tm.record("wash_shuffle", do_shuffle)
        tm.record("papa_ema", do_ema)
        tm.record("wash_average", do_avg)
    t1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    total_ms = t0.elapsed_time(t1)

    # the two analysis passes, timed on their own after the timed region (not part of a step)
    reps = 5
    weights = [1.0 / N] * N
    extra = {}
    for name, fn in (("wash_consensus_sqdist", lambda: wash.wash_consensus_sqdist(pop)),
                     ("wash_weighted_average", lambda: wash.wash_weighted_average(pop, weights, out))):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        nbytes = N * P * 4.0 if name == "wash_consensus_sqdist" else (N + 1.0) * P * 4.0
        extra[name] = {"avg_us": ms * 1e3, "alg_bytes": nbytes, "achieved": nbytes / (ms * 1e-3) / 1e9,
                       "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    selected = int(cnt.item()) / steps        # read before the extra passes below add to the counter

    # populations that fit the 256 MB Infinity Cache: the same three kernels once more, each after a
    # 1 GiB fill that evicts the caches (the fill is outside the per-kernel events)
    cold = None
    if N * P * 4 * bufs <= 256 * (1 << 20):
        evict = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        tc = Timer(torch)
        for _ in range(10):
            for key, fn in (("wash_shuffle", do_shuffle), ("papa_ema", do_ema), ("wash_average", do_avg)):
                evict.fill_(1.0)
                tc.record(key, fn)
        torch.cuda.synchronize()
        cold = {k: sum(tc.ms(k)) / len(tc.ms(k)) * 1e3 for k in ("wash_shuffle", "papa_ema", "wash_average")}
        del evict

    # the same step captured once in a HIP graph and replayed; the shuffle reads its step number from
    # device memory and advances it, so every replay is a new iteration (fresh mask and permutations)
    graph_ms, graph_bufs = None, None
    try:
        step_dev = torch.full((1,), step_no[0], dtype=torch.int64, device=dev)
        graph_bufs = state_bufs if state_bufs is not None else ([pop, mom] if mom is not None else [pop])
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            wash.wash_shuffle_device_step(graph_bufs, segs, cfg.seed, step_dev, advance=True,
                                          gap_stream=(stream == "gap"), selected_count=cnt if count else None)
            do_ema()
            do_avg()
        g.replay()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps_g = max(5, min(steps, 50))
        a.record()
        for _ in range(reps_g):
            g.replay()
        b.record()
        torch.cuda.synchronize()
        graph_ms = a.elapsed_time(b) / reps_g
        del g
    except Exception as exc:  # noqa: BLE001  (a failed capture must not cost the measurement)
        print(f"[bench] graph capture skipped: {exc}", file=sys.stderr)

    avg_ms = {k: sum(tm.ms(k)) / steps for k in ("wash_shuffle", "papa_ema", "wash_average")}
    med_ms = {k: _median(tm.ms(k)) for k in avg_ms}
    frac_sel = _expected_fraction(segs_list, P)
    res = {
        "config": cfg.index, "name": cfg.name, "stream": stream, "N": N, "P": P, "segments": len(segs_list),
        "momentum": bool(cfg.momentum), "buffers_shuffled": bufs, "expected_fraction": frac_sel,
        "selected_per_step": selected, "steps": steps,
        "ms_per_step": total_ms / steps, "wall_ms_per_step": wall * 1e3 / steps,
        "graph_replay_ms_per_step": graph_ms,
        "avg_us": {k: v * 1e3 for k, v in avg_ms.items()},
        "median_us": {k: v * 1e3 for k, v in med_ms.items()},
        "min_us": {k: min(tm.ms(k)) * 1e3 for k in avg_ms},
        "cold_cache_us": cold,
        "first_steps_us": {k: [round(x * 1e3, 1) for x in tm.ms(k)[:12]] for k in avg_ms},
        "shuffle_coords_per_s": P / (avg_ms["wash_shuffle"] * 1e-3),
        "shuffle_elements_per_s": selected * N * bufs / (avg_ms["wash_shuffle"] * 1e-3),
        "shuffle_store_units_per_s": _expected_store_units(segs_list, N, bufs) / (avg_ms["wash_shuffle"] * 1e-3),
        "pass_coords_per_s": P / (total_ms / steps * 1e-3),
        "population_bytes": N * P * 4 * bufs,
        "cache_resident": N * P * 4 * bufs <= 256 * (1 << 20),
        "roofline": kernel_rooflines(N, P, bufs, frac_sel, avg_ms),
        "analysis_passes": extra,
        "placement": ({"tuned": place_info["tuned"], "arena_GiB": place_info["arena_bytes"] / 2**30,
                       "offsets_GiB": [o / 2**30 for o in place_info["offsets"]],
                       "boundaries_GiB": [b / 2**30 for b in place_info.get("boundaries", [])],
                       "probes_ms": [[(o / 2**30, round(ms, 3)) for o, ms in t] for t in place_info["probes_ms"]]}
                      if place_info is not None else {"tuned": False}),
    }
    place_info = placed = state_bufs = graph_bufs = None
    del pop, mom, ema_buf, out
    torch.cuda.empty_cache()
    return res


def padded_rows(torch, wash, cfg, reps=10):
    """papa_ema and wash_average on the same population with every row padded to a multiple of 32 elements (128 bytes):
    what the unaligned row pitch of this configuration costs the streaming kernels."""
    N, P = cfg.N, (cfg.P + 31) // 32 * 32
    pop = torch.empty(N, P, dtype=torch.float32, device="cuda:0").normal_(0.0, 0.02)
    out = torch.empty(P, dtype=torch.float32, device="cuda:0")
    res = {"N": N, "P_padded": P}
    for name, fn, nbytes in (("papa_ema", lambda: wash.papa_ema(pop, cfg.alpha), 2.0 * N * P * 4),
                             ("wash_average", lambda: wash.wash_average(pop, out), (N + 1.0) * P * 4)):
        for _ in range(2):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        res[name] = {"avg_us": ms * 1e3, "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    del pop, out
    torch.cuda.empty_cache()
    return res


def copy_yardstick(torch, wash, n_floats=1 << 28, reps=10):
    src = torch.empty(n_floats, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        wash.wash_copy_f32(src, dst)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        wash.wash_copy_f32(src, dst)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / reps
    gbs = 2.0 * n_floats * 4 / (ms * 1e-3) / 1e9
    return {"bytes": 2 * n_floats * 4, "avg_us": ms * 1e3, "GBps": gbs, "frac_of_peak": gbs / HBM_PEAK_GBS}


def scatter_yardstick(torch, wash, lines=1 << 25, blocks=8192, rounds=16):
    """G places/s of independent scattered 4-byte loads, stores and load->store pairs, and of stores of whole
    64-byte pieces, on a 4 GiB buffer: what the memory system gives a sparse shuffle that does nothing but
    touch its values."""
    buf = torch.zeros(lines * 32, dtype=torch.float32, device="cuda:0")
    out = {}
    for mode, name in ((0, "loads"), (1, "stores"), (2, "load_then_store"), (3, "stores_of_64_byte_pieces")):
        wash.wash_probe_scattered(buf, mode, rounds, blocks)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        n = 0
        for _ in range(3):
            n += wash.wash_probe_scattered(buf, mode, rounds, blocks)
        b.record()
        torch.cuda.synchronize()
        out[name + "_Gelem_per_s"] = n / (a.elapsed_time(b) * 1e-3) / 1e9
    out["buffer_bytes"] = lines * 128
    return out


def _r(x, digits=4):
    """Round to `digits` significant digits (keeps the headline line short)."""
    if x is None or x == 0:
        return x
    return float(f"{x:.{digits}g}")


def bound_label(N, bufs, frac_selected, stream, dense):
    """Which resource binds the shuffle kernel in this regime (measured: VALU activity, counters)."""
    if dense:
        return "hbm"                      # rows streamed through LDS: a plain in-place pass over the bytes
    if frac_selected * N * bufs < 0.05:
        # the Philox mask scan (one quarter call per coordinate) outweighs the scattered accesses
        return "valu" if stream == "v1" else "latency"
    return "hbm"


def cpu_baseline_full(cfg, budget_s=3.0, mt_budget_s=0.5):
    """The oracle as it stands on whole passes (shuffle + EMA + average) of a configuration that fits
    the host: single thread, until about budget_s seconds are spent; then the shuffle alone over all cores."""
    import oracle
    from workloads import host_population

    pop, mom = host_population(cfg.tensors(), cfg.N, cfg.init, cfg.data_seed, cfg.momentum)
    segs = cfg.segments()
    ema_buf = pop.copy()
    passes, t_spent = 0, 0.0
    parts = {"wash_shuffle": 0.0, "papa_ema": 0.0, "wash_average": 0.0}
    while passes < 1 or (t_spent < budget_s and passes < 50):
        t0 = time.perf_counter()
        oracle.shuffle(pop, mom, segs, cfg.seed, passes, threads=1)
        t1 = time.perf_counter()
        oracle.ema(ema_buf, cfg.alpha)
        t2 = time.perf_counter()
        oracle.average(pop)
        t3 = time.perf_counter()
        parts["wash_shuffle"] += t1 - t0
        parts["papa_ema"] += t2 - t1
        parts["wash_average"] += t3 - t2
        t_spent += t3 - t0
        passes += 1
    threads = max(1, min(16, os.cpu_count() or 1))
    mt_calls, mt_spent = 0, 0.0
    while mt_calls < 2 or (mt_spent < mt_budget_s and mt_calls < 50):
        t0 = time.perf_counter()
        oracle.shuffle(pop, mom, segs, cfg.seed, 1000 + mt_calls, threads=threads)
        mt_spent += time.perf_counter() - t0
        mt_calls += 1
    return {
        "value": _r(cfg.P * passes / parts["wash_shuffle"], 5), "unit": "coords/s", "cores": 1, "kind": "oracle",
        "sample": f"{passes} whole passes over the full config-{cfg.index} population, {t_spent:.1f} s of CPU time",
        "us_per_call": {k: round(v / passes * 1e6, 1) for k, v in parts.items()},
        "all_cores": {"threads": threads, "us_per_call": round(mt_spent / mt_calls * 1e6, 1),
                              "coords_per_s": _r(cfg.P * mt_calls / mt_spent, 5)},
        "host_cores_available": os.cpu_count(),
    }


def cpu_baseline_sampled(cfg, steps=3, nsample=3):
    """The oracle on a bounded sample of a population that does not fit the host: whole tensor segments
    (all N rows, parameters and momentum) at their true coordinates and probabilities, shuffled with the
    oracle's window call, then EMA and average on the same columns; the per-coordinate cost is scaled to
    the whole row.  Single thread, then the shuffle over all cores."""
    import numpy as np
    import oracle

    segs = cfg.segments()
    # three segments spread over the list (first, middle, last of those long enough to time)
    long_enough = [s for s, (_, length, _) in enumerate(segs) if length >= 100_000]
    sample_segments = sorted({long_enough[(len(long_enough) - 1) * k // (nsample - 1)] for k in range(nsample)})
    rng = np.random.default_rng(cfg.data_seed)
    threads = max(1, min(16, os.cpu_count() or 1))
    parts = {"wash_shuffle": 0.0, "papa_ema": 0.0, "wash_average": 0.0}
    coords, mt_spent, mt_coords = 0, 0.0, 0
    for s in sample_segments:
        off, length, p = segs[s]
        win = (rng.standard_normal((cfg.N, length), dtype=np.float32) * np.float32(0.02))
        mom = (rng.standard_normal((cfg.N, length), dtype=np.float32) * np.float32(1e-3)) if cfg.momentum else None
        for step in range(steps):
            t0 = time.perf_counter()
            oracle.shuffle_window(win, mom, cfg.P, off, segs, cfg.seed, step)
            t1 = time.perf_counter()
            oracle.ema(win, cfg.alpha)
            t2 = time.perf_counter()
            oracle.average(win)
            t3 = time.perf_counter()
            parts["wash_shuffle"] += t1 - t0
            parts["papa_ema"] += t2 - t1
            parts["wash_average"] += t3 - t2
            coords += length
        # all cores: the same columns as a population of their own (same p, same amount of work)
        for step in range(steps):
            t0 = time.perf_counter()
            oracle.shuffle(win, mom, [(0, length, p)], cfg.seed, step, threads=threads)
            mt_spent += time.perf_counter() - t0
            mt_coords += length
    scale = cfg.P / coords                # per-coordinate cost of the sample, times the coordinates of a whole row
    total = sum(parts.values())
    return {
        "value": _r(coords / parts["wash_shuffle"], 5), "unit": "coords/s", "cores": 1, "kind": "oracle",
        "sample": f"{len(sample_segments)} of {len(segs)} segments ({coords // steps} coordinates x {cfg.N} rows, "
                  f"params{'+momentum' if cfg.momentum else ''}) x {steps} steps, {total:.1f} s CPU",
        "extrapolated_ms_per_call": {k: round(v * scale * 1e3) for k, v in parts.items()},
        "all_cores": {"threads": threads, "coords_per_s": _r(mt_coords / mt_spent, 4)},
    }


def cpu_baseline(cfg, sample_steps=3, nsample=3):
    host_bytes = cfg.N * cfg.P * 4 * (3 if cfg.momentum else 2)
    if host_bytes > 4 * (1 << 30):
        return cpu_baseline_sampled(cfg, steps=sample_steps, nsample=nsample)
    return cpu_baseline_full(cfg)


def load_traffic(workload_key, kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE in separate
    runs of this script (summaries committed under profiles/); None if that workload was not profiled."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == workload_key and parts[1] == kernel:
                    return float(parts[2])
    except (OSError, ValueError):
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5,
                    help="1..5 (default 5: N=8 models x 1.1e9 parameters with momentum, the largest single-GPU workload)")
    ap.add_argument("--p", type=float, default=None, help="override the shuffle probability of every tensor")
    ap.add_argument("--headline-only", "--skip-all-configs", dest="headline_only", action="store_true",
                    help="time only the headline workload; by default the other configs (both shuffle streams, the "
                         "oracle beside each) are timed too, with at most 20 steps each, into the detail file")
    ap.add_argument("--detail", default=os.path.join(ROOT, "gpurun_out", "bench_detail.json"),
                    help="side file for everything that does not fit the headline line ('' = none)")
    ap.add_argument("--stream", choices=["v1", "gap"], default="v1",
                    help="mask stream of the shuffle: v1 = wash_shuffle, gap = wash_shuffle_gap")
    ap.add_argument("--states", type=int, default=None, choices=[1, 2, 3, 4],
                    help="shuffle this many buffers (parameters + optimizer states) through wash_shuffle_states")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-count", action="store_true", help="do not ask wash_shuffle for the selected count")
    ap.add_argument("--stream-min-bytes", type=int, default=None,
                    help="override the population size from which average/EMA use non-temporal accesses")
    ap.add_argument("--gap-blocks", type=int, default=None, help="override blocks per wavefront of the gap kernel")
    ap.add_argument("--average-chunks", type=int, default=None, help="chunks per block of wash_average (1, 2, 4, 8)")
    ap.add_argument("--tile-coords", type=int, default=None, help="override the shuffle tile size")
    ap.add_argument("--shuffle-blocks-per-cu", type=int, default=None,
                    help="cap on resident blocks per compute unit of the gathering shuffle kernel (0 = none)")
    ap.add_argument("--dense", type=int, default=None, choices=[0, 1, 2],
                    help="wash_shuffle's dense path: 0 automatic, 1 never, 2 whenever it fits")
    ap.add_argument("--placement", choices=["tuned", "default"], default="tuned",
                    help="tuned: buffers of 512 MiB and more are placed by wash.place_population (one arena, the "
                         "position where a step runs fastest); default: torch's allocator")
    ap.add_argument("--placement-from", default=None,
                    help="detail file of an earlier run of this script: use the arena size and buffer offsets it found "
                         "instead of probing again (for runs under a profiler, where probe launches would mix into "
                         "the per-kernel statistics)")
    ap.add_argument("--only", choices=["pass", "copy"], default="pass",
                    help="copy: run only the copy yardstick (for counter calibration)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path shards along P without any exchange; "
              "no multi-GPU figure is produced). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2405_17517_amd as wash
    from workloads import CONFIGS, get_config

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)

    if args.stream_min_bytes is not None:
        wash.wash_set_option(wash.OPT_STREAM_MIN_BYTES, args.stream_min_bytes)
    if args.gap_blocks is not None:
        wash.wash_set_option(wash.OPT_GAP_BLOCKS, args.gap_blocks)
    if args.average_chunks is not None:
        wash.wash_set_option(wash.OPT_AVERAGE_CHUNKS, args.average_chunks)
    if args.tile_coords is not None:
        wash.wash_set_option(wash.OPT_TILE_COORDS, args.tile_coords)
    if args.dense is not None:
        wash.wash_set_option(wash.OPT_DENSE, args.dense)
    if args.shuffle_blocks_per_cu is not None:
        wash.wash_set_option(wash.OPT_SHUFFLE_BLOCKS_PER_CU, args.shuffle_blocks_per_cu)

    if args.only == "copy":
        print(json.dumps({"copy_yardstick": copy_yardstick(torch, wash)}))
        return

    def note(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    if args.placement_from:
        with open(args.placement_from) as f:
            earlier = json.load(f).get("placement_found", {})
        _PLACEMENT.update({(int(k) if k.isdigit() else k): v for k, v in earlier.items()})
    cfg = get_config(args.config)
    note(f"headline workload: config {cfg.index} ({cfg.name}), N={cfg.N}, P={cfg.P}")
    main_res = run_config(torch, wash, cfg, args.steps, args.warmup, p_override=args.p, count=not args.no_count,
                          stream=args.stream, states=args.states, placement=args.placement)
    note(f"config {cfg.index}: shuffle {main_res['avg_us']['wash_shuffle']:.1f} us, ema "
         f"{main_res['avg_us']['papa_ema']:.1f} us, average {main_res['avg_us']['wash_average']:.1f} us")
    # the same workload with the buffers wherever torch's allocator puts them, reported beside the placed run
    # (not under --placement-from: a traced run must hold the launches of one placement only)
    plain_res = None
    if main_res["placement"]["tuned"] and not args.placement_from:
        try:
            plain_res = run_config(torch, wash, cfg, args.steps, args.warmup, p_override=args.p, count=not args.no_count,
                                   stream=args.stream, states=args.states, placement="default")
            note(f"config {cfg.index}, allocator's placement: shuffle {plain_res['avg_us']['wash_shuffle']:.1f} us, ema "
                 f"{plain_res['avg_us']['papa_ema']:.1f} us, average {plain_res['avg_us']['wash_average']:.1f} us")
        except (MemoryError, RuntimeError) as exc:                  # the headline does not depend on this run
            note(f"run at the allocator's placement skipped: {exc}")
            plain_res = None
            torch.cuda.empty_cache()
    yard = copy_yardstick(torch, wash)
    scat = scatter_yardstick(torch, wash)

    roof = main_res["roofline"]
    workload_key = f"config{cfg.index}" + (f"_p{args.p:g}" if args.p is not None else "")
    dense = args.p is not None and args.p >= 0.08 and args.stream == "v1"
    shuffle_bound = bound_label(cfg.N, main_res["buffers_shuffled"], main_res["expected_fraction"], args.stream, dense)
    per_kernel = {}
    for k, v in roof.items():
        traffic = load_traffic(workload_key, k)
        e = {"us": _r(v["avg_us"]), "GBps": _r(v["achieved"]), "frac": _r(v["frac"], 3),
             "bound": shuffle_bound if k == "wash_shuffle" else "hbm", "traffic": traffic}
        if traffic:
            # counted HBM bytes over the kernel time: what the memory system actually moved
            e["traffic_frac"] = _r(traffic / (v["avg_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 3)
        per_kernel[k] = e
    dominant = max(roof, key=lambda k: roof[k]["avg_us"])
    r = roof[dominant]
    roofline = {"kernel": dominant, "bound": per_kernel[dominant]["bound"], "achieved": _r(r["achieved"]),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": _r(r["frac"], 3),
                "traffic": per_kernel[dominant]["traffic"], "traffic_frac": per_kernel[dominant].get("traffic_frac"),
                "alg_bytes_per_launch": _r(r["alg_bytes"], 5), "avg_us": _r(r["avg_us"])}

    roofline["traffic"] = per_kernel[dominant]["traffic"]
    for e in per_kernel.values():
        e.pop("traffic")
    cpu = None
    if not args.no_cpu_baseline:
        note("timing the CPU oracle on the headline workload")
        cpu = cpu_baseline(cfg, sample_steps=10, nsample=9)
        note(f"oracle: {cpu['value']:.3g} coords/s on one core")

    p_text = f"p={args.p:g}" if args.p is not None else (
        "p linear 0.05->0.001 over 200 segments" if cfg.index == 5 else f"p={cfg.probs(1)[0]:g}")
    line = {
        "metric": "shuffle coords/s + effective HBM GB/s (% of roofline) at N models x P params",
        "value": _r(main_res["shuffle_coords_per_s"], 5), "unit": "coords/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": _r(main_res["ms_per_step"], 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.index}: {cfg.name}, N={cfg.N}, P={cfg.P}, {p_text}, "
                               f"{'params+momentum' if cfg.momentum else 'params only'}, "
                               f"{main_res['population_bytes'] / 1e9:.1f} GB in HBM"
                               f"{' (buffers placed by place_population)' if main_res['placement']['tuned'] else ''}; "
                               "step = wash_shuffle + papa_ema + wash_average; value = P / wash_shuffle time"},
        "pass_coords_per_s": _r(main_res["pass_coords_per_s"], 5),
        "selected_per_step": main_res["selected_per_step"],
        "roofline": roofline,
        "roofline_per_kernel": per_kernel,
        "cpu_baseline": cpu,
    }
    if plain_res is not None:
        line["allocator_placement_us"] = {k: _r(v) for k, v in plain_res["avg_us"].items()}

    detail = {"headline": line, "headline_detail": main_res, "headline_allocator_placement": plain_res, "copy_yardstick": yard, "scatter_yardstick": scat,
              "shuffle_vs_scattered_stores": {
                  "bound": "scattered-store", "achieved": main_res["shuffle_store_units_per_s"] / 1e9,
                  "peak": scat["stores_Gelem_per_s"], "unit": "G half-lines/s",
                  "frac": main_res["shuffle_store_units_per_s"] / (scat["stores_Gelem_per_s"] * 1e9)}}

    default_run = (args.p is None and args.stream == "v1" and args.states is None)
    if not args.headline_only and default_run:
        # everything below goes to the detail file only: a failure there must not cost the headline line
        try:
            all_configs_detail(torch, wash, args, cfg, main_res, scat, cpu, detail, note)
        except Exception as exc:                                    # noqa: BLE001
            note(f"detail run stopped: {type(exc).__name__}: {exc}")
            detail["detail_error"] = f"{type(exc).__name__}: {exc}"

    detail["placement_found"] = {str(k): v for k, v in _PLACEMENT.items()}
    if args.detail:
        try:
            if os.path.dirname(args.detail):
                os.makedirs(os.path.dirname(args.detail), exist_ok=True)
            with open(args.detail, "w") as f:
                json.dump(detail, f, indent=1)
            line["detail_file"] = os.path.relpath(args.detail, ROOT)
        except (OSError, TypeError, ValueError) as exc:
            note(f"detail file not written: {exc}")

    sys.stderr.flush()
    print(json.dumps(line, separators=(",", ":")), flush=True)


def all_configs_detail(torch, wash, args, cfg, main_res, scat, cpu, detail, note):
    """Every other configuration with both mask streams, the streaming kernels on padded rows, and the oracle
    timed per configuration: results go into `detail`."""
    from workloads import CONFIGS
    rows = []
    for c in CONFIGS:
        ps = c.p_sweep if c.p_sweep else (None,)
        for p in ps:
            k = max(5, min(c.steps, 20))
            for st in ("v1", "gap"):
                if c.index == cfg.index and st == args.stream:
                    res = dict(main_res)
                else:
                    res = run_config(torch, wash, c, k, min(args.warmup, 3), p_override=p, stream=st,
                                     placement=args.placement)
                res["p_override"] = p
                is_dense = st == "v1" and (p if p is not None else 0.0) >= 0.08
                res["roofline"]["wash_shuffle"]["bound"] = bound_label(c.N, res["buffers_shuffled"],
                                                                       res["expected_fraction"], st, is_dense)
                res["shuffle_vs_scattered_stores_frac"] = (res["shuffle_store_units_per_s"]
                                                           / (scat["stores_Gelem_per_s"] * 1e9))
                rows.append(res)
                note(f"config {c.index} p={p} stream {st}: shuffle {res['avg_us']['wash_shuffle']:.1f} us "
                     f"({res['roofline']['wash_shuffle']['frac'] * 100:.2f} % of 2pNP4/t, "
                     f"{res['roofline']['wash_shuffle']['bound']}-bound), ema {res['avg_us']['papa_ema']:.1f} us "
                     f"({res['roofline']['papa_ema']['frac'] * 100:.1f} %), average "
                     f"{res['avg_us']['wash_average']:.1f} us ({res['roofline']['wash_average']['frac'] * 100:.1f} %)")
    detail["all_configs"] = rows
    detail["rows_padded_to_128_bytes"] = {}
    for c in CONFIGS:
        if c.P % 32 != 0 and c.N * c.P * 4 >= (256 << 20):
            r = padded_rows(torch, wash, c)
            detail["rows_padded_to_128_bytes"][f"config{c.index}"] = r
            note(f"config {c.index} with rows padded to 128 bytes: ema {r['papa_ema']['avg_us']:.1f} us "
                 f"({r['papa_ema']['frac'] * 100:.1f} %), average {r['wash_average']['avg_us']:.1f} us "
                 f"({r['wash_average']['frac'] * 100:.1f} %)")
    if not args.no_cpu_baseline:
        per_cfg = {}
        for c in CONFIGS:
            per_cfg[f"config{c.index}"] = cpu if c.index == cfg.index else cpu_baseline(c)
            b = per_cfg[f"config{c.index}"]
            note(f"oracle, config {c.index}: {b['value']:.3g} coords/s (1 core), "
                 f"{b['all_cores']['coords_per_s']:.3g} coords/s ({b['all_cores']['threads']} threads)")
        detail["cpu_baseline_per_config"] = per_cfg


if __name__ == "__main__":
    main()
