"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Shuffle: bit-exact.  Average / EMA: 1e-6 relative (the
kernels accumulate in fp64 like the definition, so they are normally identical)."""
import numpy as np
import pytest

import oracle
from workloads import distinct_population

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def wash():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2405_17517_amd as w
    yield w
    w.wash_set_option(w.OPT_TILE_COORDS, 0)


def _bits(a):
    return a.view(np.uint32)


def _ragged_segments(P, ps):
    """Cut [0, P) into len(ps) pieces at odd places, leaving a gap before the last piece."""
    k = len(ps)
    edges = sorted({0, P} | {max(1, min(P - 1, (P * i) // k + (3 * i) % 7 - 3)) for i in range(1, k)})
    segs = []
    for i in range(len(edges) - 1):
        a, b = edges[i], edges[i + 1]
        if i == len(edges) - 2 and b - a > 4:
            a += 3                                   # uncovered gap
        segs.append((a, b - a, ps[i % k]))
    return segs


STREAMS = ["v1", "gap"]


def _fn(wash, stream):
    return wash.wash_shuffle if stream == "v1" else wash.wash_shuffle_gap


def _run_shuffle(wash, pop, mom, segs, seed, step, tile=0, stream="v1"):
    wash.wash_set_option(wash.OPT_TILE_COORDS, tile)
    d = torch.from_numpy(pop).cuda()
    dm = torch.from_numpy(mom).cuda() if mom is not None else None
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    _fn(wash, stream)(d, dm, segs, seed, step, cnt)
    torch.cuda.synchronize()
    return d.cpu().numpy(), (dm.cpu().numpy() if dm is not None else None), int(cnt.item())


SHAPES = [(1, 1), (1, 77), (2, 3), (2, 255), (3, 256), (4, 257), (5, 4097), (8, 12289), (10, 70001),
          (20, 33333), (31, 5000), (32, 20011)]


@pytest.mark.parametrize("stream", STREAMS)
@pytest.mark.parametrize("N,P", SHAPES)
@pytest.mark.parametrize("p", [0.0, 0.001, 0.05, 0.5, 1.0])
def test_shuffle_one_segment(wash, N, P, p, stream):
    print(f"case N={N} P={P} p={p} stream={stream}", flush=True)
    pop = distinct_population(N, P)
    segs = [(0, P, p)]
    ref = pop.copy()
    ref_cnt = oracle.shuffle(ref, None, segs, 17, 4, stream=stream)
    got, _, cnt = _run_shuffle(wash, pop, None, segs, 17, 4, stream=stream)
    assert cnt == ref_cnt
    assert np.array_equal(_bits(got), _bits(ref))


@pytest.mark.parametrize("N,P", [(2, 1000), (5, 40001), (10, 123457), (20, 65539), (32, 9001), (8, 1_500_007)])
@pytest.mark.parametrize("tile,stream", [(0, "v1"), (256, "v1"), (4096, "v1"), (65536, "v1"), (0, "gap")])
def test_shuffle_ragged_segments_momentum(wash, N, P, tile, stream):
    print(f"case N={N} P={P} tile={tile} stream={stream}", flush=True)
    pop = distinct_population(N, P)
    mom = distinct_population(N, P, base=0x40000000)
    segs = _ragged_segments(P, [0.3, 0.0, 1.0, 0.01, 0.3, 0.3, 0.002, 0.9, 0.05])
    ref, refm = pop.copy(), mom.copy()
    ref_cnt = oracle.shuffle(ref, refm, segs, 0xABCDEF0123456789, 4294967295, stream=stream)
    got, gotm, cnt = _run_shuffle(wash, pop, mom, segs, 0xABCDEF0123456789, 4294967295, tile, stream)
    assert cnt == ref_cnt
    assert np.array_equal(_bits(got), _bits(ref))
    assert np.array_equal(_bits(gotm), _bits(refm))


@pytest.mark.parametrize("stream", STREAMS)
def test_shuffle_many_tiny_segments(wash, stream):
    # tensors of 1..70 elements back to back, probabilities cycling, some zero
    N, P = 6, 50000
    rng = np.random.default_rng(0)
    segs, off, k = [], 0, 0
    while off < P - 100:
        ln = int(rng.integers(1, 70))
        segs.append((off, ln, [0.5, 0.0, 1.0, 0.1, 0.5][k % 5]))
        off += ln + (1 if k % 11 == 0 else 0)
        k += 1
    pop = distinct_population(N, P)
    ref = pop.copy()
    ref_cnt = oracle.shuffle(ref, None, segs, 5, 6, stream=stream)
    for tile in (256, 1024, 0):
        got, _, cnt = _run_shuffle(wash, pop, None, segs, 5, 6, tile, stream)
        assert cnt == ref_cnt and np.array_equal(_bits(got), _bits(ref))


@pytest.mark.parametrize("stream", STREAMS)
def test_shuffle_consecutive_steps_and_special_values(wash, stream):
    N, P = 7, 30011
    bits = np.random.default_rng(1).integers(0, 2 ** 32, size=(N, P), dtype=np.uint64).astype(np.uint32)
    bits[:, :3] = np.array([0x7FC00001, 0xFFC12345, 0x80000000], dtype=np.uint32)   # NaN payloads, -0.0
    pop = bits.view(np.float32).copy()
    segs = [(0, P, 0.2)]
    ref = pop.copy()
    d = torch.from_numpy(pop).cuda()
    for step in range(12):
        oracle.shuffle(ref, None, segs, 3, step, stream=stream)
        _fn(wash, stream)(d, None, segs, 3, step)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(d.cpu().numpy()), _bits(ref))


@pytest.mark.parametrize("stream", STREAMS)
def test_empty_and_degenerate_inputs(wash, stream):
    N, P = 32, 5000                                   # the largest population size accepted
    pop = distinct_population(N, P)
    for segs in ([], [(0, 0, 0.5)], [(10, 0, 1.0), (10, 0, 1.0)], [(0, P, 0.0)], [(0, 1, 1.0)], [(P - 1, 1, 1.0)],
                 [(0, 0, 1.0), (0, 3, 1.0), (3, 0, 0.2), (3, 2, 1.0), (4999, 1, 1.0)]):
        ref = pop.copy()
        ref_cnt = oracle.shuffle(ref, None, segs, 3, 1, stream=stream)
        got, _, cnt = _run_shuffle(wash, pop, None, segs, 3, 1, stream=stream)
        assert cnt == ref_cnt and np.array_equal(_bits(got), _bits(ref)), segs
    one = distinct_population(1, 300)                 # a single model: nothing can move
    got, _, cnt = _run_shuffle(wash, one, None, [(0, 300, 1.0)], 3, 1, stream=stream)
    assert cnt == 300 and np.array_equal(_bits(got), _bits(one))


def test_gap_equal_p_neighbours_merge_and_p1_matches_v1(wash):
    N, P = 5, 70_003
    pop = distinct_population(N, P)
    one = _run_shuffle(wash, pop, None, [(0, P, 0.04)], 9, 1, stream="gap")
    cut = _run_shuffle(wash, pop, None, [(0, 777, 0.04), (777, 0, 0.9), (777, 3000, 0.04), (3777, P - 3777, 0.04)],
                       9, 1, stream="gap")
    assert one[2] == cut[2] and np.array_equal(_bits(one[0]), _bits(cut[0]))
    a = _run_shuffle(wash, pop, None, [(0, P, 1.0)], 9, 1, stream="gap")
    b = _run_shuffle(wash, pop, None, [(0, P, 1.0)], 9, 1, stream="v1")
    assert a[2] == b[2] == P and np.array_equal(_bits(a[0]), _bits(b[0]))


def test_gap_probabilities_below_double_resolution(wash):
    """Segments whose p is so small that 1 - p rounds to 1 select nothing (Bernoulli(p) of Eq. 3), alone
    and between ordinary segments, whose streams they leave alone."""
    N, P = 6, 40_000
    pop = distinct_population(N, P)
    for segs in ([(0, P, 1e-17)], [(0, P, 5e-324)], [(0, 100, 2.0 ** -54), (100, P - 100, 1e-300)],
                 [(0, 3000, 0.05), (3000, 2000, 1e-300), (5000, 30_000, 0.05), (35_000, 5000, 2.0 ** -53)]):
        ref = pop.copy()
        ref_cnt = oracle.shuffle(ref, None, segs, 13, 2, stream="gap")
        got, _, cnt = _run_shuffle(wash, pop, None, segs, 13, 2, stream="gap")
        assert cnt == ref_cnt and np.array_equal(_bits(got), _bits(ref)), segs
        if max(p for _, _, p in segs) < 1e-10:
            assert cnt == 0 and np.array_equal(_bits(got), _bits(pop))


def test_shuffle_is_deterministic_and_tile_independent(wash):
    N, P = 10, 1 << 18
    pop = distinct_population(N, P)
    segs = [(0, P, 0.03)]
    outs = [_run_shuffle(wash, pop, None, segs, 1, 2, tile)[0] for tile in (0, 256, 512, 8192, 0)]
    for o in outs[1:]:
        assert np.array_equal(_bits(o), _bits(outs[0]))


@pytest.mark.parametrize("N", range(1, 33))
def test_average_and_ema_streaming_shapes_every_population_size(wash, N):
    """The launch shapes used beyond the Infinity Cache (occupancy-capped blocks of 64 or 256 threads, all N
    loads in flight), forced on small inputs through the size threshold: every population size (each is its
    own kernel instantiation), rows whose pitch is a multiple of 128 bytes and rows whose pitch is not, a
    ragged last vector; average (Alg. 1 output) and EMA (Eq. 1) bit-identical to the oracle."""
    wash.wash_set_option(wash.OPT_STREAM_MIN_BYTES, 0)
    try:
        for P in (32 * 2049, 70_001 + N, 259):
            print(f"streaming shapes N={N} P={P}", flush=True)
            rng = np.random.default_rng(N * 131 + P)
            pop = (rng.standard_normal((N, P)) * 0.02).astype(np.float32)
            d = torch.from_numpy(pop).cuda()
            assert np.array_equal(wash.wash_average(d).cpu().numpy(), oracle.average(pop)), (N, P)
            wash.papa_ema(d, 0.99)
            ref = pop.copy()
            oracle.ema(ref, 0.99)
            assert np.array_equal(d.cpu().numpy(), ref), (N, P)
    finally:
        wash.wash_set_option(wash.OPT_STREAM_MIN_BYTES, 256 << 20)


@pytest.mark.parametrize("N,P", [(1, 5), (2, 1023), (4, 1 << 20), (5, 1000003), (10, 300001), (20, 70002), (32, 4099)])
def test_average_and_ema(wash, N, P):
    print(f"case N={N} P={P}", flush=True)
    rng = np.random.default_rng(N * 1000 + P % 1000)
    pop = (rng.standard_normal((N, P)) * 0.02).astype(np.float32)
    d = torch.from_numpy(pop).cuda()
    avg = wash.wash_average(d).cpu().numpy()
    ref = oracle.average(pop)
    scale = np.maximum(np.abs(ref), np.abs(pop).mean(axis=0))
    assert np.all(np.abs(avg - ref) <= 1e-6 * scale)
    assert np.array_equal(avg, ref)          # fp64 accumulation in the same order: identical
    for alpha in (0.99, 0.0, 1.0, 0.37):
        d = torch.from_numpy(pop).cuda()
        wash.papa_ema(d, alpha)
        got = d.cpu().numpy()
        e = pop.copy()
        oracle.ema(e, alpha)
        scale = np.maximum(np.abs(e), np.abs(pop).mean(axis=0, keepdims=True))
        assert np.all(np.abs(got - e) <= 1e-6 * scale)
        assert np.array_equal(got, e)


def test_shuffle_keeps_mean_and_multiset_on_device(wash):
    N, P = 5, 2_000_003
    rng = np.random.default_rng(9)
    pop = (rng.standard_normal((N, P)) * 0.02).astype(np.float32)
    d = torch.from_numpy(pop).cuda()
    before = wash.wash_average(d).clone()
    xor0 = torch.sort(d.view(torch.int32), dim=0).values.clone()
    wash.wash_shuffle(d, None, [(0, P, 0.1)], 8, 0)
    assert torch.equal(torch.sort(d.view(torch.int32), dim=0).values, xor0)
    assert not torch.equal(d.cpu(), torch.from_numpy(pop))
    after = wash.wash_average(d)
    # the sum is taken in ascending n, so a permuted column may round differently in fp64;
    # after rounding to fp32 that is below the 1e-6 bar by orders of magnitude
    assert torch.allclose(after, before, rtol=1e-6, atol=1e-9)
    # and against the oracle: the shuffled population bit for bit, its average within the bar
    ref = pop.copy()
    oracle.shuffle(ref, None, [(0, P, 0.1)], 8, 0, threads=8)
    assert np.array_equal(_bits(d.cpu().numpy()), _bits(ref))
    ref_avg = oracle.average(ref)
    scale = np.maximum(np.abs(ref_avg), np.abs(ref).mean(axis=0))
    assert np.all(np.abs(after.cpu().numpy() - ref_avg) <= 1e-6 * scale)


def test_calls_on_two_streams_do_not_share_scratch(wash):
    """The selected count and the partial sums of the consensus distance go through library-owned device
    memory that belongs to the calling stream: shuffles (both mask streams) and distance passes that
    overlap on two streams give the oracle's counts, bits and sums."""
    N = 6
    cases = []
    for k, (P, p, stream) in enumerate([(3_000_001, 0.02, "v1"), (2_500_003, 0.3, "v1"), (3_100_007, 0.01, "gap"),
                                         (2_000_003, 0.05, "gap")]):
        pop = (np.random.default_rng(70 + k).standard_normal((N, P)) * 0.02).astype(np.float32)
        cases.append((pop, [(0, P // 2, p), (P // 2, P - P // 2, p / 2)], stream))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    steps = 12
    for a, b in ((0, 1), (2, 3), (0, 3)):
        devs, cnts, dists = [], [], []
        for idx in (a, b):
            devs.append(torch.from_numpy(cases[idx][0]).cuda())
            cnts.append(torch.zeros(1, dtype=torch.int64, device="cuda"))
            dists.append(torch.zeros(N, dtype=torch.float64, device="cuda"))
        torch.cuda.synchronize()
        print(f"two streams: cases {a} and {b}", flush=True)
        for step in range(steps):
            for slot, idx in enumerate((a, b)):
                with torch.cuda.stream(streams[slot]):
                    _fn(wash, cases[idx][2])(devs[slot], None, cases[idx][1], 5, step, cnts[slot])
                    wash.wash_consensus_sqdist(devs[slot], out=dists[slot])
        torch.cuda.synchronize()
        for slot, idx in enumerate((a, b)):
            ref = cases[idx][0].copy()
            ref_cnt = sum(oracle.shuffle(ref, None, cases[idx][1], 5, step, threads=8, stream=cases[idx][2])
                          for step in range(steps))
            assert int(cnts[slot].item()) == ref_cnt
            assert np.array_equal(_bits(devs[slot].cpu().numpy()), _bits(ref))
            assert np.allclose(dists[slot].cpu().numpy(), oracle.consensus_sqdist(ref), rtol=1e-10, atol=0)


def test_host_threads_on_their_own_streams(wash):
    """Four host threads, each with a stream and a population of its own, call the library at the same time
    (ctypes releases the interpreter lock during a call): the cached tables and the per-stream workspaces are
    shared state of the library, and every thread must still get the oracle's bits, counts and sums."""
    from concurrent.futures import ThreadPoolExecutor
    N, steps = 5, 8
    cases = []
    for k, (P, p, stream) in enumerate([(1_200_001, 0.02, "v1"), (900_003, 0.2, "v1"), (1_100_007, 0.01, "gap"),
                                         (1_200_001, 0.02, "gap")]):
        pop = (np.random.default_rng(170 + k).standard_normal((N, P)) * 0.02).astype(np.float32)
        cases.append((pop, [(0, P // 3, p), (P // 3, P - P // 3, p / 4)], stream))
    devs = [torch.from_numpy(c[0]).cuda() for c in cases]
    torch.cuda.synchronize()

    def work(k):
        pop, segs, which = cases[k]
        s = torch.cuda.Stream()
        cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
        with torch.cuda.stream(s):
            cnt.zero_()
            for step in range(steps):
                _fn(wash, which)(devs[k], None, segs, 9, step, cnt)
            dist = wash.wash_consensus_sqdist(devs[k])
            mean = wash.wash_average(devs[k])
            wash.papa_ema(devs[k], 0.9)
        s.synchronize()
        return int(cnt.item()), dist.cpu().numpy(), mean.cpu().numpy(), devs[k].cpu().numpy()

    print("four threads", flush=True)
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(work, range(4)))
    for k, (cnt, dist, mean, final) in enumerate(results):
        pop, segs, which = cases[k]
        ref = pop.copy()
        ref_cnt = sum(oracle.shuffle(ref, None, segs, 9, step, threads=8, stream=which) for step in range(steps))
        assert cnt == ref_cnt, k
        assert np.allclose(dist, oracle.consensus_sqdist(ref), rtol=1e-10, atol=0), k
        assert np.array_equal(_bits(mean), _bits(oracle.average(ref))), k
        oracle.ema(ref, 0.9)
        assert np.array_equal(_bits(final), _bits(ref)), k


def test_more_streams_than_workspaces(wash):
    """A process that keeps making streams: beyond 256 workspaces the library waits for the device and takes
    the workspaces of ordinary streams back.  Every call still reports the oracle's count, also on streams
    that held a workspace before the pool was recycled."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    N, P, nstreams = 4, 20_011, 300
    pop = distinct_population(N, P)
    segs = [(0, P, 0.1)]
    want = [oracle.shuffle(pop.copy(), None, segs, 21, step) for step in range(3)]
    d = torch.from_numpy(pop).cuda()
    handles = []
    for _ in range(nstreams):
        h = ctypes.c_void_p()
        assert hip.hipStreamCreate(ctypes.byref(h)) == 0
        handles.append(h)
    assert len({h.value for h in handles}) == nstreams
    print("many streams", flush=True)
    cnts = torch.zeros(nstreams, dtype=torch.int64, device="cuda")
    works = [d.clone() for _ in range(nstreams)]
    torch.cuda.synchronize()
    again = (0, 1, 2, 150, nstreams - 1)              # these streams call once more after the pool was recycled
    for k in list(range(nstreams)) + list(again):
        with torch.cuda.stream(torch.cuda.ExternalStream(handles[k].value)):
            wash.wash_shuffle(works[k], None, segs, 21, k % 3, cnts[k:k + 1])
    torch.cuda.synchronize()
    got = cnts.cpu().numpy()
    for h in handles:
        assert hip.hipStreamDestroy(h) == 0
    for k in range(nstreams):
        assert got[k] == want[k % 3] * (2 if k in again else 1), k


def test_error_paths_launch_nothing(wash):
    d = torch.zeros((2, 100), dtype=torch.float32, device="cuda")
    d.copy_(torch.arange(200, dtype=torch.float32, device="cuda").view(2, 100))
    keep = d.clone()
    for segs in ([(0, 101, 0.5)], [(50, 60, 0.5)], [(0, 10, 1.5)], [(0, 10, float("nan"))],
                 [(10, 10, 0.5), (0, 5, 0.5)], [(0, 10, 0.5), (9, 5, 0.5)]):
        with pytest.raises(wash.WashError):
            wash.wash_shuffle(d, None, segs, 0, 0)
    with pytest.raises(wash.WashError):
        wash.wash_shuffle(d, None, [(0, 100, 0.5)], 0, 1 << 32)
    with pytest.raises(wash.WashError):
        wash.wash_shuffle(d, d, [(0, 100, 0.5)], 0, 0)
    with pytest.raises(wash.WashError):
        wash.papa_ema(d, float("nan"))
    big = torch.zeros((33, 4), dtype=torch.float32, device="cuda")
    with pytest.raises(wash.WashError):
        wash.wash_average(big)
    torch.cuda.synchronize()
    assert torch.equal(d, keep)


def test_table_cache_eviction_shutdown_and_options(wash):
    # more distinct segment lists than the library caches (16): old tables are freed and rebuilt on demand
    N, P = 4, 20_000
    pop = distinct_population(N, P)
    lists = [[(0, 1000 + 37 * k, 0.3), (5000 + k, 9000, 0.1 + 0.01 * k)] for k in range(20)]
    expect = []
    for segs in lists:
        ref = pop.copy()
        oracle.shuffle(ref, None, segs, 2, 8)
        expect.append(ref)
    for rnd in range(2):
        for segs, ref in zip(lists, expect):
            for stream in STREAMS[:1] if rnd else STREAMS:
                if stream == "v1":
                    got, _, _ = _run_shuffle(wash, pop, None, segs, 2, 8, stream="v1")
                    assert np.array_equal(_bits(got), _bits(ref))
                else:
                    refg = pop.copy()
                    oracle.shuffle(refg, None, segs, 2, 8, stream="gap")
                    got, _, _ = _run_shuffle(wash, pop, None, segs, 2, 8, stream="gap")
                    assert np.array_equal(_bits(got), _bits(refg))
    torch.cuda.synchronize()
    wash.wash_shutdown()                                  # frees every cached table and the scratch buffer
    got, _, _ = _run_shuffle(wash, pop, None, lists[0], 2, 8)
    assert np.array_equal(_bits(got), _bits(expect[0]))
    d = torch.from_numpy(pop).cuda()
    assert np.allclose(wash.wash_consensus_sqdist(d).cpu().numpy(), oracle.consensus_sqdist(pop), rtol=1e-10)
    for opt, bad in ((wash.OPT_TILE_COORDS, 100), (wash.OPT_GAP_BLOCKS, 3), (wash.OPT_AVERAGE_CHUNKS, 5),
                     (wash.OPT_STREAM_MIN_BYTES, -1), (99, 0)):
        with pytest.raises(wash.WashError):
            wash.wash_set_option(opt, bad)
    for opt, vals in ((wash.OPT_GAP_BLOCKS, (1, 64, 0)), (wash.OPT_AVERAGE_CHUNKS, (8, 2, 0)),
                      (wash.OPT_STREAM_MIN_BYTES, (0, 256 << 20))):
        for v in vals:
            wash.wash_set_option(opt, v)
            avg = wash.wash_average(d).cpu().numpy()
            assert np.array_equal(avg, oracle.average(pop))


@pytest.mark.parametrize("gap", [False, True])
@pytest.mark.parametrize("N,P,nbuf", [(2, 1000, 1), (5, 40001, 3), (10, 123457, 4), (20, 65539, 3), (32, 9001, 4),
                                      (32, 9001, 2), (8, 700_003, 4), (1, 50, 4)])
def test_shuffle_states_moves_every_buffer_with_one_permutation(wash, N, P, nbuf, gap):
    # WASH+Opt with several optimizer states (Sec. 4): each buffer ends up as if shuffled alone
    # with the same (seed, step), because mask and permutation depend on those only
    print(f"case N={N} P={P} nbuf={nbuf} gap={gap}", flush=True)
    stream = "gap" if gap else "v1"
    bufs = [distinct_population(N, P, base=0x3F000000 + k * 0x01000000) for k in range(nbuf)]
    cut = [0, P // 7, P // 7 + 3, P // 2, P - 1, P]
    segs = [(cut[k], cut[k + 1] - cut[k], pk) for k, pk in enumerate([0.3, 1.0, 0.004, 0.08, 1.0])]
    refs, ref_cnt = [], None
    for b in bufs:
        r = b.copy()
        ref_cnt = oracle.shuffle(r, None, segs, 99, 12, stream=stream)
        refs.append(r)
    dev = [torch.from_numpy(b).cuda() for b in bufs]
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    wash.wash_set_option(wash.OPT_TILE_COORDS, 0)
    wash.wash_shuffle_states(dev, segs, 99, 12, gap_stream=gap, selected_count=cnt)
    torch.cuda.synchronize()
    assert int(cnt.item()) == ref_cnt
    for d, r in zip(dev, refs):
        assert np.array_equal(_bits(d.cpu().numpy()), _bits(r))
    if nbuf >= 2:
        # the two-buffer entry points are the same operation
        d0, d1 = torch.from_numpy(bufs[0]).cuda(), torch.from_numpy(bufs[1]).cuda()
        _fn(wash, stream)(d0, d1, segs, 99, 12, None)
        assert torch.equal(d0, dev[0]) and torch.equal(d1, dev[1])


def _random_case(rng):
    N = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 10, 16, 20, 31, 32]))
    P = int(rng.choice([1, 5, 63, 64, 255, 1023, 1024, 1025, 4097, 20_000, 70_001, 300_007]))
    nbuf = int(rng.integers(1, 5))
    gap = bool(rng.integers(0, 2))
    tile = 0 if gap else int(rng.choice([0, 0, 256, 512, 1280, 4096, 65536]))
    # a sorted list of non-overlapping segments with holes, empty segments and touching neighbours
    cuts = np.unique(rng.integers(0, P + 1, size=int(rng.integers(0, 24))))
    segs, k = [], 0
    while k + 1 < len(cuts):
        p = float(rng.choice([0.0, 1.0, 0.5, 0.25, 0.03, 0.004, 1e-4, rng.random()]))
        segs.append((int(cuts[k]), int(cuts[k + 1] - cuts[k]), p))
        if rng.random() < 0.2:
            segs.append((int(cuts[k + 1]), 0, 0.7))          # empty segment
        k += 1 if rng.random() < 0.7 else 2                   # sometimes leave a hole
    seed = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
    step = int(rng.choice([0, 1, 77, 2 ** 31, 2 ** 32 - 1]))
    return N, P, nbuf, gap, tile, segs, seed, step


@pytest.mark.parametrize("case", range(96))
def test_randomised_shapes_segments_buffers(wash, case):
    rng = np.random.default_rng(20_000 + case)
    N, P, nbuf, gap, tile, segs, seed, step = _random_case(rng)
    print(f"case {case}: N={N} P={P} nbuf={nbuf} gap={gap} tile={tile} nsegs={len(segs)} seed={seed:#x} step={step}",
          flush=True)
    stream = "gap" if gap else "v1"
    bufs = [rng.integers(0, 2 ** 32, size=(N, P), dtype=np.uint64).astype(np.uint32).view(np.float32) for _ in range(nbuf)]
    refs, ref_cnt = [], 0
    for b in bufs:
        r = b.copy()
        ref_cnt = oracle.shuffle(r, None, segs, seed, step, stream=stream)
        refs.append(r)
    dev = [torch.from_numpy(b.copy()).cuda() for b in bufs]
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    wash.wash_set_option(wash.OPT_TILE_COORDS, tile)
    try:
        wash.wash_shuffle_states(dev, segs, seed, step, gap_stream=gap, selected_count=cnt)
        torch.cuda.synchronize()
    finally:
        wash.wash_set_option(wash.OPT_TILE_COORDS, 0)
    assert int(cnt.item()) == ref_cnt
    for d, r in zip(dev, refs):
        assert np.array_equal(_bits(d.cpu().numpy()), _bits(r))
    # average and EMA of the first buffer's finite stand-in
    pop = distinct_population(N, P)
    d = torch.from_numpy(pop).cuda()
    assert np.array_equal(wash.wash_average(d).cpu().numpy(), oracle.average(pop))
    alpha = float(rng.choice([0.0, 0.5, 0.99, 1.0]))
    wash.papa_ema(d, alpha)
    ref = pop.copy()
    oracle.ema(ref, alpha)
    assert np.array_equal(_bits(d.cpu().numpy()), _bits(ref))


@pytest.mark.parametrize("dense", [1, 2])
@pytest.mark.parametrize("N,P,nbuf", [(2, 3, 1), (2, 255, 2), (3, 256, 3), (4, 257, 4), (5, 4097, 1), (10, 70_001, 2),
                                      (20, 33_333, 3), (31, 5000, 2), (32, 20_011, 1), (8, 1_000_003, 2),
                                      (15, 123_457, 4)])
@pytest.mark.parametrize("p", [0.002, 0.07, 0.5, 1.0])
def test_dense_and_sparse_paths_give_the_oracle_bits(wash, N, P, nbuf, p, dense):
    # the dense path (whole strips of all rows through LDS) and the sparse path (gathers of single
    # values) implement the same stream; option 2 forces the dense one wherever it fits, 1 forbids it
    print(f"case N={N} P={P} nbuf={nbuf} p={p} dense={dense}", flush=True)
    if P >= 64:
        a, b = P // 3, P // 2
        segs = [(0, a, p), (a + 5, b - a - 5, 1.0 if p < 1.0 else 0.3), (b, P - b - 1, p)]
    else:
        segs = [(0, P, p)]
    bufs = [distinct_population(N, P, base=0x3F000000 + k * 0x01000000) for k in range(nbuf)]
    refs, ref_cnt = [], 0
    for b_ in bufs:
        r = b_.copy()
        ref_cnt = oracle.shuffle(r, None, segs, 31, 6)
        refs.append(r)
    dev = [torch.from_numpy(b_).cuda() for b_ in bufs]
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    wash.wash_set_option(wash.OPT_TILE_COORDS, 0)
    wash.wash_set_option(wash.OPT_DENSE, dense)
    try:
        wash.wash_shuffle_states(dev, segs, 31, 6, selected_count=cnt)
        torch.cuda.synchronize()
    finally:
        wash.wash_set_option(wash.OPT_DENSE, 0)
    assert int(cnt.item()) == ref_cnt
    for d, r in zip(dev, refs):
        assert np.array_equal(_bits(d.cpu().numpy()), _bits(r))


def test_place_population_returns_ordinary_buffers(wash):
    """Buffers handed out by the placement helper (one arena, positions chosen by timing the library's own
    kernels) are plain contiguous [N, P] tensors: disjoint, inside the arena, and a shuffling step with
    momentum on them gives the oracle's bits."""
    N, P = 4, 70_000_003                      # 1.12 GB per buffer: large enough for the helper to probe
    segs = [(0, P // 2, 0.01), (P // 2, P - P // 2, 0.002)]
    bufs, info = wash.place_population(N, P, 2, segs, arena_bytes=6 << 30, grid_bytes=512 << 20)
    assert info["tuned"] and len(bufs) == 2 and len(info["probes_ms"]) == 2
    assert all(0 < b < info["arena_bytes"] for b in info["boundaries"])          # often none in so small an arena
    a0 = info["arena"].data_ptr()
    spans = []
    for b in bufs:
        assert b.shape == (N, P) and b.dtype == torch.float32 and b.is_contiguous() and b.data_ptr() % 256 == 0
        assert a0 <= b.data_ptr() and b.data_ptr() + N * P * 4 <= a0 + info["arena_bytes"]
        spans.append((b.data_ptr(), b.data_ptr() + N * P * 4))
    assert spans[0][1] <= spans[1][0] or spans[1][1] <= spans[0][0]
    gen = torch.Generator(device="cuda").manual_seed(5)
    bufs[0].normal_(0.0, 0.02, generator=gen)
    bufs[1].normal_(0.0, 1e-3, generator=gen)
    ref, refm = bufs[0].cpu().numpy(), bufs[1].cpu().numpy()
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    wash.wash_shuffle(bufs[0], bufs[1], segs, 3, 7, cnt)
    ref_cnt = oracle.shuffle(ref, refm, segs, 3, 7, threads=8)
    assert int(cnt.item()) == ref_cnt
    assert np.array_equal(_bits(bufs[0].cpu().numpy()), _bits(ref))
    assert np.array_equal(_bits(bufs[1].cpu().numpy()), _bits(refm))
    # small populations are placed back to back without probing
    small, sinfo = wash.place_population(3, 1000, 2, arena_bytes=1 << 20)
    assert not sinfo["tuned"] and small[0].shape == (3, 1000) and small[1].data_ptr() >= small[0].data_ptr() + 12000
